// Internal declarations shared by the library's translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe.h"

namespace moe {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kRouteTokens = 256;    // tokens per block in the routing kernels

// Work-group barrier that orders LDS traffic only.  __syncthreads() also drains every outstanding
// global load (on gfx9 loads and stores share one counter), which would empty the register prefetch
// queues the streaming kernels depend on at each barrier.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- bf16 <-> f32 on raw 16-bit patterns -------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t v) {
    return __uint_as_float(static_cast<uint32_t>(v) << 16);
}
// round to nearest even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}
// two fp32 -> packed bf16, round to nearest even, on the hardware converter (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const bf16x2_t v = {static_cast<__bf16>(lo), static_cast<__bf16>(hi)};
    return __builtin_bit_cast(uint32_t, v);
}

// gelu_tanh(z) = 0.5 z (1 + tanh(u)), u = sqrt(2/pi) (z + 0.044715 z^3).  Since tanh(u) = 2 sigmoid(2u) - 1 this is
// z sigmoid(2u) = z / (1 + exp(-2u)): one exp2 and one rcp on the hardware units, five multiply-adds.
__device__ __forceinline__ float gelu_tanh(float z) {
    const float z2 = z * z;
    // -2u log2(e) = z (c1 + c3 z^2)
    const float e = __builtin_amdgcn_exp2f(z * fmaf(z2, -0.10294324f, -2.3022082f));
    return z * __builtin_amdgcn_rcpf(1.0f + e);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {
    static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = f32_to_bf16(v); }
};

// ---- launchers (each returns MOE_OK or MOE_ERR_HIP) ---------------------------------------

// logits[t,e] = bg[e] + sum_i x[t,i] Wg[i,e]
int launch_gate_logits(const void* x, int dtype, const float* Wg, const float* bg, float* logits,
                       int T, int d, int E, hipStream_t s);

// the same for bf16 tokens on the bf16 matrix cores (fp32 weights split into three bf16 pieces, exact);
// frag_ws: gate_bf16_ws_bytes(d, E) bytes of scratch for the split weights, rewritten by every call
bool gate_bf16_supported(int d, int E);
size_t gate_bf16_ws_bytes(int d, int E);
int launch_gate_logits_bf16(const void* x, const float* Wg, const void* Wg_packed, const float* bg, float* logits, int T,
                            int d, int E, void* frag_ws, hipStream_t s);
// the split weights written once into a caller-owned buffer of gate_bf16_ws_bytes(d, E) bytes (Wg_packed above)
int launch_pack_gate(const float* Wg, void* packed, int d, int E, hipStream_t s);

// logits, top-k, gate weights, tile-local ranks (parked in slot_idx) and per-tile histograms for bf16 tokens;
// launch_route_finalize(..., *tokens_per_hist, ..., *hist_out) completes the routing.
// scratch as for launch_route; logits is always written
bool gate_bf16_fused_supported(int T, int d, int E);
int launch_gate_bf16_fused(const void* x, const float* Wg, const void* Wg_packed, const float* bg, float* logits, int T,
                           int d, int E, int k, int32_t* expert_idx, int32_t* slot_idx, float* gate_w, void* frag_ws,
                           int32_t* scratch, int* tokens_per_hist, const int32_t** hist_out, hipStream_t s);

// the whole gate of at most 256 bf16 tokens in one launch (logits by many work-groups, routing by the last one);
// flags: kGateFlagInts uint32 of scratch, epoch: a value no earlier call left there
constexpr int kGateFlagInts = 64;
bool gate_decode_supported(int T, int d, int E);
int launch_gate_decode(const void* x, const float* Wg, const void* Wg_packed, const float* bg, float* logits, int T, int d,
                       int E, int k, int C, int32_t* expert_idx, int32_t* slot_idx, float* gate_w, int32_t* expert_rows,
                       int32_t* slot_token, int32_t* expert_order, void* frag_ws, uint32_t* flags, uint32_t epoch,
                       hipStream_t s);

// number of int32 the routing kernels need as scratch
size_t route_scratch_ints(int T, int E, int k);

// softmax + top-k + capacity slots from fp32 logits
int launch_route(const float* logits, int T, int E, int k, int C,
                 int32_t* expert_idx, int32_t* slot_idx, float* gate_w,
                 int32_t* expert_rows, int32_t* slot_token, int32_t* expert_order /* [2E + 2] or nullptr */,
                 int32_t* scratch, hipStream_t s);

// second routing kernel alone: hist = one histogram [k][E] per block of TB tokens (TB divides 256) with the
// block-local ranks parked in slot_idx
int launch_route_finalize(int T, int E, int k, int C, int TB, const int32_t* expert_idx, int32_t* slot_idx,
                          int32_t* expert_rows, int32_t* slot_token, int32_t* expert_order, const int32_t* hist,
                          hipStream_t s);

// the two launch orders of the experts (2E + 2 ints: see write_expert_order) from the row counts alone
int launch_expert_order(const int32_t* expert_rows, int E, int C, int32_t* order, hipStream_t s);

int launch_dispatch(const void* x, int dtype, const int32_t* slot_token, const int32_t* expert_rows,
                    void* xe, int E, int C, int d, hipStream_t s);

int launch_combine(const void* ye, int dtype, const int32_t* expert_idx, const int32_t* slot_idx,
                   const float* gate_w, const void* addend, void* out,
                   int T, int k, int C, int d, hipStream_t s);

// Grouped GEMM  out[g, r, :] = epi( A[row(g,r), :] . B[g] + bias[g] )  for r < rows(g).
struct GemmArgs {
    const void* A;            // activations, row-major, leading dimension K
    const void* B;            // [G, K, N] weights
    const void* bias;         // [G, N] or nullptr
    void* out;                // row-major, leading dimension N
    const int32_t* rows;      // [G] device row counts, or nullptr -> fixed_rows for every group
    const int32_t* row_map;   // [G, max_rows] A-row index per (g, r) (negative = skip), or nullptr
    int32_t fixed_rows;
    int32_t max_rows;         // upper bound of rows(g): sizes the grid
    int32_t G, K, N;
    int64_t a_group_stride;   // in rows; A-row of (g, r) = g*a_group_stride + r when row_map == nullptr
    int64_t o_group_stride;   // in rows; out-row of (g, r) = g*o_group_stride + r
    int32_t gelu;             // 1: gelu_tanh after the bias
    int32_t dtype;            // element type of A, B, bias, out
};
int launch_gemm_simple(const GemmArgs& a, hipStream_t s);

// bf16 MFMA weight-streaming grouped GEMM (ffn_mfma.hip).
enum WsEpilogue {
    EPI_STORE = 0,    // out[g*o_group_stride + r, :] = acc + bias
    EPI_GELU = 1,     // out[g*o_group_stride + r, :] = gelu_tanh(acc + bias)
    EPI_SCATTER = 2,  // out[token(g,r), :] = gate_w[token, 0] * (acc + bias)        (top-1 combine)
    EPI_COMBINE = 3,  // out[r, :] = acc + bias + sum_j keep_j g_j ye[e_j, slot_j, :]   (dense branch + combine)
    EPI_PARTIAL = 4   // partial[ks, g*o_group_stride + r, :] = acc   (split-K, fp32, no bias)
};
struct WsGemmArgs {
    const uint16_t* A;         // activations, leading dimension K
    const uint16_t* B;         // [G, K, N], or the same weights in fragment order (packed != 0)
    int32_t packed;            // B is [G, ceil(K/32), ceil(N/128), 8, 64, 8] as written by launch_pack_weights
    const uint16_t* bias;      // [G, N] or nullptr
    const int32_t* rows;       // [G] device row counts or nullptr -> fixed_rows
    const int32_t* order;      // [G + 1] groups in launch order (busiest first), then the tile-dealing flag; or nullptr -> identity
    const int32_t* row_map;    // [G, map_stride]: A-row of (g, r), or nullptr -> g*a_group_stride + r
    int32_t fixed_rows, max_rows, map_stride;
    int32_t G, K, N;
    long long a_group_stride;
    uint16_t* out;             // leading dimension N
    long long o_group_stride;
    int32_t ksplit;            // >= 1; > 1 only with EPI_PARTIAL
    int32_t spread;            // tiled kernel, tile dealing: 0 = as order[G] says, 1 = always spread, 2 = never
    float* partial;            // [ksplit, partial_rows, N]
    long long partial_rows;
    // EPI_SCATTER
    const int32_t* scatter_map;    // [G, scatter_stride] token per expert row
    int32_t scatter_stride;
    const int32_t* zero_slot_idx;  // [T*top_k]: rows t with zero_slot_idx[t*top_k] < 0 are zero-filled (top_k == 1)
    int32_t T;
    // EPI_SCATTER / EPI_COMBINE
    const float* gate_w;           // [T, top_k]
    int32_t top_k;
    const uint16_t* ye;            // [E, C, N]
    const int32_t* expert_idx;     // [T, top_k]
    const int32_t* slot_idx;       // [T, top_k]
    int32_t C;
};
bool wsgemm_supported(int K, int N);
void wsgemm_pick_tile(int max_rows, int G, int N, int* MT, int* NW);
int launch_wsgemm(const WsGemmArgs& a, int epi, int MT, int NW, int NBUF, hipStream_t s);
int wsgemm_chunk_k(int MT);

// Tiled variant for groups with many rows (ffn_tile.hip); same arguments, ksplit must be 1.
int launch_tgemm(const WsGemmArgs& a, int epi, hipStream_t s);
// two grouped products in one launch (same K, N, packing, epilogue; both with 256-row tiles): twice the tiles
bool tgemm_pair_fusable(const WsGemmArgs& a, const WsGemmArgs& b);
int launch_tgemm_pair(const WsGemmArgs& a, const WsGemmArgs& b, int epi, hipStream_t s);
bool tgemm_supported(int K, int N);   // K a multiple of 32   // k-extent of one LDS chunk = granularity of split-K

// Weights in the fragment order of v_mfma_f32_16x16x32_bf16's second operand (pack.hip).  Element (k, n) of group g
// goes to  ((((g*KB + k/32)*NG + n/128)*8 + n%8)*64 + (k%32/8)*16 + (n%128)/8)*8 + k%8,  KB = ceil(K/32),
// NG = ceil(N/128); positions past K or N hold zeros.  A lane's 16 bytes are then 8 consecutive k of one column,
// a wave's 1 KB is one fragment, and fragment j of a 128-column group holds columns 8c + j (c = lane % 16): a lane's
// 8 accumulators of a row are 8 consecutive columns.
inline size_t packed_weight_elems(int G, int K, int N) {
    return (size_t)G * ((K + 31) / 32) * ((N + 127) / 128) * 4096;
}
int launch_pack_weights(const uint16_t* W, uint16_t* packed, int G, int K, int N, hipStream_t s);

// Sums split-K partials in split order, adds the bias and finishes like EPI_STORE (scatter_map ==
// nullptr) or EPI_SCATTER (scatter_map given; also zero-fills rows of dropped tokens).
struct SplitKReduceArgs {
    const float* partial;      // [ksplit, G*group_stride, N]
    int32_t ksplit, G, N;
    long long group_stride;
    const int32_t* rows;       // [G], or nullptr: max_rows for every group
    int32_t max_rows;
    const uint16_t* bias;      // [G, N] or nullptr
    uint16_t* out;
    const int32_t* scatter_map;
    const float* gate_w;
    int32_t top_k;
    const int32_t* zero_slot_idx;
    int32_t T;
};
int launch_splitk_reduce(const SplitKReduceArgs& a, hipStream_t s);

// ---- the non-expert half of a decoder block, one decode step (block.hip) --------------------------------------
int launch_add_layernorm(const uint16_t* x, const uint16_t* r /* or nullptr */, const float* gamma, const float* beta,
                         uint16_t* sum_out /* x + r, or nullptr */, uint16_t* y, int T, int d, float eps, hipStream_t s);
int launch_add_rows(const uint16_t* a, const uint16_t* b, uint16_t* out, long long n, hipStream_t s);
bool attn_supported(int d, int H);
size_t attn_partial_floats(int T, int H, int dh, int Lmax);
int launch_attn_decode(const uint16_t* qkv, uint16_t* cache_k, uint16_t* cache_v, const int32_t* pos, float* partial,
                       uint16_t* attn, int T, int H, int dh, int Lmax, hipStream_t s);

}  // namespace moe
