// Gate logits for bf16 tokens on the bf16 matrix cores, exact to fp32 level (paper Sec. 5.4: the gate
// is the first of the three MoE components; its matrix product is small but sits on the critical path
// before every other kernel of the layer).
//
//   logits[t,e] = bg[e] + sum_i x[t,i] Wg[i,e],   x bf16, Wg and bg fp32, fp32 accumulation.
//
// An fp32 weight is the exact sum of three bf16 numbers (3 x 8 significant bits = the 24 of fp32):
// Wg = hi + mid + lo with hi = bf16(Wg), mid = bf16(Wg - hi), lo = bf16(Wg - hi - mid).  A bf16 token
// value times a bf16 piece is exact in fp32, so three v_mfma_f32_16x16x32_bf16 per tile give the same
// sum of exact products as an fp32 multiply-add chain, at a fraction of the fp32 matrix-core time.
//
// Two kernels:
//   * wg_split_kernel writes the three pieces as ready-made MFMA B fragments (1 KB each: lane l holds
//     k = 8*(l/16)..+7 of expert column l%16), ordered [k-block][expert tile][piece];
//   * gate_logits_bf16_kernel: a work-group owns a tile of 16*MA tokens x 16*NE experts; its four waves
//     split the k-blocks (wave w takes blocks w, w+4, ...) and each computes the whole tile for its
//     blocks, so no operand byte is fetched twice by a work-group; the four partial tiles are summed
//     through LDS in fixed order.  Every operand fragment is one 16-byte load per lane from global
//     memory straight into registers, several k-blocks ahead; no LDS traffic and no barrier in the
//     loop.  The kernel is bound by the rate at which a CU can pull operands out of L2 (about
//     50-70 GB/s per CU measured, direct-to-LDS loads no faster), so the tile is chosen to minimise
//     bytes per CU while still giving every CU a work-group.
// Requires d_model to be a multiple of 32 and at most 128 experts; other shapes use the fp32 kernel.
#include "moe_internal.h"

namespace moe {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kKB = 32;                  // k per MFMA
constexpr int kFragElems = 512;          // bf16 elements of one fragment (64 lanes x 8)
// KB k-blocks x ET expert tiles x 3 pieces; one thread per (k-block, expert tile, lane)
__global__ __launch_bounds__(256) void wg_split_kernel(const float* __restrict__ Wg, uint16_t* __restrict__ frags, int d,
                                                       int E, int KB, int ET) {
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)KB * ET * 64) return;
    const int lane = (int)(idx & 63);
    const long long fe = idx >> 6;
    const int et = (int)(fe % ET), kb = (int)(fe / ET);
    const int n = et * 16 + (lane & 15);
    const int k0 = kb * kKB + (lane >> 4) * 8;
    uint16_t p[3][8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int k = k0 + j;
        const float w = (k < d && n < E) ? Wg[(size_t)k * E + n] : 0.f;
        const uint16_t hi = f32_to_bf16(w);
        const float r1 = w - bf16_to_f32(hi);                 // exact
        const uint16_t mid = f32_to_bf16(r1);
        const float r2 = r1 - bf16_to_f32(mid);               // exact
        p[0][j] = hi; p[1][j] = mid; p[2][j] = f32_to_bf16(r2);
    }
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        uint4 o;
        o.x = p[q][0] | ((uint32_t)p[q][1] << 16); o.y = p[q][2] | ((uint32_t)p[q][3] << 16);
        o.z = p[q][4] | ((uint32_t)p[q][5] << 16); o.w = p[q][6] | ((uint32_t)p[q][7] << 16);
        *reinterpret_cast<uint4*>(frags + ((size_t)(fe * 3 + q)) * kFragElems + lane * 8) = o;
    }
}

template <int MA, int NE> struct GateCfg {
    static constexpr int PER = MA + 3 * NE;                                  // 16-byte loads per lane and k-block
    static constexpr int D = 48 / PER < 3 ? 3 : (48 / PER > 6 ? 6 : 48 / PER);   // k-blocks held in registers
};

// tile: MA token tiles (16 tokens each) x NE expert tiles; blockIdx.x = token tile, blockIdx.y = expert group;
// ET = expert tiles in all (fragment stride)
template <int MA, int NE>
__global__ __launch_bounds__(256) void gate_logits_bf16_kernel(const uint16_t* __restrict__ x,
                                                               const uint16_t* __restrict__ frags,
                                                               const float* __restrict__ bg, float* __restrict__ logits,
                                                               int T, int d, int E, int ET) {
    constexpr int D = GateCfg<MA, NE>::D, PER = GateCfg<MA, NE>::PER, WE = 1, WK = 4;
    __shared__ f32x4_t red[(WK - 1) * WE * MA * NE * 64];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int we = 0, wk = w;
    const int et0 = blockIdx.y * NE;                              // first expert tile of this work-group
    const int t0 = blockIdx.x * (16 * MA);
    const int KB = d / kKB;
    const int nkb = KB > wk ? (KB - wk + WK - 1) / WK : 0;        // k-blocks wk, wk + WK, ... of this wave

    f32x4_t acc[MA][NE];
#pragma unroll
    for (int m = 0; m < MA; ++m)
#pragma unroll
        for (int e = 0; e < NE; ++e) acc[m][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    if (nkb > 0) {
        // per-lane sources: token rows (clamped into the matrix: their results are never stored) and fragments
        const uint16_t* a_src[MA];
#pragma unroll
        for (int m = 0; m < MA; ++m)
            a_src[m] = x + (size_t)min(t0 + 16 * m + (lane & 15), T - 1) * d + (lane >> 4) * 8;
        const uint16_t* b_src = frags + (size_t)et0 * 3 * kFragElems + lane * 8;
        const size_t b_kb_stride = (size_t)ET * 3 * kFragElems;

        // Operands of one k-block: A fragments straight from the token rows, B fragments as stored.  The
        // loads and the waits for them are written by hand: the compiler's own bookkeeping of outstanding
        // loads gives up at the back edge of a rotating register ring and waits for nearly all of them.
        // Loads return in order, so "all but the newest (D-1)*PER" means the oldest k-block has arrived;
        // the wait names that block's registers as operands, which orders every use after it.
        struct Stage {
            u32x4_t r[PER];                                       // MA token fragments, then 3*NE weight fragments
        };
        auto load = [&](Stage& st, int step) {
            const int kb = wk + min(step, nkb - 1) * WK;          // past the end: harmless re-read, dropped
#pragma unroll
            for (int m = 0; m < MA; ++m)
                asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(st.r[m]) : "v"(a_src[m] + kb * kKB) : "memory");
            const uint16_t* bp = b_src + (size_t)kb * b_kb_stride;
#pragma unroll
            for (int i = 0; i < 3 * NE; ++i)
                asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(st.r[MA + i]) : "v"(bp + i * kFragElems) : "memory");
        };
        auto arrived = [&](Stage& st) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                if (i == 0) asm volatile("s_waitcnt vmcnt(%1)" : "+v"(st.r[i]) : "n"((D - 1) * PER) : "memory");
                else asm volatile("" : "+v"(st.r[i]));
            }
        };
        // `live` is false for the steps past the last k-block of a partly filled round: their token
        // fragments are replaced by zeros, so the loop needs no branches.
        auto mma = [&](const Stage& st, bool live) {
            bf16x8_t af[MA];
#pragma unroll
            for (int m = 0; m < MA; ++m) {
                const u32x4_t v = st.r[m];
                const u32x4_t z = {live ? v.x : 0u, live ? v.y : 0u, live ? v.z : 0u, live ? v.w : 0u};
                af[m] = __builtin_bit_cast(bf16x8_t, z);
            }
#pragma unroll
            for (int e = 0; e < NE; ++e)
#pragma unroll
                for (int q = 0; q < 3; ++q)
#pragma unroll
                    for (int m = 0; m < MA; ++m)
                        acc[m][e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[m], __builtin_bit_cast(bf16x8_t, st.r[MA + e * 3 + q]),
                                                                            acc[m][e], 0, 0, 0);
        };

        Stage st[D];
#pragma unroll
        for (int s = 0; s < D - 1; ++s) load(st[s], s);
        for (int s0 = 0; s0 < nkb; s0 += D) {
#pragma unroll
            for (int i = 0; i < D; ++i) {
                load(st[(i + D - 1) % D], s0 + i + D - 1);
                arrived(st[i]);
                mma(st[i], s0 + i < nkb);
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // the loads fetched ahead past the end
    }

    // ---- sum over the k-splits (fixed order), then bias and store ------------------------------------
    if (WK > 1) {
        if (wk > 0) {
#pragma unroll
            for (int m = 0; m < MA; ++m)
#pragma unroll
                for (int e = 0; e < NE; ++e) red[((((wk - 1) * WE + we) * MA + m) * NE + e) * 64 + lane] = acc[m][e];
        }
        __syncthreads();
        if (wk == 0) {
#pragma unroll
            for (int k = 1; k < WK; ++k)
#pragma unroll
                for (int m = 0; m < MA; ++m)
#pragma unroll
                    for (int e = 0; e < NE; ++e) acc[m][e] += red[((((k - 1) * WE + we) * MA + m) * NE + e) * 64 + lane];
        }
    }
    if (wk == 0) {
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const int col = (et0 + e) * 16 + (lane & 15);     // D: column lane%16, rows 4*(lane/16)+r
            if (col >= E) continue;
            const float b = bg ? bg[col] : 0.f;
#pragma unroll
            for (int m = 0; m < MA; ++m)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int t = t0 + 16 * m + 4 * (lane >> 4) + r;
                    if (t < T) logits[(size_t)t * E + col] = acc[m][e][r] + b;
                }
        }
    }
}

template <int MA, int NE>
int launch_cfg(const uint16_t* x, const uint16_t* frags, const float* bg, float* logits, int T, int d, int E, int ET,
               hipStream_t s) {
    const dim3 grid((T + 16 * MA - 1) / (16 * MA), ET / NE);
    hipLaunchKernelGGL((gate_logits_bf16_kernel<MA, NE>), grid, dim3(256), 0, s, x, frags, bg, logits, T, d, E, ET);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// expert tiles, padded to 1, 2, 4 or 8
int padded_expert_tiles(int E) {
    const int et = (E + 15) / 16;
    return et <= 1 ? 1 : et <= 2 ? 2 : et <= 4 ? 4 : 8;
}

}  // namespace

bool gate_bf16_supported(int d, int E) { return d % kKB == 0 && d >= kKB && E >= 1 && E <= 128; }

size_t gate_bf16_ws_bytes(int d, int E) {
    if (!gate_bf16_supported(d, E)) return 0;
    return (size_t)(d / kKB) * padded_expert_tiles(E) * 3 * kFragElems * sizeof(uint16_t);
}

int launch_gate_logits_bf16(const void* x, const float* Wg, const float* bg, float* logits, int T, int d, int E,
                            void* frag_ws, hipStream_t s) {
    if (!gate_bf16_supported(d, E) || !frag_ws) return MOE_ERR_INVALID_ARG;
    const int KB = d / kKB, ET = padded_expert_tiles(E);
    uint16_t* frags = static_cast<uint16_t*>(frag_ws);
    const long long threads = (long long)KB * ET * 64;
    hipLaunchKernelGGL(wg_split_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, Wg, frags, d, E, KB, ET);
    if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
    const uint16_t* xb = static_cast<const uint16_t*>(x);
    // Largest tile (fewest operand bytes per output) that still gives every CU a work-group; when even
    // the smallest tile cannot (few tokens), the smallest one: most work-groups, least time per CU.
    int MA = 2, NE = 1;
    bool found = false;
    for (int ma = 4; ma >= 2 && !found; ma -= 2)
        for (int ne = ET < 4 ? ET : 4; ne >= 1 && !found; ne /= 2)
            if ((long long)((T + 16 * ma - 1) / (16 * ma)) * (ET / ne) >= 256) { MA = ma; NE = ne; found = true; }
#define MOE_GATE_CASE(ma, ne) \
    if (MA == ma && NE == ne) return launch_cfg<ma, ne>(xb, frags, bg, logits, T, d, E, ET, s)
    MOE_GATE_CASE(4, 4); MOE_GATE_CASE(4, 2); MOE_GATE_CASE(4, 1);
    MOE_GATE_CASE(2, 4); MOE_GATE_CASE(2, 2); MOE_GATE_CASE(2, 1);
#undef MOE_GATE_CASE
    return MOE_ERR_INVALID_ARG;
}

}  // namespace moe
