// Gating kernels for gfx950: gate logits, softmax + top-k, and the capacity
// prefix count that gives every (token, choice) its row inside its expert.
//
// Paper Sec. 5.4: the gating function is top-k, a cumulative sum that yields the
// position of each token among those processed by its expert (bounded by the
// capacity), and a scatter, all driven by a dense token-to-expert mapping table
// instead of one-hot masks.  The paper parallelises the cumsum with a Blelloch
// scan on its hardware; here the count is done with 64-wide wavefront ballots
// (rank inside a wave), a per-block histogram and a prefix over blocks, which
// is deterministic (no atomics) and needs two small launches.
#include <cstdlib>

#include "route_device.h"

namespace moe {

// ------------------------------------------------------------------------------------------
// logits[t,e] = bg[e] + sum_i x[t,i] Wg[i,e]     fp32 in, fp32 accumulate, on the fp32 matrix cores
//
// v_mfma_f32_16x16x4_f32: a wave owns 16 tokens x 64 experts (4 accumulator tiles).  Per 32-wide
// k-chunk a lane reads 8 consecutive k of its token row straight from global memory (16 bytes of
// bf16, widened by a shift, or 32 bytes of fp32) and feeds them to 8 successive MFMAs; lane group
// g = lane/16 therefore holds k = 8g + j in MFMA j, and reads the matching Wg row 8g + j from an
// LDS tile kept in Wg's own [k][e] layout (columns rotated by 16 per 8 rows so that the four lane
// groups hit different banks).  No transposition anywhere.  A work-group is WT x WE x WK waves:
// token tiles x 64-expert tiles x k-splits (the k-split, summed through LDS in fixed order, keeps
// every CU busy when there are few tokens).
// ------------------------------------------------------------------------------------------
typedef float f32x4_t __attribute__((ext_vector_type(4)));
constexpr int kGK = 32;      // k-rows per step
constexpr int kGPD = 3;      // steps of operands kept in flight in registers

// 8 consecutive k of a token row as raw 16-byte words (bf16: one word; fp32: two), widened later
template <typename XT> struct XRaw;
template <> struct XRaw<uint16_t> {
    uint4 w;
    __device__ __forceinline__ void load(const uint16_t* row, int k, int d) {
        w = *reinterpret_cast<const uint4*>(row + min(k, d - 8));
    }
    __device__ __forceinline__ void widen(int k, int d, float (&v)[8]) const {
        const bool in = k < d;                              // d % 8 == 0: all eight or none
        const uint4 a = in ? w : make_uint4(0, 0, 0, 0);
        v[0] = __uint_as_float(a.x << 16); v[1] = __uint_as_float(a.x & 0xffff0000u);
        v[2] = __uint_as_float(a.y << 16); v[3] = __uint_as_float(a.y & 0xffff0000u);
        v[4] = __uint_as_float(a.z << 16); v[5] = __uint_as_float(a.z & 0xffff0000u);
        v[6] = __uint_as_float(a.w << 16); v[7] = __uint_as_float(a.w & 0xffff0000u);
    }
};
template <> struct XRaw<float> {
    float4 lo, hi;
    __device__ __forceinline__ void load(const float* row, int k, int d) {
        lo = *reinterpret_cast<const float4*>(row + min(k, d - 4));
        hi = *reinterpret_cast<const float4*>(row + min(k + 4, d - 4));
    }
    __device__ __forceinline__ void widen(int k, int d, float (&v)[8]) const {
        const bool in0 = k < d, in1 = k + 4 < d;            // d % 4 == 0
        v[0] = in0 ? lo.x : 0.f; v[1] = in0 ? lo.y : 0.f; v[2] = in0 ? lo.z : 0.f; v[3] = in0 ? lo.w : 0.f;
        v[4] = in1 ? hi.x : 0.f; v[5] = in1 ? hi.y : 0.f; v[6] = in1 ? hi.z : 0.f; v[7] = in1 ? hi.w : 0.f;
    }
};

// VEC = 4: E is a multiple of 4 and Wg rows are read as float4; VEC = 1: any E, scalar reads.
// FULL: d is a multiple of 32*WK and E of the work-group's expert width, so no operand is ever out
// of range and the selects that zero them disappear from the loop.
template <typename XT, int WT, int WE, int WK, int VEC, bool FULL>
__global__ __launch_bounds__(256) void gate_logits_kernel(const XT* __restrict__ x, const float* __restrict__ Wg,
                                                          const float* __restrict__ bg, float* __restrict__ logits,
                                                          int T, int d, int E) {
    static_assert(WT * WE * WK == 4, "four waves");
    constexpr int EN = WE * 64;                       // experts per pass of the work-group
    constexpr int TM = WT * 16;                       // tokens per work-group
    constexpr int NB = WK * kGK * EN / 256 / VEC;     // Wg words staged per thread and step
    __shared__ __attribute__((aligned(16))) float Bs[WK][kGK][EN];
    __shared__ float red[WK > 1 ? (WK - 1) * WT * WE * 16 * 64 : 1];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int wk = w % WK, we = (w / WK) % WE, wt = w / (WK * WE);
    const int t0 = blockIdx.x * TM + wt * 16;
    const XT* xrow = x + (size_t)min(t0 + n, T - 1) * d;           // A row of this lane (clamped, not stored)

    // k is cut into 32-row chunks; split s of the WK k-splits owns chunks [s*cper, (s+1)*cper).
    // In step c the work-group stages chunk s*cper + c of every split and each wave multiplies its
    // own split's tile.  Operands of the next kGPD steps are always in flight: all loads are
    // unconditional (addresses clamped, values zeroed when consumed), so no branch separates a load
    // from its use and the compiler can count outstanding loads exactly.
    const int chunks = (d + kGK - 1) / kGK;
    const int cper = (chunks + WK - 1) / WK;

    for (int e0 = 0; e0 < E; e0 += EN) {
        f32x4_t acc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        typedef float bword_t __attribute__((ext_vector_type(VEC)));
        bword_t breg[kGPD][NB];
        XRaw<XT> areg[kGPD];

        auto b_load = [&](bword_t (&dst)[NB], int c) {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int p = (tid + i * 256) * VEC;
                const int s = p / (kGK * EN), kk = (p / EN) % kGK, ee = p % EN;
                const int k = min((s * cper + c) * kGK + kk, d - 1), e = min(e0 + ee, E - VEC);
                dst[i] = *reinterpret_cast<const bword_t*>(Wg + (size_t)k * E + e);
            }
        };
        auto b_store = [&](const bword_t (&src)[NB], int c) {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int p = (tid + i * 256) * VEC;
                const int s = p / (kGK * EN), kk = (p / EN) % kGK, ee = p % EN;
                bword_t v = src[i];
                if (!FULL) {
                    const bool in = (s * cper + c) * kGK + kk < d && e0 + ee < E && c < cper;
#pragma unroll
                    for (int q = 0; q < VEC; ++q) v[q] = in ? v[q] : 0.f;
                }
                // columns rotated by 16 per 8 rows: the four lane groups of a B read hit distinct banks
                *reinterpret_cast<bword_t*>(&Bs[s][kk][(ee + 16 * (kk >> 3)) % EN]) = v;
            }
        };
        // one step: tile of chunk c to LDS, refill the register slot kGPD steps ahead, multiply
        auto step = [&](bword_t (&bslot)[NB], XRaw<XT>& aslot, int c) {
            lds_barrier();                            // the previous step has finished reading the tile
            b_store(bslot, c);
            float av[8];
            const int ka = (wk * cper + c) * kGK + 8 * g;
            aslot.widen(FULL ? 0 : (c < cper ? ka : d), d, av);
            lds_barrier();
            b_load(bslot, c + kGPD);
            aslot.load(xrow, (wk * cper + c + kGPD) * kGK + 8 * g, d);
            __builtin_amdgcn_sched_barrier(0);
            float bv[8][4];
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) bv[j][nt] = Bs[wk][8 * g + j][(we * 64 + nt * 16 + n + 16 * g) % EN];
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[j], bv[j][nt], acc[nt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        };

#pragma unroll
        for (int s = 0; s < kGPD; ++s) {
            b_load(breg[s], s);
            areg[s].load(xrow, (wk * cper + s) * kGK + 8 * g, d);
        }
        int c0 = 0;
        for (; c0 + kGPD <= cper; c0 += kGPD) {
#pragma unroll
            for (int s = 0; s < kGPD; ++s) step(breg[s], areg[s], c0 + s);
        }
        if (c0 < cper) step(breg[0], areg[0], c0);
        if (c0 + 1 < cper) step(breg[1], areg[1], c0 + 1);

        if (WK > 1) {
            __syncthreads();
            float* mine = red + ((size_t)((wk - 1) * WT * WE + wt * WE + we) * 16) * 64;
            if (wk > 0) {
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) mine[(nt * 4 + r) * 64 + lane] = acc[nt][r];
            }
            __syncthreads();
            if (wk == 0) {
                for (int s = 1; s < WK; ++s) {
                    const float* o = red + ((size_t)((s - 1) * WT * WE + wt * WE + we) * 16) * 64;
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[nt][r] += o[(nt * 4 + r) * 64 + lane];
                }
            }
        }
        if (wk == 0) {
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                const int e = e0 + we * 64 + nt * 16 + n;
                if (e >= E) continue;
                const float b = bg ? bg[e] : 0.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int t = t0 + 4 * g + r;
                    if (t < T) logits[(size_t)t * E + e] = acc[nt][r] + b;
                }
            }
        }
        __syncthreads();      // the next expert pass restages the tile
    }
}

template <typename XT>
static int launch_logits_t(const XT* x, const float* Wg, const float* bg, float* logits, int T, int d, int E,
                           hipStream_t s) {
#define MOE_LOGITS_CASE(WT, WE, WK)                                                                          \
    do {                                                                                                     \
        const dim3 grid((T + WT * 16 - 1) / (WT * 16));                                                      \
        const bool full = d % (kGK * WK) == 0 && E % (WE * 64) == 0;                                         \
        if (full)                                                                                            \
            hipLaunchKernelGGL((gate_logits_kernel<XT, WT, WE, WK, 4, true>), grid, dim3(256), 0, s, x, Wg, bg,     \
                               logits, T, d, E);                                                             \
        else if (E % 4 == 0)                                                                                 \
            hipLaunchKernelGGL((gate_logits_kernel<XT, WT, WE, WK, 4, false>), grid, dim3(256), 0, s, x, Wg, bg,    \
                               logits, T, d, E);                                                             \
        else                                                                                                 \
            hipLaunchKernelGGL((gate_logits_kernel<XT, WT, WE, WK, 1, false>), grid, dim3(256), 0, s, x, Wg, bg,    \
                               logits, T, d, E);                                                             \
    } while (0)
    const bool wide = E > 64;          // 128 experts per pass, else 64
    const bool few = T <= 1024;        // few tokens: waves go to k-splits, not token tiles
    if (wide) {
        if (few) MOE_LOGITS_CASE(1, 2, 2);
        else MOE_LOGITS_CASE(2, 2, 1);
    } else {
        if (few) MOE_LOGITS_CASE(1, 1, 4);
        else MOE_LOGITS_CASE(4, 1, 1);
    }
#undef MOE_LOGITS_CASE
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int launch_gate_logits(const void* x, int dtype, const float* Wg, const float* bg, float* logits, int T, int d,
                       int E, hipStream_t s) {
    if (dtype == MOE_F32) return launch_logits_t(static_cast<const float*>(x), Wg, bg, logits, T, d, E, s);
    return launch_logits_t(static_cast<const uint16_t*>(x), Wg, bg, logits, T, d, E, s);
}

template <int K, int NV>
__global__ __launch_bounds__(kRouteTokens) void route_local_kernel(const float* __restrict__ logits, int T, int E,
                                                                   int32_t* __restrict__ expert_idx,
                                                                   int32_t* __restrict__ slot_idx,
                                                                   float* __restrict__ gate_w,
                                                                   int32_t* __restrict__ hist) {
    extern __shared__ int32_t smem[];
    route_local_body<K, NV>(smem, logits, T, E, expert_idx, slot_idx, gate_w, hist);
}

// ------------------------------------------------------------------------------------------
// Routing, kernel 2 of 2: every block sums the histograms of the blocks before it (its base)
// and of all blocks (totals), then turns block-local ranks into rows:
//   first choices:  row = base_1[e] + rank
//   second choices: row = total_1[e] + base_2[e] + rank      (all first choices rank first)
// row >= C -> dropped (-1).  Rows >= expert_rows[e] of slot_token are set to -1.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void expert_order_kernel(const int32_t* __restrict__ expert_rows, int E, int C,
                                                           int32_t* __restrict__ order) {
    extern __shared__ int32_t smem[];                 // rows [E], sorted [E + 2]
    for (int e = threadIdx.x; e < E; e += 256) smem[e] = min(expert_rows[e], C);
    __syncthreads();
    write_expert_order(smem, E, order, smem + E, threadIdx.x, 256);
}

int launch_expert_order(const int32_t* expert_rows, int E, int C, int32_t* order, hipStream_t s) {
    hipLaunchKernelGGL(expert_order_kernel, dim3(1), dim3(256), sizeof(int32_t) * (2 * E + 2), s, expert_rows, E, C, order);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

constexpr int kMaxFine = 8;      // fine blocks per 256 tokens at most (32-token tiles)

// hist holds one histogram [K][E] per block of TB tokens (TB divides 256, TB >= 32).  A work-group finalises 256
// tokens.  Every work-group sums the histograms of all blocks before its own: the reads grow with the square of the
// number of blocks (T = 16384, E = 64, top-2: 8 MB in all, served by L2), a stated limit of this kernel.
template <int K>
__device__ __forceinline__ void route_finalize_body(int32_t* smem, int T, int E, int C, int nblocks, int TB,
                                                    const int32_t* __restrict__ expert_idx, int32_t* __restrict__ slot_idx,
                                                    int32_t* __restrict__ expert_rows, int32_t* __restrict__ slot_token,
                                                    int32_t* __restrict__ expert_order, const int32_t* __restrict__ hist) {
    const int ncol = K * E;                                // column = (choice j, expert e)
    const int q = kRouteTokens / TB;                       // fine blocks per work-group
    int32_t* base = smem;                                  // [q][K][E] rows before the fine block's tokens
    int32_t* rows_sh = base + q * ncol;                    // [E]
    int32_t* part = rows_sh + E;                           // [2][R][ncol]: before-me sums, all-blocks sums
    const int tid = threadIdx.x;
    const int b = blockIdx.x;

    // the blocks' histograms are summed with all 256 threads: R row groups each take every R-th block,
    // partial sums meet in LDS
    const int R = ncol >= kRouteTokens ? 1 : kRouteTokens / ncol;
    for (int idx = tid; idx < R * ncol; idx += kRouteTokens) {
        const int col = idx % ncol, rg = idx / ncol;
        int pre = 0, tot = 0;
        // every TB-token block's histogram once; those of 256-token blocks before this one also count as "before me"
        const int nfine = (T + TB - 1) / TB, first_own = b * q;
#pragma unroll 16
        for (int fb = rg; fb < nfine; fb += R) {
            const int v = hist[(size_t)fb * ncol + col];
            tot += v;
            pre += fb < first_own ? v : 0;
        }
        part[rg * ncol + col] = pre;
        part[(R + rg) * ncol + col] = tot;
    }
    __syncthreads();
    for (int e = tid; e < E; e += kRouteTokens) {
        int pre[K], tot[K];
#pragma unroll
        for (int j = 0; j < K; ++j) {
            pre[j] = tot[j] = 0;
            for (int rg = 0; rg < R; ++rg) {
                pre[j] += part[rg * ncol + j * E + e];
                tot[j] += part[(R + rg) * ncol + j * E + e];
            }
        }
        // first choices: rows before = first choices of earlier tokens; second choices rank behind ALL first ones
        int run[K];
        run[0] = pre[0];
        int total = tot[0];
        if (K == 2) {
            run[1] = tot[0] + pre[1];
            total += tot[1];
        }
        // the fine histograms of this block, fetched together (one memory round trip, not one per fine block)
        int fine[kMaxFine - 1][K];
#pragma unroll
        for (int f = 0; f < kMaxFine - 1; ++f)
#pragma unroll
            for (int j = 0; j < K; ++j)
                fine[f][j] = (f + 1 < q && (b * q + f) * TB < T) ? hist[((size_t)(b * q + f) * K + j) * E + e] : 0;
#pragma unroll
        for (int f = 0; f < kMaxFine; ++f) {
            if (f < q) {
#pragma unroll
                for (int j = 0; j < K; ++j) {
                    base[(f * K + j) * E + e] = run[j];
                    if (f < kMaxFine - 1) run[j] += fine[f < kMaxFine - 1 ? f : 0][j];
                }
            }
        }
        rows_sh[e] = min(total, C);
    }
    __syncthreads();

    const int t = b * kRouteTokens + tid;
    if (t < T) {
        const int f = tid / TB;
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const int e = expert_idx[(size_t)t * K + j];
            const int loc = base[(f * K + j) * E + e] + slot_idx[(size_t)t * K + j];
            if (loc < C) {
                slot_idx[(size_t)t * K + j] = loc;
                slot_token[(size_t)e * C + loc] = t;
            } else {
                slot_idx[(size_t)t * K + j] = -1;
            }
        }
    }

    const long long total_slots = (long long)E * C;
    const long long chunk = (total_slots + nblocks - 1) / nblocks;
    const long long lo = (long long)b * chunk;
    const long long hi = min(lo + chunk, total_slots);
    for (long long i = lo + tid; i < hi; i += kRouteTokens) {
        const int e = (int)(i / C), c = (int)(i % C);
        if (c >= rows_sh[e]) slot_token[i] = -1;
    }
    // The rows per expert and the launch order are the work of one block: with an order to write, of an extra block
    // behind the last one (no tokens, no slots: everything above ran empty for it), so that the ranking does not
    // lengthen a block that also has tokens to place.
    if (b == (expert_order ? nblocks : 0)) {
        for (int e = tid; e < E; e += kRouteTokens) expert_rows[e] = rows_sh[e];
        if (expert_order) write_expert_order(rows_sh, E, expert_order, part, tid, kRouteTokens);   // part: free by now
    }
}

template <int K>
__global__ __launch_bounds__(kRouteTokens) void route_finalize_kernel(int T, int E, int C, int nblocks, int TB,
                                                                      const int32_t* __restrict__ expert_idx,
                                                                      int32_t* __restrict__ slot_idx,
                                                                      int32_t* __restrict__ expert_rows,
                                                                      int32_t* __restrict__ slot_token,
                                                                      int32_t* __restrict__ expert_order,
                                                                      const int32_t* __restrict__ hist) {
    extern __shared__ int32_t smem[];
    route_finalize_body<K>(smem, T, E, C, nblocks, TB, expert_idx, slot_idx, expert_rows, slot_token, expert_order, hist);
}

// At most 256 tokens (decode): one block, whose local ranks are already global ones -- the whole routing in one
// launch with a single memory round trip (the logits): totals and ranks stay in LDS and registers.
template <int K, int NV>
__global__ __launch_bounds__(kRouteTokens) void route_single_kernel(const float* __restrict__ logits, int T, int E, int C,
                                                                    int32_t* __restrict__ expert_idx,
                                                                    int32_t* __restrict__ slot_idx,
                                                                    float* __restrict__ gate_w,
                                                                    int32_t* __restrict__ expert_rows,
                                                                    int32_t* __restrict__ slot_token,
                                                                    int32_t* __restrict__ expert_order,
                                                                    int32_t* __restrict__ hist) {
    extern __shared__ int32_t smem[];
    route_single_body<K, NV>(smem, logits, T, E, C, expert_idx, slot_idx, gate_w, expert_rows, slot_token, expert_order, hist);
}

size_t route_finalize_lds_bytes(int E, int k, int TB) {
    const int ncol = k * E;
    const int R = ncol >= kRouteTokens ? 1 : kRouteTokens / ncol;
    size_t ints = (size_t)(kRouteTokens / TB) * ncol + E + 2 * (size_t)R * ncol;
    if (ints < (size_t)(kRouteTokens / TB) * ncol + 2 * (size_t)E + 2) ints = (size_t)(kRouteTokens / TB) * ncol + 2 * (size_t)E + 2;
    return ints * sizeof(int32_t);
}

int launch_route_finalize(int T, int E, int k, int C, int TB, const int32_t* expert_idx, int32_t* slot_idx,
                          int32_t* expert_rows, int32_t* slot_token, int32_t* expert_order, const int32_t* hist,
                          hipStream_t s) {
    const int nb = (T + kRouteTokens - 1) / kRouteTokens;
    const size_t sm = route_finalize_lds_bytes(E, k, TB);
    const int grid = nb + (expert_order ? 1 : 0);               // + the block that ranks the experts
    if (k == 1)
        hipLaunchKernelGGL((route_finalize_kernel<1>), dim3(grid), dim3(kRouteTokens), sm, s, T, E, C, nb, TB, expert_idx,
                           slot_idx, expert_rows, slot_token, expert_order, hist);
    else
        hipLaunchKernelGGL((route_finalize_kernel<2>), dim3(grid), dim3(kRouteTokens), sm, s, T, E, C, nb, TB, expert_idx,
                           slot_idx, expert_rows, slot_token, expert_order, hist);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// histograms for blocks of 32 tokens at the finest
size_t route_scratch_ints(int T, int E, int k) {
    const size_t fine = ((size_t)T + 31) / 32;
    return fine * (size_t)k * (size_t)E;
}

int launch_route(const float* logits, int T, int E, int k, int C, int32_t* expert_idx, int32_t* slot_idx,
                 float* gate_w, int32_t* expert_rows, int32_t* slot_token, int32_t* expert_order, int32_t* scratch,
                 hipStream_t s) {
    const int nb = (T + kRouteTokens - 1) / kRouteTokens;
    const int NW = kRouteTokens / kWave;
    const size_t sm1 = sizeof(int32_t) * ((size_t)k * kRouteTokens + (size_t)NW * k * E);
    if (nb == 1) {
        const size_t sm = sm1 + sizeof(int32_t) * ((size_t)k * E + 2 * (size_t)E + 2);   // + totals, rows, order scratch
#define MOE_ROUTE_SINGLE(K, NV)                                                                                      \
    hipLaunchKernelGGL((route_single_kernel<K, NV>), dim3(1), dim3(kRouteTokens), sm, s, logits, T, E, C, expert_idx, \
                       slot_idx, gate_w, expert_rows, slot_token, expert_order, scratch)
        if (k == 1) {
            if (E <= 16) MOE_ROUTE_SINGLE(1, 1);
            else if (E <= 32) MOE_ROUTE_SINGLE(1, 2);
            else if (E <= 64) MOE_ROUTE_SINGLE(1, 4);
            else if (E <= 128) MOE_ROUTE_SINGLE(1, 8);
            else MOE_ROUTE_SINGLE(1, 0);
        } else {
            if (E <= 16) MOE_ROUTE_SINGLE(2, 1);
            else if (E <= 32) MOE_ROUTE_SINGLE(2, 2);
            else if (E <= 64) MOE_ROUTE_SINGLE(2, 4);
            else if (E <= 128) MOE_ROUTE_SINGLE(2, 8);
            else MOE_ROUTE_SINGLE(2, 0);
        }
#undef MOE_ROUTE_SINGLE
        return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
    }
#define MOE_ROUTE_LOCAL(K, NV)                                                                                   \
    hipLaunchKernelGGL((route_local_kernel<K, NV>), dim3(nb), dim3(kRouteTokens), sm1, s, logits, T, E, expert_idx, \
                       slot_idx, gate_w, scratch)
    if (k == 1) {
        if (E <= 16) MOE_ROUTE_LOCAL(1, 1);
        else if (E <= 32) MOE_ROUTE_LOCAL(1, 2);
        else if (E <= 64) MOE_ROUTE_LOCAL(1, 4);
        else if (E <= 128) MOE_ROUTE_LOCAL(1, 8);
        else MOE_ROUTE_LOCAL(1, 0);
    } else {
        if (E <= 16) MOE_ROUTE_LOCAL(2, 1);
        else if (E <= 32) MOE_ROUTE_LOCAL(2, 2);
        else if (E <= 64) MOE_ROUTE_LOCAL(2, 4);
        else if (E <= 128) MOE_ROUTE_LOCAL(2, 8);
        else MOE_ROUTE_LOCAL(2, 0);
    }
#undef MOE_ROUTE_LOCAL
    if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
    // the block histograms are per 256 tokens
    return launch_route_finalize(T, E, k, C, kRouteTokens, expert_idx, slot_idx, expert_rows, slot_token, expert_order,
                                 scratch, s);
}

}  // namespace moe
