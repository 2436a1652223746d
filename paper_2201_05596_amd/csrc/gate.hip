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
#include "moe_internal.h"

namespace moe {

// ------------------------------------------------------------------------------------------
// logits[t,e] = bg[e] + sum_i x[t,i] Wg[i,e]     fp32 accumulate
//
// Block = 256 threads = EB expert lanes x (256/EB) token groups, 8 tokens per
// thread.  The x tile is staged in LDS as fp32 and read back as broadcast
// 16-byte vectors; Wg rows are read coalesced straight from L2.
// ------------------------------------------------------------------------------------------
constexpr int kLogitKC = 64;     // k-chunk of the x tile
constexpr int kLogitTPT = 8;     // tokens per thread

template <typename XT, int EB>
__global__ __launch_bounds__(256) void gate_logits_kernel(const XT* __restrict__ x, const float* __restrict__ Wg,
                                                          const float* __restrict__ bg, float* __restrict__ logits,
                                                          int T, int d, int E) {
    constexpr int NTH = 256 / EB;
    constexpr int TM = NTH * kLogitTPT;
    __shared__ __attribute__((aligned(16))) float xs[TM][kLogitKC + 4];

    const int tid = threadIdx.x;
    const int el = tid % EB;
    const int th = tid / EB;
    const int t0 = blockIdx.x * TM;

    for (int e0 = 0; e0 < E; e0 += EB) {
        const int e = e0 + el;
        const bool e_ok = e < E;
        float acc[kLogitTPT];
#pragma unroll
        for (int i = 0; i < kLogitTPT; ++i) acc[i] = 0.f;

        for (int k0 = 0; k0 < d; k0 += kLogitKC) {
            __syncthreads();
            for (int i = tid; i < TM * kLogitKC; i += 256) {
                const int r = i / kLogitKC, c = i % kLogitKC;
                const int t = t0 + r, k = k0 + c;
                xs[r][c] = (t < T && k < d) ? Elem<XT>::load(x + (size_t)t * d + k) : 0.f;
            }
            __syncthreads();
            const int kmax = min(kLogitKC, d - k0);
            if (e_ok) {
                for (int kk = 0; kk < kmax; kk += 4) {
                    float w[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) w[i] = (kk + i < kmax) ? Wg[(size_t)(k0 + kk + i) * E + e] : 0.f;
#pragma unroll
                    for (int tt = 0; tt < kLogitTPT; ++tt) {
                        const float4 xv = *reinterpret_cast<const float4*>(&xs[th * kLogitTPT + tt][kk]);
                        acc[tt] = fmaf(xv.x, w[0], acc[tt]);
                        acc[tt] = fmaf(xv.y, w[1], acc[tt]);
                        acc[tt] = fmaf(xv.z, w[2], acc[tt]);
                        acc[tt] = fmaf(xv.w, w[3], acc[tt]);
                    }
                }
            }
        }
        if (e_ok) {
            const float b = bg ? bg[e] : 0.f;
#pragma unroll
            for (int tt = 0; tt < kLogitTPT; ++tt) {
                const int t = t0 + th * kLogitTPT + tt;
                if (t < T) logits[(size_t)t * E + e] = acc[tt] + b;
            }
        }
    }
}

template <typename XT>
static int launch_logits_t(const XT* x, const float* Wg, const float* bg, float* logits, int T, int d, int E,
                           hipStream_t s) {
#define MOE_LOGITS_CASE(EB)                                                                           \
    {                                                                                                 \
        constexpr int TM = (256 / EB) * kLogitTPT;                                                    \
        hipLaunchKernelGGL((gate_logits_kernel<XT, EB>), dim3((T + TM - 1) / TM), dim3(256), 0, s, x, \
                           Wg, bg, logits, T, d, E);                                                  \
    }
    if (E <= 16) MOE_LOGITS_CASE(16)
    else if (E <= 32) MOE_LOGITS_CASE(32)
    else if (E <= 64) MOE_LOGITS_CASE(64)
    else if (E <= 128) MOE_LOGITS_CASE(128)
    else MOE_LOGITS_CASE(256)
#undef MOE_LOGITS_CASE
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int launch_gate_logits(const void* x, int dtype, const float* Wg, const float* bg, float* logits, int T, int d,
                       int E, hipStream_t s) {
    if (dtype == MOE_F32) return launch_logits_t(static_cast<const float*>(x), Wg, bg, logits, T, d, E, s);
    return launch_logits_t(static_cast<const uint16_t*>(x), Wg, bg, logits, T, d, E, s);
}

// ------------------------------------------------------------------------------------------
// Routing, kernel 1 of 2: per block of 256 tokens
//   phase A  one wave per token: top-k by logit (lowest index on ties), softmax weight(s)
//   phase B  one lane per token: rank of the token among the wave's tokens that chose the same
//            expert, by ballot; per-wave histogram
//   phase C  prefix over the block's waves; block histogram to global scratch; the rank inside
//            the block is parked in slot_idx until kernel 2 adds the block's base.
// scratch layout: hist[block][choice][E]
// ------------------------------------------------------------------------------------------
struct Best {
    float v;
    int i;
};
__device__ __forceinline__ Best better(Best a, Best b) {
    return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;
}
__device__ __forceinline__ Best wave_best(Best a) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        Best o;
        o.v = __shfl_xor(a.v, m, kWave);
        o.i = __shfl_xor(a.i, m, kWave);
        a = better(a, o);
    }
    return a;
}
__device__ __forceinline__ float wave_sum(float a) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) a += __shfl_xor(a, m, kWave);
    return a;
}

template <int K>
__global__ __launch_bounds__(kRouteTokens) void route_local_kernel(const float* __restrict__ logits, int T, int E,
                                                                   int32_t* __restrict__ expert_idx,
                                                                   int32_t* __restrict__ slot_idx,
                                                                   float* __restrict__ gate_w,
                                                                   int32_t* __restrict__ hist) {
    constexpr int NW = kRouteTokens / kWave;
    extern __shared__ int32_t smem[];
    int32_t* e_sh = smem;                          // [K][256] chosen expert per token of the block
    int32_t* whist = smem + K * kRouteTokens;      // [NW][K][E]

    const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave;
    const int tb = blockIdx.x * kRouteTokens;

    for (int i = tid; i < NW * K * E; i += kRouteTokens) whist[i] = 0;

    // phase A
    for (int q = 0; q < kWave; ++q) {
        const int tl = w * kWave + q;
        const int t = tb + tl;
        if (t >= T) {                                 // wave-uniform
            if (lane == 0) {
                e_sh[tl] = -1;
                if (K == 2) e_sh[kRouteTokens + tl] = -1;
            }
            continue;
        }
        const float* row = logits + (size_t)t * E;
        Best b1{-INFINITY, 0x7fffffff}, b2{-INFINITY, 0x7fffffff};
        for (int e = lane; e < E; e += kWave) {
            const float v = row[e];
            if (v > b1.v) { b2 = b1; b1.v = v; b1.i = e; }
            else if (v > b2.v) { b2.v = v; b2.i = e; }
        }
        const Best g1 = wave_best(b1);
        Best g2{-INFINITY, 0x7fffffff};
        if (K == 2) g2 = wave_best(b1.i == g1.i ? b2 : b1);
        float s = 0.f;
        for (int e = lane; e < E; e += kWave) s += expf(row[e] - g1.v);
        s = wave_sum(s);
        if (lane == 0) {
            e_sh[tl] = g1.i;
            expert_idx[(size_t)t * K] = g1.i;
            if (K == 1) {
                gate_w[t] = 1.0f / s;
            } else {
                const float r = expf(g2.v - g1.v);
                e_sh[kRouteTokens + tl] = g2.i;
                expert_idx[(size_t)t * K + 1] = g2.i;
                gate_w[(size_t)t * K] = 1.0f / (1.0f + r);
                gate_w[(size_t)t * K + 1] = r / (1.0f + r);
            }
        }
    }
    __syncthreads();

    // phase B
    int my_e[K], my_rank[K];
    const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const int e = e_sh[j * kRouteTokens + tid];
        my_e[j] = e;
        my_rank[j] = 0;
        unsigned long long todo = __ballot(e >= 0);
        while (todo) {
            const int leader = __ffsll((long long)todo) - 1;
            const int le = __shfl(e, leader, kWave);
            const unsigned long long m = __ballot(e == le);
            if (e == le) my_rank[j] = __popcll(m & lt_mask);
            if (lane == leader) whist[(w * K + j) * E + le] = __popcll(m);
            todo &= ~m;
        }
    }
    __syncthreads();

    // phase C
    for (int i = tid; i < K * E; i += kRouteTokens) {
        const int j = i / E, e = i % E;
        int run = 0;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) {
            const int c = whist[(ww * K + j) * E + e];
            whist[(ww * K + j) * E + e] = run;
            run += c;
        }
        hist[((size_t)blockIdx.x * K + j) * E + e] = run;
    }
    __syncthreads();
    const int t = tb + tid;
    if (t < T) {
#pragma unroll
        for (int j = 0; j < K; ++j)
            slot_idx[(size_t)t * K + j] = my_rank[j] + whist[(w * K + j) * E + my_e[j]];
    }
}

// ------------------------------------------------------------------------------------------
// Routing, kernel 2 of 2: every block sums the histograms of the blocks before it (its base)
// and of all blocks (totals), then turns block-local ranks into rows:
//   first choices:  row = base_1[e] + rank
//   second choices: row = total_1[e] + base_2[e] + rank      (all first choices rank first)
// row >= C -> dropped (-1).  Rows >= expert_rows[e] of slot_token are set to -1.
// ------------------------------------------------------------------------------------------
template <int K>
__global__ __launch_bounds__(kRouteTokens) void route_finalize_kernel(int T, int E, int C, int nblocks,
                                                                      const int32_t* __restrict__ expert_idx,
                                                                      int32_t* __restrict__ slot_idx,
                                                                      int32_t* __restrict__ expert_rows,
                                                                      int32_t* __restrict__ slot_token,
                                                                      const int32_t* __restrict__ hist) {
    extern __shared__ int32_t smem[];
    int32_t* base = smem;             // [K][E]
    int32_t* rows_sh = smem + K * E;  // [E]
    const int tid = threadIdx.x;
    const int b = blockIdx.x;

    for (int e = tid; e < E; e += kRouteTokens) {
        int pre[K], tot[K];
#pragma unroll
        for (int j = 0; j < K; ++j) pre[j] = tot[j] = 0;
        for (int bb = 0; bb < nblocks; ++bb) {
#pragma unroll
            for (int j = 0; j < K; ++j) {
                const int v = hist[((size_t)bb * K + j) * E + e];
                tot[j] += v;
                if (bb < b) pre[j] += v;
            }
        }
        base[e] = pre[0];
        int total = tot[0];
        if (K == 2) {
            base[E + e] = tot[0] + pre[1];
            total += tot[1];
        }
        rows_sh[e] = min(total, C);
    }
    __syncthreads();

    const int t = b * kRouteTokens + tid;
    if (t < T) {
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const int e = expert_idx[(size_t)t * K + j];
            const int loc = base[j * E + e] + slot_idx[(size_t)t * K + j];
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
    if (b == 0)
        for (int e = tid; e < E; e += kRouteTokens) expert_rows[e] = rows_sh[e];
}

size_t route_scratch_ints(int T, int E, int k) {
    const size_t nb = ((size_t)T + kRouteTokens - 1) / kRouteTokens;
    return nb * (size_t)k * (size_t)E;
}

int launch_route(const float* logits, int T, int E, int k, int C, int32_t* expert_idx, int32_t* slot_idx,
                 float* gate_w, int32_t* expert_rows, int32_t* slot_token, int32_t* scratch, hipStream_t s) {
    const int nb = (T + kRouteTokens - 1) / kRouteTokens;
    const int NW = kRouteTokens / kWave;
    const size_t sm1 = sizeof(int32_t) * ((size_t)k * kRouteTokens + (size_t)NW * k * E);
    const size_t sm2 = sizeof(int32_t) * ((size_t)k * E + E);
    if (k == 1) {
        hipLaunchKernelGGL((route_local_kernel<1>), dim3(nb), dim3(kRouteTokens), sm1, s, logits, T, E,
                           expert_idx, slot_idx, gate_w, scratch);
        hipLaunchKernelGGL((route_finalize_kernel<1>), dim3(nb), dim3(kRouteTokens), sm2, s, T, E, C, nb,
                           expert_idx, slot_idx, expert_rows, slot_token, scratch);
    } else {
        hipLaunchKernelGGL((route_local_kernel<2>), dim3(nb), dim3(kRouteTokens), sm1, s, logits, T, E,
                           expert_idx, slot_idx, gate_w, scratch);
        hipLaunchKernelGGL((route_finalize_kernel<2>), dim3(nb), dim3(kRouteTokens), sm2, s, T, E, C, nb,
                           expert_idx, slot_idx, expert_rows, slot_token, scratch);
    }
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace moe
