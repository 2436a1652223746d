// Device-side pieces of the routing shared by the routing kernels and by the decode gate, which runs the whole
// routing at the end of its logits kernel (paper Sec. 5.4: top-k, the cumulative count that places a token inside
// its expert, the capacity cut and the mapping tables, fused into as few launches as the dependences allow).
#pragma once

#include "gate_common.h"

namespace moe {

// ------------------------------------------------------------------------------------------
// Routing, kernel 1 of 2: per block of 256 tokens
//   phase A  16 lanes per token: top-k by logit (lowest index on ties), softmax weight(s)
//   phase B  one lane per token: rank of the token among the wave's tokens that chose the same
//            expert, by ballot; per-wave histogram
//   phase C  prefix over the block's waves; block histogram to global scratch; the rank inside
//            the block is parked in slot_idx until kernel 2 adds the block's base.
// scratch layout: hist[block][choice][E]
// ------------------------------------------------------------------------------------------
// SINGLE (at most 256 tokens, one block): the block's totals stay in LDS (tot_sh [K][E]) and the ranks in registers
// (my_e, my_slot: expert and rank within the expert's choice-j tokens of this thread's token), nothing is parked
// in global memory.
template <int K, int NV, bool SINGLE = false>
__device__ __forceinline__ void route_local_body(int32_t* smem, const float* __restrict__ logits, int T, int E,
                                                 int32_t* __restrict__ expert_idx, int32_t* __restrict__ slot_idx,
                                                 float* __restrict__ gate_w, int32_t* __restrict__ hist,
                                                 int32_t* tot_sh = nullptr, int* my_e_out = nullptr,
                                                 int* my_slot_out = nullptr) {
    constexpr int NW = kRouteTokens / kWave;
    int32_t* e_sh = smem;                          // [K][256] chosen expert per token of the block
    int32_t* whist = smem + K * kRouteTokens;      // [NW][K][E]

    const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave;
    const int tb = SINGLE ? 0 : blockIdx.x * kRouteTokens;     // SINGLE: whichever block runs it, the tokens are 0..T-1

    for (int i = tid; i < NW * K * E; i += kRouteTokens) whist[i] = 0;

    // phase A: 16 lanes per token, 16 tokens of the block at a time.  When the row fits in registers
    // (E <= 128) the logits of all 16 rounds are fetched first, in one memory round trip.
    {
        const int grp = tid >> 4, sub = tid & 15;
        constexpr int ROUNDS = kRouteTokens / 16;
        auto publish = [&](int tl, Best g1, Best g2, float w1, float w2) {
            const int t = tb + tl;
            if (sub == 0) {
                const bool ok = t < T;
                e_sh[tl] = ok ? g1.i : -1;
                if (K == 2) e_sh[kRouteTokens + tl] = ok ? g2.i : -1;
                if (ok) {
                    expert_idx[(size_t)t * K] = g1.i;
                    gate_w[(size_t)t * K] = w1;
                    if (K == 2) {
                        expert_idx[(size_t)t * K + 1] = g2.i;
                        gate_w[(size_t)t * K + 1] = w2;
                    }
                }
            }
        };
        if (NV > 0) {
            constexpr int NVV = NV > 0 ? NV : 1;
            float v[ROUNDS][NVV];
            const int live_rounds = min(ROUNDS, (T - tb + 15) / 16);      // rounds that hold a token (uniform over the block)
#pragma unroll
            for (int it = 0; it < ROUNDS; ++it) {
                if (it >= live_rounds) break;
                const float* row = logits + (size_t)min(tb + it * 16 + grp, T - 1) * E;   // clamped: lanes stay in the shuffles
#pragma unroll
                for (int i = 0; i < NVV; ++i) v[it][i] = row[min(sub + 16 * i, E - 1)];
            }
#pragma unroll
            for (int it = 0; it < ROUNDS; ++it) {
                if (it >= live_rounds) {                                   // no token: only the table entries
                    if (sub == 0) {
                        e_sh[it * 16 + grp] = -1;
                        if (K == 2) e_sh[kRouteTokens + it * 16 + grp] = -1;
                    }
                    continue;
                }
#pragma unroll
                for (int i = 0; i < NVV; ++i) v[it][i] = sub + 16 * i < E ? v[it][i] : -INFINITY;
                Best g1, g2;
                float w1, w2;
                token_gate_regs<K, NVV>(v[it], sub, g1, g2, w1, w2);
                publish(it * 16 + grp, g1, g2, w1, w2);
            }
        } else {
#pragma unroll 4
            for (int it = 0; it < ROUNDS; ++it) {
                const int tl = it * 16 + grp;
                Best g1, g2;
                float w1, w2;
                token_gate_mem<K>(logits + (size_t)min(tb + tl, T - 1) * E, E, sub, g1, g2, w1, w2);
                publish(tl, g1, g2, w1, w2);
            }
        }
    }
    __syncthreads();

    // phase B
    int my_e[K], my_rank[K];
#pragma unroll
    for (int j = 0; j < K; ++j) {
        my_e[j] = e_sh[j * kRouteTokens + tid];
        my_rank[j] = wave_rank_by_expert(my_e[j], lane, whist + (w * K + j) * E);
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
        if (SINGLE) tot_sh[j * E + e] = run;
        else hist[((size_t)blockIdx.x * K + j) * E + e] = run;
    }
    __syncthreads();
    const int t = tb + tid;
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const int slot = t < T ? my_rank[j] + whist[(w * K + j) * E + my_e[j]] : 0;
        if (SINGLE) {
            my_e_out[j] = my_e[j];
            my_slot_out[j] = slot;
        } else if (t < T) {
            slot_idx[(size_t)t * K + j] = slot;
        }
    }
}

// Launch order of the experts for the grouped GEMMs, which deal consecutive entries round-robin to
// the 8 XCDs.  Experts are ranked by kept rows (most first, ties by index); active ones are then
// handed out so that every XCD alternates between a busy expert (matrix-core bound) and a light one
// (weight-bandwidth bound), neighbouring XCDs in opposite phase: entry p = 8j + x (j-th expert of XCD
// x) takes the next busiest remaining expert when j + x is even, the next lightest when odd.  All
// XCDs get the same number of active experts, and while half of them multiply the others stream
// weights.  Experts without rows follow at the end.  O(E^2) compares, E <= 1024.
// order[E] (one entry past the list) tells the tiled GEMM how to deal its tiles to the XCDs: 1 when the active
// experts are of very different sizes (at least a quarter of them hold at most a quarter of the largest one's
// rows), so that dealing whole experts would leave the XCDs with unequal work; 0 otherwise.
// A second list follows at order[E + 1 ..]: the experts plainly by rows, busiest first, and the same flag at
// order[2E + 1] (for products whose tiles are long and few per compute unit: longest first, short ones fill the end).
// `order` holds 2E + 2 ints.  `sorted` is LDS scratch of E + 2 ints; every thread of the block must call.
__device__ __forceinline__ void write_expert_order(const int32_t* rows /* LDS */, int E, int32_t* __restrict__ order,
                                                   int32_t* sorted /* LDS */, int tid, int nthreads) {
    if (tid == 0) sorted[E] = sorted[E + 1] = 0;
    __syncthreads();
    // rank of expert e = number of experts that come before it.  With fewer experts than threads, `parts` adjacent
    // lanes share an expert, each comparing it with a slice of the others (8 independent LDS reads at a time).
    int parts = 1;
    while (parts < 16 && parts * 2 * E <= nthreads) parts *= 2;
    const int part = tid % parts, slice = (E + parts - 1) / parts;
    const int lo = part * slice, hi = min(E, lo + slice);
    int active = 0;
    for (int e0 = 0; e0 < E; e0 += nthreads / parts) {          // same trip count for every thread
        const int e = e0 + tid / parts;
        const bool ok = e < E;
        const int r = ok ? rows[e] : 0;
        int rank = 0, o = lo;
        for (; o + 8 <= hi; o += 8) {
            int ro[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) ro[i] = rows[o + i];
#pragma unroll
            for (int i = 0; i < 8; ++i) rank += (ro[i] > r || (ro[i] == r && o + i < e)) ? 1 : 0;
        }
        for (; o < hi; ++o) {
            const int ro = rows[o];
            rank += (ro > r || (ro == r && o < e)) ? 1 : 0;
        }
        for (int m = 1; m < parts; m <<= 1) rank += __shfl_xor(rank, m);
        if (ok && part == 0) {
            sorted[rank] = e;
            active += r > 0 ? 1 : 0;
        }
    }
    if (active) atomicAdd(&sorted[E], active);          // integer count in LDS: order-independent
    __syncthreads();
    const int na = sorted[E];
    {
        const int largest = rows[sorted[0]];
        int small = 0;
        for (int e = tid; e < E; e += nthreads) small += rows[e] > 0 && rows[e] * 4 <= largest ? 1 : 0;
        if (small) atomicAdd(&sorted[E + 1], small);
        __syncthreads();
        if (tid == 0) order[E] = order[2 * E + 1] = sorted[E + 1] * 4 >= na && na > 0 ? 1 : 0;
    }
    for (int p = tid; p < E; p += nthreads) {
        int e;
        if (p >= na) {
            e = sorted[p];
        } else {
            const int j = p >> 3, x = p & 7;
            // busy takes among positions 8j .. 8j+x-1: those x' with (j + x') even
            const int busy_before = 4 * j + ((j & 1) ? (x >> 1) : ((x + 1) >> 1));
            const int light_before = p - busy_before;
            e = ((j + x) & 1) ? sorted[na - 1 - light_before] : sorted[busy_before];
        }
        order[p] = e;
        order[E + 1 + p] = sorted[p];                     // second list: plainly by rows, busiest first
    }
}

// At most 256 tokens: the whole routing by one block of 256 threads, whose block-local ranks are already global ones;
// totals and ranks stay in LDS and registers, one memory round trip (the logits).  smem: route_single_lds_ints(E, K) ints.
template <int K, int NV>
__device__ __forceinline__ void route_single_body(int32_t* smem, const float* __restrict__ logits, int T, int E, int C,
                                                  int32_t* __restrict__ expert_idx, int32_t* __restrict__ slot_idx,
                                                  float* __restrict__ gate_w, int32_t* __restrict__ expert_rows,
                                                  int32_t* __restrict__ slot_token, int32_t* __restrict__ expert_order,
                                                  int32_t* __restrict__ hist) {
    constexpr int NW = kRouteTokens / kWave;
    int32_t* tot_sh = smem + K * kRouteTokens + NW * K * E;     // [K][E] tokens per (choice, expert)
    int32_t* rows_sh = tot_sh + K * E;                          // [E]
    int32_t* sorted = rows_sh + E;                              // [E + 2]
    const int tid = threadIdx.x;
    int my_e[K], my_slot[K];
    route_local_body<K, NV, true>(smem, logits, T, E, expert_idx, slot_idx, gate_w, hist, tot_sh, my_e, my_slot);
    for (int e = tid; e < E; e += kRouteTokens) {
        const int rows = min(tot_sh[e] + (K == 2 ? tot_sh[E + e] : 0), C);
        rows_sh[e] = rows;
        expert_rows[e] = rows;
    }
    if (tid < T) {
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const int e = my_e[j];
            const int loc = my_slot[j] + (j == 1 ? tot_sh[e] : 0);   // second choices rank behind all first ones
            if (loc < C) slot_token[(size_t)e * C + loc] = tid;
            slot_idx[(size_t)tid * K + j] = loc < C ? loc : -1;
        }
    }
    __syncthreads();
    for (long long i = tid; i < (long long)E * C; i += kRouteTokens)
        if ((int)(i % C) >= rows_sh[i / C]) slot_token[i] = -1;
    if (expert_order) write_expert_order(rows_sh, E, expert_order, sorted, tid, kRouteTokens);
}
// LDS ints of route_single_body: chosen experts, per-wave histograms, totals, rows, order scratch
__host__ __device__ inline size_t route_single_lds_ints(int E, int k) {
    return (size_t)k * kRouteTokens + (size_t)(kRouteTokens / kWave) * k * E + (size_t)k * E + 2 * (size_t)E + 2;
}

}  // namespace moe
