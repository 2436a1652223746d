// Per-token gate arithmetic shared by the routing kernels: top-k by logit with ties to the lowest
// expert index, softmax weight(s), computed by an aligned group of 16 lanes (paper Sec. 5.4: the
// gating function's top-k selection and its probability-domain weights).
#pragma once

#include "moe_internal.h"

namespace moe {

struct Best {
    float v;
    int i;
};
__device__ __forceinline__ Best better(Best a, Best b) {
    return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;
}
// All-reduce inside aligned groups of 16 lanes (one DPP "row") with data-parallel-primitive moves:
// swap inside pairs, swap pairs inside quads, mirror the two quads of each half row, mirror the two
// half rows.  After step i every aligned group of 2^i lanes holds one common value, which is what
// makes the mirrors (which reverse lane order) as good as butterflies.  No LDS traffic, unlike
// __shfl_xor.
constexpr int kDppSwap1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppSwap2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // row_half_mirror
constexpr int kDppMirror = 0x140;      // row_mirror
template <int CTRL> __device__ __forceinline__ int dpp_i(int v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
template <int CTRL> __device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(dpp_i<CTRL>(__float_as_int(v)));
}
template <int CTRL> __device__ __forceinline__ Best best_step(Best a) {
    Best o;
    o.v = dpp_f<CTRL>(a.v);
    o.i = dpp_i<CTRL>(a.i);
    return better(a, o);
}
__device__ __forceinline__ Best group_best(Best a) {
    a = best_step<kDppSwap1>(a);
    a = best_step<kDppSwap2>(a);
    a = best_step<kDppHalfMirror>(a);
    a = best_step<kDppMirror>(a);
    return a;
}
// Sum in a fixed tree order; every lane ends with the same bits (each step adds the same two
// partial sums on both sides, and fp add commutes).
__device__ __forceinline__ float group_sum(float a) {
    a += dpp_f<kDppSwap1>(a);
    a += dpp_f<kDppSwap2>(a);
    a += dpp_f<kDppHalfMirror>(a);
    a += dpp_f<kDppMirror>(a);
    return a;
}

// exp on the hardware exp2 unit; the argument is <= 0 here and the dominant terms have a small
// argument, which keeps the softmax weights within ~1e-7 of the exact value
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }

template <int K>
__device__ __forceinline__ void gate_weights(float s, Best g1, Best g2, float& w1, float& w2) {
    if (K == 1) {
        w1 = 1.0f / s;                          // softmax probability of the arg-max
        w2 = 0.f;
    } else {
        const float r = fast_exp(g2.v - g1.v);  // p2/p1; renormalised pair = (1, r)/(1 + r)
        w1 = 1.0f / (1.0f + r);
        w2 = r / (1.0f + r);
    }
}

// Top-K experts and gate weights of one token, computed by a group of 16 lanes; lane `sub` looks
// at experts sub, sub+16, ...  Every lane of the group returns the same result.
// Register version: the lane's NV logits are already loaded (padding = -inf).
template <int K, int NV>
__device__ __forceinline__ void token_gate_regs(const float (&v)[NV], int sub, Best& g1, Best& g2, float& w1,
                                                float& w2) {
    const Best none{-INFINITY, 0x7fffffff};
    Best b1 = none, b2 = none;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int e = sub + 16 * i;
        if (v[i] > b1.v) { b2 = b1; b1.v = v[i]; b1.i = e; }
        else if (v[i] > b2.v) { b2.v = v[i]; b2.i = e; }
    }
    g1 = group_best(b1);
    g2 = none;
    if (K == 2) g2 = group_best(b1.i == g1.i ? b2 : b1);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) s += fast_exp(v[i] - g1.v);       // exp(-inf) = 0 for the padding
    gate_weights<K>(group_sum(s), g1, g2, w1, w2);
}
// Any E: two passes over the row in memory.
template <int K>
__device__ __forceinline__ void token_gate_mem(const float* __restrict__ row, int E, int sub, Best& g1, Best& g2,
                                               float& w1, float& w2) {
    const Best none{-INFINITY, 0x7fffffff};
    Best b1 = none, b2 = none;
    for (int e = sub; e < E; e += 16) {
        const float v = row[e];
        if (v > b1.v) { b2 = b1; b1.v = v; b1.i = e; }
        else if (v > b2.v) { b2.v = v; b2.i = e; }
    }
    g1 = group_best(b1);
    g2 = none;
    if (K == 2) g2 = group_best(b1.i == g1.i ? b2 : b1);
    float s = 0.f;
    for (int e = sub; e < E; e += 16) s += fast_exp(row[e] - g1.v);
    gate_weights<K>(group_sum(s), g1, g2, w1, w2);
}

// Rank of each lane's token among the wave's tokens that chose the same expert (e < 0: no token), by
// ballots: returns the number of lower lanes with the same e; the lowest lane of every group of equal e
// adds the group's size to count[e] (LDS or global, one writer per expert and wave).
__device__ __forceinline__ int wave_rank_by_expert(int e, int lane, int32_t* count) {
    const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
    int rank = 0;
    unsigned long long todo = __ballot(e >= 0);
    while (todo) {
        const int leader = __ffsll((long long)todo) - 1;
        const int le = __shfl(e, leader, kWave);
        const unsigned long long m = __ballot(e == le);
        if (e == le) rank = __popcll(m & lt_mask);
        if (lane == leader) count[le] = __popcll(m);
        todo &= ~m;
    }
    return rank;
}

}  // namespace moe
