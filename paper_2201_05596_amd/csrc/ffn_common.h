// Pieces shared by the two bf16 MFMA grouped-GEMM kernels (weight-streaming and tiled): operand
// types, the register transpose of K-major weights, the XCD-aware tile numbering and the epilogues.
#pragma once

#include "moe_internal.h"

namespace moe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kXcd = 8;             // L2 domains; consecutive work-group ids rotate over them

__device__ __forceinline__ uint32_t dw(const uint4& v, int q) {
    return q == 0 ? v.x : q == 1 ? v.y : q == 2 ? v.z : v.w;
}

// MFMA B fragments from K-major weights.  src[j] holds 8 consecutive columns of k-row j (j = 0..7):
// an 8x8 block of 16-bit values, k down, n across.  The MFMA wants, per output column, 8 consecutive
// k in one register quad: an 8x8 transpose, done with v_perm_b32.  Pair qq of the block's columns
// (2qq, 2qq+1) comes out as two fragments.
__device__ __forceinline__ void b_frag_pair(const uint4 (&src)[8], int qq, bf16x8_t& lo_col, bf16x8_t& hi_col) {
    uint32_t lo[4], hi[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t r0 = dw(src[2 * p], qq), r1 = dw(src[2 * p + 1], qq);
        lo[p] = __builtin_amdgcn_perm(r1, r0, 0x05040100u);   // column 2qq   : k = 2p, 2p+1
        hi[p] = __builtin_amdgcn_perm(r1, r0, 0x07060302u);   // column 2qq+1
    }
    lo_col = __builtin_bit_cast(bf16x8_t, make_uint4(lo[0], lo[1], lo[2], lo[3]));
    hi_col = __builtin_bit_cast(bf16x8_t, make_uint4(hi[0], hi[1], hi[2], hi[3]));
}

// Consecutive work-group ids rotate over the 8 XCDs (each with its own L2).  With at least 8
// groups, all tiles of one expert are placed on one XCD: its activation rows (read by every
// column tile) and its weights (read by every row tile) are then fetched into that L2 once.
// Experts are taken from `order` (busiest first), dealt round-robin to the XCDs, so that each
// XCD streams the same number of active experts.  With fewer groups (the dense branch) column
// tiles are spread over the XCDs instead.  inner_n = row tiles x k-splits per (group, column tile).
struct TileId {
    int g, nt, inner;
    bool live;
};
__device__ __forceinline__ TileId tile_of_block(const WsGemmArgs& a, int n_tiles, int inner_n, int block) {
    TileId t;
    const int xcd = block % kXcd;
    const int q = block / kXcd;
    if (a.G >= kXcd) {
        const int per_group = n_tiles * inner_n;
        const int slot = (q / per_group) * kXcd + xcd;
        t.nt = (q % per_group) / inner_n;
        t.inner = q % inner_n;
        t.live = slot < a.G;
        t.g = t.live ? (a.order ? a.order[slot] : slot) : 0;
    } else if (a.ksplit == 1 && inner_n >= kXcd) {
        // few groups with many row tiles (the dense branch): every XCD takes a contiguous range of
        // row tiles and walks it column tile by column tile, so the work-groups running together on
        // an XCD share a few activation row tiles (kept in its L2) while the weights stream through
        const int per_xcd = (inner_n + kXcd - 1) / kXcd;
        const int per_group = per_xcd * n_tiles;
        t.g = q / per_group;
        t.nt = q % n_tiles;
        t.inner = xcd * per_xcd + (q % per_group) / n_tiles;
        t.live = t.g < a.G && t.inner < inner_n;
    } else {
        const int u = (q / inner_n) * kXcd + xcd;
        t.g = u / n_tiles;
        t.nt = u % n_tiles;
        t.inner = q % inner_n;
        t.live = u < a.G * n_tiles;
    }
    return t;
}
// Second mapping, for the tiled kernel with many groups of very different sizes (config 5: a few experts at capacity,
// many with a handful of rows): every XCD takes 1/8 of the column tiles of EVERY group and walks the groups in launch
// order, row tiles innermost.  All XCDs then carry the same work whatever the row counts are; a weight column tile
// still enters exactly one L2 (its row tiles run back to back there); only the groups' activation rows are read by
// all eight.  Because the launch order alternates busy and light groups, the CUs of an XCD run matrix-bound and
// weight-streaming tiles at the same time, instead of one phase after the other.
// Which mapping applies is decided on the device, by the flag behind the launch order (only the device knows the row
// counts); the host sizes the grid for either.
__host__ __device__ __forceinline__ bool tile_spread_possible(const WsGemmArgs& a, int n_tiles) {
    return a.order != nullptr && a.spread != 2 && a.ksplit == 1 && a.G >= kXcd && n_tiles % kXcd == 0;
}
__device__ __forceinline__ bool tile_spread(const WsGemmArgs& a, int n_tiles) {
    return tile_spread_possible(a, n_tiles) && (a.spread == 1 || a.order[a.G] != 0);
}
__device__ __forceinline__ TileId tile_of_block_spread(const WsGemmArgs& a, int n_tiles, int inner_n, int block) {
    TileId t;
    const int xcd = block % kXcd, q = block / kXcd;
    const int per_x = n_tiles / kXcd, per_group = per_x * inner_n;
    const int slot = q / per_group, rem = q % per_group;
    t.nt = xcd * per_x + rem / inner_n;
    t.inner = rem % inner_n;
    t.live = slot < a.G;
    t.g = t.live ? (a.order ? a.order[slot] : slot) : 0;
    return t;
}
inline long long tile_grid_blocks(const WsGemmArgs& a, int n_tiles, int inner_n) {
    // (the spread mapping needs G * n_tiles * inner_n blocks, never more than the first case below)
    if (a.G >= kXcd) return (long long)(a.G + kXcd - 1) / kXcd * kXcd * n_tiles * inner_n;
    if (a.ksplit == 1 && inner_n >= kXcd) return (long long)a.G * ((inner_n + kXcd - 1) / kXcd) * n_tiles * kXcd;
    return ((long long)a.G * n_tiles + kXcd - 1) / kXcd * kXcd * inner_n;
}

// Top-1 combine fused into GEMM-2 leaves rows of dropped tokens unwritten: zero them, spread over
// all work-groups (a dropped token has no other writer).
__device__ __forceinline__ void zero_dropped_rows(const WsGemmArgs& a, int tid, int nthreads) {
    if (!a.zero_slot_idx) return;
    for (int t = blockIdx.x; t < a.T; t += gridDim.x) {
        if (a.zero_slot_idx[t] < 0) {
            uint4* o = reinterpret_cast<uint4*>(a.out + (size_t)t * a.N);
            for (int i = tid; i < a.N / 8; i += nthreads) o[i] = make_uint4(0, 0, 0, 0);
        }
    }
}

// 16-byte loads and stores with the non-temporal hint: data that passes through once (expert weights at a
// few rows per expert, results nobody reads soon) should not push reusable lines out of the caches.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream16(void* p, const uint4 o) {
    const u32x4_t v = {o.x, o.y, o.z, o.w};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(p));
}

// 8 bf16 biases of columns n_lane.. as loaded (zero without a bias vector), and their fp32 values
__device__ __forceinline__ uint4 load_bias_raw(const WsGemmArgs& a, int g, int n_lane) {
    return a.bias ? *reinterpret_cast<const uint4*>(a.bias + (size_t)g * a.N + n_lane) : make_uint4(0, 0, 0, 0);
}
__device__ __forceinline__ void unpack_bias8(const uint4 bv, float (&bias)[8]) {
    bias[0] = __uint_as_float(bv.x << 16); bias[1] = __uint_as_float(bv.x & 0xffff0000u);
    bias[2] = __uint_as_float(bv.y << 16); bias[3] = __uint_as_float(bv.y & 0xffff0000u);
    bias[4] = __uint_as_float(bv.z << 16); bias[5] = __uint_as_float(bv.z & 0xffff0000u);
    bias[6] = __uint_as_float(bv.w << 16); bias[7] = __uint_as_float(bv.w & 0xffff0000u);
}
__device__ __forceinline__ void load_bias8(const WsGemmArgs& a, int g, int n_lane, float (&bias)[8]) {
    unpack_bias8(load_bias_raw(a, g, n_lane), bias);
}

// Token and gate probability of expert row `row` of group g (top-1 combine fused into GEMM-2)
__device__ __forceinline__ void scatter_lookup(const WsGemmArgs& a, int g, int row, int& t, float& gw) {
    t = a.scatter_map[(size_t)g * a.scatter_stride + row];
    gw = a.gate_w[(size_t)t * a.top_k];
}

// Finishes NC (8 or 4) consecutive columns n_lane.. of row `row` (index inside group g): v = acc + bias on entry.
// EPI_SCATTER: (t, gw) = scatter_lookup of the row, fetched by the caller.
template <int EPI, int NC = 8>
__device__ __forceinline__ void finish_row(const WsGemmArgs& a, int g, int row, int ks, int n_lane, float (&v)[NC],
                                           int t = 0, float gw = 1.f) {
    static_assert(NC == 8 || NC == 4, "columns per lane");
    const long long grow = (long long)g * a.o_group_stride + row;   // row in [G, o_group_stride]
    if (EPI == EPI_PARTIAL) {
        float* o = a.partial + ((size_t)ks * a.partial_rows + grow) * a.N + n_lane;
#pragma unroll
        for (int q = 0; q < NC / 4; ++q)
            *reinterpret_cast<float4*>(o + 4 * q) = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
        return;
    }
    size_t orow = (size_t)grow;
    if (EPI == EPI_GELU) {
#pragma unroll
        for (int i = 0; i < NC; ++i) v[i] = gelu_tanh(v[i]);
    } else if (EPI == EPI_SCATTER) {
#pragma unroll
        for (int i = 0; i < NC; ++i) v[i] *= gw;
        orow = (size_t)t;
    } else if (EPI == EPI_COMBINE) {
        // dense branch + sum_j keep_j g_j ye[e_j, slot_j, :] for token grow
        for (int j = 0; j < a.top_k; ++j) {
            const int s = a.slot_idx[grow * a.top_k + j];
            if (s < 0) continue;
            const int e = a.expert_idx[grow * a.top_k + j];
            const float gw = a.gate_w[grow * a.top_k + j];
            const uint16_t* yp = a.ye + ((size_t)e * a.C + s) * a.N + n_lane;
            uint32_t y[NC / 2];
            if (NC == 8) {
                const uint4 yv = *reinterpret_cast<const uint4*>(yp);
                y[0] = yv.x; y[1] = yv.y; y[NC / 2 - 2] = yv.z; y[NC / 2 - 1] = yv.w;
            } else {
                const uint2 yv = *reinterpret_cast<const uint2*>(yp);
                y[0] = yv.x; y[1] = yv.y;
            }
#pragma unroll
            for (int q = 0; q < NC / 2; ++q) {
                v[2 * q] = fmaf(gw, __uint_as_float(y[q] << 16), v[2 * q]);
                v[2 * q + 1] = fmaf(gw, __uint_as_float(y[q] & 0xffff0000u), v[2 * q + 1]);
            }
        }
    }
    uint32_t o[NC / 2];
#pragma unroll
    for (int q = 0; q < NC / 2; ++q) o[q] = pack_bf16x2(v[2 * q], v[2 * q + 1]);
    // h and the layer output are written once and read much later or never: streaming stores keep them
    // from displacing the activation rows in L2.  Expert outputs and split-K partials are read back at once.
    uint16_t* dst = a.out + orow * a.N + n_lane;
    if (NC == 8) {
        const uint4 ov = make_uint4(o[0], o[1], o[NC / 2 - 2], o[NC / 2 - 1]);
        if (EPI == EPI_STORE) *reinterpret_cast<uint4*>(dst) = ov;
        else store_stream16(dst, ov);
    } else {
        const uint2 ov = make_uint2(o[0], o[1]);
        if (EPI == EPI_STORE) *reinterpret_cast<uint2*>(dst) = ov;
        else __builtin_nontemporal_store(__builtin_bit_cast(unsigned long long, ov), reinterpret_cast<unsigned long long*>(dst));
    }
}

}  // namespace moe
