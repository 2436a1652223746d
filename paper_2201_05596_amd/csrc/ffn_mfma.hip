// bf16 grouped GEMM for the expert FFNs on gfx950 matrix cores (paper Sec. 3.1:
// every expert is an FFN; Sec. 5.1: at inference the time to read the parameters
// from memory dominates).  One kernel template serves both products of the FFN,
// the dense branch of Residual-MoE (Sec. 4.1.1) and, through its epilogues, the
// two layout transforms of Sec. 5.4 fused into the GEMMs:
//   * GEMM-1 may read its rows straight from the token matrix through the
//     slot->token table (dispatch without a dispatch buffer);
//   * GEMM-2 may scale by the gate probability and write straight to the
//     token's output row (top-1 combine without an expert-output buffer), or
//     add the gathered expert outputs to the dense branch.
//
// Design: weight-streaming.  With tens of rows per expert the arithmetic
// intensity is ~rows flop/byte, far below the MI355X ridge, so the kernel is
// organised around reading every weight byte exactly once at full HBM rate:
//   * a wave owns 128 output columns and marches down K; weights go
//     HBM -> registers with 16-byte loads (8 columns of one k-row per lane),
//     never through LDS, several 32-row "super-fragments" in flight;
//   * the MFMA B operand needs 8 consecutive k per lane, the loads deliver 8
//     consecutive n: an 8x8 16-bit transpose in registers (v_perm_b32) turns
//     eight loads into eight B fragments, whose columns are interleaved
//     (fragment i holds columns 8c+i) -- harmless, the epilogue then finds 8
//     consecutive columns per lane and stores 16 bytes;
//   * the small activation tile (MT rows x K) is shared by the block's waves
//     through LDS in double-buffered k-chunks, rows padded by 16 bytes so the
//     16-lane A-fragment reads hit distinct banks;
//   * v_mfma_f32_16x16x32_bf16, fp32 accumulation.
// Work-groups are numbered so that all row tiles of one (expert, column tile)
// run on the same XCD back to back and share the weights through that XCD's L2.
#include "ffn_common.h"

namespace moe {

constexpr int kSF = 32;             // k-rows per super-fragment (one 16x16x32 MFMA deep)
constexpr int kWaveCols = 128;      // output columns per wave
constexpr int kLdsTileElems = 8192; // MT * KC: bf16 elements of one LDS activation buffer

// One tile of work: virtual block vb computes rows m0.. of group g, column tile nt, k-split ks.
struct WsWork {
    int vb, g, nt, m0, nrows, ch_beg, ch_end;
};

// Compile-time shape of a tile and what follows from it
template <int MT, int NW> struct WsTile {
    static constexpr int NT = NW * 64;
    static constexpr int MSUB = MT / 16;
    static constexpr int KC = kLdsTileElems / MT;        // k-extent of one LDS chunk
    static constexpr int STRIDE = KC * 2 + 16;           // bytes per LDS row
    static constexpr int PIECES = MT * KC / 8;           // 16-byte pieces per chunk
    static constexpr int NP = PIECES / NT;               // pieces per thread
    static constexpr int SFC = KC / kSF;                 // super-fragments per chunk
    static constexpr int LDS_A = 2 * MT * STRIDE;        // the two activation buffers
    static_assert(PIECES % NT == 0 && SFC >= 1, "tile configuration");
};

// Tile counts of one GEMM (uniform over the grid)
struct WsGeo {
    int n_tiles, m_tiles, inner_n, chunks_total, chunks_per;
};
template <int MT, int NW> __device__ __forceinline__ WsGeo ws_geo(const WsGemmArgs& a) {
    WsGeo g;
    g.n_tiles = (a.N + NW * kWaveCols - 1) / (NW * kWaveCols);
    g.m_tiles = (a.max_rows + MT - 1) / MT;
    g.inner_n = g.m_tiles * a.ksplit;
    g.chunks_total = (a.K + WsTile<MT, NW>::KC - 1) / WsTile<MT, NW>::KC;
    g.chunks_per = (g.chunks_total + a.ksplit - 1) / a.ksplit;     // whole chunks per k-split
    return g;
}

// The first virtual block vb, vb + stride, ... below `limit` that has work, as a tile; t.vb >= limit if none.
// Uniform over the work-group.
template <int MT, int EPI>
__device__ __forceinline__ WsWork ws_find_work(const WsGemmArgs& a, const WsGeo& geo, int vb, int limit, int stride) {
    WsWork t{};
    for (; vb < limit; vb += stride) {
        const TileId tile = tile_of_block(a, geo.n_tiles, geo.inner_n, vb);
        if (!tile.live) continue;
        const int rows = a.rows ? min(a.rows[tile.g], a.max_rows) : a.fixed_rows;
        const int mt = tile.inner % geo.m_tiles, ks = tile.inner / geo.m_tiles;
        if (mt * MT >= rows) continue;
        t.ch_beg = ks * geo.chunks_per;
        t.ch_end = min(t.ch_beg + geo.chunks_per, geo.chunks_total);
        if (t.ch_beg >= t.ch_end && EPI != EPI_PARTIAL) continue;
        t.g = tile.g; t.nt = tile.nt; t.m0 = mt * MT; t.nrows = min(MT, rows - t.m0);
        break;
    }
    t.vb = vb;
    return t;
}

// One tile: prologue (row table, first activation chunk), the weight stream down K, epilogue.  `nxt` is the
// work-group's next tile OF THE SAME GEMM (has_next false if there is none): the fragments fetched ahead at the
// end of this tile are its first ones, and `primed` tells the next call that they are in `raw` already.
template <int MT, int NW, int EPI, int NBUF, bool PACKED>
__device__ __forceinline__ void ws_tile(const WsGemmArgs& a, const WsGeo& geo, const WsWork& cur, const WsWork& nxt,
                                        const bool has_next, uint4 (&raw)[NBUF][8], bool& primed, char* lds,
                                        long long* arow_sh, int* tok_sh, float* gw_sh) {
    typedef WsTile<MT, NW> TC;
    constexpr int NT = TC::NT, MSUB = TC::MSUB, KC = TC::KC, STRIDE = TC::STRIDE, NP = TC::NP, SFC = TC::SFC;
    static_assert(SFC % NBUF == 0, "tile configuration");
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int c = lane & 15, kg = lane >> 4;
    const int chunks_per = geo.chunks_per;
    // first of the 8 columns of this lane in column tile nt
    auto lane_col = [&](int nt) { return nt * (NW * kWaveCols) + w * kWaveCols + c * 8; };
    int akp[NP];                                   // k-offset of this thread's activation pieces
#pragma unroll
    for (int i = 0; i < NP; ++i) akp[i] = ((tid + i * NT) % (KC / 8)) * 8;

    const int g = cur.g, m0 = cur.m0, nrows = cur.nrows, ch_beg = cur.ch_beg, ch_end = cur.ch_end;

    // ---- per-lane weight pointers: 8 columns n_lane..n_lane+7 of rows k, this tile and the next ----
    const int n_lane_raw = lane_col(cur.nt);
    const bool col_ok = n_lane_raw < a.N;
    const int n_lane = col_ok ? n_lane_raw : a.N - 8;             // clamp: loads stay in bounds, never stored
    // K-major weights: 8 columns n_lane.. of a k-row.  Packed weights: the wave's 128-column group (column tile nt,
    // wave w), whose eight fragments of one 32-deep k-block are 8 KB in a row; a lane takes 16 bytes of each.
    const int p_kb = (a.K + 31) / 32, p_ng = (a.N + 127) / 128;
    auto packed_base = [&](int gg, int nt) {
        const int grp = min(nt * NW + w, p_ng - 1);               // clamped like the column: loaded, never stored
        return a.B + ((size_t)gg * p_kb * p_ng + grp) * 4096 + lane * 8;
    };
    const uint16_t* Bg = PACKED ? packed_base(g, cur.nt) : a.B + (size_t)g * a.K * a.N + n_lane;
    // everything the epilogue needs from memory is fetched here: a load issued after the weight
    // fragments that run ahead into the next tile could only be waited for together with them
    const uint4 bias_raw = EPI != EPI_PARTIAL ? load_bias_raw(a, g, n_lane) : make_uint4(0, 0, 0, 0);
    const uint16_t* Bn = PACKED ? packed_base(has_next ? nxt.g : g, has_next ? nxt.nt : cur.nt)
                                : a.B + (size_t)(has_next ? nxt.g : g) * a.K * a.N + min(lane_col(has_next ? nxt.nt : cur.nt), a.N - 8);
    const int k_end_pad = ch_end * KC;                          // first k that belongs to the next tile
    const int k_next = has_next ? nxt.ch_beg * KC : 0;

    // weight super-fragment: rows k0 + kg*8 + j, j = 0..7.  K is a multiple of 8: a lane's 8 rows are all
    // inside or all outside.  Rows in [K, k_end_pad) re-read the last 8 rows (in bounds) and meet zeros on
    // the activation side; rows from k_end_pad on are the first rows of the NEXT tile of this work-group,
    // so the fragments fetched ahead at the end of a tile are the next tile's first ones and the weight
    // stream does not stop for the epilogue (without a next tile they re-read this tile's first rows).
    // Packed: dst[j] is fragment j of k-block k0/32 (k0 is a multiple of 32), same rules per k-block.
    auto b_load = [&](uint4 (&dst)[8], int k0) {
        if constexpr (PACKED) {
            const bool own = k0 < k_end_pad;
            const int kb = min((own ? k0 : k0 - k_end_pad + k_next) / kSF, p_kb - 1);
            const uint16_t* p = (own ? Bg : Bn) + (size_t)kb * p_ng * 4096;
#pragma unroll
            for (int j = 0; j < 8; ++j) dst[j] = load_stream16(p + j * 512);
        } else {
            const int kk = k0 + kg * 8;
            const bool own = kk < k_end_pad;
            const uint16_t* p = (own ? Bg : Bn) + (size_t)min(own ? kk : kk - k_end_pad + k_next, a.K - 8) * a.N;
#pragma unroll
            for (int j = 0; j < 8; ++j) dst[j] = load_stream16(p + (size_t)j * a.N);
        }
    };
    // The tile's first weight fragments go out before anything else (unless the previous tile already fetched
    // them): the row table and the epilogue inputs below cost another memory round trip or two, which the
    // weights now share instead of following.
    if (!primed && ch_beg < ch_end) {
#pragma unroll
        for (int b = 0; b < NBUF - 1; ++b) b_load(raw[b], ch_beg * KC + b * kSF);
    }

    // ---- A rows of the tile ----------------------------------------------------------
    lds_barrier();                                              // the previous tile's readers are done
    if (tid < MT) {
        const int r = m0 + min(tid, nrows - 1);                 // rows past the end alias the last valid one
        long long ar;
        if (a.row_map) ar = a.row_map[(size_t)g * a.map_stride + r];
        else ar = (long long)g * a.a_group_stride + r;
        arow_sh[tid] = ar;
        if (EPI == EPI_SCATTER) scatter_lookup(a, g, r, tok_sh[tid], gw_sh[tid]);
    }
    lds_barrier();

    f32x4_t acc[MSUB][8];
#pragma unroll
    for (int i = 0; i < MSUB; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // activation chunk: global -> registers -> LDS.  Each thread moves NP 16-byte pieces per chunk;
    // their rows and k-offsets never change, so the row pointers are formed once.  The loads are
    // unconditional (k clamped into the row, the value replaced by zero past K) so that the main
    // loop has no branches around memory operations and the prefetches really stay in flight.
    const uint16_t* arow_ptr[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) arow_ptr[i] = a.A + (size_t)arow_sh[(tid + i * NT) / (KC / 8)] * a.K;
    uint4 areg[NP];
    auto a_load = [&](int ch) {                     // loads only: nothing here waits for them
        const int k0 = ch * KC;
#pragma unroll
        for (int i = 0; i < NP; ++i)
            areg[i] = *reinterpret_cast<const uint4*>(arow_ptr[i] + min(k0 + akp[i], a.K - 8));
    };
    auto a_store = [&](int ch, int buf) {           // zero past K, then registers -> LDS
        char* base = lds + buf * MT * STRIDE;
        const int k0 = ch * KC;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int p = tid + i * NT;
            const int r = p / (KC / 8), kp = p % (KC / 8);
            const bool in = k0 + akp[i] < a.K;
            const uint4 v = areg[i];
            *reinterpret_cast<uint4*>(base + r * STRIDE + kp * 16) =
                make_uint4(in ? v.x : 0u, in ? v.y : 0u, in ? v.z : 0u, in ? v.w : 0u);
        }
    };

    auto sf_compute = [&](const uint4 (&src)[8], const char* a_lane) {
        bf16x8_t af[MSUB];
#pragma unroll
        for (int ms = 0; ms < MSUB; ++ms)
            af[ms] = *reinterpret_cast<const bf16x8_t*>(a_lane + ms * 16 * STRIDE);
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) {
            bf16x8_t blo, bhi;
            if constexpr (PACKED) {
                blo = __builtin_bit_cast(bf16x8_t, src[2 * qq]);
                bhi = __builtin_bit_cast(bf16x8_t, src[2 * qq + 1]);
            } else {
                b_frag_pair(src, qq, blo, bhi);
            }
#pragma unroll
            for (int ms = 0; ms < MSUB; ++ms) {
                acc[ms][2 * qq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[ms], blo, acc[ms][2 * qq], 0, 0, 0);
                acc[ms][2 * qq + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[ms], bhi, acc[ms][2 * qq + 1], 0, 0, 0);
            }
        }
    };

    if (ch_beg < ch_end) {
        // prologue: first activation chunk in LDS (the first weight super-fragments are in flight already)
        a_load(ch_beg);
        a_store(ch_beg, 0);
        lds_barrier();

        const char* a_lane0 = lds + (lane & 15) * STRIDE + kg * 16;
        for (int ch = ch_beg; ch < ch_end; ++ch) {
            const int buf = (ch - ch_beg) & 1;
            a_load(ch + 1);                    // next chunk (past the end: clamped and zeroed, never used)
            __builtin_amdgcn_sched_barrier(0);
            const char* a_lane = a_lane0 + buf * MT * STRIDE;
            const int kbase = ch * KC;
#pragma unroll
            for (int s = 0; s < SFC; s += NBUF) {
#pragma unroll
                for (int b = 0; b < NBUF; ++b) {
                    // keep NBUF-1 super-fragments in flight: fetch the one NBUF-1 ahead, then use slot b.
                    // The scheduling barriers pin that order: left alone, the compiler sinks the loads
                    // down to their first use and the prefetch distance collapses to zero.
                    b_load(raw[(b + NBUF - 1) % NBUF], kbase + (s + b + NBUF - 1) * kSF);
                    __builtin_amdgcn_sched_barrier(0);
                    sf_compute(raw[b], a_lane + (s + b) * kSF * 2);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            a_store(ch + 1, buf ^ 1);
            lds_barrier();
        }
        primed = has_next;
    } else {
        primed = false;
    }

    // ---- epilogue ------------------------------------------------------------------------
    if (col_ok) {
        const int mg = kg;                                     // D: rows 4*(lane/16)+r, column lane%16
        const int ks = ch_beg / chunks_per;
        float bias[8];
        unpack_bias8(bias_raw, bias);
#pragma unroll
        for (int ms = 0; ms < MSUB; ++ms) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int rl = ms * 16 + mg * 4 + r;
                if (rl >= nrows) continue;
                float v[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = acc[ms][i][r] + bias[i];
                finish_row<EPI>(a, g, m0 + rl, ks, n_lane, v, EPI == EPI_SCATTER ? tok_sh[rl] : 0,
                                EPI == EPI_SCATTER ? gw_sh[rl] : 1.f);
            }
        }
    }
}

template <int MT, int NW, int EPI, int NBUF, bool PACKED>
__global__ __launch_bounds__(NW * 64) void wsgemm_kernel(const WsGemmArgs a, const int total_blocks) {
    typedef WsTile<MT, NW> TC;
    __shared__ __attribute__((aligned(16))) char lds[TC::LDS_A];
    __shared__ long long arow_sh[MT];
    __shared__ int tok_sh[MT];                     // EPI_SCATTER: token and gate probability of the tile's rows
    __shared__ float gw_sh[MT];

    const WsGeo geo = ws_geo<MT, NW>(a);
    if (EPI == EPI_SCATTER) zero_dropped_rows(a, threadIdx.x, TC::NT);

    // The grid holds as many work-groups as fit on the chip at once; work-group b takes the virtual
    // blocks b, b + gridDim.x, ... that have work (the XCD of a virtual block is that of b: the grid
    // is a multiple of the XCD count).  Knowing the next tile early lets the weight stream run on
    // across tile boundaries.
    uint4 raw[NBUF][8];                            // weight super-fragments in flight
    bool primed = false;                           // raw[0..NBUF-2] already hold the tile's first fragments
    WsWork cur = ws_find_work<MT, EPI>(a, geo, blockIdx.x, total_blocks, gridDim.x);
    while (cur.vb < total_blocks) {
        const WsWork nxt = ws_find_work<MT, EPI>(a, geo, cur.vb + gridDim.x, total_blocks, gridDim.x);
        ws_tile<MT, NW, EPI, NBUF, PACKED>(a, geo, cur, nxt, nxt.vb < total_blocks, raw, primed, lds, arow_sh, tok_sh, gw_sh);
        cur = nxt;
    }
}

// ------------------------------------------------------------------------------------------
// Split-K finish: out = epilogue( sum_s partial[s] + bias ), splits summed in index order so the
// result does not depend on scheduling.  One wave per expert row and 512-column piece of it.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const SplitKReduceArgs a) {
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long nwaves = (long long)gridDim.x * 4;
    const long long total_rows = (long long)a.G * a.group_stride;
    if (a.scatter_map && a.zero_slot_idx) {
        for (long long t = wave; t < a.T; t += nwaves) {
            if (a.zero_slot_idx[t] < 0) {
                uint4* o = reinterpret_cast<uint4*>(a.out + (size_t)t * a.N);
                for (int i = lane; i < a.N / 8; i += 64) o[i] = make_uint4(0, 0, 0, 0);
            }
        }
    }
    // one wave per (row, 512-column piece): few rows (a decode step) still spread over the chip
    const int pieces = (a.N / 8 + 63) / 64;
    for (long long item = wave; item < total_rows * pieces; item += nwaves) {
        const long long row = item / pieces;
        const int i = (int)(item % pieces) * 64 + lane;
        const int g = (int)(row / a.group_stride), r = (int)(row % a.group_stride);
        if (r >= (a.rows ? min(a.rows[g], a.max_rows) : a.max_rows) || i >= a.N / 8) continue;
        float gw = 1.f;
        size_t orow = (size_t)row;
        if (a.scatter_map) {
            const int t = a.scatter_map[row];
            gw = a.gate_w[(size_t)t * a.top_k];
            orow = (size_t)t;
        }
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = 0.f;
        const float* p0 = a.partial + (size_t)row * a.N + (size_t)i * 8;
        const size_t sstride = (size_t)total_rows * a.N;
        int s = 0;
        for (; s + 4 <= a.ksplit; s += 4) {                     // four splits' loads in flight, summed in split order
            float4 x0[4], x1[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float* p = p0 + (size_t)(s + u) * sstride;
                x0[u] = *reinterpret_cast<const float4*>(p);
                x1[u] = *reinterpret_cast<const float4*>(p + 4);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                v[0] += x0[u].x; v[1] += x0[u].y; v[2] += x0[u].z; v[3] += x0[u].w;
                v[4] += x1[u].x; v[5] += x1[u].y; v[6] += x1[u].z; v[7] += x1[u].w;
            }
        }
        for (; s < a.ksplit; ++s) {
            const float* p = p0 + (size_t)s * sstride;
            const float4 x0 = *reinterpret_cast<const float4*>(p), x1 = *reinterpret_cast<const float4*>(p + 4);
            v[0] += x0.x; v[1] += x0.y; v[2] += x0.z; v[3] += x0.w;
            v[4] += x1.x; v[5] += x1.y; v[6] += x1.z; v[7] += x1.w;
        }
        if (a.bias) {
            const uint4 bv = *reinterpret_cast<const uint4*>(a.bias + (size_t)g * a.N + (size_t)i * 8);
            v[0] += __uint_as_float(bv.x << 16); v[1] += __uint_as_float(bv.x & 0xffff0000u);
            v[2] += __uint_as_float(bv.y << 16); v[3] += __uint_as_float(bv.y & 0xffff0000u);
            v[4] += __uint_as_float(bv.z << 16); v[5] += __uint_as_float(bv.z & 0xffff0000u);
            v[6] += __uint_as_float(bv.w << 16); v[7] += __uint_as_float(bv.w & 0xffff0000u);
        }
        uint4 o;
        o.x = pack_bf16x2(gw * v[0], gw * v[1]); o.y = pack_bf16x2(gw * v[2], gw * v[3]);
        o.z = pack_bf16x2(gw * v[4], gw * v[5]); o.w = pack_bf16x2(gw * v[6], gw * v[7]);
        *reinterpret_cast<uint4*>(a.out + orow * a.N + (size_t)i * 8) = o;
    }
}

int launch_splitk_reduce(const SplitKReduceArgs& a, hipStream_t s) {
    const long long total_rows = (long long)a.G * a.group_stride;
    long long blocks = (total_rows * ((a.N / 8 + 63) / 64) + 3) / 4;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// ------------------------------------------------------------------------------------------
// work-groups of `kernel` that fit on the chip at once (a multiple of the XCD count), cached by the caller
static int resident_blocks(const void* kernel, int threads) {
    int per_cu = 0, dev = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess || per_cu < 1) per_cu = 1;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < kXcd)
        cus = 256;
    return per_cu * cus / kXcd * kXcd;
}

template <int MT, int NW, int EPI, int NBUF, bool PACKED>
static bool launch_cfg_p(const WsGemmArgs& a, hipStream_t s) {
    const int n_tiles = (a.N + NW * kWaveCols - 1) / (NW * kWaveCols);
    const int m_tiles = (a.max_rows + MT - 1) / MT;
    const long long total = tile_grid_blocks(a, n_tiles, m_tiles * a.ksplit);      // a multiple of the XCD count
    if (total > (1ll << 30)) return false;
    static int resident = 0;                                                       // one per instantiation
    if (!resident) resident = resident_blocks(reinterpret_cast<const void*>(&wsgemm_kernel<MT, NW, EPI, NBUF, PACKED>), NW * 64);
    const long long blocks = total < resident ? total : resident;
    hipLaunchKernelGGL((wsgemm_kernel<MT, NW, EPI, NBUF, PACKED>), dim3((unsigned)blocks), dim3(NW * 64), 0, s, a, (int)total);
    return true;
}
template <int MT, int NW, int EPI, int NBUF>
static bool launch_cfg(const WsGemmArgs& a, hipStream_t s) {
    return a.packed ? launch_cfg_p<MT, NW, EPI, NBUF, true>(a, s) : launch_cfg_p<MT, NW, EPI, NBUF, false>(a, s);
}

template <int EPI>
static bool launch_epi(const WsGemmArgs& a, int MT, int NW, int NBUF, hipStream_t s) {
#define MOE_WS_CASE(mt, nw, nb) if (MT == mt && NW == nw && NBUF == nb) return launch_cfg<mt, nw, EPI, nb>(a, s);
    MOE_WS_CASE(16, 4, 2) MOE_WS_CASE(16, 2, 2) MOE_WS_CASE(32, 4, 2) MOE_WS_CASE(32, 2, 2)
    MOE_WS_CASE(64, 4, 2) MOE_WS_CASE(64, 2, 2)
#undef MOE_WS_CASE
    return false;
}

bool wsgemm_supported(int K, int N) { return K % 8 == 0 && N % 8 == 0 && K >= 8 && N >= 8; }

void wsgemm_pick_tile(int max_rows, int G, int N, int* MT, int* NW) {
    *MT = max_rows <= 16 ? 16 : max_rows <= 32 ? 32 : 64;
    // enough work-groups to put two on every CU, otherwise narrower ones
    const long long m_tiles = (max_rows + *MT - 1) / *MT;
    const long long blocks4 = (long long)G * ((N + 4 * kWaveCols - 1) / (4 * kWaveCols)) * m_tiles;
    *NW = blocks4 >= 512 ? 4 : 2;
}

int wsgemm_chunk_k(int MT) { return kLdsTileElems / MT; }

int launch_wsgemm(const WsGemmArgs& a, int epi, int MT, int NW, int NBUF, hipStream_t s) {
    if (a.G <= 0 || a.max_rows <= 0) return MOE_OK;
    if (a.ksplit < 1 || (a.ksplit > 1 && epi != EPI_PARTIAL)) return MOE_ERR_INVALID_ARG;
    bool ok = false;
    switch (epi) {
        case EPI_STORE: ok = launch_epi<EPI_STORE>(a, MT, NW, NBUF, s); break;
        case EPI_GELU: ok = launch_epi<EPI_GELU>(a, MT, NW, NBUF, s); break;
        case EPI_SCATTER: ok = launch_epi<EPI_SCATTER>(a, MT, NW, NBUF, s); break;
        case EPI_COMBINE: ok = launch_epi<EPI_COMBINE>(a, MT, NW, NBUF, s); break;
        case EPI_PARTIAL: ok = launch_epi<EPI_PARTIAL>(a, MT, NW, NBUF, s); break;
        default: return MOE_ERR_INVALID_ARG;
    }
    if (!ok) return MOE_ERR_INVALID_ARG;
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace moe
