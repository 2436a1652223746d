// Tiled bf16 MFMA grouped GEMM for groups with many rows: experts holding more than 64 tokens and
// the dense branch of Residual-MoE (paper Sec. 4.1.1), where the products are bound by the matrix
// cores, not by weight traffic.
//
// A work-group of NWM x 2 waves owns a (NWM*64) x (2*WN) output tile; a wave owns 64 x WN of it (WN = 128, or 64
// for products with few columns).  Both operands pass through LDS in 32-deep k-stages, 3 to 6 stages deep, filled by direct
// global->LDS loads (global_load_lds_dwordx4: 16 bytes per lane, a wave writes 1 KB of contiguous
// LDS per instruction, no staging registers), so all stages but one are always in flight:
//   * weights: 32 k-rows x 2*WN columns, K-major exactly as in memory (a wave instruction copies
//     two or four whole rows); a wave reads its WN columns as eight row pieces per lane and turns
//     them into WN/16 MFMA B fragments with the same in-register transpose as the streaming
//     kernel.  Each weight byte is fetched from L2 once per work-group and serves NWM*WM rows;
//   * activations: NWM*WM rows x 64 bytes.  Direct loads leave no room for row padding, so bank
//     conflicts of the A-fragment reads (16 lanes, 16 rows, same k) are avoided by a swizzle done
//     on the global side: 16-byte slot `pos` of row r holds k-piece pos ^ a_swizzle(r).
// The direct loads are issued through inline asm: the compiler then does not know they write LDS
// and does not put a full vmcnt(0) wait in front of every LDS read; completion is tracked by hand
// (in-order vmcnt: 8 loads per wave and stage).
// v_mfma_f32_16x16x32_bf16, fp32 accumulation; epilogues shared with the streaming kernel.
// Requires K to be a multiple of 32 (no zero fill is possible on the way into LDS).
#include "ffn_common.h"
#include <type_traits>

namespace moe {

constexpr int kTK = 32;            // k-rows per stage

// 16 bytes per lane from global memory straight into LDS at lds_wave_base + lane*16
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_wave_base) : "memory", "m0");
}
// A 64-lane 16-byte LDS read is served in four passes of 16 lanes, and the passes are not runs of
// consecutive lanes: pass 0 takes lanes 0-3, 12-15, 20-23, 24-27, pass 1 lanes 4-7, 8-11, 16-19,
// 28-31, passes 2 and 3 the same +32.  With rows of 64 bytes a lane (row m, k-group kg) reads 16-byte
// unit 4*(m%4) + slot, so the four lanes of a pass that share m%4 need four different slots.  Taking
// slot = kg ^ f(m/4) with f = {0, 2, 3, 1} does that for every pass.
__device__ __forceinline__ int a_swizzle(int row) { return (0x78 >> (((row >> 2) & 3) * 2)) & 3; }

template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// NWM waves along the rows x 2 along the columns; each owns WM rows x WN columns (WN = 128, or 64 for products
// with so few columns that 256-column tiles would leave CUs without work)
template <int WM, int NWM, int NS_, int WN> struct TileCfg {
    static constexpr int NWAVES = NWM * 2;
    static constexpr int BM = NWM * WM;
    static constexpr int TBN = 2 * WN;                         // tile columns
    static constexpr int B_BYTES = kTK * TBN * 2;              // weight bytes per stage (16 or 8 KB)
    static constexpr int A_BYTES = BM * 64;                    // activation bytes per stage
    static constexpr int STAGE = A_BYTES + B_BYTES;
    // 256-row tiles: 4 stages of 32 KB, one work-group of 8 waves per CU.  128-row tiles: 5 stages of 24 KB and one
    // work-group of 4 waves per CU, or 3 stages and at most 256 registers per lane, so that two work-groups share a
    // CU and one multiplies while the other waits at its barrier: much faster for short K (8192 x 1024 x 4096:
    // 92 against 141 us), slightly slower for long K, where the deeper ring counts.
    static constexpr int NS = NS_;
    static constexpr int WGS_PER_CU = NS_ * (NWM * WM * 64 + B_BYTES) + NWM * WM * 8 <= 80 * 1024 && NWM == 2 ? 2 : 1;
    static constexpr int NIA = A_BYTES / 1024 / NWAVES;        // activation loads per wave and stage
    static constexpr int NIB = B_BYTES / 1024 / NWAVES;        // weight loads per wave and stage
    static constexpr int RPI = 1024 / (TBN * 2);               // k-rows one weight load (1 KB) covers: 2 or 4
    // Tiles of 256 rows that hold at most 128 valid ones (lightly loaded experts, the last rows of a busy one) need
    // only half of the activation space; the ring is then cut into 6 stages of 24 KB instead of 4 of 32 KB, which
    // keeps 80 KB of weights in flight instead of 48 KB: such tiles are bound by the rate one CU can stream at.
    static constexpr bool HAS_LIGHT = NWM == 4 && WN == 128;
    static constexpr int L_ROWS = NWAVES * 16;                 // one activation load per wave and stage
    static constexpr int L_A_BYTES = L_ROWS * 64;
    static constexpr int L_STAGE = L_A_BYTES + B_BYTES;
    static constexpr int L_NS = 6;
    static constexpr int RING = HAS_LIGHT && L_NS * L_STAGE > NS * STAGE ? L_NS * L_STAGE : NS * STAGE;
    static constexpr int LDS_BYTES = RING + BM * 8;
};

template <int WM, int NWM, int NSX, int EPI, int WN, bool PACKED>
__global__ __launch_bounds__(NWM * 128, (TileCfg<WM, NWM, NSX, WN>::WGS_PER_CU)) void tgemm_kernel(const WsGemmArgs a0,
                                                                                                   const WsGemmArgs a1,
                                                                                                   const int split) {
    // One launch may carry two grouped products of the same shape class (the experts' and the dense branch's of a
    // Residual-MoE layer): work-groups below `split` belong to the first, the others to the second.  Twice the tiles
    // let products with few columns use the large tile and still give every CU one.
    const bool second = (int)blockIdx.x >= split;                // uniform over the work-group
    const WsGemmArgs& a = second ? a1 : a0;
    const int block = second ? (int)blockIdx.x - split : (int)blockIdx.x;
    typedef TileCfg<WM, NWM, NSX, WN> Cfg;
    constexpr int TBN = Cfg::TBN, NCF = WN / 16;               // column fragments (= columns per lane) of a wave
    constexpr int BM = Cfg::BM, MSUB = WM / 16, NIB = Cfg::NIB, NTHREADS = NWM * 128;

    extern __shared__ __attribute__((aligned(16))) char lds[];   // the ring of stages, then BM row indices
    long long* arow_sh = reinterpret_cast<long long*>(lds + Cfg::RING);
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds));   // LDS byte offset of the segment

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave number, in a scalar register
    const int c = lane & 15, kg = lane >> 4;
    const int wm = w >> 1, wn = w & 1;

    const int n_tiles = (a.N + TBN - 1) / TBN;
    const int m_tiles = (a.max_rows + BM - 1) / BM;
    const TileId tile = tile_spread(a, n_tiles) ? tile_of_block_spread(a, n_tiles, m_tiles, block)
                                                : tile_of_block(a, n_tiles, m_tiles, block);
    const int g = tile.g, nt = tile.nt, mt = tile.inner;

    if (EPI == EPI_SCATTER) zero_dropped_rows(a, tid, NTHREADS);
    if (!tile.live) return;
    const int rows = a.rows ? min(a.rows[g], a.max_rows) : a.fixed_rows;
    const int m0 = mt * BM;
    if (m0 >= rows) return;
    const int nrows = min(BM, rows - m0);

    for (int i = tid; i < BM; i += NTHREADS) {
        const int r = m0 + min(i, nrows - 1);                   // rows past the end alias the last valid one
        arow_sh[i] = a.row_map ? (long long)a.row_map[(size_t)g * a.map_stride + r] : (long long)g * a.a_group_stride + r;
    }
    __syncthreads();

    // The rest of the kernel exists once per number ACT of 16-row sub-tiles that a wave works on:
    // a tile of a lightly loaded expert is pure weight streaming and must not pay matrix-core time
    // (or LDS reads) for rows that do not exist.  The choice is wave-uniform; a wave without valid rows
    // still takes part in the loads and barriers.  Separate copies (not branches inside one loop) keep
    // the accumulators of each copy in place in the register file.
    // A wave without valid rows (ACT = 0) still takes part in the loads and barriers, nothing else.
    const int nsub = __builtin_amdgcn_readfirstlane(max(0, (min(nrows - wm * WM, WM) + 15) / 16));
    auto run = [&](auto act_c, auto light_c, auto loada_c) {
    constexpr int ACT = decltype(act_c)::value;
    constexpr bool LIGHT = decltype(light_c)::value;
    constexpr bool LOADA = decltype(loada_c)::value;           // false: the 16 rows this wave would load do not exist
    constexpr int NA = ACT > 0 ? ACT : 1;                       // array extents
    constexpr int NS = LIGHT ? Cfg::L_NS : Cfg::NS, STAGE = LIGHT ? Cfg::L_STAGE : Cfg::STAGE;
    constexpr int A_BYTES = LIGHT ? Cfg::L_A_BYTES : Cfg::A_BYTES, NIA = !LOADA ? 0 : LIGHT ? 1 : Cfg::NIA;
    constexpr int PER_STAGE = NIA + NIB;                       // loads per wave and stage
    // The hand-written waits below count on this: every issue() puts exactly PER_STAGE direct loads of this wave in
    // flight (its two loops have compile-time trip counts NIA and NIB, no lane or wave skips one), loads complete in
    // order, NS - 1 stages are issued before the first wait, and each step issues one stage after waiting for all
    // but the NS - 3 youngest.  vmcnt is a 6-bit counter.
    static_assert(NS >= 3, "the ring needs a stage being read, one landing and one in flight");
    static_assert(PER_STAGE >= 1 && (NS - 1) * PER_STAGE < 64, "outstanding direct loads must fit the vmcnt field");
    static_assert(NIB * Cfg::NWAVES * 1024 == Cfg::B_BYTES, "the waves' weight loads tile a stage exactly");
    static_assert(!LOADA || NIA * Cfg::NWAVES * 1024 == A_BYTES, "the waves' activation loads tile a stage exactly");

    // ---- per-lane sources of the direct loads (fixed for the whole k-loop) ---------------------------
    // activations: wave w, load i copies rows (w*NIA + i)*16 .. +15; lane L -> row +L/4, slot L%4
    const uint16_t* a_src[NIA > 0 ? NIA : 1];
#pragma unroll
    for (int i = 0; i < NIA; ++i) {
        const int r = (w * NIA + i) * 16 + (lane >> 2);
        const int kp = (lane & 3) ^ a_swizzle(r);                 // swizzle
        a_src[i] = a.A + (size_t)arow_sh[r] * a.K + kp * 8;
    }
    // weights: wave w, load i copies the RPI k-rows (w*NIB + i)*RPI ..; lane L -> row +L/LPR, 16-byte column piece L%LPR
    constexpr int RPI = Cfg::RPI, LPR = 64 / RPI;
    const int n0 = nt * TBN;
    // With 128-column tiles a k-row is 256 bytes and a lane reads 8 bytes of it, so the two k-groups (rows 8 apart =
    // 2 KB) that one pass of such an LDS read serves would meet on the same banks: k-rows with bit 3 set are
    // stored with their two 128-byte halves swapped (b_half_swap), on this side by fetching the other half.
    static_assert(WN == 128 || NIB == 1, "the half swap assumes one weight load per wave and stage");
    const int b_row = w * NIB * RPI + lane / LPR;
    const int b_piece = (lane % LPR) ^ (WN == 64 ? ((b_row >> 3) & 1) * 8 : 0);
    // Packed weights: a stage of the tile is TBN/16 ready-made fragments of 1 KB; load i of wave w copies fragment
    // w*NIB + i (all of one wave's fragments lie in one 128-column group: NIB divides 8), whole and in place.
    static_assert(8 % NIB == 0, "a wave's weight loads stay inside one 128-column group");
    const int p_ng = (a.N + 127) / 128;
    const int p_grp = min(n0 / 128 + (w * NIB) / 8, p_ng - 1);             // clamped group: loaded, never stored
    const uint16_t* b_src = PACKED
        ? a.B + (((size_t)g * (a.K / kTK) * p_ng + p_grp) * 8 + (w * NIB) % 8) * 512 + lane * 8
        : a.B + (size_t)g * a.K * a.N + (size_t)b_row * a.N + min(n0 + b_piece * 8, a.N - 8);   // clamped column
    const size_t b_step2 = PACKED ? (size_t)512 : (size_t)RPI * a.N;        // from one load of a stage to the next
    const size_t b_kstep = PACKED ? (size_t)p_ng * 4096 : (size_t)kTK * a.N;   // from one stage to the next
    const int steps = a.K / kTK;
    auto issue = [&](int step) {                                // all loads of one stage, this wave's share
        const int st = min(step, steps - 1);                    // past the end: harmless re-read, keeps the count uniform
        const uint32_t base = lds0 + (step % NS) * STAGE;
        const int k0 = st * kTK;
#pragma unroll
        for (int i = 0; i < NIA; ++i)
            dma16(a_src[i] + k0, __builtin_amdgcn_readfirstlane(base + (w * NIA + i) * 1024));
        const uint16_t* bp = b_src + (size_t)st * b_kstep;
#pragma unroll
        for (int i = 0; i < NIB; ++i)
            dma16(bp + i * b_step2, __builtin_amdgcn_readfirstlane(base + A_BYTES + (w * NIB + i) * 1024));
    };

    f32x4_t acc[NA][NCF];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int j = 0; j < NCF; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // A fragment of sub-tile ms: row R = wm*WM + ms*16 + c, k-piece kg -> slot kg ^ a_swizzle(R);
    // a_swizzle(R) == a_swizzle(c) because the other terms are multiples of 16
    const int a_lane = (wm * WM + c) * 64 + ((kg ^ a_swizzle(c)) * 16);
    const int b_lane = PACKED ? A_BYTES + wn * (NCF * 1024) + lane * 16
                              : A_BYTES + (kg * 8) * (TBN * 2) + (((wn * WN + c * NCF) * 2) ^ (WN == 64 ? (kg & 1) * 128 : 0));

    // operand fragments of one stage in registers.  K-major weights: per k-row the lane's NCF columns (16 or 8
    // bytes), transposed in registers before use; packed weights: the NCF fragments as they are.
    typedef typename std::conditional<NCF == 8, uint4, uint2>::type BRaw;
    struct Frags {
        BRaw braw[PACKED ? 1 : 8];
        bf16x8_t bf[PACKED ? NCF : 1];
        bf16x8_t af[NA];
    };
    auto read_frags = [&](Frags& f, int buf) {
        if (ACT == 0) return;
        const char* base = lds + buf * STAGE;
        if constexpr (PACKED) {
#pragma unroll
            for (int j = 0; j < NCF; ++j) f.bf[j] = *reinterpret_cast<const bf16x8_t*>(base + b_lane + j * 1024);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) f.braw[j] = *reinterpret_cast<const BRaw*>(base + b_lane + j * (TBN * 2));
        }
#pragma unroll
        for (int ms = 0; ms < ACT; ++ms) f.af[ms] = *reinterpret_cast<const bf16x8_t*>(base + a_lane + ms * 16 * 64);
    };
    // dword q of a lane's row piece
    auto raw_dw = [](const BRaw& v, int q) -> uint32_t {
        if constexpr (NCF == 8) return dw(v, q);
        else return q == 0 ? v.x : v.y;
    };
    auto mma = [&](const Frags& f) {
        if (ACT == 0) return;
        if constexpr (PACKED) {
#pragma unroll
            for (int j = 0; j < NCF; ++j)
#pragma unroll
                for (int ms = 0; ms < ACT; ++ms)
                    acc[ms][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.af[ms], f.bf[j], acc[ms][j], 0, 0, 0);
        } else {
#pragma unroll
        for (int qq = 0; qq < NCF / 2; ++qq) {
            // 8 k-rows x 2 columns of 16-bit values -> two fragments (v_perm_b32), as in the streaming kernel
            uint32_t lo[4], hi[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t r0 = raw_dw(f.braw[2 * p], qq), r1 = raw_dw(f.braw[2 * p + 1], qq);
                lo[p] = __builtin_amdgcn_perm(r1, r0, 0x05040100u);   // column 2qq   : k = 2p, 2p+1
                hi[p] = __builtin_amdgcn_perm(r1, r0, 0x07060302u);   // column 2qq+1
            }
            const bf16x8_t blo = __builtin_bit_cast(bf16x8_t, make_uint4(lo[0], lo[1], lo[2], lo[3]));
            const bf16x8_t bhi = __builtin_bit_cast(bf16x8_t, make_uint4(hi[0], hi[1], hi[2], hi[3]));
#pragma unroll
            for (int ms = 0; ms < ACT; ++ms) {
                acc[ms][2 * qq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.af[ms], blo, acc[ms][2 * qq], 0, 0, 0);
                acc[ms][2 * qq + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.af[ms], bhi, acc[ms][2 * qq + 1], 0, 0, 0);
            }
        }
        }
    };

    // ---- main loop ---------------------------------------------------------------------------------
    // In step s the fragments of stage s are already in registers; the step waits for this wave's
    // share of stage s+1 (in-order completion: NS-3 later stages may stay outstanding), meets the
    // other waves (their shares have landed too, and nobody reads the buffer of stage s-1 any more),
    // refills that buffer with stage s+NS-1, then reads the fragments of stage s+1 from LDS while the
    // matrix cores work on stage s: LDS reads and MFMAs of a wave overlap instead of alternating.
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue(s);
    Frags f0, f1;
    wait_vmcnt<(NS - 2) * PER_STAGE>();
    __builtin_amdgcn_s_barrier();
    read_frags(f0, 0);
    auto step = [&](const Frags& cur, Frags& nxt, int s) {
        wait_vmcnt<(NS - 3) * PER_STAGE>();
        __builtin_amdgcn_s_barrier();
        issue(s + NS - 1);
        read_frags(nxt, (s + 1) % NS);
        mma(cur);
        // Pin the order: the LDS reads of the next stage go out one at a time between the matrix instructions of
        // this one (left alone, the compiler sinks them to the end of the step, just in front of their first use).
        // Only in the bias + GELU kernel and only for full tiles, by measurement: there it is worth 7 % on K = 1024
        // products (c3a GEMM-1: 91 -> 85 us) and nothing on K = 4096 ones; the store kernel with the same pins loses
        // 2 % on c5's K = 16384 tiles.
        if (EPI == EPI_GELU && ACT == MSUB && !LIGHT) {
            constexpr int READS = (PACKED ? NCF : 8) + ACT, MFMAS = NCF * ACT, PER = MFMAS / READS > 0 ? MFMAS / READS : 1;
            constexpr int GROUPS = MFMAS / PER < READS ? MFMAS / PER : READS;
#pragma unroll
            for (int i = 0; i < GROUPS; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // one LDS read
                __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);    // PER matrix instructions
            }
            if (READS > GROUPS) __builtin_amdgcn_sched_group_barrier(0x100, READS - GROUPS, 0);
            if (MFMAS > PER * GROUPS) __builtin_amdgcn_sched_group_barrier(0x008, MFMAS - PER * GROUPS, 0);
        }
    };
    int s = 0;
    for (; s + 2 <= steps; s += 2) {
        step(f0, f1, s);
        step(f1, f0, s + 1);
    }
    if (s < steps) step(f0, f1, s);
    wait_vmcnt<0>();                      // drain the over-issued tail loads before LDS is released

    // ---- epilogue ------------------------------------------------------------------------------
    // packed weights, 64-column waves: wave wn holds fragments 4wn..4wn+3 of the tile's one 128-column group,
    // i.e. columns 8c + 4wn + i of it
    const int n_lane = PACKED && WN == 64 ? n0 + c * 8 + wn * 4 : n0 + wn * WN + c * NCF;
    if (ACT == 0 || n_lane >= a.N) return;
    float bias[NCF];
    {
        float b8[8];
        if (NCF == 8) load_bias8(a, g, n_lane, b8);
        else {                                                   // 4 columns: 8 bytes of bias
#pragma unroll
            for (int i = 0; i < 8; ++i) b8[i] = 0.f;
            if (a.bias) {
                const uint2 bv = *reinterpret_cast<const uint2*>(a.bias + (size_t)g * a.N + n_lane);
                b8[0] = __uint_as_float(bv.x << 16); b8[1] = __uint_as_float(bv.x & 0xffff0000u);
                b8[2] = __uint_as_float(bv.y << 16); b8[3] = __uint_as_float(bv.y & 0xffff0000u);
            }
        }
#pragma unroll
        for (int i = 0; i < NCF; ++i) bias[i] = b8[i];
    }
#pragma unroll
    for (int ms = 0; ms < ACT; ++ms) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int rl = wm * WM + ms * 16 + kg * 4 + r;       // D: rows 4*(lane/16)+r, column lane%16
            if (rl >= nrows) continue;
            float v[NCF];
#pragma unroll
            for (int i = 0; i < NCF; ++i) v[i] = acc[ms][i][r] + bias[i];
            int t = 0;
            float gw = 1.f;
            if (EPI == EPI_SCATTER) scatter_lookup(a, g, m0 + rl, t, gw);
            finish_row<EPI, NCF>(a, g, m0 + rl, 0, n_lane, v, t, gw);
        }
        __builtin_amdgcn_sched_barrier(0);      // keep the accumulators' live ranges short
    }
    };
    typedef std::integral_constant<bool, false> No;
    typedef std::integral_constant<bool, true> Yes;
    bool done = false;
    if constexpr (Cfg::HAS_LIGHT) {
        if (nrows <= Cfg::L_ROWS) {                             // uniform over the work-group
            done = true;
            // a tile of a nearly empty expert is pure streaming: waves whose 16 activation rows lie past the last
            // valid row do not load them (the copies would only repeat the last row and take a third of the load slots)
            if (__builtin_amdgcn_readfirstlane(w * 16 < nrows) || nsub > 2) {
                if (nsub > 2) run(std::integral_constant<int, MSUB>(), Yes(), Yes());
                else if (nsub == 2) run(std::integral_constant<int, 2>(), Yes(), Yes());
                else if (nsub == 1) run(std::integral_constant<int, 1>(), Yes(), Yes());
                else run(std::integral_constant<int, 0>(), Yes(), Yes());
            } else {
                if (nsub == 2) run(std::integral_constant<int, 2>(), Yes(), No());
                else if (nsub == 1) run(std::integral_constant<int, 1>(), Yes(), No());
                else run(std::integral_constant<int, 0>(), Yes(), No());
            }
        }
    }
    if (!done) {
        if (nsub > 2) run(std::integral_constant<int, MSUB>(), No(), Yes());
        else if (nsub == 2) run(std::integral_constant<int, 2>(), No(), Yes());
        else if (nsub == 1) run(std::integral_constant<int, 1>(), No(), Yes());
        else run(std::integral_constant<int, 0>(), No(), Yes());
    }
}

// b == nullptr: one product; otherwise the two products share the launch (same K, N, packing)
template <int WM, int NWM, int NSX, int EPI, int WN, bool PACKED>
static int launch_tp(const WsGemmArgs& a, const WsGemmArgs* b, hipStream_t s) {
    constexpr int BM = NWM * WM, TBN = 2 * WN;
    const int n_tiles = (a.N + TBN - 1) / TBN;
    const long long blocks_a = tile_grid_blocks(a, n_tiles, (a.max_rows + BM - 1) / BM);
    const long long blocks_b = b ? tile_grid_blocks(*b, n_tiles, (b->max_rows + BM - 1) / BM) : 0;
    const long long blocks = blocks_a + blocks_b;                // both multiples of the XCD count
    if (blocks > (1ll << 30)) return MOE_ERR_UNSUPPORTED;        // block indices are ints in the kernel
    const size_t smem = TileCfg<WM, NWM, NSX, WN>::LDS_BYTES;
    static_assert(TileCfg<WM, NWM, NSX, WN>::LDS_BYTES <= 160 * 1024, "a work-group's ring must fit one CU's LDS");
    static_assert(TileCfg<WM, NWM, NSX, WN>::WGS_PER_CU * TileCfg<WM, NWM, NSX, WN>::LDS_BYTES <= 160 * 1024,
                  "the promised work-groups per CU must fit its LDS together");
    static bool attr_set = false;            // one flag per instantiation
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&tgemm_kernel<WM, NWM, NSX, EPI, WN, PACKED>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return MOE_ERR_HIP;
        attr_set = true;
    }
    hipLaunchKernelGGL((tgemm_kernel<WM, NWM, NSX, EPI, WN, PACKED>), dim3((unsigned)blocks), dim3(NWM * 128), smem, s, a,
                       b ? *b : a, (int)blocks_a);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}
template <int WM, int NWM, int NSX, int EPI, int WN>
static int launch_t(const WsGemmArgs& a, const WsGemmArgs* b, hipStream_t s) {
    return a.packed ? launch_tp<WM, NWM, NSX, EPI, WN, true>(a, b, s) : launch_tp<WM, NWM, NSX, EPI, WN, false>(a, b, s);
}

// Tile shapes.  256 x 256 (4 x 2 waves of 64 x 128: the accumulators take 128 registers, which the compiler updates
// in place; 128 rows per wave fill the file and cost copies) wherever that gives every CU a tile.  Products with few
// columns (N = d_model in GEMM-2) get 256 x 128 tiles of 4 x 2 waves of 64 x 64 instead: as many tiles, but eight waves
// per CU rather than the four of a 128 x 256 tile, which is what hides the LDS and barrier latencies.  Groups of at
// most 128 rows: 128 x 256 tiles; for short K as 2 x 2 waves of 64 x 128, 3 stages, two work-groups per CU; for long K
// (few, long tiles: one per CU) as 4 x 2 waves of 32 x 128 with 6 stages of 24 KB -- eight waves hide the latencies
// better than four there (c3b GEMM-2: 113 against 116 us), for short K the two work-groups do (121 against 127 us).
enum TileShape { TILE_128x256, TILE_256x256, TILE_256x128 };
static TileShape pick_tile(int max_rows, int G, int N) {
    if (max_rows <= 128) return TILE_128x256;
    const long long row_tiles = (long long)G * ((max_rows + 255) / 256);
    if (row_tiles * ((N + 255) / 256) >= 256) return TILE_256x256;
    if (row_tiles * ((N + 127) / 128) >= 256) return TILE_256x128;
    return TILE_128x256;
}

// Two products in one launch (same K, N and packing; the tile is picked for the tiles of both together).  Both with
// groups of more than 128 rows: 256-row tiles, the large 256 x 256 one if the pair has enough tiles for it.  One of
// them with groups of at most 128 rows: 128 x 256 tiles for both, but only if the other product alone could not fill
// the chip with 256 x 256 tiles (a product with few columns), since 128-row tiles are the less efficient ones.
static bool pair_shape(const WsGemmArgs& a, const WsGemmArgs& b, TileShape* shape) {
    if (a.K != b.K || a.N != b.N || (a.packed != 0) != (b.packed != 0) || a.ksplit != 1 || b.ksplit != 1) return false;
    const long long n256 = (a.N + 255) / 256;
    if (a.max_rows <= 128 || b.max_rows <= 128) {
        const WsGemmArgs& big = a.max_rows <= 128 ? b : a;
        if (big.max_rows <= 128 || (long long)big.G * ((big.max_rows + 255) / 256) * n256 >= 256) return false;
        *shape = TILE_128x256;
        return true;
    }
    const long long row_tiles = (long long)a.G * ((a.max_rows + 255) / 256) + (long long)b.G * ((b.max_rows + 255) / 256);
    if (row_tiles * n256 >= 256) *shape = TILE_256x256;
    else if (row_tiles * ((a.N + 127) / 128) >= 256) *shape = TILE_256x128;
    else return false;
    return true;
}
bool tgemm_pair_fusable(const WsGemmArgs& a, const WsGemmArgs& b) {
    TileShape t;
    return tgemm_supported(a.K, a.N) && pair_shape(a, b, &t);
}

template <int EPI>
static int launch_t_epi(const WsGemmArgs& a, const WsGemmArgs* b, hipStream_t s) {
    TileShape shape = pick_tile(a.max_rows, a.G, a.N);
    if (b && !pair_shape(a, *b, &shape)) return MOE_ERR_INVALID_ARG;
    switch (shape) {
        case TILE_256x256: return launch_t<64, 4, 4, EPI, 128>(a, b, s);
        case TILE_256x128: return launch_t<64, 4, 5, EPI, 64>(a, b, s);
        default: return a.K <= 2048 ? launch_t<64, 2, 3, EPI, 128>(a, b, s) : launch_t<32, 4, 5, EPI, 128>(a, b, s);
    }
}

bool tgemm_supported(int K, int N) { return K % kTK == 0 && K >= kTK && N % 8 == 0 && N >= 8; }

static int launch_tgemm_any(const WsGemmArgs& a, const WsGemmArgs* b, int epi, hipStream_t s) {
    if (a.G <= 0 || a.max_rows <= 0) return b ? MOE_ERR_INVALID_ARG : MOE_OK;
    if (a.ksplit != 1 || !tgemm_supported(a.K, a.N)) return MOE_ERR_INVALID_ARG;
    switch (epi) {
        case EPI_STORE: return launch_t_epi<EPI_STORE>(a, b, s);
        case EPI_GELU: return launch_t_epi<EPI_GELU>(a, b, s);
        case EPI_SCATTER: return b ? MOE_ERR_INVALID_ARG : launch_t_epi<EPI_SCATTER>(a, b, s);   // zeroes rows grid-wide
        case EPI_COMBINE: return launch_t_epi<EPI_COMBINE>(a, b, s);
        case EPI_PARTIAL: return launch_t_epi<EPI_PARTIAL>(a, b, s);      // ksplit == 1: one fp32 partial, no bias
        default: return MOE_ERR_INVALID_ARG;
    }
}
int launch_tgemm(const WsGemmArgs& a, int epi, hipStream_t s) { return launch_tgemm_any(a, nullptr, epi, s); }
int launch_tgemm_pair(const WsGemmArgs& a, const WsGemmArgs& b, int epi, hipStream_t s) {
    return launch_tgemm_any(a, &b, epi, s);
}

}  // namespace moe
