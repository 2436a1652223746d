// Gate for bf16 tokens on the bf16 matrix cores, exact to fp32 level (paper Sec. 5.4: the gating
// function -- logits, top-k, the count that places a token inside its expert -- fused into as few
// kernels as the data dependences allow; it is small but sits on the critical path before every other
// kernel of the layer).
//
//   logits[t,e] = bg[e] + sum_i x[t,i] Wg[i,e],   x bf16, Wg and bg fp32, fp32 accumulation.
//
// An fp32 weight is the exact sum of three bf16 numbers (3 x 8 significant bits = the 24 of fp32):
// Wg = hi + mid + lo with hi = bf16(Wg), mid = bf16(Wg - hi), lo = bf16(Wg - hi - mid).  A bf16 token
// value times a bf16 piece is exact in fp32, so three v_mfma_f32_16x16x32_bf16 per tile give the same
// sum of exact products as an fp32 multiply-add chain, at a fraction of the fp32 matrix-core time.
//
// Kernels:
//   * gate_prepare_kernel writes the three pieces as ready-made MFMA B fragments (1 KB each: lane l
//     holds k = 8*(l/16)..+7 of expert column l%16), ordered [k-block][expert tile][piece]: into the
//     workspace at every call, or once into a buffer the caller keeps (packed gate weights);
//   * gate_bf16_kernel: a work-group owns a tile of 16*MA tokens x 16*NE experts; its four waves
//     split the k-blocks (wave w takes blocks w, w+4, ...) and each computes the whole tile for its
//     blocks, so no operand byte is fetched twice by a work-group.  Every operand fragment is one
//     16-byte load per lane from global memory straight into registers, several k-blocks ahead; no LDS
//     traffic and no barrier in the loop.  The four partial tiles are summed through LDS in a fixed
//     order, the finished tile is laid out [token][expert] in LDS and written with 16-byte stores.
//     When the tile spans all experts (K = 1 or 2) the kernel goes on to the first half of the
//     routing on the tile it holds: top-k and gate weights per token (16 lanes per token), the rank of
//     each token among the tile's tokens with the same expert (ballots) and the tile's histogram.
//     route_finalize_kernel turns ranks into rows.
//     With few tokens the experts are split over work-groups instead (K = 0: logits only) so that
//     more CUs take part, and the routing runs as a kernel of its own.
// Requires d_model to be a multiple of 32 and at most 128 experts; other shapes use the fp32 kernel.
#include "route_device.h"

namespace moe {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kKB = 32;                  // k per MFMA
constexpr int kFragElems = 512;          // bf16 elements of one fragment (64 lanes x 8)
// KB k-blocks x ET expert tiles x 3 pieces; one thread per (k-block, expert tile, lane).
__global__ __launch_bounds__(256) void gate_prepare_kernel(const float* __restrict__ Wg, uint16_t* __restrict__ frags, int d,
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
    // k-blocks held in registers: as many as fit beside the accumulators (4 registers per load and per tile)
    static constexpr int D_WANT = 48 / PER < 3 ? 3 : (48 / PER > 6 ? 6 : 48 / PER);
    static constexpr int D = 4 * (MA * NE + D_WANT * PER) <= 400 ? D_WANT : 2;
};

// tile: MA token tiles (16 tokens each) x NE expert tiles; blockIdx.x = token tile, blockIdx.y = expert group;
// ET = expert tiles in all (fragment stride).  K = 0: logits only.  K = 1, 2 (needs NE == ET): also top-K, gate
// weights, tile-local ranks (parked in slot_idx) and histograms.
template <int MA, int NE, int K> struct GateLds {
    static constexpr int TM = 16 * MA, TN = 16 * NE;
    static constexpr int STRIDE = TN + 4;                         // floats per tile row: 4 rows apart fall 16 banks apart
    static constexpr int RED = 2 * MA * NE * 64 * 16;             // two partial tiles, bytes
    static constexpr int TILE = TM * STRIDE * 4;
    static constexpr int MAIN = RED > TILE ? RED : TILE;          // the finished tile reuses the partial tiles' space
    static constexpr int ROUTE = K > 0 ? (K * TM + K * TN) * 4 : 0;   // chosen experts, histogram
    static constexpr int BYTES = MAIN + ROUTE;
};

template <int MA, int NE, int K>
__device__ __forceinline__ void gate_bf16_body(char* lds, const uint16_t* __restrict__ x, const uint16_t* __restrict__ frags,
                                               const float* __restrict__ bg, float* __restrict__ logits, int T, int d,
                                               int E, int ET, int32_t* __restrict__ expert_idx,
                                               int32_t* __restrict__ slot_idx, float* __restrict__ gate_w,
                                               int32_t* __restrict__ hist) {
    typedef GateLds<MA, NE, K> L;
    constexpr int D = GateCfg<MA, NE>::D, PER = GateCfg<MA, NE>::PER, WK = 4, TM = L::TM, TN = L::TN, STRIDE = L::STRIDE;
    f32x4_t* red = reinterpret_cast<f32x4_t*>(lds);               // [2][MA][NE][64]
    float* tile = reinterpret_cast<float*>(lds);                  // [TM][STRIDE], after the reduction

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wk = w;
    const int et0 = blockIdx.y * NE;                              // first expert tile of this work-group
    const int t0 = blockIdx.x * TM;
    const int KB = d / kKB;
    const int nkb = KB > wk ? (KB - wk + WK - 1) / WK : 0;        // k-blocks wk, wk + WK, ... of this wave

    // bias of this lane's expert columns, fetched before anything else is in flight
    float bias[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        const int col = (et0 + e) * 16 + (lane & 15);
        bias[e] = (bg && col < E) ? bg[col] : 0.f;
    }

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

        // Operands of one k-block: A fragments straight from the token rows, B fragments as stored.
        // Plain loads: the compiler tracks their completion.  (Loads issued from inline asm with
        // hand-placed waits are NOT an option here: the compiler regards an asm output as valid at once
        // and, under register pressure, copies it elsewhere before the data has arrived.)
        struct Stage {
            u32x4_t r[PER];                                       // MA token fragments, then 3*NE weight fragments
        };
        auto load = [&](Stage& st, int step) {
            const int kb = wk + min(step, nkb - 1) * WK;          // past the end: harmless re-read, dropped
#pragma unroll
            for (int m = 0; m < MA; ++m) st.r[m] = *reinterpret_cast<const u32x4_t*>(a_src[m] + kb * kKB);
            const uint16_t* bp = b_src + (size_t)kb * b_kb_stride;
#pragma unroll
            for (int i = 0; i < 3 * NE; ++i) st.r[MA + i] = *reinterpret_cast<const u32x4_t*>(bp + i * kFragElems);
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
                // the scheduling barriers pin "fetch the block D-1 ahead, then use the oldest": left alone,
                // the compiler sinks the loads to their first use
                load(st[(i + D - 1) % D], s0 + i + D - 1);
                __builtin_amdgcn_sched_barrier(0);
                mma(st[i], s0 + i < nkb);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // ---- sum of the four partial tiles, always as (w0 + w2) + (w1 + w3) ------------------------------
    if (w >= 2) {
#pragma unroll
        for (int m = 0; m < MA; ++m)
#pragma unroll
            for (int e = 0; e < NE; ++e) red[(((w - 2) * MA + m) * NE + e) * 64 + lane] = acc[m][e];
    }
    __syncthreads();
    if (w < 2) {
#pragma unroll
        for (int m = 0; m < MA; ++m)
#pragma unroll
            for (int e = 0; e < NE; ++e) acc[m][e] += red[((w * MA + m) * NE + e) * 64 + lane];
    }
    __syncthreads();
    if (w == 1) {
#pragma unroll
        for (int m = 0; m < MA; ++m)
#pragma unroll
            for (int e = 0; e < NE; ++e) red[(m * NE + e) * 64 + lane] = acc[m][e];
    }
    __syncthreads();
    if (w == 0) {
        // finished logits (bias added) go to LDS as [token][expert]; D fragment: column lane%16, rows 4*(lane/16)+r
#pragma unroll
        for (int m = 0; m < MA; ++m)
#pragma unroll
            for (int e = 0; e < NE; ++e) acc[m][e] += red[(m * NE + e) * 64 + lane];
        asm volatile("" ::: "memory");                                // keep the reads above ahead of the writes below
        // the partial tile just read and the finished tile share LDS: only this wave touches either here,
        // and its LDS operations execute in order
#pragma unroll
        for (int m = 0; m < MA; ++m)
#pragma unroll
            for (int e = 0; e < NE; ++e)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    tile[(16 * m + 4 * (lane >> 4) + r) * STRIDE + 16 * e + (lane & 15)] = acc[m][e][r] + bias[e];
    }
    __syncthreads();

    // ---- logits out: 16 bytes per thread, rows contiguous ------------------------------------------------
    {
        constexpr int V = TN / 4;                                 // float4 per tile row
        const int col0 = et0 * 16;
        for (int i = tid; i < TM * V; i += 256) {
            const int tl = i / V, c4 = (i % V) * 4;
            const int t = t0 + tl, col = col0 + c4;
            if (t >= T || col >= E) continue;
            const float4 v = *reinterpret_cast<const float4*>(tile + tl * STRIDE + c4);
            float* o = logits + (size_t)t * E + col;
            if ((E & 3) == 0) *reinterpret_cast<float4*>(o) = v;              // col + 3 < E and 16-byte aligned
            else {
                o[0] = v.x;
                if (col + 1 < E) o[1] = v.y;
                if (col + 2 < E) o[2] = v.z;
                if (col + 3 < E) o[3] = v.w;
            }
        }
    }

    if (K > 0) {
        constexpr int KK = K > 0 ? K : 1;
        int32_t* e_sh = reinterpret_cast<int32_t*>(lds + L::MAIN);    // [K][TM] chosen expert per token of the tile
        int32_t* h_sh = e_sh + KK * TM;                               // [K][TN] histogram of the tile
        for (int i = tid; i < KK * TN; i += 256) h_sh[i] = 0;
        // 16 lanes per token, 16 tokens at a time
        const int grp = tid >> 4, sub = tid & 15;
#pragma unroll
        for (int it = 0; it < MA; ++it) {
            const int tl = it * 16 + grp;
            float v[NE];
#pragma unroll
            for (int i = 0; i < NE; ++i) v[i] = sub + 16 * i < E ? tile[tl * STRIDE + sub + 16 * i] : -INFINITY;
            Best g1, g2;
            float w1, w2;
            token_gate_regs<KK, NE>(v, sub, g1, g2, w1, w2);
            if (sub == 0) {
                const int t = t0 + tl;
                const bool ok = t < T;
                e_sh[tl] = ok ? g1.i : -1;
                if (KK == 2) e_sh[TM + tl] = ok ? g2.i : -1;
                if (ok) {
                    expert_idx[(size_t)t * KK] = g1.i;
                    gate_w[(size_t)t * KK] = w1;
                    if (KK == 2) {
                        expert_idx[(size_t)t * KK + 1] = g2.i;
                        gate_w[(size_t)t * KK + 1] = w2;
                    }
                }
            }
        }
        __syncthreads();
        // one lane per token (the tile has at most 64): rank among the tile's tokens with the same expert
        if (w == 0) {
#pragma unroll
            for (int j = 0; j < KK; ++j) {
                const int e = lane < TM ? e_sh[j * TM + lane] : -1;
                const int rank = wave_rank_by_expert(e, lane, h_sh + j * TN);
                if (e >= 0) slot_idx[(size_t)(t0 + lane) * KK + j] = rank;
            }
        }
        __syncthreads();
        // histogram [K][E] of this tile
        for (int i = tid; i < KK * E; i += 256) {
            const int j = i / E, e = i % E;
            hist[(size_t)blockIdx.x * KK * E + i] = h_sh[j * TN + e];
        }
    }
}

template <int MA, int NE, int K>
__global__ __launch_bounds__(256) void gate_bf16_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ frags,
                                                        const float* __restrict__ bg, float* __restrict__ logits, int T, int d,
                                                        int E, int ET, int32_t* __restrict__ expert_idx,
                                                        int32_t* __restrict__ slot_idx, float* __restrict__ gate_w,
                                                        int32_t* __restrict__ hist) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    gate_bf16_body<MA, NE, K>(lds, x, frags, bg, logits, T, d, E, ET, expert_idx, slot_idx, gate_w, hist);
}

// The whole gate of a decode step (at most 256 tokens) in ONE launch: the work-groups compute the logits tile by tile
// (experts split over work-groups, so that many CUs share the read of the gate weights); every work-group then
// publishes a flag, and the one with the highest index waits for all flags and runs the whole routing on the finished
// logits.  The flags hold the call's epoch (never 0, and not repeated by the host from one call to the next), so they
// need no clearing beforehand: what nobody or an earlier call left there is not this call's epoch, and the waiting
// work-group puts every flag it has seen back to 0, which also makes a replayed graph launch (same epoch) safe.  Hand-over across the XCDs'
// separate L2s: the writers release at device scope after their stores (write-back of the L2), the reader acquires at
// device scope before its loads (invalidate).  The wait cannot hang: work-groups are started in index order, so all
// others are running or done when the last one starts (and the whole grid, at most 64 work-groups, fits on the chip
// at once); it is bounded all the same, and gives up (leaving wrong tables, never a hung GPU) after about 10^6 polls.
template <int MA, int NE, int RK, int NV>
__global__ __launch_bounds__(256) void gate_decode_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ frags,
                                                          const float* __restrict__ bg, float* __restrict__ logits, int T,
                                                          int d, int E, int ET, int C, int32_t* __restrict__ expert_idx,
                                                          int32_t* __restrict__ slot_idx, float* __restrict__ gate_w,
                                                          int32_t* __restrict__ expert_rows, int32_t* __restrict__ slot_token,
                                                          int32_t* __restrict__ expert_order, uint32_t* __restrict__ flags,
                                                          uint32_t epoch) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    gate_bf16_body<MA, NE, 0>(lds, x, frags, bg, logits, T, d, E, ET, nullptr, nullptr, nullptr, nullptr);
    const int nblocks = gridDim.x * gridDim.y, bid = blockIdx.y * gridDim.x + blockIdx.x;
    __syncthreads();                                   // every thread's logits stores are issued
    if (threadIdx.x == 0) {
        __atomic_thread_fence(__ATOMIC_RELEASE);       // device scope: this work-group's stores become visible ...
        __hip_atomic_store(flags + bid, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ... before its flag
    }
    if (bid != nblocks - 1) return;
    if ((int)threadIdx.x < nblocks) {
        int polls = 0;
        while (__hip_atomic_load(flags + threadIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch && polls < (1 << 20)) {
            __builtin_amdgcn_s_sleep(2);
            ++polls;
        }
    }
    __atomic_thread_fence(__ATOMIC_ACQUIRE);           // device scope: nothing read below comes from a stale cache line
    // Each flag goes back to 0 (never an epoch) once it has been seen: a captured launch that is replayed carries the
    // same epoch every time and must not find it in the flags of its own previous run.
    if ((int)threadIdx.x < nblocks) __hip_atomic_store(flags + threadIdx.x, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    route_single_body<RK, NV>(reinterpret_cast<int32_t*>(lds), logits, T, E, C, expert_idx, slot_idx, gate_w, expert_rows,
                              slot_token, expert_order, nullptr);
}

template <int MA, int NE, int K>
int launch_cfg(const uint16_t* x, const uint16_t* frags, const float* bg, float* logits, int T, int d, int E, int ET,
               int32_t* expert_idx, int32_t* slot_idx, float* gate_w, int32_t* hist, hipStream_t s) {
    constexpr int smem = GateLds<MA, NE, K>::BYTES;
    static bool attr_set = false;             // one flag per instantiation
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gate_bf16_kernel<MA, NE, K>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return MOE_ERR_HIP;
        attr_set = true;
    }
    const dim3 grid((T + 16 * MA - 1) / (16 * MA), ET / NE);
    hipLaunchKernelGGL((gate_bf16_kernel<MA, NE, K>), grid, dim3(256), smem, s, x, frags, bg, logits, T, d, E, ET, expert_idx,
                       slot_idx, gate_w, hist);
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

static int launch_prepare(const float* Wg, uint16_t* frags, int d, int E, int KB, int ET, hipStream_t s) {
    const long long threads = (long long)KB * ET * 64;
    hipLaunchKernelGGL(gate_prepare_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, Wg, frags, d, E, KB, ET);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int launch_pack_gate(const float* Wg, void* packed, int d, int E, hipStream_t s) {
    if (!gate_bf16_supported(d, E)) return MOE_ERR_UNSUPPORTED;
    return launch_prepare(Wg, static_cast<uint16_t*>(packed), d, E, d / kKB, padded_expert_tiles(E), s);
}

// Wg_packed != nullptr: the gate weights as launch_pack_gate wrote them (Wg and frag_ws are then not used)
int launch_gate_logits_bf16(const void* x, const float* Wg, const void* Wg_packed, const float* bg, float* logits, int T,
                            int d, int E, void* frag_ws, hipStream_t s) {
    if (!gate_bf16_supported(d, E) || (!frag_ws && !Wg_packed)) return MOE_ERR_INVALID_ARG;
    const int KB = d / kKB, ET = padded_expert_tiles(E);
    const uint16_t* frags = static_cast<const uint16_t*>(Wg_packed);
    if (!frags) {
        const int rc = launch_prepare(Wg, static_cast<uint16_t*>(frag_ws), d, E, KB, ET, s);
        if (rc != MOE_OK) return rc;
        frags = static_cast<const uint16_t*>(frag_ws);
    }
    const uint16_t* xb = static_cast<const uint16_t*>(x);
    // Largest tile (fewest operand bytes per output) that still gives every CU a work-group; when even
    // the smallest tile cannot (few tokens), the smallest one: most work-groups, least time per CU.
    int MA = 2, NE = 1;
    bool found = false;
    for (int ma = 4; ma >= 2 && !found; ma -= 2)
        for (int ne = ET < 4 ? ET : 4; ne >= 1 && !found; ne /= 2)
            if ((long long)((T + 16 * ma - 1) / (16 * ma)) * (ET / ne) >= 256) { MA = ma; NE = ne; found = true; }
#define MOE_GATE_CASE(ma, ne) \
    if (MA == ma && NE == ne)   \
    return launch_cfg<ma, ne, 0>(xb, frags, bg, logits, T, d, E, ET, nullptr, nullptr, nullptr, nullptr, s)
    MOE_GATE_CASE(4, 4); MOE_GATE_CASE(4, 2); MOE_GATE_CASE(4, 1);
    MOE_GATE_CASE(2, 4); MOE_GATE_CASE(2, 2); MOE_GATE_CASE(2, 1);
#undef MOE_GATE_CASE
    return MOE_ERR_INVALID_ARG;
}

// The decode gate in one launch: bf16 tokens, at most 256 of them.  flags: 64 uint32 of scratch; epoch: a value that
// differs from what any earlier call left in `flags`.
bool gate_decode_supported(int T, int d, int E) { return gate_bf16_supported(d, E) && T <= kRouteTokens; }

template <int RK, int NV>
static int launch_decode_cfg(const uint16_t* x, const uint16_t* frags, const float* bg, float* logits, int T, int d, int E,
                             int ET, int C, int32_t* expert_idx, int32_t* slot_idx, float* gate_w, int32_t* expert_rows,
                             int32_t* slot_token, int32_t* expert_order, uint32_t* flags, uint32_t epoch, hipStream_t s) {
    constexpr int MA = 2, NE = 1;                       // smallest tile: most work-groups (at most 8 x 8)
    const size_t route = route_single_lds_ints(E, RK) * sizeof(int32_t);
    const size_t smem = route > (size_t)GateLds<MA, NE, 0>::BYTES ? route : (size_t)GateLds<MA, NE, 0>::BYTES;
    const dim3 grid((T + 16 * MA - 1) / (16 * MA), ET / NE);
    if (grid.x * grid.y > 64) return MOE_ERR_INVALID_ARG;
    static size_t attr_bytes = 0;                       // one per instantiation
    if (smem > attr_bytes) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gate_decode_kernel<MA, NE, RK, NV>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return MOE_ERR_HIP;
        attr_bytes = smem;
    }
    hipLaunchKernelGGL((gate_decode_kernel<MA, NE, RK, NV>), grid, dim3(256), smem, s, x, frags, bg, logits, T, d, E, ET, C,
                       expert_idx, slot_idx, gate_w, expert_rows, slot_token, expert_order, flags, epoch);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int launch_gate_decode(const void* x, const float* Wg, const void* Wg_packed, const float* bg, float* logits, int T, int d,
                       int E, int k, int C, int32_t* expert_idx, int32_t* slot_idx, float* gate_w, int32_t* expert_rows,
                       int32_t* slot_token, int32_t* expert_order, void* frag_ws, uint32_t* flags, uint32_t epoch,
                       hipStream_t s) {
    if (!gate_decode_supported(T, d, E) || (!frag_ws && !Wg_packed) || !flags || k < 1 || k > 2) return MOE_ERR_INVALID_ARG;
    const int KB = d / kKB, ET = padded_expert_tiles(E);
    const uint16_t* frags = static_cast<const uint16_t*>(Wg_packed);
    if (!frags) {
        const int rc = launch_prepare(Wg, static_cast<uint16_t*>(frag_ws), d, E, KB, ET, s);
        if (rc != MOE_OK) return rc;
        frags = static_cast<const uint16_t*>(frag_ws);
    }
    const uint16_t* xb = static_cast<const uint16_t*>(x);
#define MOE_DECODE_CASE(kk, nv) \
    return launch_decode_cfg<kk, nv>(xb, frags, bg, logits, T, d, E, ET, C, expert_idx, slot_idx, gate_w, expert_rows, \
                                     slot_token, expert_order, flags, epoch, s)
    if (k == 1) {
        if (E <= 16) MOE_DECODE_CASE(1, 1);
        if (E <= 32) MOE_DECODE_CASE(1, 2);
        if (E <= 64) MOE_DECODE_CASE(1, 4);
        MOE_DECODE_CASE(1, 8);
    }
    if (E <= 16) MOE_DECODE_CASE(2, 1);
    if (E <= 32) MOE_DECODE_CASE(2, 2);
    if (E <= 64) MOE_DECODE_CASE(2, 4);
    MOE_DECODE_CASE(2, 8);
#undef MOE_DECODE_CASE
}

// With fewer tokens the fused kernel would leave most CUs idle; logits over expert groups plus a separate
// routing kernel is faster then.
bool gate_bf16_fused_supported(int T, int d, int E) { return gate_bf16_supported(d, E) && T >= 2048; }

int launch_gate_bf16_fused(const void* x, const float* Wg, const void* Wg_packed, const float* bg, float* logits, int T,
                           int d, int E, int k, int32_t* expert_idx, int32_t* slot_idx, float* gate_w, void* frag_ws,
                           int32_t* scratch, int* tokens_per_hist, const int32_t** hist_out, hipStream_t s) {
    if (!gate_bf16_fused_supported(T, d, E) || (!frag_ws && !Wg_packed) || !scratch || k < 1 || k > 2)
        return MOE_ERR_INVALID_ARG;
    const int KB = d / kKB, ET = padded_expert_tiles(E);
    const uint16_t* frags = static_cast<const uint16_t*>(Wg_packed);
    // 64-token tiles once they give every CU a work-group, else 32-token ones
    const int MA = (T + 63) / 64 >= 256 ? 4 : 2;
    const int TM = 16 * MA;
    int32_t* hist = scratch;                                      // one histogram per tile: route_scratch_ints(T, E, k)
    int rc = MOE_OK;
    if (!frags) {
        rc = launch_prepare(Wg, static_cast<uint16_t*>(frag_ws), d, E, KB, ET, s);
        if (rc != MOE_OK) return rc;
        frags = static_cast<const uint16_t*>(frag_ws);
    }
    const uint16_t* xb = static_cast<const uint16_t*>(x);
    rc = MOE_ERR_INVALID_ARG;
#define MOE_GATE_CASE(ma, ne, kk) \
    if (MA == ma && ET == ne && k == kk) \
    rc = launch_cfg<ma, ne, kk>(xb, frags, bg, logits, T, d, E, ET, expert_idx, slot_idx, gate_w, hist, s)
    MOE_GATE_CASE(4, 8, 1); MOE_GATE_CASE(4, 4, 1); MOE_GATE_CASE(4, 2, 1); MOE_GATE_CASE(4, 1, 1);
    MOE_GATE_CASE(2, 8, 1); MOE_GATE_CASE(2, 4, 1); MOE_GATE_CASE(2, 2, 1); MOE_GATE_CASE(2, 1, 1);
    MOE_GATE_CASE(4, 8, 2); MOE_GATE_CASE(4, 4, 2); MOE_GATE_CASE(4, 2, 2); MOE_GATE_CASE(4, 1, 2);
    MOE_GATE_CASE(2, 8, 2); MOE_GATE_CASE(2, 4, 2); MOE_GATE_CASE(2, 2, 2); MOE_GATE_CASE(2, 1, 2);
#undef MOE_GATE_CASE
    *tokens_per_hist = TM;
    *hist_out = hist;
    return rc;
}

}  // namespace moe
