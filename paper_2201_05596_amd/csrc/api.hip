// C ABI of the library: argument checks, workspace carving and launch sequencing.
// Every check happens on the host before the first HIP call.
#include <vector>

#include "moe_internal.h"

using namespace moe;

namespace {

// ---- optional stage timing of moe_layer_forward (benchmark aid) ----------------------------------
// When enabled, an event is recorded on the call's stream before the first kernel and after every
// stage; nothing is read back until moe_profile_elapsed() is called.
enum Stage { ST_LOGITS, ST_ROUTE, ST_DISPATCH, ST_GEMM1, ST_GEMM2, ST_REDUCE, ST_DENSE1, ST_DENSE2, ST_COMBINE, ST_COUNT };
const char* const kStageNames[ST_COUNT] = {"gate_logits", "gate_route", "dispatch", "expert_gemm1", "expert_gemm2",
                                           "splitk_reduce", "dense_gemm1", "dense_gemm2", "combine"};
struct Profiler {
    int max_calls = 0, calls = 0, cur = -1;
    int stride = 1, seen = 0;       // only every stride-th call since the last enable is timed
    unsigned mask = ~0u;            // stages that get their own time
    bool dirty = false;             // kernels were launched since the last recorded event
    std::vector<hipEvent_t> ev;     // [max_calls][kMarks]
    std::vector<int> stage;         // stage that ended at each mark; -1: the mark only opens the next stage
    std::vector<int> nmarks;        // [max_calls]
} g_prof;
constexpr int kMarks = 2 * ST_COUNT + 1;

void prof_record(int stage, hipStream_t st) {
    const int m = g_prof.nmarks[g_prof.cur];
    if (m >= kMarks) return;
    g_prof.stage[(size_t)g_prof.cur * kMarks + m] = stage;
    (void)hipEventRecord(g_prof.ev[(size_t)g_prof.cur * kMarks + m], st);
    g_prof.nmarks[g_prof.cur] = m + 1;
    g_prof.dirty = false;
}
void prof_begin(hipStream_t st) {
    g_prof.cur = -1;
    if (g_prof.max_calls == 0 || g_prof.calls >= g_prof.max_calls) return;
    if (g_prof.seen++ % g_prof.stride != 0) return;
    g_prof.cur = g_prof.calls++;
    g_prof.nmarks[g_prof.cur] = 0;
    g_prof.dirty = true;            // whatever ran before the call
}
// before a stage's first launch: open it with an event unless one was just recorded
void prof_pre(int stage, hipStream_t st) {
    if (g_prof.cur < 0 || !(g_prof.mask >> stage & 1u)) return;
    if (g_prof.dirty || g_prof.nmarks[g_prof.cur] == 0) prof_record(-1, st);
}
// after a stage's last launch
void prof_mark(int stage, hipStream_t st) {
    if (g_prof.cur < 0) return;
    if (g_prof.mask >> stage & 1u) prof_record(stage, st);
    else g_prof.dirty = true;
}

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t esize(int dtype) { return dtype == MOE_F32 ? 4 : 2; }

int check_shape(const moe_shape_t* s) {
    if (!s) return MOE_ERR_INVALID_ARG;
    if (s->T < 1 || s->d_model < 1 || s->d_ffn < 1 || s->E < 1 || s->capacity < 1) return MOE_ERR_INVALID_ARG;
    if (s->top_k < 1 || s->top_k > s->E) return MOE_ERR_INVALID_ARG;
    if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) return MOE_ERR_INVALID_ARG;
    if (s->residual != 0 && s->residual != 1) return MOE_ERR_INVALID_ARG;
    if (s->flags & ~(MOE_FLAG_PACKED_WEIGHTS | MOE_FLAG_PACKED_GATE)) return MOE_ERR_INVALID_ARG;
    if ((s->flags & MOE_FLAG_PACKED_WEIGHTS) && s->dtype != MOE_BF16) return MOE_ERR_UNSUPPORTED;
    if ((s->flags & MOE_FLAG_PACKED_GATE) && (s->dtype != MOE_BF16 || !gate_bf16_supported(s->d_model, s->E)))
        return MOE_ERR_UNSUPPORTED;
    if (s->top_k > 2 || s->E > 1024) return MOE_ERR_UNSUPPORTED;
    const int mult = s->dtype == MOE_F32 ? 4 : 8;
    if (s->d_model % mult || s->d_ffn % mult) return MOE_ERR_UNSUPPORTED;
    if ((long long)s->T * s->top_k >= (1ll << 31) || (long long)s->E * s->capacity >= (1ll << 31))
        return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

// Tile shapes and split-K factor of the two expert GEMMs (bf16 MFMA path).
struct FfnPlan {
    bool mfma;          // false: plain fp32-ALU GEMM (fp32 layers)
    int MT, NW1, NW2;   // row tile; waves per work-group of GEMM-1 / GEMM-2
    int ksplit2;        // split-K factor of GEMM-2 (1 = none)
    bool tiled;         // more than 64 rows per expert: the tiled (matrix-core-bound) kernel
    int NBUF;           // weight super-fragments kept in flight per wave, plus one
};

FfnPlan plan_ffn(const moe_shape_t* s) {
    FfnPlan p{};
    p.mfma = s->dtype == MOE_BF16 && wsgemm_supported(s->d_model, s->d_ffn);
    p.ksplit2 = 1;
    p.NBUF = 2;
    if (!p.mfma) return p;
    p.tiled = s->capacity > 64 && tgemm_supported(s->d_model, s->d_ffn) && tgemm_supported(s->d_ffn, s->d_model);
    wsgemm_pick_tile(s->capacity, s->E, s->d_ffn, &p.MT, &p.NW1);
    int mt2;
    wsgemm_pick_tile(s->capacity, s->E, s->d_model, &mt2, &p.NW2);
    // GEMM-2 has few output columns; when that leaves the chip short of waves, split K
    const long long touched = s->E < (long long)s->T * s->top_k ? s->E : (long long)s->T * s->top_k;
    const long long m_tiles = (s->capacity + p.MT - 1) / p.MT;
    const long long waves = touched * ((s->d_model + 127) / 128) * m_tiles;
    if (waves < 1024 && !p.tiled) {
        const int chunks = (s->d_ffn + wsgemm_chunk_k(p.MT) - 1) / wsgemm_chunk_k(p.MT);
        long long ks = (2048 + waves - 1) / waves;
        if (ks > 8) ks = 8;
        if (ks > chunks) ks = chunks;
        p.ksplit2 = (int)(ks < 1 ? 1 : ks);
    }
    return p;
}

// Carving of the caller's workspace.  Offsets in bytes; every region 256-byte aligned.
struct WsLayout {
    size_t logits, wg_frags, hist, flags, expert_idx, slot_idx, gate_w, rows, order, slot_token, xe, h, ye, hd, dense, partial, total;
};

WsLayout ws_layout(const moe_shape_t* s) {
    WsLayout L{};
    const size_t T = s->T, d = s->d_model, f = s->d_ffn, E = s->E, k = s->top_k, C = s->capacity;
    const size_t es = esize(s->dtype);
    const FfnPlan plan = plan_ffn(s);
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes); return o; };
    L.logits = take(T * E * 4);
    L.wg_frags = take(s->dtype == MOE_BF16 ? gate_bf16_ws_bytes(s->d_model, s->E) : 0);
    L.hist = take(route_scratch_ints(s->T, s->E, s->top_k) * 4);
    L.flags = take(kGateFlagInts * 4);                 // hand-over flags of the one-launch decode gate
    L.expert_idx = take(T * k * 4);
    L.slot_idx = take(T * k * 4);
    L.gate_w = take(T * k * 4);
    L.rows = take(E * 4);
    L.order = take(2 * (E + 1) * 4);  // two launch orders of the experts, each followed by the tile-dealing flag
    L.slot_token = take(E * C * 4);
    L.xe = take(plan.mfma ? 0 : E * C * d * es);       // the MFMA path gathers rows inside GEMM-1
    L.h = take(E * C * f * es);
    L.ye = take(E * C * d * es);
    L.hd = take(s->residual ? T * f * es : 0);
    L.dense = take(s->residual ? T * d * es : 0);      // the dense branch's output where it is not combined in place
    L.partial = take(plan.ksplit2 > 1 ? (size_t)plan.ksplit2 * E * C * d * 4 : 0);
    L.total = off;
    return L;
}

template <typename T> inline T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(ws) + off); }

int check_ws(const moe_shape_t* s, const void* ws, size_t ws_bytes) {
    if (!ws || !aligned16(ws) || ws_bytes < ws_layout(s).total) return MOE_ERR_WORKSPACE;
    return MOE_OK;
}

// The gate's share of the workspace: the leading regions of the layout (logits, split gate weights, histograms).
size_t gate_scratch_bytes(const moe_shape_t* s) { return ws_layout(s).expert_idx; }

// Scratch of moe_gate_noalloc: one array per GPU, inside the library's code object, so that the call needs no
// workspace from its caller and no allocation.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels get the device address that call returns, looked up once per device.
constexpr size_t kStaticScratchBytes = 8u << 20;
constexpr int kMaxDevices = 64;
__device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
void* g_static_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOE_ERR_HIP;
    if (!g_static_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess || !p) return MOE_ERR_HIP;
        g_static_scratch_ptr[dev] = p;
    }
    *out = g_static_scratch_ptr[dev];
    return MOE_OK;
}

// gate logits: bf16 tokens go to the bf16 matrix cores when the shape allows, everything else to the fp32 ones.
// With MOE_FLAG_PACKED_GATE, Wg is the buffer moe_pack_gate wrote and no weight is split at call time.
int run_gate_logits(const moe_shape_t* s, const void* x, const float* Wg, const float* bg, float* logits, void* ws,
                    const WsLayout& L, hipStream_t st) {
    const bool packed = s->flags & MOE_FLAG_PACKED_GATE;
    if (s->dtype == MOE_BF16 && gate_bf16_supported(s->d_model, s->E))
        return launch_gate_logits_bf16(x, packed ? nullptr : Wg, packed ? Wg : nullptr, bg, logits, s->T, s->d_model, s->E,
                                       at<void>(ws, L.wg_frags), st);
    return launch_gate_logits(x, s->dtype, Wg, bg, logits, s->T, s->d_model, s->E, st);
}

// the whole gate from tokens: logits (ST_LOGITS; with bf16 tokens and enough of them this kernel also does the
// top-k and the tile-local ranking) and the rest of the routing (ST_ROUTE)
int run_gate(const moe_shape_t* s, const void* x, const float* Wg, const float* bg, float* logits, int32_t* expert_idx,
             int32_t* slot_idx, float* gate_w, int32_t* rows, int32_t* slot_token, int32_t* order, void* ws,
             const WsLayout& L, bool profile, hipStream_t st) {
    int32_t* scratch = at<int32_t>(ws, L.hist);
    int rc;
    if (s->dtype == MOE_BF16 && gate_bf16_fused_supported(s->T, s->d_model, s->E)) {
        int tb = 0;
        const int32_t* hist = nullptr;
        const bool packed = s->flags & MOE_FLAG_PACKED_GATE;
        if (profile) prof_pre(ST_LOGITS, st);
        rc = launch_gate_bf16_fused(x, packed ? nullptr : Wg, packed ? Wg : nullptr, bg, logits, s->T, s->d_model, s->E,
                                    s->top_k, expert_idx, slot_idx, gate_w, at<void>(ws, L.wg_frags), scratch, &tb, &hist, st);
        if (profile) prof_mark(ST_LOGITS, st);
        if (rc != MOE_OK) return rc;
        if (profile) prof_pre(ST_ROUTE, st);
        rc = launch_route_finalize(s->T, s->E, s->top_k, s->capacity, tb, expert_idx, slot_idx, rows, slot_token, order,
                                   hist, st);
        if (profile) prof_mark(ST_ROUTE, st);
        return rc;
    }
    if (s->dtype == MOE_BF16 && gate_decode_supported(s->T, s->d_model, s->E)) {
        // decode: logits and the whole routing in one launch (counted under ST_LOGITS)
        static uint32_t epoch = 0;                     // never repeats: a flag left by an earlier call is never "done"
        epoch = epoch + 1 == 0 ? 1 : epoch + 1;
        const bool packed = s->flags & MOE_FLAG_PACKED_GATE;
        if (profile) prof_pre(ST_LOGITS, st);
        rc = launch_gate_decode(x, packed ? nullptr : Wg, packed ? Wg : nullptr, bg, logits, s->T, s->d_model, s->E,
                                s->top_k, s->capacity, expert_idx, slot_idx, gate_w, rows, slot_token, order,
                                at<void>(ws, L.wg_frags), at<uint32_t>(ws, L.flags), epoch, st);
        if (profile) prof_mark(ST_LOGITS, st);
        return rc;
    }
    if (profile) prof_pre(ST_LOGITS, st);
    rc = run_gate_logits(s, x, Wg, bg, logits, ws, L, st);
    if (profile) prof_mark(ST_LOGITS, st);
    if (rc != MOE_OK) return rc;
    if (profile) prof_pre(ST_ROUTE, st);
    rc = launch_route(logits, s->T, s->E, s->top_k, s->capacity, expert_idx, slot_idx, gate_w, rows, slot_token, order,
                      scratch, st);
    if (profile) prof_mark(ST_ROUTE, st);
    return rc;
}

// the two GEMMs of an FFN on the plain fp32-ALU kernel (fp32 layers)
int run_ffn_simple(int dtype, int G, int max_rows, const int32_t* rows, int fixed_rows, int d, int f, const void* xin,
                   const void* W1, const void* b1, const void* W2, const void* b2, void* h, void* yout, hipStream_t st) {
    GemmArgs a{};
    a.A = xin; a.B = W1; a.bias = b1; a.out = h; a.rows = rows; a.row_map = nullptr;
    a.fixed_rows = fixed_rows; a.max_rows = max_rows; a.G = G; a.K = d; a.N = f;
    a.a_group_stride = max_rows; a.o_group_stride = max_rows; a.gelu = 1; a.dtype = dtype;
    int rc = launch_gemm_simple(a, st);
    if (rc != MOE_OK) return rc;
    a.A = h; a.B = W2; a.bias = b2; a.out = yout; a.K = f; a.N = d; a.gelu = 0;
    return launch_gemm_simple(a, st);
}

inline const uint16_t* u16(const void* p) { return static_cast<const uint16_t*>(p); }
inline uint16_t* u16(void* p) { return static_cast<uint16_t*>(p); }

// Expert GEMM-1 on the MFMA kernel: h[e, r, :] = gelu_tanh(A_row(e, r) W1[e] + b1[e]).
// row_map == nullptr: A rows are xin[e*C + r]; otherwise xin[row_map[e*C + r]] (dispatch fused in).
int run_expert_gemm1(const moe_shape_t* s, const FfnPlan& p, const void* xin, const int32_t* row_map,
                     const int32_t* rows, const int32_t* order, const void* W1, const void* b1, void* h,
                     hipStream_t st) {
    WsGemmArgs a{};
    a.A = u16(xin); a.B = u16(W1); a.bias = u16(b1); a.rows = rows; a.order = order; a.row_map = row_map;
    a.packed = s->flags & MOE_FLAG_PACKED_WEIGHTS;
    a.max_rows = s->capacity; a.map_stride = s->capacity; a.G = s->E; a.K = s->d_model; a.N = s->d_ffn;
    a.a_group_stride = s->capacity; a.out = u16(h); a.o_group_stride = s->capacity; a.ksplit = 1;
    prof_pre(ST_GEMM1, st);
    const int rc = p.tiled ? launch_tgemm(a, EPI_GELU, st) : launch_wsgemm(a, EPI_GELU, p.MT, p.NW1, p.NBUF, st);
    prof_mark(ST_GEMM1, st);
    return rc;
}

// Expert GEMM-2 on the MFMA kernel.  scatter == false: ye[e, r, :] = h[e, r, :] W2[e] + b2[e].
// scatter == true (top-1): out[token(e, r), :] = gate_w[token] * (...), rows of dropped tokens zeroed.
int run_expert_gemm2(const moe_shape_t* s, const FfnPlan& p, const void* h, const int32_t* rows,
                     const int32_t* order, const void* W2, const void* b2, bool scatter, const int32_t* slot_token, const int32_t* slot_idx,
                     const float* gate_w, void* dst, float* partial, hipStream_t st) {
    WsGemmArgs a{};
    a.A = u16(h); a.B = u16(W2); a.bias = u16(b2); a.rows = rows; a.row_map = nullptr;
    // The tiled kernel's tiles of this product are long (K = d_ffn) and few per CU: the busiest experts go first, so
    // that the short tiles of the light ones fill the end (the second list).  GEMM-1 and the streaming kernel keep
    // the list that alternates busy and light experts.
    a.order = order && p.tiled ? order + s->E + 1 : order;
    a.packed = s->flags & MOE_FLAG_PACKED_WEIGHTS;
    a.max_rows = s->capacity; a.G = s->E; a.K = s->d_ffn; a.N = s->d_model;
    a.a_group_stride = s->capacity; a.out = u16(dst); a.o_group_stride = s->capacity; a.ksplit = p.ksplit2;
    a.scatter_map = slot_token; a.scatter_stride = s->capacity; a.zero_slot_idx = slot_idx; a.T = s->T;
    a.gate_w = gate_w; a.top_k = s->top_k;
    prof_pre(ST_GEMM2, st);
    if (p.ksplit2 == 1) {
        const int epi = scatter ? EPI_SCATTER : EPI_STORE;
        const int rc1 = p.tiled ? launch_tgemm(a, epi, st) : launch_wsgemm(a, epi, p.MT, p.NW2, p.NBUF, st);
        prof_mark(ST_GEMM2, st);
        return rc1;
    }
    a.partial = partial;
    a.partial_rows = (long long)s->E * s->capacity;
    int rc = launch_wsgemm(a, EPI_PARTIAL, p.MT, p.NW2, p.NBUF, st);
    prof_mark(ST_GEMM2, st);
    if (rc != MOE_OK) return rc;
    SplitKReduceArgs r{};
    r.partial = partial; r.ksplit = p.ksplit2; r.G = s->E; r.N = s->d_model; r.group_stride = s->capacity;
    r.rows = rows; r.max_rows = s->capacity; r.bias = u16(b2); r.out = u16(dst);
    r.scatter_map = scatter ? slot_token : nullptr; r.gate_w = gate_w; r.top_k = s->top_k;
    r.zero_slot_idx = scatter ? slot_idx : nullptr; r.T = s->T;
    prof_pre(ST_REDUCE, st);
    rc = launch_splitk_reduce(r, st);
    prof_mark(ST_REDUCE, st);
    return rc;
}

// Dense branch of Residual-MoE on the MFMA kernel, with the combine fused into its second GEMM:
// out[t, :] = gelu_tanh(x[t] Wd1 + bd1) Wd2 + bd2 + sum_j keep_j g_j ye[e_j, slot_j, :].
int run_dense_branch(const moe_shape_t* s, const void* x, const void* Wd1, const void* bd1, const void* Wd2,
                     const void* bd2, void* hd, const void* ye, const int32_t* expert_idx, const int32_t* slot_idx,
                     const float* gate_w, void* out, hipStream_t st) {
    int MT, NW;
    WsGemmArgs a{};
    a.A = u16(x); a.B = u16(Wd1); a.bias = u16(bd1); a.fixed_rows = s->T; a.max_rows = s->T; a.G = 1;
    a.packed = s->flags & MOE_FLAG_PACKED_WEIGHTS;
    a.K = s->d_model; a.N = s->d_ffn; a.out = u16(hd); a.ksplit = 1;
    wsgemm_pick_tile(s->T, 1, s->d_ffn, &MT, &NW);
    const bool tiled = s->T > 64 && tgemm_supported(s->d_model, s->d_ffn) && tgemm_supported(s->d_ffn, s->d_model);
    prof_pre(ST_DENSE1, st);
    int rc = tiled ? launch_tgemm(a, EPI_GELU, st) : launch_wsgemm(a, EPI_GELU, MT, NW, 2, st);
    prof_mark(ST_DENSE1, st);
    if (rc != MOE_OK) return rc;
    a.A = u16(hd); a.B = u16(Wd2); a.bias = u16(bd2); a.K = s->d_ffn; a.N = s->d_model; a.out = u16(out);
    a.ye = u16(ye); a.expert_idx = expert_idx; a.slot_idx = slot_idx; a.gate_w = gate_w; a.top_k = s->top_k;
    a.C = s->capacity;
    wsgemm_pick_tile(s->T, 1, s->d_model, &MT, &NW);
    prof_pre(ST_DENSE2, st);
    rc = tiled ? launch_tgemm(a, EPI_COMBINE, st) : launch_wsgemm(a, EPI_COMBINE, MT, NW, 2, st);
    prof_mark(ST_DENSE2, st);
    return rc;
}

// Residual-MoE with experts and dense branch both on 256-row tiles: the experts' and the dense branch's products of
// each FFN half share one launch (same inner and outer sizes), so that the second half, with only d_model columns,
// has twice the tiles and can use the large tile; the combine then is a kernel of its own on the two outputs.
// Returns MOE_ERR_UNSUPPORTED (nothing launched) when the pair does not fit that pattern.
int run_residual_paired(const moe_shape_t* s, const FfnPlan& p, const void* x, const int32_t* slot_token,
                        const int32_t* rows, const int32_t* order, const void* W1, const void* b1, const void* W2,
                        const void* b2, const void* Wd1, const void* bd1, const void* Wd2, const void* bd2, void* h,
                        void* hd, void* ye, void* dense_out, const int32_t* expert_idx, const int32_t* slot_idx,
                        const float* gate_w, void* out, hipStream_t st) {
    if (!p.tiled || s->T <= 128) return MOE_ERR_UNSUPPORTED;
    const int packed = s->flags & MOE_FLAG_PACKED_WEIGHTS;
    WsGemmArgs e1{}, d1{}, e2{}, d2{};
    e1.A = u16(x); e1.B = u16(W1); e1.bias = u16(b1); e1.rows = rows; e1.order = order; e1.row_map = slot_token;
    e1.packed = packed; e1.max_rows = s->capacity; e1.map_stride = s->capacity; e1.G = s->E; e1.K = s->d_model;
    e1.N = s->d_ffn; e1.a_group_stride = s->capacity; e1.out = u16(h); e1.o_group_stride = s->capacity; e1.ksplit = 1;
    d1.A = u16(x); d1.B = u16(Wd1); d1.bias = u16(bd1); d1.fixed_rows = s->T; d1.max_rows = s->T; d1.G = 1;
    d1.packed = packed; d1.K = s->d_model; d1.N = s->d_ffn; d1.out = u16(hd); d1.ksplit = 1;
    e2 = e1; e2.A = u16(h); e2.B = u16(W2); e2.bias = u16(b2); e2.row_map = nullptr; e2.K = s->d_ffn; e2.N = s->d_model;
    e2.out = u16(ye);
    d2 = d1; d2.A = u16(hd); d2.B = u16(Wd2); d2.bias = u16(bd2); d2.K = s->d_ffn; d2.N = s->d_model; d2.out = u16(dense_out);
    if (!tgemm_pair_fusable(e2, d2)) return MOE_ERR_UNSUPPORTED;
    int rc;
    if (tgemm_pair_fusable(e1, d1)) {
        prof_pre(ST_GEMM1, st);
        rc = launch_tgemm_pair(e1, d1, EPI_GELU, st);
        prof_mark(ST_GEMM1, st);
    } else {                                  // the first halves each on the tile that suits them
        prof_pre(ST_GEMM1, st);
        rc = launch_tgemm(e1, EPI_GELU, st);
        prof_mark(ST_GEMM1, st);
        if (rc != MOE_OK) return rc;
        prof_pre(ST_DENSE1, st);
        rc = launch_tgemm(d1, EPI_GELU, st);
        prof_mark(ST_DENSE1, st);
    }
    if (rc != MOE_OK) return rc;
    prof_pre(ST_GEMM2, st);
    rc = launch_tgemm_pair(e2, d2, EPI_STORE, st);
    prof_mark(ST_GEMM2, st);
    if (rc != MOE_OK) return rc;
    prof_pre(ST_COMBINE, st);
    rc = launch_combine(ye, s->dtype, expert_idx, slot_idx, gate_w, dense_out, out, s->T, s->top_k, s->capacity,
                        s->d_model, st);
    prof_mark(ST_COMBINE, st);
    return rc;
}

}  // namespace

extern "C" {

size_t moe_workspace_bytes(const moe_shape_t* shape) {
    if (check_shape(shape) != MOE_OK) return 0;
    return ws_layout(shape).total;
}

const char* moe_status_string(int status) {
    switch (status) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID_ARG: return "invalid argument";
        case MOE_ERR_UNSUPPORTED: return "unsupported shape";
        case MOE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case MOE_ERR_HIP: return "HIP launch failed";
        case MOE_ERR_SCRATCH_LIMIT: return "shape needs more scratch than the no-allocation entry point holds";
        default: return "unknown status";
    }
}

const char* moe_version(void) { return "0.2"; }

size_t moe_packed_weights_bytes(int32_t G, int32_t K, int32_t N) {
    if (G < 1 || K < 8 || N < 8 || K % 8 || N % 8) return 0;
    return packed_weight_elems(G, K, N) * 2;
}

size_t moe_packed_gate_bytes(int32_t d_model, int32_t E) {
    if (d_model < 1 || E < 1) return 0;
    return gate_bf16_ws_bytes(d_model, E);            // 0 for shapes the bf16 gate kernel does not cover
}

int moe_pack_gate(int32_t d_model, int32_t E, const float* Wg, void* packed, void* stream) {
    if (d_model < 1 || E < 1 || !Wg || !packed || !aligned16(Wg) || !aligned16(packed)) return MOE_ERR_INVALID_ARG;
    return launch_pack_gate(Wg, packed, d_model, E, static_cast<hipStream_t>(stream));
}

int moe_pack_weights(int32_t G, int32_t K, int32_t N, const void* W, void* packed, void* stream) {
    if (G < 1 || K < 8 || N < 8 || !W || !packed || !aligned16(W) || !aligned16(packed)) return MOE_ERR_INVALID_ARG;
    if (K % 8 || N % 8) return MOE_ERR_UNSUPPORTED;
    return launch_pack_weights(u16(W), u16(packed), G, K, N, static_cast<hipStream_t>(stream));
}

// argument checks shared by moe_gate and moe_gate_noalloc (everything but the scratch memory)
static int check_gate_args(const moe_shape_t* shape, const void* x, const float* Wg, const float* bg, float* logits,
                           int32_t* expert_idx, int32_t* slot_idx, float* gate_w, int32_t* expert_rows,
                           int32_t* slot_token) {
    const int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    if (!expert_idx || !slot_idx || !gate_w || !expert_rows || !slot_token) return MOE_ERR_INVALID_ARG;
    if (!x && !logits) return MOE_ERR_INVALID_ARG;
    if (x && !Wg) return MOE_ERR_INVALID_ARG;
    const void* ptrs[] = {x, Wg, bg, logits, expert_idx, slot_idx, gate_w, expert_rows, slot_token};
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return MOE_ERR_INVALID_ARG;
    return MOE_OK;
}

// the gate on checked arguments; `ws` holds at least gate_scratch_bytes(shape) bytes
static int gate_checked(const moe_shape_t* shape, const void* x, const float* Wg, const float* bg, float* logits,
                        int32_t* expert_idx, int32_t* slot_idx, float* gate_w, int32_t* expert_rows,
                        int32_t* slot_token, void* ws, hipStream_t st) {
    const WsLayout L = ws_layout(shape);
    float* lg = logits ? logits : at<float>(ws, L.logits);
    if (x)
        return run_gate(shape, x, Wg, bg, lg, expert_idx, slot_idx, gate_w, expert_rows, slot_token, nullptr, ws, L, false, st);
    return launch_route(lg, shape->T, shape->E, shape->top_k, shape->capacity, expert_idx, slot_idx, gate_w,
                        expert_rows, slot_token, nullptr, at<int32_t>(ws, L.hist), st);
}

int moe_gate(const moe_shape_t* shape, const void* x, const float* Wg, const float* bg, float* logits,
             int32_t* expert_idx, int32_t* slot_idx, float* gate_w, int32_t* expert_rows, int32_t* slot_token,
             void* ws, size_t ws_bytes, void* stream) {
    int rc = check_gate_args(shape, x, Wg, bg, logits, expert_idx, slot_idx, gate_w, expert_rows, slot_token);
    if (rc != MOE_OK) return rc;
    rc = check_ws(shape, ws, ws_bytes);
    if (rc != MOE_OK) return rc;
    return gate_checked(shape, x, Wg, bg, logits, expert_idx, slot_idx, gate_w, expert_rows, slot_token, ws,
                        static_cast<hipStream_t>(stream));
}

size_t moe_gate_noalloc_max_bytes(void) { return kStaticScratchBytes; }

size_t moe_gate_noalloc_bytes(const moe_shape_t* shape) {
    if (check_shape(shape) != MOE_OK) return 0;
    return gate_scratch_bytes(shape);
}

int moe_gate_noalloc(const moe_shape_t* shape, const void* x, const float* Wg, const float* bg, float* logits,
                     int32_t* expert_idx, int32_t* slot_idx, float* gate_w, int32_t* expert_rows, int32_t* slot_token,
                     void* stream) {
    int rc = check_gate_args(shape, x, Wg, bg, logits, expert_idx, slot_idx, gate_w, expert_rows, slot_token);
    if (rc != MOE_OK) return rc;
    if (gate_scratch_bytes(shape) > kStaticScratchBytes) return MOE_ERR_SCRATCH_LIMIT;
    void* scratch = nullptr;
    rc = static_scratch(&scratch);
    if (rc != MOE_OK) return rc;
    return gate_checked(shape, x, Wg, bg, logits, expert_idx, slot_idx, gate_w, expert_rows, slot_token, scratch,
                        static_cast<hipStream_t>(stream));
}

int moe_dispatch(const moe_shape_t* shape, const void* x, const int32_t* slot_token, const int32_t* expert_rows,
                 void* xe, void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    if (!x || !slot_token || !expert_rows || !xe) return MOE_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(slot_token) || !aligned16(expert_rows) || !aligned16(xe)) return MOE_ERR_INVALID_ARG;
    return launch_dispatch(x, shape->dtype, slot_token, expert_rows, xe, shape->E, shape->capacity, shape->d_model,
                           static_cast<hipStream_t>(stream));
}

int moe_expert_ffn(const moe_shape_t* shape, const void* xe, const int32_t* expert_rows, const void* W1,
                   const void* b1, const void* W2, const void* b2, void* ye, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    if (!xe || !expert_rows || !W1 || !W2 || !ye) return MOE_ERR_INVALID_ARG;
    const void* ptrs[] = {xe, expert_rows, W1, b1, W2, b2, ye};
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return MOE_ERR_INVALID_ARG;
    rc = check_ws(shape, ws, ws_bytes);
    if (rc != MOE_OK) return rc;
    const WsLayout L = ws_layout(shape);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const FfnPlan plan = plan_ffn(shape);
    if (!plan.mfma)
        return run_ffn_simple(shape->dtype, shape->E, shape->capacity, expert_rows, 0, shape->d_model, shape->d_ffn, xe,
                              W1, b1, W2, b2, at<void>(ws, L.h), ye, st);
    int32_t* order = at<int32_t>(ws, L.order);
    rc = launch_expert_order(expert_rows, shape->E, shape->capacity, order, st);
    if (rc != MOE_OK) return rc;
    rc = run_expert_gemm1(shape, plan, xe, nullptr, expert_rows, order, W1, b1, at<void>(ws, L.h), st);
    if (rc != MOE_OK) return rc;
    return run_expert_gemm2(shape, plan, at<void>(ws, L.h), expert_rows, order, W2, b2, false, nullptr, nullptr, nullptr, ye,
                            at<float>(ws, L.partial), st);
}

int moe_expert_ffn_slice(const moe_shape_t* shape, const void* xe, const int32_t* expert_rows, const void* W1s,
                         const void* b1s, const void* W2s, float* ye_partial, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    if (shape->dtype != MOE_BF16) return MOE_ERR_UNSUPPORTED;
    if (!xe || !expert_rows || !W1s || !W2s || !ye_partial) return MOE_ERR_INVALID_ARG;
    const void* ptrs[] = {xe, expert_rows, W1s, b1s, W2s, ye_partial};
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return MOE_ERR_INVALID_ARG;
    rc = check_ws(shape, ws, ws_bytes);
    if (rc != MOE_OK) return rc;
    const WsLayout L = ws_layout(shape);
    hipStream_t st = static_cast<hipStream_t>(stream);
    FfnPlan plan = plan_ffn(shape);
    plan.ksplit2 = 1;                                  // the slice itself is the split of the inner dimension
    int32_t* order = at<int32_t>(ws, L.order);
    rc = launch_expert_order(expert_rows, shape->E, shape->capacity, order, st);
    if (rc != MOE_OK) return rc;
    rc = run_expert_gemm1(shape, plan, xe, nullptr, expert_rows, order, W1s, b1s, at<void>(ws, L.h), st);
    if (rc != MOE_OK) return rc;
    WsGemmArgs a{};
    a.A = at<uint16_t>(ws, L.h); a.B = u16(W2s); a.rows = expert_rows; a.order = order;
    a.packed = shape->flags & MOE_FLAG_PACKED_WEIGHTS;
    a.max_rows = shape->capacity; a.G = shape->E; a.K = shape->d_ffn; a.N = shape->d_model;
    a.a_group_stride = shape->capacity; a.o_group_stride = shape->capacity; a.ksplit = 1;
    a.partial = ye_partial; a.partial_rows = (long long)shape->E * shape->capacity;
    return plan.tiled ? launch_tgemm(a, EPI_PARTIAL, st) : launch_wsgemm(a, EPI_PARTIAL, plan.MT, plan.NW2, plan.NBUF, st);
}

int moe_expert_ffn_slice_reduce(const moe_shape_t* shape, int32_t n_slices, const float* ye_partials,
                                const int32_t* expert_rows, const void* b2, void* ye, void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    if (shape->dtype != MOE_BF16) return MOE_ERR_UNSUPPORTED;
    if (n_slices < 1 || n_slices > 64 || !ye_partials || !expert_rows || !ye) return MOE_ERR_INVALID_ARG;
    if (!aligned16(ye_partials) || !aligned16(expert_rows) || !aligned16(ye) || (b2 && !aligned16(b2)))
        return MOE_ERR_INVALID_ARG;
    SplitKReduceArgs r{};
    r.partial = ye_partials; r.ksplit = n_slices; r.G = shape->E; r.N = shape->d_model; r.group_stride = shape->capacity;
    r.rows = expert_rows; r.max_rows = shape->capacity; r.bias = u16(b2); r.out = u16(ye); r.top_k = shape->top_k;
    r.T = shape->T;
    return launch_splitk_reduce(r, static_cast<hipStream_t>(stream));
}

int moe_combine(const moe_shape_t* shape, const void* ye, const int32_t* expert_idx, const int32_t* slot_idx,
                const float* gate_w, const void* addend, void* out, void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    if (!ye || !expert_idx || !slot_idx || !gate_w || !out) return MOE_ERR_INVALID_ARG;
    const void* ptrs[] = {ye, expert_idx, slot_idx, gate_w, addend, out};
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return MOE_ERR_INVALID_ARG;
    return launch_combine(ye, shape->dtype, expert_idx, slot_idx, gate_w, addend, out, shape->T, shape->top_k,
                          shape->capacity, shape->d_model, static_cast<hipStream_t>(stream));
}

static int layer_forward_checked(const moe_shape_t* shape, const void* x, const float* Wg, const float* bg, const void* W1,
                      const void* b1, const void* W2, const void* b2, const void* Wd1, const void* bd1, const void* Wd2,
                      const void* bd2, void* out, float* logits_out, int32_t* expert_idx_out, int32_t* slot_idx_out,
                      float* gate_w_out, int32_t* expert_rows_out, int32_t* slot_token_out, void* ws, size_t ws_bytes,
                      void* stream) {
    int rc = check_shape(shape);
    if (rc != MOE_OK) return rc;
    if (!x || !Wg || !W1 || !W2 || !out) return MOE_ERR_INVALID_ARG;
    if (shape->residual && (!Wd1 || !Wd2)) return MOE_ERR_INVALID_ARG;
    if (!shape->residual && (Wd1 || Wd2 || bd1 || bd2)) return MOE_ERR_INVALID_ARG;
    const void* ptrs[] = {x, Wg, bg, W1, b1, W2, b2, Wd1, bd1, Wd2, bd2, out, logits_out, expert_idx_out,
                          slot_idx_out, gate_w_out, expert_rows_out, slot_token_out};
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return MOE_ERR_INVALID_ARG;
    rc = check_ws(shape, ws, ws_bytes);
    if (rc != MOE_OK) return rc;

    const WsLayout L = ws_layout(shape);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int T = shape->T, d = shape->d_model, f = shape->d_ffn, E = shape->E, k = shape->top_k, C = shape->capacity;
    const int dt = shape->dtype;

    float* logits = logits_out ? logits_out : at<float>(ws, L.logits);
    int32_t* expert_idx = expert_idx_out ? expert_idx_out : at<int32_t>(ws, L.expert_idx);
    int32_t* slot_idx = slot_idx_out ? slot_idx_out : at<int32_t>(ws, L.slot_idx);
    float* gate_w = gate_w_out ? gate_w_out : at<float>(ws, L.gate_w);
    int32_t* rows = expert_rows_out ? expert_rows_out : at<int32_t>(ws, L.rows);
    int32_t* slot_token = slot_token_out ? slot_token_out : at<int32_t>(ws, L.slot_token);

    prof_begin(st);
    int32_t* order = at<int32_t>(ws, L.order);
    rc = run_gate(shape, x, Wg, bg, logits, expert_idx, slot_idx, gate_w, rows, slot_token, order, ws, L, true, st);
    if (rc != MOE_OK) return rc;
    const FfnPlan plan = plan_ffn(shape);
    if (!plan.mfma) {
        // fp32 layer: the unfused sequence dispatch -> FFN -> [dense branch] -> combine
        prof_pre(ST_DISPATCH, st);
        rc = launch_dispatch(x, dt, slot_token, rows, at<void>(ws, L.xe), E, C, d, st);
        prof_mark(ST_DISPATCH, st);
        if (rc != MOE_OK) return rc;
        prof_pre(ST_GEMM2, st);
        rc = run_ffn_simple(dt, E, C, rows, 0, d, f, at<void>(ws, L.xe), W1, b1, W2, b2, at<void>(ws, L.h),
                            at<void>(ws, L.ye), st);
        prof_mark(ST_GEMM2, st);
        if (rc != MOE_OK) return rc;
        const void* addend = nullptr;
        if (shape->residual) {
            prof_pre(ST_DENSE2, st);
            rc = run_ffn_simple(dt, 1, T, nullptr, T, d, f, x, Wd1, bd1, Wd2, bd2, at<void>(ws, L.hd),
                                at<void>(ws, L.dense), st);
            prof_mark(ST_DENSE2, st);
            if (rc != MOE_OK) return rc;
            addend = at<void>(ws, L.dense);
        }
        prof_pre(ST_COMBINE, st);
        rc = launch_combine(at<void>(ws, L.ye), dt, expert_idx, slot_idx, gate_w, addend, out, T, k, C, d, st);
        prof_mark(ST_COMBINE, st);
        return rc;
    }

    if (shape->residual) {
        rc = run_residual_paired(shape, plan, x, slot_token, rows, order, W1, b1, W2, b2, Wd1, bd1, Wd2, bd2,
                                 at<void>(ws, L.h), at<void>(ws, L.hd), at<void>(ws, L.ye), at<void>(ws, L.dense),
                                 expert_idx, slot_idx, gate_w, out, st);
        if (rc != MOE_ERR_UNSUPPORTED) return rc;
    }
    // bf16: dispatch is fused into GEMM-1 (rows gathered through slot_token) ...
    rc = run_expert_gemm1(shape, plan, x, slot_token, rows, order, W1, b1, at<void>(ws, L.h), st);
    if (rc != MOE_OK) return rc;
    // ... and, for top-1 Standard-MoE, combine into GEMM-2 (scale by the gate weight, write the token's row)
    if (k == 1 && !shape->residual)
        return run_expert_gemm2(shape, plan, at<void>(ws, L.h), rows, order, W2, b2, true, slot_token, slot_idx, gate_w, out,
                                at<float>(ws, L.partial), st);
    rc = run_expert_gemm2(shape, plan, at<void>(ws, L.h), rows, order, W2, b2, false, nullptr, nullptr, nullptr,
                          at<void>(ws, L.ye), at<float>(ws, L.partial), st);
    if (rc != MOE_OK) return rc;
    if (shape->residual)
        return run_dense_branch(shape, x, Wd1, bd1, Wd2, bd2, at<void>(ws, L.hd), at<void>(ws, L.ye), expert_idx,
                                slot_idx, gate_w, out, st);
    prof_pre(ST_COMBINE, st);
    rc = launch_combine(at<void>(ws, L.ye), dt, expert_idx, slot_idx, gate_w, nullptr, out, T, k, C, d, st);
    prof_mark(ST_COMBINE, st);
    return rc;
}

int moe_layer_forward(const moe_shape_t* shape, const void* x, const float* Wg, const float* bg, const void* W1,
                      const void* b1, const void* W2, const void* b2, const void* Wd1, const void* bd1, const void* Wd2,
                      const void* bd2, void* out, float* logits_out, int32_t* expert_idx_out, int32_t* slot_idx_out,
                      float* gate_w_out, int32_t* expert_rows_out, int32_t* slot_token_out, void* ws, size_t ws_bytes,
                      void* stream) {
    const int rc = layer_forward_checked(shape, x, Wg, bg, W1, b1, W2, b2, Wd1, bd1, Wd2, bd2, out, logits_out,
                                         expert_idx_out, slot_idx_out, gate_w_out, expert_rows_out, slot_token_out, ws,
                                         ws_bytes, stream);
    g_prof.cur = -1;       // stage events belong to this call only: a later moe_expert_ffn must not add to them
    return rc;
}

// ---- one decode step of a whole decoder block ---------------------------------------------------------------------
namespace {

struct BlockLayout {
    size_t qkv, attn, proj, x1, xn, moe_out, attn_partial, lin_partial, moe_ws, total;
};
constexpr int kLinearMaxSplit = 8;

BlockLayout block_layout(const moe_shape_t* s, const moe_block_shape_t* b) {
    BlockLayout L{};
    const size_t T = s->T, d = s->d_model;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes); return o; };
    L.qkv = take(T * 3 * d * 2);
    L.attn = take(T * d * 2);
    L.proj = take(T * d * 2);
    L.x1 = take(T * d * 2);
    L.xn = take(T * d * 2);
    L.moe_out = take(T * d * 2);
    L.attn_partial = take(attn_partial_floats(s->T, b->n_heads, s->d_model / b->n_heads, b->max_len) * 4);
    L.lin_partial = take((size_t)kLinearMaxSplit * T * 3 * d * 4);
    L.moe_ws = take(ws_layout(s).total);
    L.total = off;
    return L;
}

int check_block_shape(const moe_shape_t* s, const moe_block_shape_t* b) {
    const int rc = check_shape(s);
    if (rc != MOE_OK) return rc;
    if (!b || b->n_heads < 1 || b->max_len < 1) return MOE_ERR_INVALID_ARG;
    if (s->dtype != MOE_BF16) return MOE_ERR_UNSUPPORTED;
    if (!attn_supported(s->d_model, b->n_heads)) return MOE_ERR_UNSUPPORTED;
    if ((long long)s->T * b->n_heads >= (1ll << 31) || b->max_len > (1 << 24)) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

// out[T, N] = x[T, K] W[K, N] + bias on the weight-streaming kernel (a decode step has few rows: the product is a
// read of W); with few output columns the inner dimension is split over more waves and summed in a fixed order
int run_linear(const uint16_t* x, const uint16_t* W, const uint16_t* bias, uint16_t* out, int T, int K, int N,
               float* partial, hipStream_t st) {
    WsGemmArgs a{};
    a.A = x; a.B = W; a.bias = bias; a.fixed_rows = T; a.max_rows = T; a.G = 1; a.K = K; a.N = N; a.out = out;
    a.o_group_stride = T; a.a_group_stride = T; a.ksplit = 1;
    int MT, NW;
    wsgemm_pick_tile(T, 1, N, &MT, &NW);
    const long long waves = (long long)((N + 127) / 128) * ((T + MT - 1) / MT);
    const int chunks = (K + wsgemm_chunk_k(MT) - 1) / wsgemm_chunk_k(MT);
    long long ks = waves < 1024 ? (2048 + waves - 1) / waves : 1;
    if (ks > kLinearMaxSplit) ks = kLinearMaxSplit;
    if (ks > chunks) ks = chunks;
    if (ks <= 1) return launch_wsgemm(a, EPI_STORE, MT, NW, 2, st);
    a.ksplit = (int)ks; a.partial = partial; a.partial_rows = T;
    int rc = launch_wsgemm(a, EPI_PARTIAL, MT, NW, 2, st);
    if (rc != MOE_OK) return rc;
    SplitKReduceArgs r{};
    r.partial = partial; r.ksplit = (int)ks; r.G = 1; r.N = N; r.group_stride = T; r.rows = nullptr; r.max_rows = T;
    r.bias = bias; r.out = out; r.top_k = 1; r.T = T;
    return launch_splitk_reduce(r, st);
}

}  // namespace

size_t moe_decode_block_workspace_bytes(const moe_shape_t* shape, const moe_block_shape_t* block) {
    if (check_block_shape(shape, block) != MOE_OK) return 0;
    return block_layout(shape, block).total;
}

int moe_decode_block_forward(const moe_shape_t* shape, const moe_block_shape_t* block, const moe_block_weights_t* w,
                             const void* x, void* k_cache, void* v_cache, const int32_t* pos, void* out, void* x1_out,
                             void* moe_in_out, float* logits_out, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_block_shape(shape, block);
    if (rc != MOE_OK) return rc;
    if (!w || !x || !k_cache || !v_cache || !pos || !out) return MOE_ERR_INVALID_ARG;
    if (!w->ln1_gamma || !w->ln1_beta || !w->Wqkv || !w->Wo || !w->ln2_gamma || !w->ln2_beta || !w->Wg || !w->W1 || !w->W2)
        return MOE_ERR_INVALID_ARG;
    if (shape->residual && (!w->Wd1 || !w->Wd2)) return MOE_ERR_INVALID_ARG;
    if (!shape->residual && (w->Wd1 || w->Wd2 || w->bd1 || w->bd2)) return MOE_ERR_INVALID_ARG;
    const void* ptrs[] = {x, k_cache, v_cache, pos, out, x1_out, moe_in_out, logits_out, w->ln1_gamma, w->ln1_beta, w->Wqkv,
                          w->bqkv, w->Wo, w->bo, w->ln2_gamma, w->ln2_beta, w->Wg, w->bg, w->W1, w->b1, w->W2, w->b2,
                          w->Wd1, w->bd1, w->Wd2, w->bd2};
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return MOE_ERR_INVALID_ARG;
    const BlockLayout L = block_layout(shape, block);
    if (!ws || !aligned16(ws) || ws_bytes < L.total) return MOE_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const int T = shape->T, d = shape->d_model, H = block->n_heads, dh = d / H;
    const float eps = 1e-5f;
    uint16_t* qkv = at<uint16_t>(ws, L.qkv);
    uint16_t* attn = at<uint16_t>(ws, L.attn);
    uint16_t* proj = at<uint16_t>(ws, L.proj);
    uint16_t* x1 = x1_out ? u16(x1_out) : at<uint16_t>(ws, L.x1);
    uint16_t* xn = at<uint16_t>(ws, L.xn);
    uint16_t* moe_in = moe_in_out ? u16(moe_in_out) : xn;
    uint16_t* moe_out = at<uint16_t>(ws, L.moe_out);
    float* lin_partial = at<float>(ws, L.lin_partial);

    // a = LayerNorm(x); qkv = a Wqkv + bqkv
    rc = launch_add_layernorm(u16(x), nullptr, w->ln1_gamma, w->ln1_beta, nullptr, xn, T, d, eps, st);
    if (rc != MOE_OK) return rc;
    rc = run_linear(xn, u16(w->Wqkv), u16(w->bqkv), qkv, T, d, 3 * d, lin_partial, st);
    if (rc != MOE_OK) return rc;
    // the new token over its sequence's cache (its own key/value rows join the cache)
    rc = launch_attn_decode(qkv, u16(k_cache), u16(v_cache), pos, at<float>(ws, L.attn_partial), attn, T, H, dh,
                            block->max_len, st);
    if (rc != MOE_OK) return rc;
    rc = run_linear(attn, u16(w->Wo), u16(w->bo), proj, T, d, d, lin_partial, st);
    if (rc != MOE_OK) return rc;
    // x1 = x + attention; the MoE layer sees LayerNorm(x1)
    rc = launch_add_layernorm(u16(x), proj, w->ln2_gamma, w->ln2_beta, x1, moe_in, T, d, eps, st);
    if (rc != MOE_OK) return rc;
    rc = layer_forward_checked(shape, moe_in, w->Wg, w->bg, w->W1, w->b1, w->W2, w->b2, w->Wd1, w->bd1, w->Wd2, w->bd2,
                               moe_out, logits_out, nullptr, nullptr, nullptr, nullptr, nullptr,
                               at<void>(ws, L.moe_ws), ws_layout(shape).total, stream);
    g_prof.cur = -1;
    if (rc != MOE_OK) return rc;
    return launch_add_rows(x1, moe_out, u16(out), (long long)T * d, st);
}

int moe_profile_enable(int max_calls) {
    for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
    g_prof.ev.clear(); g_prof.stage.clear(); g_prof.nmarks.clear();
    g_prof.max_calls = 0; g_prof.calls = 0; g_prof.cur = -1; g_prof.seen = 0;
    if (max_calls <= 0) return MOE_OK;
    if (max_calls > 4096) return MOE_ERR_INVALID_ARG;
    const size_t n = (size_t)max_calls * kMarks;
    g_prof.ev.resize(n);
    for (size_t i = 0; i < n; ++i)
        if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) { g_prof.ev.resize(i); moe_profile_enable(0); return MOE_ERR_HIP; }
    g_prof.stage.assign(n, -1);
    g_prof.nmarks.assign(max_calls, 0);
    g_prof.max_calls = max_calls;
    return MOE_OK;
}

int moe_profile_select(unsigned stage_mask) {
    g_prof.mask = stage_mask;
    return MOE_OK;
}

int moe_profile_stride(int every_nth_call) {
    if (every_nth_call < 1) return MOE_ERR_INVALID_ARG;
    g_prof.stride = every_nth_call;
    return MOE_OK;
}

int moe_profile_calls(void) { return g_prof.calls; }
int moe_profile_stage_count(void) { return ST_COUNT; }
const char* moe_profile_stage_name(int i) { return (i >= 0 && i < ST_COUNT) ? kStageNames[i] : ""; }

int moe_profile_elapsed(int call, float* ms) {
    if (!ms || call < 0 || call >= g_prof.calls) return MOE_ERR_INVALID_ARG;
    for (int i = 0; i < ST_COUNT; ++i) ms[i] = 0.f;
    const size_t base = (size_t)call * kMarks;
    const int m = g_prof.nmarks[call];
    if (m < 2) return MOE_OK;
    if (hipEventSynchronize(g_prof.ev[base + m - 1]) != hipSuccess) return MOE_ERR_HIP;
    for (int i = 1; i < m; ++i) {
        const int st = g_prof.stage[base + i];
        if (st < 0) continue;                  // that event only opened the next stage
        float t = 0.f;
        if (hipEventElapsedTime(&t, g_prof.ev[base + i - 1], g_prof.ev[base + i]) != hipSuccess) return MOE_ERR_HIP;
        ms[st] += t;
    }
    return MOE_OK;
}

}  // extern "C"
