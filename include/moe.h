/* moe.h -- C ABI of the MI355X (gfx950) MoE-layer forward library.
 *
 * The library computes the forward pass of one Mixture-of-Experts layer as the
 * DeepSpeed-MoE paper (arXiv 2201.05596) states it in Sec. 5.4: a gating
 * function assigns tokens to experts, the tokens are sorted by assigned expert
 * (dispatch), each expert's FFN runs on its tokens, and the expert outputs are
 * scaled by the gate probability and put back in token order (combine).  As in
 * Sec. 5.4 the one-hot/einsum formulation is replaced by a dense
 * token-to-expert mapping table and explicit data-layout transforms.  The
 * Residual-MoE variant of Sec. 4.1.1 adds a dense MLP branch to every token.
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library
 *     never allocates, frees or synchronises.  All work is enqueued on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Tensors are row-major and densely packed; base pointers must be 16-byte
 *     aligned.  Element type of x / xe / ye / out and of the FFN weights and
 *     biases is `shape.dtype`; gate weights, gate bias, logits and gate_w are
 *     always float; indices are int32_t.
 *   - `shape` is a HOST pointer, read before the call returns.
 *   - Return value: MOE_OK, or a negative moe_status_t.  On
 *     MOE_ERR_INVALID_ARG / MOE_ERR_UNSUPPORTED / MOE_ERR_WORKSPACE nothing
 *     was launched, no HIP call was made and no output was touched.
 *     MOE_ERR_HIP reports a failed launch; outputs are then unspecified.
 *   - `capacity` (rows per expert, C) is always given explicitly; the library
 *     never derives it from a capacity factor.
 *   - Non-finite gate logits give unspecified routing.
 *   - Calls on one stream are ordered; two calls that share a workspace and
 *     run concurrently on different streams race.
 *   - Entry points are called from one host thread at a time (the library
 *     keeps small host-side caches: kernel attributes, occupancy, profiler).
 *   - Stream capture: after one ordinary call with the same shape (kernel
 *     attributes and occupancy are looked up at first use) a call only
 *     enqueues kernels and may be recorded into a HIP graph; every replay
 *     gives what the ordinary call gives.  Keep the stage profiler off then.
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = -1,  /* null pointer, misaligned pointer, bad size        */
    MOE_ERR_UNSUPPORTED = -2,  /* valid request outside what the kernels cover      */
    MOE_ERR_WORKSPACE = -3,    /* ws is NULL or smaller than moe_workspace_bytes()  */
    MOE_ERR_HIP = -4,          /* a kernel launch failed                            */
    MOE_ERR_SCRATCH_LIMIT = -5 /* moe_gate_noalloc: shape beyond its fixed scratch   */
} moe_status_t;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype_t;

/* Bits of moe_shape_t.flags. */
enum {
    /* W1, W2 (and Wd1, Wd2) are not the plain [E,d,f] / [E,f,d] arrays but the
     * buffers moe_pack_weights() wrote from them (bf16 only). */
    MOE_FLAG_PACKED_WEIGHTS = 1,
    /* Wg is not the plain float [d,E] array but the buffer moe_pack_gate() wrote
     * from it (bf16 tokens, d_model a multiple of 32, at most 128 experts). */
    MOE_FLAG_PACKED_GATE = 2
};

/* Shape of one MoE layer.  Limits: T >= 1, 1 <= E <= 1024, top_k in {1,2} and
 * <= E, capacity >= 1, T*top_k and E*capacity below 2^31; d_model and d_ffn
 * multiples of 8 (bf16) or 4 (f32).  `flags`: 0 or MOE_FLAG_* bits. */
typedef struct {
    int32_t T;         /* tokens (paper: S)                                    */
    int32_t d_model;   /* hidden size (paper: M)                               */
    int32_t d_ffn;     /* expert FFN inner width                               */
    int32_t E;         /* experts                                              */
    int32_t top_k;     /* experts per token                                    */
    int32_t capacity;  /* rows per expert (paper: c_e)                         */
    int32_t dtype;     /* moe_dtype_t                                          */
    int32_t residual;  /* 1: Residual-MoE (dense MLP branch added), else 0     */
    int32_t flags;     /* MOE_FLAG_* bits, 0 = plain weights                   */
} moe_shape_t;

/* Upper bound, in bytes, of the workspace any entry point needs for this
 * shape.  Returns 0 for an invalid shape.  Pure host arithmetic. */
size_t moe_workspace_bytes(const moe_shape_t* shape);

/* Static string for a status code. */
const char* moe_status_string(int status);

/* Library version, "major.minor". */
const char* moe_version(void);

/* moe_pack_weights -- optional one-time re-tiling of bf16 FFN weights for the
 * matrix cores (inference weights do not change between calls; Sec. 5.1: what
 * an inference step costs is reading the parameters).  W is a plain row-major
 * [G,K,N] array (W1: G=E, K=d_model, N=d_ffn; W2: G=E, K=d_ffn, N=d_model; the
 * dense branch: G=1); `packed` receives moe_packed_weights_bytes(G,K,N) bytes
 * (K rounded up to 32, N to 128, zero filled) in which every 16 bytes are 8
 * consecutive k of one column, in the order the matrix instructions consume
 * them.  Pass the packed buffers as W1/W2/Wd1/Wd2 together with
 * MOE_FLAG_PACKED_WEIGHTS in shape.flags (all of a call's FFN weights packed,
 * or none).  The plain layout stays the default input of every entry point;
 * results are the same either way up to fp32 summation order.  K and N must be
 * multiples of 8.  moe_packed_weights_bytes returns 0 for sizes it rejects. */
size_t moe_packed_weights_bytes(int32_t G, int32_t K, int32_t N);
int moe_pack_weights(int32_t G, int32_t K, int32_t N, const void* W, void* packed, void* stream);

/* moe_pack_gate -- optional one-time preparation of the gate weights for bf16
 * layers: every fp32 weight as the exact sum of three bf16 numbers, laid out as
 * matrix-instruction operands (the gate kernel otherwise does this split into
 * its workspace at every call, one kernel launch more; Sec. 5.4 counts kernel
 * launches among the gate's costs).  `packed` receives moe_packed_gate_bytes(d,E)
 * bytes (0 = shape not covered: d_model not a multiple of 32, or E > 128); pass it
 * as Wg (cast to const float*) with MOE_FLAG_PACKED_GATE.  Logits are bit-identical
 * to those from the plain weights. */
size_t moe_packed_gate_bytes(int32_t d_model, int32_t E);
int moe_pack_gate(int32_t d_model, int32_t E, const float* Wg, void* packed, void* stream);

/* moe_gate -- the fused gating function of Sec. 5.4: gate logits, softmax,
 * top-k, the cumulative sum that gives each token its position inside its
 * expert, the capacity cut, and the mapping tables.
 *
 *   x          [T,d]   tokens, or NULL to route from given logits
 *   Wg         [d,E]   float gate weights (ignored when x == NULL)
 *   bg         [E]     float gate bias or NULL
 *   logits     [T,E]   float.  x == NULL: INPUT.  Otherwise OUTPUT,
 *                      l[t,e] = bg[e] + sum_i x[t,i] Wg[i,e]; may be NULL.
 *   expert_idx [T,k]   out: chosen experts, highest logit first; ties go to the
 *                      lowest expert index
 *   slot_idx   [T,k]   out: row inside the expert, or -1 if dropped.  The row
 *                      is the number of earlier claims on that expert: claims
 *                      are ordered by choice rank first (every first choice
 *                      before any second choice), then by token index; a claim
 *                      whose position is >= capacity is dropped.
 *   gate_w     [T,k]   out: top-1: softmax probability of the chosen expert;
 *                      top-2: the two chosen probabilities divided by their sum
 *   expert_rows[E]     out: kept rows per expert (<= capacity)
 *   slot_token [E,C]   out: token held by each row, -1 for rows >= expert_rows
 *   ws                 workspace, >= moe_workspace_bytes(shape)
 * Routing (expert_idx, slot_idx, expert_rows, slot_token) is a deterministic
 * function of the fp32 logits. */
int moe_gate(const moe_shape_t* shape, const void* x, const float* Wg, const float* bg,
             float* logits, int32_t* expert_idx, int32_t* slot_idx, float* gate_w,
             int32_t* expert_rows, int32_t* slot_token,
             void* ws, size_t ws_bytes, void* stream);

/* moe_gate_noalloc -- moe_gate for callers that cannot allocate device memory or
 * hand over a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and kernels as
 * moe_gate, without `ws`: the scratch (logits when `logits` is NULL, the split
 * gate weights, the block histograms) lives in a fixed array of
 * moe_gate_noalloc_max_bytes() = 8 MiB inside the library's code object, one
 * copy per GPU, held until the process ends.  A shape whose gate scratch
 * (moe_gate_noalloc_bytes(shape); roughly 4*T*E + 6*d*E bytes) exceeds that
 * returns MOE_ERR_SCRATCH_LIMIT before anything is launched.  The call makes no
 * allocation and frees nothing; the first call on a device looks the array's
 * address up once (make that call outside graph capture).  Every call on a GPU
 * uses that GPU's one array and nothing in it is assumed to survive between
 * calls: calls that overlap on one GPU (different streams or host threads) race. */
size_t moe_gate_noalloc_max_bytes(void);
size_t moe_gate_noalloc_bytes(const moe_shape_t* shape);
int moe_gate_noalloc(const moe_shape_t* shape, const void* x, const float* Wg, const float* bg,
                     float* logits, int32_t* expert_idx, int32_t* slot_idx, float* gate_w,
                     int32_t* expert_rows, int32_t* slot_token, void* stream);

/* moe_dispatch -- first layout transform of Sec. 5.4 (replaces the sparse
 * einsum that sorts tokens by expert): xe[e,c,:] = x[slot_token[e,c],:] for
 * c < expert_rows[e].  Rows c >= expert_rows[e] of xe are left untouched. */
int moe_dispatch(const moe_shape_t* shape, const void* x, const int32_t* slot_token,
                 const int32_t* expert_rows, void* xe /* [E,C,d] */, void* stream);

/* moe_expert_ffn -- the expert FFNs (Sec. 3.1: each expert is an FFN of the
 * base model): for c < expert_rows[e]
 *   ye[e,c,:] = gelu_tanh(xe[e,c,:] W1[e] + b1[e]) W2[e] + b2[e].
 *   W1 [E,d,f], b1 [E,f] or NULL, W2 [E,f,d], b2 [E,d] or NULL.
 * Rows c >= expert_rows[e] of ye are left untouched; weights of experts with
 * no rows are not read. */
int moe_expert_ffn(const moe_shape_t* shape, const void* xe, const int32_t* expert_rows,
                   const void* W1, const void* b1, const void* W2, const void* b2,
                   void* ye /* [E,C,d] */, void* ws, size_t ws_bytes, void* stream);

/* moe_expert_ffn_slice -- one device's share of expert-slicing (Sec. 5.2: when
 * there are more devices than experts, an expert's parameters are themselves
 * split across devices, horizontally and vertically as in tensor-slicing).
 * The slice is a range of the FFN's inner dimension: the caller holds
 * W1s [E,d,fs] (the slice's columns of W1), b1s [E,fs] or NULL, W2s [E,fs,d]
 * (the same rows of W2), and shape.d_ffn = fs is the slice's width.  For
 * c < expert_rows[e]
 *   ye_partial[e,c,:] = gelu_tanh(xe[e,c,:] W1s[e] + b1s[e]) W2s[e]      (fp32, no b2)
 * which is the slice's term of the sum over the inner dimension; the slices'
 * partials add up to the expert output (the all-reduce between the devices of
 * a sliced expert; on one device: moe_expert_ffn_slice_reduce).  ye_partial is
 * [E,C,d] float; other rows are left untouched.  bf16 only. */
int moe_expert_ffn_slice(const moe_shape_t* shape, const void* xe, const int32_t* expert_rows,
                         const void* W1s, const void* b1s, const void* W2s, float* ye_partial,
                         void* ws, size_t ws_bytes, void* stream);

/* moe_expert_ffn_slice_reduce -- the sum that ends expert-slicing, done locally:
 *   ye[e,c,:] = b2[e] + sum_s ye_partials[s,e,c,:]     (slices added in index order, fp32)
 * for c < expert_rows[e]; ye_partials is [n_slices,E,C,d] float, 1 <= n_slices <= 64,
 * b2 [E,d] or NULL, ye [E,C,d] in shape.dtype.  shape.d_ffn is not used. */
int moe_expert_ffn_slice_reduce(const moe_shape_t* shape, int32_t n_slices, const float* ye_partials,
                                const int32_t* expert_rows, const void* b2, void* ye, void* stream);

/* moe_combine -- second layout transform of Sec. 5.4 (replaces the final
 * einsum; scales by the gate probability and restores token order):
 *   out[t,:] = addend[t,:] + sum_j [slot_idx[t,j] >= 0] gate_w[t,j] ye[expert_idx[t,j], slot_idx[t,j], :]
 * with fp32 accumulation.  addend ([T,d], same dtype) may be NULL (= 0).  A token
 * whose choices were all dropped gets exactly addend (exactly 0 without one). */
int moe_combine(const moe_shape_t* shape, const void* ye, const int32_t* expert_idx,
                const int32_t* slot_idx, const float* gate_w, const void* addend,
                void* out /* [T,d] */, void* stream);

/* moe_layer_forward -- the whole layer behind one call (Sec. 5.4 fuses the gate
 * and the layout transforms; Sec. 4.1.1 defines the residual branch):
 *   out = combine(expert_ffn(dispatch(x))) [+ gelu_tanh(x Wd1 + bd1) Wd2 + bd2].
 * Wd1 [d,f], bd1 [f] or NULL, Wd2 [f,d], bd2 [d] or NULL are required iff
 * shape.residual.  The *_out pointers are optional (NULL) exports of the gate's
 * results, shaped as in moe_gate.  No host synchronisation happens inside. */
int moe_layer_forward(const moe_shape_t* shape, const void* x, const float* Wg, const float* bg,
                      const void* W1, const void* b1, const void* W2, const void* b2,
                      const void* Wd1, const void* bd1, const void* Wd2, const void* bd2,
                      void* out /* [T,d] */,
                      float* logits_out, int32_t* expert_idx_out, int32_t* slot_idx_out,
                      float* gate_w_out, int32_t* expert_rows_out, int32_t* slot_token_out,
                      void* ws, size_t ws_bytes, void* stream);

/* moe_decode_block_forward -- one decode step (one new token per sequence) of a
 * whole decoder block whose feed-forward part is the MoE layer: the models of
 * Sec. 3.1 are GPT-like decoders with experts on every other feed-forward layer,
 * and Sec. 5.4 runs transformer kernels for the non-expert part beside the MoE
 * kernels.  With T = shape.T sequences, d = d_model, H heads of dh = d/H (64 or
 * 128), bf16:
 *   a      = LayerNorm(x; ln1_gamma, ln1_beta)            (eps 1e-5, biased variance)
 *   q,k,v  = a Wqkv + bqkv                                Wqkv [d,3d], columns q | k | v, head h at h*dh
 *   o[b,h] = softmax(q[b,h] . K^T / sqrt(dh)) V           K, V = the sequence's pos[b] cached rows + the new one
 *   x1     = x + o Wo + bo                                Wo [d,d]
 *   out    = x1 + moe_layer_forward(LayerNorm(x1; ln2_gamma, ln2_beta))
 * k_cache, v_cache [T,H,max_len,dh]: rows 0..pos[b]-1 of sequence b are read, row
 * pos[b] is WRITTEN with the new token's key/value (pos[b] is clamped into
 * 0..max_len-1); the caller advances pos.  LayerNorm parameters are float [d];
 * biases (bqkv [3d], bo [d]) may be NULL.  The MoE weights are those of
 * moe_layer_forward (MOE_FLAG_PACKED_WEIGHTS applies to them only); a dense
 * feed-forward block is E = 1, capacity = T.  Optional exports for parity tests:
 * x1_out [T,d], moe_in_out [T,d] (the MoE layer's input), logits_out [T,E].
 * ws >= moe_decode_block_workspace_bytes(shape, block). */
typedef struct {
    int32_t n_heads;   /* attention heads; d_model / n_heads must be 64 or 128 */
    int32_t max_len;   /* positions per sequence in the key/value caches       */
} moe_block_shape_t;

typedef struct {
    const float* ln1_gamma; const float* ln1_beta;
    const void* Wqkv; const void* bqkv;
    const void* Wo; const void* bo;
    const float* ln2_gamma; const float* ln2_beta;
    const float* Wg; const float* bg;
    const void* W1; const void* b1; const void* W2; const void* b2;
    const void* Wd1; const void* bd1; const void* Wd2; const void* bd2;
} moe_block_weights_t;

size_t moe_decode_block_workspace_bytes(const moe_shape_t* shape, const moe_block_shape_t* block);
int moe_decode_block_forward(const moe_shape_t* shape, const moe_block_shape_t* block, const moe_block_weights_t* weights,
                             const void* x, void* k_cache, void* v_cache, const int32_t* pos, void* out,
                             void* x1_out, void* moe_in_out, float* logits_out,
                             void* ws, size_t ws_bytes, void* stream);

/* Stage timing of moe_layer_forward, for benchmarks (the paper reports the MoE
 * kernels' latency as a whole, Sec. 5.4; this splits it per kernel).
 * moe_profile_enable(n > 0) creates events for the next n calls (the one place
 * where the library creates a HIP resource), n = 0 disables and destroys them.
 * While enabled, each moe_layer_forward call records events on its stream around
 * the selected stages (one before a stage unless the previous stage just
 * recorded one, one after it); nothing is read back.  moe_profile_select takes
 * a bit mask over stage indices (default: all stages); fewer selected stages
 * mean fewer events and less disturbance of the call being timed.
 * moe_profile_elapsed(call, ms) waits for that call's last event and fills
 * ms[moe_profile_stage_count()] with the milliseconds per stage (0 for stages
 * the call did not run).  moe_profile_stride(n >= 1, default 1) times only every
 * n-th call after the last moe_profile_enable (the first, the (n+1)-th, ...),
 * so that a long timed run is disturbed by events in 1/n of its calls only;
 * "the next n calls" of moe_profile_enable then means the next n timed calls.
 * Not thread-safe. */
int moe_profile_enable(int max_calls);
int moe_profile_select(unsigned stage_mask);
int moe_profile_stride(int every_nth_call);
int moe_profile_calls(void);
int moe_profile_stage_count(void);
const char* moe_profile_stage_name(int stage);
int moe_profile_elapsed(int call, float* ms);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
