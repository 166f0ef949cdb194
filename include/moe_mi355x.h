/*
 * moe_mi355x.h -- C ABI of the single-GPU Mixture-of-Experts layer hot path for AMD MI355X (gfx950).
 *
 * One GPU's share of one MoE layer, forward and backward, as the FSMoE paper states the layer
 * (Sec. 2.1): a gating function, an ordering function and its reverse, and E expert FFNs.
 * Notation follows the paper's Table 1: N = B*L tokens, M embedding size, E experts, k top-k,
 * f capacity factor, H expert hidden size, T capacity (maximum tokens per expert).
 *
 * Conventions that hold for every entry point
 *   - Every tensor pointer is a DEVICE pointer to a dense row-major array owned by the caller.
 *     The library never allocates, frees or keeps device memory and never synchronises: it
 *     enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = the default stream)
 *     and returns.  Configuration structs and the size_t* outputs are HOST memory.  Tensor pointers,
 *     the workspace and the saved blob must be 16-byte aligned (rows move as 16-byte vectors);
 *     a misaligned required pointer is MOE_ERR_INVALID_ARG.
 *   - Activations and weights have the element type cfg->dtype (fp32 or bf16 bit patterns).
 *     Logits, probabilities, gate weights and their gradients are fp32.  Indices are int32.
 *   - A, the number of kept (token, choice) assignments, is data dependent.  Buffers indexed by
 *     expert rows are sized by the caller for N*k rows; kernels read A = offsets[E] on the device.
 *     Rows at and beyond A are never read or written.
 *   - Arguments are validated on the host before any launch.  A failed call launches nothing,
 *     returns a status other than MOE_OK and leaves a message for moe_last_error().
 *   - Device data are assumed finite.  With NaN/Inf logits the values are unspecified, but the routing
 *     stays valid (k distinct experts in range per token, consistent counts and index maps).
 *   - Calls that share output or workspace buffers must be ordered by the caller (same stream).
 *   - Stream capture: no call records a memset, allocates or synchronises, so calls can be captured into a
 *     HIP graph.  The first gate call on each device makes one host-side hipFuncSetAttribute call (it lifts
 *     the 64 KB limit on the LDS of the gate kernels; per device, thread-safe, MOE_ERR_DEVICE if the runtime
 *     refuses it): make one eager call per device before capturing.  The chunked calls with an aux_stream
 *     create and destroy n_chunks + 1 events per call (host cost of a few microseconds each).
 *   - Expert rows given by the caller (moe_expert_ffn_fwd/bwd, moe_layer_*_routed with a gate of the caller's):
 *     offsets must be non-decreasing with offsets[0] = 0, no expert may hold more than min(N, capacity) rows
 *     (capacity <= 0: N), and offsets[E] <= N*k.  The launch grids are sized from these bounds on the host;
 *     rows beyond them would silently stay uncomputed.
 *   - Diagnostics: with MOE_FORCE_PLAIN_GEMM=1 in the environment (read at every expert-FFN call) every
 *     expert product runs on the plain FMA kernel instead of the MFMA kernel; for A/B checks only.
 */
#ifndef MOE_MI355X_H
#define MOE_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = 1, /* NULL pointer, non-positive size, k > E, ... */
  MOE_ERR_UNSUPPORTED = 2, /* a dtype / activation / size this build has no kernel for */
  MOE_ERR_WORKSPACE = 3,   /* workspace or saved blob smaller than moe_workspace_bytes reports */
  MOE_ERR_DEVICE = 4       /* the HIP runtime refused a launch */
} moe_status_t;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype_t;

/* Expert FFN types (Sec. 3.1 "Expert"): the two-layer GPT FFN with an element-wise activation,
 * or the three-matrix Mixtral FFN (MOE_ACT_SWIGLU). */
typedef enum { MOE_ACT_RELU = 0, MOE_ACT_GELU_TANH = 1, MOE_ACT_SWIGLU = 2, MOE_ACT_GELU_ERF = 3 } moe_act_t;

/* Gate-weight functions of Sec. 2.1 (values of moe_config_t.renormalize). */
typedef enum {
  MOE_GATE_SOFTMAX_ALL = 0, MOE_GATE_SOFTMAX_TOPK = 1, MOE_GATE_SIGMOID = 2, MOE_GATE_EXPERT_CHOICE = 3
} moe_gate_t;

typedef struct moe_config {
  int32_t n_tokens;         /* N = B*L */
  int32_t d_model;          /* M */
  int32_t n_experts;        /* E, at most 256 */
  int32_t d_hidden;         /* H */
  int32_t top_k;            /* k, 1 <= k <= min(E, 8) */
  int32_t capacity;         /* T, rows per expert; <= 0 means nothing is dropped (the paper's f = *) */
  int32_t dtype;            /* moe_dtype_t of activations and weights */
  int32_t act;              /* moe_act_t */
  int32_t renormalize;      /* gate weights, moe_gate_t.  The k experts are always those of the k largest logits.
                               1: G = Softmax(KeepTopK(H, k)) as printed in Sec. 2.1;
                               0: softmax over all E, selected probabilities used as they are;
                               2: the sigmoid gate of Sec. 2.1 (BASE, StableMoE): weight sigma(H_i);
                               3: expert choice (Sec. 2.1), G = Softmax(KeepTopK(H^T, k)): every expert keeps the
                                  `capacity` tokens with its largest logits (ties: earlier token) and weighs them
                                  by the softmax over those logits.  A token has one slot per expert, so top_k
                                  must equal n_experts (hence E <= 8), slot j is expert j, and capacity > 0 is the
                                  number of tokens per expert.  See moe_route. */
  int32_t add_residual;     /* 1: y = x + MoE(x) (and dx += dy) */
  int32_t accumulate_wgrad; /* 0: expert weight gradients are overwritten; 1: added to */
} moe_config_t;

/* T := k*f*N/E (Sec. 2.1, ordering function), evaluated as ((k*f)*N)/E in double and rounded up.
 * Host function, no GPU work.  Returns -1 on non-positive arguments. */
int32_t moe_capacity(int32_t n_tokens, int32_t n_experts, int32_t top_k, double f);

/* Sizes in bytes of the scratch workspace every call below accepts (one size fits all calls
 * with this cfg) and of the `saved` blob moe_layer_fwd fills for moe_layer_bwd.  Host function. */
moe_status_t moe_workspace_bytes(const moe_config_t* cfg, size_t* workspace_bytes, size_t* saved_bytes);

/* Gate + capacity (Sec. 2.1 "Gating Function" and the capacity rule of the ordering function).
 *   logits[t,e] = sum_m x[t,m] * w_gate[m,e] + b_gate[e], returned as fp32.
 *                 fp32 inputs, more than 64 experts, expert choice: the sum is carried in fp64 and rounded once.
 *                 bf16 inputs, up to 64 experts: the (exact) products are summed on the matrix cores in fp32 chains
 *                 of 64 and the chains in fp64; such a logit lies within 2^-17 * |x[t,:]|_2 * |w_gate[:,e]|_2 of the
 *                 exact sum (in practice 1e-7 .. 1e-6 of the largest logit), and every logit that a top-k decision
 *                 depends on within that bound is recomputed as the fp64 sum.
 *   topk_idx[t,j] = expert with the j-th largest logit (ties: lower index), j = 0 is the largest; in both cases the
 *                 decision is the one the fp64 sums, rounded once to fp32, give
 *   probs = G(I): renormalize=1 -> softmax over the k kept logits, exactly 0 elsewhere;
 *                 renormalize=0 -> softmax over all E; renormalize=2 -> sigma(logits), all E
 *   topk_w[t,j] = probs[t, topk_idx[t,j]]
 *   pos[t,j]    = slot inside the expert: choices are served rank by rank (all j=0, then j=1, ...),
 *                 tokens in order inside a rank, while the expert has fewer than T rows; else -1
 *   count[e] = rows kept by expert e, offsets = exclusive prefix sum of count (offsets[E] = A)
 *   row_of[t,j] = offsets[e] + pos[t,j] or -1;  src_of_row[row] = t*k + j  (entries >= A: -1)
 * renormalize=3 (expert choice), k = E: topk_idx[t,j] = j; pos[t,j] = rank of token t among the tokens expert j
 *   kept, in token order, or -1; topk_w = probs = softmax over the kept logits of the expert's column, 0 elsewhere;
 *   count[e] = min(capacity, N) for every expert; row_of, offsets, src_of_row as above.
 * in : x [N,M] dtype, w_gate [M,E] dtype, b_gate [E] fp32 or NULL
 * out: logits [N,E] f32, probs [N,E] f32, topk_idx [N,k] i32, topk_w [N,k] f32, pos [N,k] i32,
 *      row_of [N,k] i32, count [E] i32, offsets [E+1] i32, src_of_row [N*k] i32
 * workspace: moe_workspace_bytes. */
moe_status_t moe_route(const moe_config_t* cfg, const void* x, const void* w_gate, const float* b_gate,
                       float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos,
                       int32_t* row_of, int32_t* count, int32_t* offsets, int32_t* src_of_row,
                       void* workspace, size_t workspace_bytes, void* stream);

/* moe_route for callers that cannot allocate device memory or carry a workspace around: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs, gates and errors as
 * moe_route, without the workspace: the scratch of the gate kernels lives in a device array of
 * MOE_ROUTE_STATIC_SCRATCH_BYTES that is part of the library (every GPU the library runs on holds it until the
 * process ends).  The call allocates and frees nothing; its first use on a device looks up the array's address
 * (hipGetSymbolAddress, host side) and, like moe_route, sets one kernel attribute.
 * Limit: 256-byte-rounded  8 * ceil(M/64)*64 * Ep  (Ep = E rounded up to 8, 16, 32 or a multiple of 64)
 *        + 4 * E * k * ceil(N/64)  + 4 * E  bytes must fit; all five benchmark shapes do (the largest, N = 32768,
 *        M = 2048, E = 64, k = 6, needs 1.8 MB).  Larger shapes: MOE_ERR_WORKSPACE, nothing launched.
 * All calls on one GPU share the one array, which keeps the last call's contents (nothing in it has to be
 * cleared between calls): two moe_route_static calls that overlap on one GPU (different streams, no ordering
 * between them) race and give undefined results; calls ordered on one stream are safe. */
#define MOE_ROUTE_STATIC_SCRATCH_BYTES (4u << 20)
moe_status_t moe_route_static(const moe_config_t* cfg, const void* x, const void* w_gate, const float* b_gate,
                              float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos,
                              int32_t* row_of, int32_t* count, int32_t* offsets, int32_t* src_of_row, void* stream);

/* Ordering function (Sec. 2.1): xe[row_of[t,j], :] = x[t, :] for every kept assignment.  The
 * compact expert-major buffer xe [A,M] is the paper's (E,T,M) layout without its padding rows:
 * expert e owns rows offsets[e] .. offsets[e+1]-1.  Pure copy, bit exact. */
moe_status_t moe_dispatch(const moe_config_t* cfg, const void* x, const int32_t* row_of, void* xe, void* stream);

/* Backward of the ordering function: dx[t,:] = sum over kept j of dxe[row_of[t,j], :]
 * (+ dy[t,:] when cfg->add_residual; dy may be NULL otherwise).  dx is overwritten. */
moe_status_t moe_dispatch_bwd(const moe_config_t* cfg, const void* dxe, const int32_t* row_of, const void* dy,
                              void* dx, void* stream);

/* Experts (Sec. 2.1 "Experts", Sec. 3.1 "Expert"): Q_e = e_e(rows of expert e) for every expert.
 *   two-layer: a1 = xe.W1_e, hh = act(a1), q = hh.W2_e
 *   Mixtral:   a1 = xe.W1_e, a3 = xe.W3_e, hh = silu(a1)*a3, q = hh.W2_e
 * in : xe [A,M], offsets [E+1], w1 [E,M,H], w3 [E,M,H] (NULL unless SWIGLU), w2 [E,H,M]
 * out: q [A,M]; stored activations for the backward pass (Sec. 4.4): a1 [A,H], a3 [A,H]
 *      (NULL unless SWIGLU), hh [A,H]; all dtype, all sized for N*k rows.
 * bf16 needs M and H to be multiples of 8 (16-byte rows). */
moe_status_t moe_expert_ffn_fwd(const moe_config_t* cfg, const void* xe, const int32_t* offsets, const void* w1,
                                const void* w3, const void* w2, void* q, void* a1, void* a3, void* hh,
                                void* workspace, size_t workspace_bytes, void* stream);

/* Backward of the experts (Sec. 4.4: gradients of input and of weights, twice the forward work).
 *   dhh = dq.W2_e^T, dW2_e = hh^T.dq, da1/da3 through the activation, dxe = da1.W1_e^T (+ da3.W3_e^T),
 *   dW1_e = xe^T.da1, dW3_e = xe^T.da3.  Experts with no rows get zero gradients (or are left
 *   unchanged when cfg->accumulate_wgrad).
 * out: dxe [A,M], dw1 [E,M,H], dw3 [E,M,H] (NULL unless SWIGLU), dw2 [E,H,M], all dtype. */
moe_status_t moe_expert_ffn_bwd(const moe_config_t* cfg, const void* dq, const void* xe, const int32_t* offsets,
                                const void* w1, const void* w3, const void* w2, const void* a1, const void* a3,
                                const void* hh, void* dxe, void* dw1, void* dw3, void* dw2, void* workspace,
                                size_t workspace_bytes, void* stream);

/* I-ordering function (Sec. 2.1): expert outputs go back to token order, scaled by the gate value:
 * y[t,:] = sum over kept j of topk_w[t,j] * q[row_of[t,j], :]  (+ x[t,:] when cfg->add_residual).
 * A token whose every choice was dropped gets 0 (or x[t,:]).  The sum is carried in fp32. */
moe_status_t moe_combine(const moe_config_t* cfg, const void* q, const float* topk_w, const int32_t* row_of,
                         const void* x, void* y, void* stream);

/* Backward of the I-ordering: dq[row_of[t,j], :] = topk_w[t,j] * dy[t, :] and
 * dtopk_w[t,j] = <dy[t,:], q[row_of[t,j],:]> (0 for dropped choices). */
moe_status_t moe_combine_bwd(const moe_config_t* cfg, const void* dy, const void* q, const float* topk_w,
                             const int32_t* row_of, void* dq, float* dtopk_w, void* stream);

/* Backward of the gate with the routing decision held fixed: g[t,e] = dtopk_w[t,j] where
 * e = topk_idx[t,j] and the choice was kept, else 0; dlogits = probs * (g - <g, probs>);
 * dw_gate = x^T.dlogits, db_gate = column sums of dlogits, dx += dlogits.W_g^T.
 * in : x [N,M], w_gate [M,E], probs [N,E] (as written by moe_route), topk_idx, pos, dtopk_w [N,k]
 * out: dw_gate [M,E] dtype, db_gate [E] f32 or NULL, dx [N,M] dtype ACCUMULATED INTO (read-modify-write).
 * workspace: moe_workspace_bytes. */
moe_status_t moe_route_bwd(const moe_config_t* cfg, const void* x, const void* w_gate, const float* probs,
                           const int32_t* topk_idx, const int32_t* pos, const float* dtopk_w, void* dw_gate,
                           float* db_gate, void* dx, void* workspace, size_t workspace_bytes, void* stream);

/* The whole layer forward: gate, ordering, experts, I-ordering in one call (Sec. 2.1, Fig. 1).
 * out: y [N,M]; `saved` (saved_bytes from moe_workspace_bytes) keeps the routing and the stored
 * activations for moe_layer_bwd. */
moe_status_t moe_layer_fwd(const moe_config_t* cfg, const void* x, const void* w_gate, const float* b_gate,
                           const void* w1, const void* w3, const void* w2, void* y, void* saved, size_t saved_bytes,
                           void* workspace, size_t workspace_bytes, void* stream);

/* The whole layer backward (Sec. 4.4) from the blob moe_layer_fwd left.
 * out: dx [N,M] (overwritten), dw_gate [M,E], db_gate [E] f32 or NULL, dw1, dw3 (NULL unless SWIGLU), dw2. */
moe_status_t moe_layer_bwd(const moe_config_t* cfg, const void* dy, const void* x, const void* w_gate,
                           const void* w1, const void* w3, const void* w2, const void* saved, size_t saved_bytes,
                           void* dx, void* dw_gate, float* db_gate, void* dw1, void* dw3, void* dw2,
                           void* workspace, size_t workspace_bytes, void* stream);

/* The layer in chunks (Sec. 4.2, Fig. 5: the capacity dimension of the dispatched tensor is cut into r
 * parts that move through dispatch -> experts one after the other so that the steps of neighbouring
 * parts can overlap).  Chunk c of n_chunks holds rows floor(c n / r) .. floor((c+1) n / r) - 1 of the
 * n rows of every expert.  The gate runs once over all tokens, the I-ordering once at the end.
 * Every output and every byte of `saved` is identical to moe_layer_fwd: rows are independent in the
 * ordering function and in the expert FFN, and no contraction is split.
 * n_chunks: 1 .. MOE_MAX_CHUNKS (1 = moe_layer_fwd).  aux_stream: NULL, or a second hipStream_t on which
 * the dispatch of chunk c+1 is enqueued while chunk c is in the expert FFN on `stream`; on return all work
 * of aux_stream is ordered before what the caller enqueues next on `stream` (the library records and
 * waits on events that it creates for the call and destroys before it returns).  Other arguments and
 * errors as moe_layer_fwd. */
#define MOE_MAX_CHUNKS 16
moe_status_t moe_layer_fwd_chunked(const moe_config_t* cfg, const void* x, const void* w_gate, const float* b_gate,
                                   const void* w1, const void* w3, const void* w2, void* y, void* saved,
                                   size_t saved_bytes, void* workspace, size_t workspace_bytes, int32_t n_chunks,
                                   void* stream, void* aux_stream);

/* Backward of the layer in chunks: the row-wise products (dq.W2^T with the activation derivative, and
 * da.W1^T) run chunk by chunk; the weight gradients contract over the rows of an expert and are computed
 * whole, after the last chunk, so that every output is identical to moe_layer_bwd.  Single stream.
 * `saved` may come from moe_layer_fwd or moe_layer_fwd_chunked with any n_chunks. */
moe_status_t moe_layer_bwd_chunked(const moe_config_t* cfg, const void* dy, const void* x, const void* w_gate,
                                   const void* w1, const void* w3, const void* w2, const void* saved, size_t saved_bytes,
                                   void* dx, void* dw_gate, float* db_gate, void* dw1, void* dw3, void* dw2,
                                   void* workspace, size_t workspace_bytes, int32_t n_chunks, void* stream);

/* The layer after the gate, for any gate (Sec. 3.1 keeps Gate, Order and Expert as separate sub-modules):
 * ordering, experts and I-ordering on a routing that is already in `saved`.  The caller first runs one of the
 * moe_route* calls (or a gate of its own) with the output pointers set to the routing tensors inside `saved`
 * (moe_saved_offset: LOGITS, PROBS, TOPK_IDX, TOPK_W, POS, ROW_OF, COUNT, OFFSETS, SRC_OF_ROW), on the same
 * stream.  n_chunks, aux_stream as moe_layer_fwd_chunked (n_chunks = 1: the plain layer).
 * out: y [N,M]; the activation tensors of `saved`. */
moe_status_t moe_layer_fwd_routed(const moe_config_t* cfg, const void* x, const void* w1, const void* w3,
                                  const void* w2, void* y, void* saved, size_t saved_bytes, void* workspace,
                                  size_t workspace_bytes, int32_t n_chunks, void* stream, void* aux_stream);

/* Backward of the same part, i.e. of everything but the gate.
 * out: dx [N,M] (OVERWRITTEN: the experts' share, plus dy with add_residual), dw1, dw3, dw2 as moe_layer_bwd,
 *      dtopk_w [N,k] f32: the gradient of the gate weights (0 for dropped choices).  The gate's own backward
 *      (moe_route_bwd, moe_route_noisy_bwd, moe_route_xmoe_bwd, ...) takes dtopk_w and adds its share to dx. */
moe_status_t moe_layer_bwd_routed(const moe_config_t* cfg, const void* dy, const void* w1, const void* w3,
                                  const void* w2, const void* saved, size_t saved_bytes, void* dx, void* dw1,
                                  void* dw3, void* dw2, float* dtopk_w, void* workspace, size_t workspace_bytes,
                                  int32_t n_chunks, void* stream);

/* Where inside `saved` a tensor lives (for inspection and tests).  Host function. */
typedef enum {
  MOE_SAVED_LOGITS = 0, MOE_SAVED_PROBS, MOE_SAVED_TOPK_IDX, MOE_SAVED_TOPK_W, MOE_SAVED_POS, MOE_SAVED_ROW_OF,
  MOE_SAVED_COUNT, MOE_SAVED_OFFSETS, MOE_SAVED_SRC_OF_ROW, MOE_SAVED_XE, MOE_SAVED_A1, MOE_SAVED_A3,
  MOE_SAVED_HH, MOE_SAVED_Q, MOE_SAVED_N_
} moe_saved_tensor_t;
moe_status_t moe_saved_offset(const moe_config_t* cfg, int32_t which, size_t* byte_offset, size_t* n_bytes);

/* The noisy gate of Sec. 2.1: H(I) = I.W_g (+ b_g) + noise * Softplus(I.W_noise), then everything moe_route
 * does with H in place of I.W_g.  The standard-normal draws are an input, so the call is a function of its
 * arguments.  Both products are accumulated in fp64 and rounded once to fp32; H is formed from the two fp32
 * tensors in fp64 and rounded once.
 * in : as moe_route, plus w_noise [M,E] dtype and noise [N,E] f32.
 * out: as moe_route (logits = H), plus noise_logits [N,E] f32 = I.W_noise (moe_route_noisy_bwd needs it). */
moe_status_t moe_route_noisy(const moe_config_t* cfg, const void* x, const void* w_gate, const float* b_gate,
                             const void* w_noise, const float* noise, float* logits, float* noise_logits, float* probs,
                             int32_t* topk_idx, float* topk_w, int32_t* pos, int32_t* row_of, int32_t* count,
                             int32_t* offsets, int32_t* src_of_row, void* workspace, size_t workspace_bytes, void* stream);

/* Backward of the noisy gate, routing decision and noise draws held fixed: with dH = dlogits as in
 * moe_route_bwd, dw_gate = x^T.dH, db_gate = column sums of dH, and for the noise product
 * dN = dH * noise * sigma(noise_logits): dw_noise = x^T.dN; dx += dH.W_g^T + dN.W_noise^T (ACCUMULATED INTO).
 * out: dw_gate, dw_noise [M,E] dtype, db_gate [E] f32 or NULL. */
moe_status_t moe_route_noisy_bwd(const moe_config_t* cfg, const void* x, const void* w_gate, const void* w_noise,
                                 const float* noise, const float* noise_logits, const float* probs,
                                 const int32_t* topk_idx, const int32_t* pos, const float* dtopk_w, void* dw_gate,
                                 float* db_gate, void* dw_noise, void* dx, void* workspace, size_t workspace_bytes,
                                 void* stream);

/* The X-MoE gate of Sec. 2.1: s_i = cos(W_proj I, W_g[:, i]).  The token is projected to d_proj dimensions,
 * projection and expert embeddings are scaled to unit l2 length, and the cosine scores take the place of I.W_g
 * in everything moe_route does (top-k, gate-weight function cfg->renormalize, capacity positions).
 * The projection is accumulated in fp64 and rounded once to fp32; the scores are formed from it in fp64 and
 * rounded once to fp32.  No temperature and no epsilon: a token whose projection is exactly zero gets NaN
 * scores (its choices are then valid expert indices, but not meaningful).
 * in : x [N,M] dtype; w_proj [M,d_proj] dtype (applied as x.W_proj); w_gate [d_proj,E] dtype, one expert
 *      embedding per column; d_proj a multiple of 4, at most 256.
 * out: proj [N,d_proj] f32 = x.W_proj (moe_route_xmoe_bwd needs it); logits [N,E] f32 = the scores; the rest
 *      as moe_route.  All device pointers.
 * workspace: moe_route_xmoe_workspace_bytes (device memory; MOE_ERR_WORKSPACE if smaller). */
moe_status_t moe_route_xmoe_workspace_bytes(const moe_config_t* cfg, int32_t d_proj, size_t* ws_bytes);
moe_status_t moe_route_xmoe(const moe_config_t* cfg, const void* x, const void* w_proj, const void* w_gate,
                            int32_t d_proj, float* proj, float* logits, float* probs, int32_t* topk_idx, float* topk_w,
                            int32_t* pos, int32_t* row_of, int32_t* count, int32_t* offsets, int32_t* src_of_row,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Backward of the X-MoE gate, routing decision held fixed.  With ds = dlogits as in moe_route_bwd, pn and wn
 * the unit-length projection rows and embedding columns: d(pn) = ds.wn^T, d(wn) = pn^T.ds; a unit scaling
 * u = v / |v| has the adjoint dv = (du - u <u, du>) / |v|; then dw_proj = x^T.dp and dx += dp.W_proj^T
 * (ACCUMULATED INTO dx).  The two small steps run in fp64/fp32; the products with x as in moe_route_bwd.
 * out: dw_proj [M,d_proj] dtype, dw_gate [d_proj,E] dtype. */
moe_status_t moe_route_xmoe_bwd(const moe_config_t* cfg, const void* x, const void* w_proj, const void* w_gate,
                                int32_t d_proj, const float* proj, const float* probs, const int32_t* topk_idx,
                                const int32_t* pos, const float* dtopk_w, void* dw_proj, void* dw_gate, void* dx,
                                void* workspace, size_t workspace_bytes, void* stream);

/* ---- pipeline degree (Sec. 4): host functions, no GPU work ------------------------------------------
 * Linear performance models of Sec. 4.1, Eq. (1): one of r chunks of AlltoAll (dispatch or combine),
 * ESP-AllGather, ESP-ReduceScatter and expert computation takes alpha + (n / r) * beta; n is the message
 * size or the amount of computation of the whole layer, alpha the start-up time.  t_gar: time of the
 * Gradient-AllReduce to hide behind the layer (0 in the forward phase, Sec. 4.4).  All >= 0, any one unit
 * of time.  On one GPU the three communication models are zero; alpha_exp, beta_exp come from timing the
 * expert FFN at several chunk sizes (bench.py --fit-expert-model). */
typedef struct moe_pipeline_model {
  double alpha_a2a, beta_a2a, n_a2a;
  double alpha_ag, beta_ag, n_ag;
  double alpha_rs, beta_rs, n_rs;
  double alpha_exp, beta_exp, n_exp;
  double t_gar;
} moe_pipeline_model_t;

/* Time of the MoE layer at pipeline degree r >= 1 (Sec. 4.2): the conditions Q1..Q7 decide which of the
 * four cases r falls into (every r falls into exactly one), the result is that case's closed form
 * t^moe_1..4.  *which_case (may be NULL) receives 1..4.  NaN for an invalid model or r < 1. */
double moe_pipeline_time(const moe_pipeline_model_t* model, double r, int32_t* which_case);

/* Algorithm 1 (FindOptimalPipelineDegree) over the integer degrees 1..r_max: for each case the minimum
 * of its closed form over the degrees that satisfy the case's condition, then the smallest of the four
 * minima; ties go to the smaller degree.  Enumeration replaces the paper's SLSQP solves on a real r.
 * out: *r; *t_moe and *which_case may be NULL.  MOE_ERR_INVALID_ARG for an invalid model or r_max < 1. */
moe_status_t moe_find_pipeline_degree(const moe_pipeline_model_t* model, int32_t r_max, int32_t* r, double* t_moe,
                                      int32_t* which_case);

/* Message of the last failed call on this host thread ("" if none).  Static storage. */
const char* moe_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MOE_MI355X_H */
