/* armt.h -- C ABI of the MI355X (gfx950) ARMT forward library.
 *
 * The library computes the forward pass of an Associative Recurrent Memory Transformer
 * (paper Section 2.1, Eq. 2-6) over one long input, either cell by cell in the order the
 * model is defined (Section 3.1: for each segment, for each layer) or with Diagonal
 * Batching (Section 3.2, Algorithm 1, Lemma 3.1): all (layer, segment) cells of one
 * anti-diagonal run together as one group.  Both produce the same result; only the
 * order of independent cells differs.
 *
 * Conventions, valid for every call unless stated otherwise:
 *   - every pointer is a DEVICE pointer unless marked [host];
 *   - the caller owns all memory; the library allocates and frees no device memory;
 *     scratch space comes in through `workspace` (armt_lm_head_static alone uses a fixed
 *     array inside the library instead);
 *   - no call keeps state for a later call.  Excluded from this, and NOT thread safe: the
 *     process-wide benchmarking and debugging knobs at the end of this header
 *     (armt_set_gemm_tile_config, armt_profile_begin / armt_profile_end, the environment
 *     variable ARMT_DEBUG_GENERIC), which change kernel selection or event recording for every
 *     later call of the process on any stream.  Leave them alone and the calls are re-entrant;
 *   - work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and the call returns without waiting for the GPU or for earlier work on the
 *     stream: the small host tables a call builds (per-layer operand pointers) travel as kernel
 *     arguments, not as copies, so nothing synchronises and the host arrays passed in
 *     (`layers`, `grads`, pointer lists) may be freed as soon as the call returns;
 *   - errors are return codes; argument errors are detected before anything is launched
 *     and leave all outputs untouched;
 *   - matrices are row-major; a weight W is [out_features, in_features] and is applied as
 *     y = x W^T; there are no biases;
 *   - the memory state A, z is always fp32, whatever the activation type.
 */
#ifndef ARMT_H_
#define ARMT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ARMT_OK = 0,
  ARMT_ERR_NULL = 1,        /* a required pointer is NULL */
  ARMT_ERR_SHAPE = 2,       /* sizes inconsistent (n_tokens not a multiple of seg_len, heads, ...) */
  ARMT_ERR_DTYPE = 3,       /* dtype is not one of armt_dtype */
  ARMT_ERR_WORKSPACE = 4,   /* workspace missing, misaligned (256 B) or smaller than armt_workspace_bytes */
  ARMT_ERR_HIP = 5,         /* a HIP runtime call failed; see armt_last_hip_error */
  ARMT_ERR_UNSUPPORTED = 6, /* valid ARMT shape this build has no kernel for (see armt_config) */
  ARMT_ERR_TOO_LARGE = 7    /* input needs more scratch than the fixed array of a *_static call holds */
} armt_status;

typedef enum { ARMT_F32 = 0, ARMT_BF16 = 1 } armt_dtype;   /* type of weights, embeddings, hidden_out */

/* Model and segmentation sizes.  Notation of the paper: L layers, segments of seg_len tokens
 * followed by n_mem memory tokens (a cell has T = seg_len + n_mem rows, Eq. 2 "[H, M]"),
 * associative hidden size d_mem, feature map DPFP-nu of width Phi = 2 * dpfp_nu * d_mem
 * (Section 2.1: A in R^{d_model x 6 d_mem} for nu = 3).
 * Valid (else ARMT_ERR_SHAPE): all sizes >= 1, n_heads * head_dim == d_model, n_heads % n_kv_heads == 0,
 * head_dim even, 1 <= dpfp_nu < 2 * d_mem.  Of the valid shapes this build has kernels for (else
 * ARMT_ERR_UNSUPPORTED): Phi <= 512; dtype BF16 additionally needs d_model, d_ff and Phi multiples of 64, d_mem a
 * multiple of 8, n_mem a multiple of 16, head_dim 64 or 128 and at most 8 query heads per KV head. */
typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ff;
  int32_t seg_len, n_mem, d_mem, dpfp_nu;
  int32_t dtype;             /* armt_dtype */
  float rms_eps;             /* RMSNorm epsilon (LLaMA-3: 1e-5) */
  float rope_theta;          /* rotary base (LLaMA-3: 500000); positions restart at 0 in every cell */
  float assoc_eps;           /* added to the denominators z.phi and |phi|^2 of Eq. 4 and 6; 0 = as printed */
} armt_config;

/* Weights of one layer: the decoder block (TransformerLayer of Eq. 2; LLaMA-3: pre-norm RMSNorm,
 * grouped-query attention with rotate-half RoPE, SwiGLU) and the associative block (Eq. 3-6).
 * All of type cfg.dtype.  A [host] array of n_layers of these is the "per-group weight pointers"
 * of the grouped layer (Section 3.3): the weights are never copied or stacked. */
typedef struct {
  const void *rms1;                 /* [d_model]                      gain of the first norm   */
  const void *wq, *wk, *wv;         /* [H*dh, d] [Hkv*dh, d] [Hkv*dh, d]                        */
  const void *wo;                   /* [d, H*dh]                                                */
  const void *rms2;                 /* [d_model]                      gain of the second norm  */
  const void *wgate, *wup;          /* [d_ff, d] [d_ff, d]                                      */
  const void *wdown;                /* [d, d_ff]                                                */
  const void *wm_q, *wm_k;          /* [d_mem, d] [d_mem, d]          W_Q (Eq. 6), W_K (Eq. 3) */
  const void *wm_v;                 /* [d, d]                         W_V (Eq. 3)              */
  const void *wm_b;                 /* [1, d]                         W_beta (Eq. 3)           */
} armt_layer_weights;

/* Bytes of scratch space armt_forward_* needs for this configuration; 0 if cfg is invalid.  The size depends on
 * neither n_tokens nor the execution order (one slot of every intermediate per layer: a step of the diagonal order
 * has at most n_layers live cells, the sequential order uses the same slots one at a time), which is why this query
 * takes the configuration only.  The workspace must be 256-byte aligned.  Its contents need not be initialised and
 * are undefined afterwards. */
size_t armt_workspace_bytes(const armt_config *cfg /* [host] */);

/* Forward pass, cells visited segment by segment, layer by layer (Section 3.1; Fig. 3a):
 * n_segments * n_layers dependent cell executions, every kernel launched for one cell.
 *
 *   layers      [host] array of cfg->n_layers armt_layer_weights (device pointers inside)
 *   mem_emb     [n_mem, d_model]  memory-token embeddings appended to every segment at layer 0
 *   x           [n_tokens, d_model] token embeddings; n_tokens must be a positive multiple of seg_len
 *   A_in, z_in  [L, d_model, Phi], [L, Phi] fp32 memory state to start from, or both NULL for the
 *               empty memory A_0 = z_0 = 0 (Eq. 3).  With an empty memory the first segment skips
 *               the associative read and uses v_bar = 0 (Algorithm 1 applies Associate only from
 *               the second group on).
 *   hidden_out  [n_tokens, d_model] of cfg.dtype: output of the last layer at the seg_len token rows
 *               of every segment (no final norm, no LM head)
 *   A_out,z_out [L, d_model, Phi], [L, Phi] fp32 memory state after the last segment; may alias
 *               A_in, z_in (state is updated in place in A_out, z_out).
 */
armt_status armt_forward_sequential(const armt_config *cfg, const armt_layer_weights *layers,
                                    const void *mem_emb, const void *x, int64_t n_tokens,
                                    const float *A_in, const float *z_in,
                                    void *hidden_out, float *A_out, float *z_out,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/* Forward pass with Diagonal Batching (Algorithm 1): step t = 0 .. L + N - 2 runs every cell
 * (layer l, segment t - l) with max(0, t - N + 1) <= l <= min(L - 1, t) in one group (Lemma 3.1):
 * grouped GEMMs with one weight set per cell, attention batched over the cells, and the memory
 * read / update of every live layer.  Same arguments and same result as armt_forward_sequential. */
armt_status armt_forward_diagonal(const armt_config *cfg, const armt_layer_weights *layers,
                                  const void *mem_emb, const void *x, int64_t n_tokens,
                                  const float *A_in, const float *z_in,
                                  void *hidden_out, float *A_out, float *z_out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

/* Choice between the two orders (the paper's appendix notes that one can fall back to the original order at run time
 * where Diagonal Batching does not pay off; its timing tables have such entries at 4096 - 8192 tokens).
 * armt_auto_order returns 1 (diagonal) or 0 (sequential) for a configuration and length, -1 if they are invalid.
 * Rule: diagonal from two segments and two layers on, else sequential.  With one segment (or one layer) every
 * anti-diagonal holds a single cell and both orders launch the same kernels; from two segments on a diagonal step
 * runs the kernels of the sequential order on larger launches and was never slower in any measured case, the
 * 4096-token column of the paper's tables included (table in the design notes).
 * armt_forward_auto runs the order armt_auto_order picks (arguments and result as armt_forward_sequential) and
 * reports it in *order_used ([host], may be NULL). */
int32_t armt_auto_order(const armt_config *cfg, int64_t n_tokens);
armt_status armt_forward_auto(const armt_config *cfg, const armt_layer_weights *layers,
                              const void *mem_emb, const void *x, int64_t n_tokens,
                              const float *A_in, const float *z_in,
                              void *hidden_out, float *A_out, float *z_out,
                              void *workspace, size_t workspace_bytes, void *hip_stream, int32_t *order_used);

/* The hybrid of the two orders: Diagonal Batching in which a group of at most split_upto cells (the small groups at
 * both ends of the schedule) is launched cell by cell instead of as one group.  split_upto = 0 is
 * armt_forward_diagonal; split_upto >= n_layers launches every cell on its own, in anti-diagonal order.  Same result
 * bit for bit.  Measured slower than the plain diagonal order for every split_upto >= 1 (a group launch is never
 * slower than its cells one after the other here); exported so that the comparison can be repeated. */
armt_status armt_forward_diagonal_split(const armt_config *cfg, const armt_layer_weights *layers,
                                        const void *mem_emb, const void *x, int64_t n_tokens,
                                        const float *A_in, const float *z_in,
                                        void *hidden_out, float *A_out, float *z_out,
                                        void *workspace, size_t workspace_bytes, void *hip_stream, int32_t split_upto);

/* Batch of B independent sequences of the same length (the paper's batched setting, Section 4.3): step t
 * runs the cells (layer l, segment t - l) of all B sequences as one group of up to B * n_layers cells; the B
 * cells of a layer share its weights.  The sequential variant runs, per (segment, layer), the B cells of that
 * layer as one group: ordinary batching, the baseline of the paper's batch-size comparison.
 * x, hidden_out: [B][n_tokens][d_model]; A_in, A_out: [B][n_layers][d_model][Phi]; z_in, z_out: [B][n_layers][Phi];
 * workspace: armt_workspace_bytes_batched(cfg, B) bytes (0 = configuration or batch rejected; B * n_layers
 * must not exceed 32768).  Everything else as in the calls above, which are the case B = 1; sequence b of a
 * batched call gets bit for bit the result of a call on sequence b alone. */
size_t armt_workspace_bytes_batched(const armt_config *cfg, int32_t batch);
armt_status armt_forward_sequential_batched(const armt_config *cfg, const armt_layer_weights *layers,
                                            const void *mem_emb, const void *x, int32_t batch, int64_t n_tokens,
                                            const float *A_in, const float *z_in,
                                            void *hidden_out, float *A_out, float *z_out,
                                            void *workspace, size_t workspace_bytes, void *hip_stream);
armt_status armt_forward_diagonal_batched(const armt_config *cfg, const armt_layer_weights *layers,
                                          const void *mem_emb, const void *x, int32_t batch, int64_t n_tokens,
                                          const float *A_in, const float *z_in,
                                          void *hidden_out, float *A_out, float *z_out,
                                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---- training: forward with a tape, and the backward pass (the paper's appendix on implementation notes states that
 * a backward pass of the diagonal schedule exists; it computes the gradient of the forward of Section 2.1, Eq. 2-6).
 *
 * armt_forward_train is armt_forward_diagonal (diagonal != 0) or armt_forward_sequential (diagonal == 0) for one
 * sequence, and in addition records in `tape`, per (segment, layer) cell, the cell's input [T][d_model] and the layer's
 * A, z from before the cell's update (fp32; armt_tape_bytes(cfg, n_tokens) bytes, 256-byte aligned, device memory
 * owned by the caller; 0 = configuration rejected).  Same results as the inference calls.
 * Tape layout (one sequence): record (s, l) starts at float ((s * n_layers + l) * R), R = T * d_model + d_model * Phi + Phi
 * rounded up to a multiple of 64, and holds the cell input [T][d_model], then A^l [d_model][Phi], then z^l [Phi]; a caller
 * may fill a tape itself (from another forward implementation, or a checkpoint) and hand it to armt_backward.
 *
 * armt_backward consumes the tape: for J = <hidden_out, d_hidden> + <A_out, dA_out> + <z_out, dz_out> it ADDS dJ/dW to
 * the caller's fp32 gradient buffers (`grads[l]` mirrors `layers[l]`: one device pointer per weight, same shapes; the
 * caller zeroes them, or keeps accumulating over calls), ADDS the gradient of the memory-token embeddings to d_mem_emb
 * [n_mem][d_model], and writes (not adds) dx [n_tokens][d_model] (may be NULL), dA_in [L][d_model][Phi] and dz_in
 * [L][Phi] (both or neither NULL).  All gradients are fp32; d_hidden [n_tokens][d_model] has the activation type;
 * dA_out, dz_out may both be NULL (= zero).  carry_in != 0 iff the forward call was given A_in, z_in (otherwise the
 * cells of segment 0 met an empty memory, and dA_in, dz_in are meaningless).  The cells are visited in the reverse of
 * the diagonal order (diagonal != 0: one group per anti-diagonal, grouped GEMMs as in the forward pass) or of the
 * sequential order; each step restores the inputs of its cells from the tape, recomputes their forward and runs the
 * backward kernels, so no activation other than the tape outlives a step.  `layers` must be the weights of the
 * forward call.  workspace: armt_backward_workspace_bytes(cfg) bytes, 256-byte aligned.
 * Supported here: head_dim <= 128 and the limits of the forward calls; anything else is rejected with
 * ARMT_ERR_UNSUPPORTED (the size queries return 0).  Two cells of one layer never run in the same step, so the
 * accumulation into a layer's gradient buffers has a fixed order and the result is deterministic. */
typedef struct {
  float *rms1, *wq, *wk, *wv, *wo;
  float *rms2, *wgate, *wup, *wdown;
  float *wm_q, *wm_k, *wm_v, *wm_b;
} armt_layer_grads;
size_t armt_tape_bytes(const armt_config *cfg, int64_t n_tokens);
size_t armt_backward_workspace_bytes(const armt_config *cfg);
armt_status armt_forward_train(const armt_config *cfg, const armt_layer_weights *layers,
                               const void *mem_emb, const void *x, int64_t n_tokens,
                               const float *A_in, const float *z_in,
                               void *hidden_out, float *A_out, float *z_out,
                               void *tape, size_t tape_bytes,
                               void *workspace, size_t workspace_bytes, void *hip_stream, int32_t diagonal);
armt_status armt_backward(const armt_config *cfg, const armt_layer_weights *layers, int64_t n_tokens,
                          const void *tape, size_t tape_bytes, int32_t carry_in,
                          const void *d_hidden, const float *dA_out, const float *dz_out,
                          const armt_layer_grads *grads /* [host] array of n_layers */,
                          float *d_mem_emb, float *dx, float *dA_in, float *dz_in,
                          void *workspace, size_t workspace_bytes, void *hip_stream, int32_t diagonal);

/* The training calls for a batch of B sequences of equal length (x, hidden_out, d_hidden, dx: [B][n_tokens][d_model];
 * A_in, A_out, dA_out, dA_in: [B][n_layers][d_model][Phi]; z likewise): the cells of a step are those of the batched
 * forward calls; the B cells of a layer put their operands side by side in the reduction dimension of the layer's
 * weight-gradient GEMMs, so the gradients of the shared weights (and of mem_emb) are the sums over the sequences, added in
 * a fixed order.  The calls above are the case B = 1.  B * n_layers must not exceed 32768. */
size_t armt_tape_bytes_batched(const armt_config *cfg, int32_t batch, int64_t n_tokens);
size_t armt_backward_workspace_bytes_batched(const armt_config *cfg, int32_t batch);
armt_status armt_forward_train_batched(const armt_config *cfg, const armt_layer_weights *layers,
                                       const void *mem_emb, const void *x, int32_t batch, int64_t n_tokens,
                                       const float *A_in, const float *z_in,
                                       void *hidden_out, float *A_out, float *z_out,
                                       void *tape, size_t tape_bytes,
                                       void *workspace, size_t workspace_bytes, void *hip_stream, int32_t diagonal);
armt_status armt_backward_batched(const armt_config *cfg, const armt_layer_weights *layers, int32_t batch, int64_t n_tokens,
                                  const void *tape, size_t tape_bytes, int32_t carry_in,
                                  const void *d_hidden, const float *dA_out, const float *dz_out,
                                  const armt_layer_grads *grads /* [host] array of n_layers */,
                                  float *d_mem_emb, float *dx, float *dA_in, float *dz_in,
                                  void *workspace, size_t workspace_bytes, void *hip_stream, int32_t diagonal);

/* Backward of the token-level ends (Algorithm 1 ends in logits; a training step differentiates a loss on them).
 * armt_lm_head_backward: for logits = rmsnorm(hidden; final_gain, rms_eps) W_lm^T and an upstream gradient d_logits
 * [n_rows][vocab] fp32, WRITES d_hidden [n_rows][d_model] fp32 and ADDS to d_final_gain [d_model] and d_w_lm
 * [vocab][d_model] (fp32; the caller zeroes them or keeps accumulating).  hidden, final_gain, w_lm as in armt_lm_head.
 * The rows are taken 8192 at a time (the weight gradient is read and written once per pass).  workspace:
 * armt_lm_head_backward_workspace_bytes(cfg, n_rows, vocab) bytes, 256-byte aligned (0 = rejected).
 * armt_embed_tokens_backward: d_emb_table[ids[i]][:] += dx[i][:] (fp32, [vocab][d_model]); ids outside the vocabulary
 * are clamped as in the forward gather; rows that share an id are added with atomics in an unspecified order. */
size_t armt_lm_head_backward_workspace_bytes(const armt_config *cfg, int64_t n_rows, int32_t vocab);
armt_status armt_lm_head_backward(const armt_config *cfg, const void *hidden, int64_t n_rows, const void *final_gain,
                                  const void *w_lm, int32_t vocab, const float *d_logits,
                                  float *d_hidden, float *d_final_gain, float *d_w_lm,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);
armt_status armt_embed_tokens_backward(const armt_config *cfg, const float *dx, const int32_t *ids /* device */,
                                       int64_t n_tokens, int32_t vocab, float *d_emb_table, void *hip_stream);

/* Anti-diagonal schedule (Lemma 3.1), host only: for step t of an L-layer model over N segments,
 * *l_lo .. *l_hi (inclusive) are the live layers; layer l runs segment t - l.  Returns the group
 * size, or 0 (and leaves the outputs alone) if t is outside 0 .. L + N - 2 or L, N < 1. */
int32_t armt_diagonal_group(int32_t n_layers, int32_t n_segments, int32_t t,
                            int32_t *l_lo /* [host] */, int32_t *l_hi /* [host] */);

/* ---- single steps of the path, exactly as the forward calls run them (for tests and micro-benchmarks).
 * Each works on a group of g cells, like one step of Algorithm 1 does.  Those that take a cfg use its
 * sizes (T = seg_len + n_mem rows per cell), need 1 <= g <= cfg->n_layers, and accept the same workspace
 * as the forward calls (armt_workspace_bytes(cfg) bytes, 256-byte aligned). ---- */

/* Grouped GEMM (Section 3.3 item 1, Section 4.1): C_i = A_i B_i^T for i < g, every group with its own
 * operand pointers.  a, b, c are [host] arrays of g device pointers: A_i [M, K], B_i [N, K] (a weight,
 * [out, in]) and C_i [M, N], all of type dtype (fp32 accumulation).  dtype BF16 needs K % 64 == 0.
 * workspace: g * 128 bytes, 256-byte aligned (holds the pointer table). */
armt_status armt_grouped_gemm(int32_t dtype, int32_t g, int32_t M, int32_t N, int32_t K,
                              const void *const *a, const void *const *b, void *const *c,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* Segment attention batched over the group (Section 4.2): rotary embedding of q and k (positions
 * 0..T-1), then causal softmax(q k^T / sqrt(dh)) v over the T rows of each cell with grouped-query
 * heads.  qkv [g, T, (H + 2 Hkv) * dh] of cfg->dtype, each row laid out [q heads | k heads | v heads],
 * is rotated in place; out [g, T, H * dh] of cfg->dtype. */
armt_status armt_segment_attention(const armt_config *cfg, int32_t g, void *qkv, void *out,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/* Associative read of a group (Eq. 6, added to its input): for every cell i and row r,
 * x[i][r] += A_i phi(Wq_i x[i][r]) / (z_i . phi(Wq_i x[i][r]) + assoc_eps).
 * x [g, T, d] fp32, updated in place; wm_q: [host] array of g device pointers to [d_mem, d] of
 * cfg->dtype; A [g, d, Phi], z [g, Phi] fp32 (read only). */
armt_status armt_assoc_read(const armt_config *cfg, int32_t g, float *x, const void *const *wm_q,
                            const float *A, const float *z, void *workspace, size_t workspace_bytes,
                            void *hip_stream);

/* Delta-rule memory update of a group (Eq. 3-5): for every cell i, from its n_mem memory-token outputs
 * ym [g, n_mem, d] fp32: k = Wk ym, v = Wv ym, beta = sigmoid(Wb ym), v_bar = A phi(k) / (z.phi(k) + eps)
 * (0 for the cell empty_group, whose memory is still empty; -1 = none), gamma = 1 - z.phi(k) / (|phi(k)|^2
 * + eps); then A_i += sum_j beta_j (v_j - v_bar_j) (x) phi(k_j), z_i += sum_j gamma_j phi(k_j), every j
 * using the state from before the update.  wm_k, wm_v, wm_b: [host] arrays of g device pointers
 * (cfg->dtype); A [g, d, Phi], z [g, Phi] fp32, updated in place. */
armt_status armt_assoc_update(const armt_config *cfg, int32_t g, const float *ym,
                              const void *const *wm_k, const void *const *wm_v, const void *const *wm_b,
                              int32_t empty_group, float *A, float *z,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---- token-level ends of Algorithm 1 (token ids in, logits out), to be called around a forward call. ---- */

/* Embedding gather: x_out[i] = emb_table[ids[i]] for i < n_tokens.  emb_table [vocab, d_model] and x_out
 * [n_tokens, d_model] of cfg->dtype, ids [n_tokens] int32 (device).  Ids must lie in [0, vocab); the kernel
 * clamps them into that range instead of reading outside the table.  No workspace. */
armt_status armt_embed_tokens(const armt_config *cfg, const void *emb_table, int32_t vocab,
                              const int32_t *ids, int64_t n_tokens, void *x_out, void *hip_stream);

/* Final RMSNorm + linear head (Algorithm 1 returns logits): logits = rmsnorm(hidden; final_gain, cfg->rms_eps)
 * w_lm^T.  hidden [n_rows, d_model] of cfg->dtype (e.g. hidden_out of a forward call, or its last rows),
 * final_gain [d_model] and w_lm [vocab, d_model] of cfg->dtype (w_lm may be the embedding table), logits
 * [n_rows, vocab] fp32.  workspace: armt_lm_head_workspace_bytes(cfg, n_rows) bytes, 256-byte aligned
 * (normalised operand, row scales, pointer table).  Returns ARMT_ERR_SHAPE for n_rows < 1 or vocab < 1. */
size_t armt_lm_head_workspace_bytes(const armt_config *cfg, int64_t n_rows);
armt_status armt_lm_head(const armt_config *cfg, const void *hidden, int64_t n_rows, const void *final_gain,
                         const void *w_lm, int32_t vocab, float *logits,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* armt_lm_head for callers that cannot allocate or carry a workspace: code under HIP graph capture, tight serving
 * loops that turn the last rows of a forward call into logits, harnesses that forbid hipMalloc.  Same arguments,
 * kernels and result (bit for bit) as armt_lm_head, but the scratch memory (normalised operand rows, row scales,
 * pointer table) is a fixed array of ARMT_LM_HEAD_STATIC_BYTES bytes inside the library, of which every GPU the
 * library runs on holds one copy until the process ends.  The call allocates nothing, on the device or on the host
 * heap.  Limit: armt_lm_head_workspace_bytes(cfg, n_rows) <= ARMT_LM_HEAD_STATIC_BYTES and n_rows < 64512 (for
 * example 2047 rows at d_model 2048 in bf16, 1023 rows at d_model 4096); anything larger returns ARMT_ERR_TOO_LARGE
 * before anything is launched.  All calls on one GPU share that GPU's array, which keeps the contents of the last
 * call (nothing in it has to be cleared: every byte a call reads it has written first): two calls whose kernels
 * overlap on one GPU (different streams, or threads) race; calls on one stream are safe. */
#define ARMT_LM_HEAD_STATIC_BYTES ((size_t)8454144)        /* 8 MiB + 64 KiB */
armt_status armt_lm_head_static(const armt_config *cfg, const void *hidden, int64_t n_rows, const void *final_gain,
                                const void *w_lm, int32_t vocab, float *logits, void *hip_stream);

/* Environment: ARMT_DEBUG_GENERIC=1 (read once per process) makes bf16 configurations run the plain
 * fp32-FMA GPU kernels of the fp32 path on bf16 operands instead of the MFMA kernels: slow, for telling an
 * error of a fast kernel from an error of the method.  Nothing ever runs on the host. */

/* ---- process-wide benchmarking and debugging knobs (not part of the re-entrant contract above, not thread safe) ---- */

/* Force the tile configuration of the bf16 grouped GEMM for all later calls of this process (1: 128x128 tile, 4 waves;
 * 2: 64x128, 4 waves; 3: 64x64, 4 waves, for the plain fp32 store only, and 4: 32x128, 4 waves, for the feature-map
 * epilogue of the W_Q projection only (other epilogues run 2 instead);
 * 5: 256x256, 16 waves; 6: as 1; 5 and 6 address the tile copies by scalar base + lane offset
 * where the shape allows; anything else below 100: choose by shape and tile count, the default).  config = 100 *
 * switches + tile configuration (or + 99 for the default choice) additionally turns fusions off, for A/B timing:
 * switch 16 the feature map of the read in the epilogue of the W_Q projection, 32 the strip of memory rows in the last
 * M-tile, 64 the transposed V written by the QKV epilogue, 128 the rotary embedding in the QKV epilogue (plain kernels
 * run instead).  Results do not depend on any of this beyond
 * rounding order.  Returns the previous tile configuration. */
int32_t armt_set_gemm_tile_config(int32_t config);

/* Kernel timing for benchmarks: between armt_profile_begin and armt_profile_end every launch of one
 * kernel kind of the step (up to max_launches of them) made by this process is bracketed by a pair of
 * HIP events on the launch stream.  gemm_kind: 0 W_Q projection of the read, 1 read A phi, 2 QKV,
 * 3 attention output, 4 gate/up with SwiGLU, 5 down, 6 W_K / W_V projections of the update (the grouped GEMMs);
 * 7 feature map + denominator of the read, 8 feature map + coefficients of the update, 9 the delta rule's pass over A,
 * 10 segment attention.
 * armt_profile_end waits for the recorded events and returns the summed kernel time in milliseconds,
 * the number of launches timed and the number of groups (cells) they covered; any pointer may be NULL.
 * Not thread safe; the events are created in begin and destroyed in end. */
armt_status armt_profile_begin(int32_t gemm_kind, int32_t max_launches);
armt_status armt_profile_end(double *total_ms /* [host] */, int64_t *launches /* [host] */,
                             int64_t *groups /* [host] */);

/* Text for a status code (static string). */
const char *armt_status_str(armt_status s);

/* Text of the HIP error behind the last ARMT_ERR_HIP returned on the calling thread ("" if none). */
const char *armt_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ARMT_H_ */
