/*
 * tide_draft.h -- C ABI of the TIDE online draft-training step for AMD MI355X (gfx950).
 *
 * The operation.  TIDE keeps a speculative-decoding draft model aligned with a
 * served target model by fine-tuning the draft on hidden states that the target
 * already produced while serving, instead of running the target a second time
 * (paper Sec. 3.3, "Online Draft Model Adaptation").  The draft is one decoder
 * layer plus an LM head that reads the concatenation of the target's hidden
 * states at a low, a middle and a high layer (Sec. 3.2, "Serving-Time Training
 * Signal Extraction") and predicts, over the target's own vocabulary (Sec. 5.1,
 * "Draft Model Configuration"), the token the target emitted (Fig. 7 caption:
 * accuracy is the top-1 match with the target).  One call of
 * tide_draft_train_step is one optimizer step of that fine-tuning on one batch
 * of captured signals:
 *
 *   x0 = Hcat W_fc^T                                 feature projection
 *   a  = rmsnorm(x0; g1); [q|k|v] = a W_qkv^T; rotate-half RoPE on q, k
 *   A  = causal grouped-query softmax attention(q, k, v)
 *   x1 = x0 + A W_o^T
 *   b  = rmsnorm(x1; g2); h = silu(b W_gate^T) * (b W_up^T); x2 = x1 + h W_down^T
 *   y  = rmsnorm(x2; g3); z = y W_lm^T   (computed by row block, never whole)
 *   loss = (1/N) sum_t keep_t (logsumexp(z_t) - z_t[tokens_t]),  N = max(1, sum keep)
 *   keep_t = loss_mask_t != 0 and 0 <= tokens_t < vocab
 *   grads = d loss / d params (no gradient w.r.t. the captured states), then AdamW.
 *
 * The paper gives no layer equations; the block internals above are the
 * standard definitions of those blocks (no biases anywhere, RMSNorm epsilon
 * inside the square root, softmax scale 1/sqrt(head_dim), AdamW with bias
 * correction and decoupled decay applied to every tensor).
 *
 * Conventions common to all entry points
 *   - Every pointer marked DEVICE is GPU memory owned by the caller; the library
 *     allocates and frees nothing.  Buffers must stay valid until the work
 *     enqueued on `stream` has completed.  Calls are asynchronous: no host
 *     synchronisation is performed; outputs are valid after the stream is
 *     synchronised.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Matrices are row-major; weights are stored [out_features, in_features].
 *   - dtype TIDE_DTYPE_FP32: params, hidden_buf are float.  dtype TIDE_DTYPE_BF16:
 *     params and hidden_buf are bfloat16 (raw 16-bit), compute accumulates in
 *     fp32.  Gradients, Adam moments and master weights are always float.
 *   - HIP graphs: the forward-only calls (tide_draft_forward, _eval, _forward_packed, _forward_tok, _eval_unroll, _eval_unroll_packed) enqueue
 *     kernels and nothing else, so they can be captured on `stream` and replayed (call once before the capture:
 *     the first call on a device sets function attributes).  A training step bakes adam_state->step (bias
 *     corrections) and lr into its launch: a captured step would replay with the captured values;
 *     tide_draft_train_step_dev keeps both in device memory and can be captured and replayed.
 *   - Return value: 0 on success, a negative TIDE_ERR_* code otherwise, with
 *     tide_last_error() describing the problem.  Arguments are validated before
 *     any work is enqueued: on TIDE_ERR_NULL / _CONFIG / _WORKSPACE nothing has
 *     been enqueued.  On TIDE_ERR_HIP (a launch failed midway) earlier kernels of
 *     the call may already be queued and the outputs are undefined.  On any error
 *     adam_state->step is unchanged.  The library never aborts and never throws
 *     across this boundary.
 */
#ifndef TIDE_DRAFT_H
#define TIDE_DRAFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TIDE_OK             0
#define TIDE_ERR_NULL      (-1)  /* a required pointer is NULL */
#define TIDE_ERR_CONFIG    (-2)  /* inconsistent or unsupported tide_draft_config */
#define TIDE_ERR_WORKSPACE (-3)  /* workspace too small or not 256-byte aligned */
#define TIDE_ERR_HIP       (-4)  /* a HIP call or kernel launch failed */

#define TIDE_DTYPE_FP32 0
#define TIDE_DTYPE_BF16 1

/* Shape and hyper-parameters of the draft (host memory, read on every call).
 * Requirements: all sizes > 0; hidden == n_heads*head_dim; n_heads % n_kv_heads
 * == 0; head_dim even; rms_eps > 0; rope_theta > 0; dtype is one of TIDE_DTYPE_*.
 * batch*seq*max(vocab, ...) must fit the 32-bit tile arithmetic documented in
 * the sources (batch*seq <= 2^22 positions, every dimension < 2^24). */
typedef struct tide_draft_config {
  int32_t batch, seq;                 /* B, S: hidden_buf is [B, S, n_capture*target_hidden] */
  int32_t n_capture, target_hidden;   /* K (3 in the paper) captured layers of width H_t */
  int32_t hidden;                     /* d: draft width (projection output) */
  int32_t n_heads, n_kv_heads, head_dim;
  int32_t ffn;                        /* F: SwiGLU inner width */
  int32_t vocab;                      /* V: the target's vocabulary */
  float rope_theta, rms_eps;
  float beta1, beta2, adam_eps, weight_decay;
  int32_t dtype;
  /* LM head.  The logits z = y W_lm^T exist for ONE block of rows at a time (bf16, overwritten in place by their
   * gradient); the forward product, the row statistics, the logit gradient and the input-gradient product run
   * block by block, and dW_lm accumulates over the blocks.
   *   lm_block_rows      rows per block; 0 = the library's choice (half of batch*seq rounded up to 64, at most
   *                      16384 rows and 6 GiB of logits, at least min(batch*seq, 4096) rows).  Other values are
   *                      rounded up to a multiple of 64.
   *   lm_keep_all_rows   0 (default) = as above, the logit buffer is one block.  Non-zero = opt-in: the buffer
   *                      holds the bf16 logit GRADIENT of every block until the end of the LM head and dW_lm is
   *                      one product over all rows, which saves the read-modify-write of dW_lm per further
   *                      block at the price of batch*seq x vocab x 2 bytes of workspace (8.4 GB at batch 16 x
   *                      seq 2048, vocab 128256).  Forward-only calls never keep more than one block. */
  int32_t lm_block_rows;
  int32_t lm_keep_all_rows;
} tide_draft_config;

/* The ten tensors of the draft; the same struct describes parameters, gradients,
 * Adam moments and master weights (identical shapes).  All DEVICE pointers. */
typedef struct tide_draft_tensors {
  void *w_fc;    /* [d, K*H_t] */
  void *g1;      /* [d]   gain of the attention-input RMSNorm */
  void *w_qkv;   /* [(n_heads + 2*n_kv_heads)*head_dim, d]: q rows, then k rows, then v rows */
  void *w_o;     /* [d, n_heads*head_dim] */
  void *g2;      /* [d]   gain of the MLP-input RMSNorm */
  void *w_gate;  /* [F, d] */
  void *w_up;    /* [F, d] */
  void *w_down;  /* [d, F] */
  void *g3;      /* [d]   gain of the final RMSNorm */
  void *w_lm;    /* [V, d] */
} tide_draft_tensors;

/* Optimizer state.  m, v: float first/second moments.  master: float master
 * copy of the parameters, used and updated only in bf16 mode (the bf16 params
 * are re-rounded from it every step); ignored (may be all NULL) in fp32 mode.
 * step: number of updates applied so far; host memory, incremented by a
 * successful tide_draft_train_step. */
typedef struct tide_adam_state {
  tide_draft_tensors m, v, master;
  int64_t step;
} tide_adam_state;

/* Bytes of DEVICE scratch the two calls below need for this config (the larger
 * of the two).  Returns 0 if the config is invalid (see tide_last_error).  The logit buffer in it is one row
 * block (cfg->lm_block_rows x vocab elements; 4.2 GB at the 8B shape) unless cfg->lm_keep_all_rows asks for all. */
size_t tide_draft_workspace_bytes(const tide_draft_config *cfg);

/* Forward only (what the evaluation step of the paper's Algorithm 1 runs on held-out signals):
 * writes the masked mean cross-entropy to *loss_out (DEVICE float) and, if
 * top1_out (DEVICE int32 [B*S]) is not NULL, the arg-max token of every
 * position (lowest index on exact ties).  Mutates nothing else.
 *   hidden_buf DEVICE [B,S,K*H_t] (dtype per cfg), read-only
 *   tokens     DEVICE int32 [B,S]: the token the target emitted after position s
 *              (the caller aligns labels; the library does not shift)
 *   loss_mask  DEVICE uint8 [B,S]: non-zero = position contributes to the loss
 *   workspace  DEVICE, >= tide_draft_workspace_bytes(cfg), 256-byte aligned */
int tide_draft_forward(const tide_draft_config *cfg, const tide_draft_tensors *params,
                       const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                       float *loss_out, int32_t *top1_out,
                       void *workspace, size_t workspace_bytes, void *stream);

/* Packed (variable-length) batches.  The paper's training signals are the hidden states of the tokens the
 * target accepted (Sec. 3.2, Fig. 3 caption): segments of different lengths.  Instead of right-padding
 * every segment to `seq`, the T = batch*seq rows of hidden_buf / tokens / loss_mask hold the segments back to
 * back: sequence i owns rows [cu_seqlens[i], cu_seqlens[i+1]).  cu_seqlens is a DEVICE array of n_seqs+1
 * ascending int32 values with cu_seqlens[0] >= 0 and cu_seqlens[n_seqs] <= T (neither can be checked without
 * a sync: rows outside [cu_seqlens[0], cu_seqlens[n_seqs]) are padding, they must hold finite values and
 * never carry loss; an empty sequence is allowed).  max_seqlen (host) bounds every sequence length: it sizes
 * the attention grid and the RoPE table, and a longer sequence gives undefined results for its tail.
 * Attention is causal inside each sequence and never crosses a boundary; RoPE positions restart at 0 in each
 * sequence; everything else is per row, so the result for a sequence equals that of the same sequence
 * right-padded in a fixed batch (loss and gradients are normalised by the N of the whole batch either way).
 * cfg.batch and cfg.seq only fix the row capacity T and the workspace size here.  Other arguments, errors
 * and ownership as in tide_draft_forward / tide_draft_train_step; extra errors: TIDE_ERR_NULL for a NULL
 * cu_seqlens, TIDE_ERR_CONFIG for n_seqs outside [1, 65535] or max_seqlen outside [1, T]. */
int tide_draft_forward_packed(const tide_draft_config *cfg, const tide_draft_tensors *params,
                              const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                              const int32_t *cu_seqlens, int32_t n_seqs, int32_t max_seqlen,
                              float *loss_out, int32_t *top1_out,
                              void *workspace, size_t workspace_bytes, void *stream);
int tide_draft_train_step_packed(const tide_draft_config *cfg, tide_draft_tensors *params,
                                 tide_draft_tensors *grads, tide_adam_state *adam_state,
                                 const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                                 const int32_t *cu_seqlens, int32_t n_seqs, int32_t max_seqlen,
                                 float lr, float *loss_out,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* Evaluation pass of the paper's Algorithm 1 (the held-out check that gates deployment of a newly trained
 * draft) in the paper's accuracy metric (Fig. 7 caption: top-1 match rate between draft and target): writes
 * the masked mean cross-entropy to *loss_out and, to *accuracy_out (DEVICE float), the fraction of the N
 * loss-carrying positions whose arg-max token (lowest index on ties) equals tokens.  Forward only, LM head on
 * the loss-carrying rows only.  Arguments as in tide_draft_forward. */
int tide_draft_eval(const tide_draft_config *cfg, const tide_draft_tensors *params,
                    const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                    float *loss_out, float *accuracy_out,
                    void *workspace, size_t workspace_bytes, void *stream);

/* One training step: forward, full backward, AdamW (Sec. 3.3: the draft is
 * fine-tuned on the signals accumulated from serving).
 *   params     in/out: updated in place (bf16 mode: re-rounded from master)
 *   grads      out: float gradients of this batch, overwritten (not accumulated)
 *   adam_state in/out: m, v (and master) updated; step incremented on success
 *   lr         learning rate of this step
 *   loss_out   DEVICE float: loss of this batch before the update
 * Other arguments as in tide_draft_forward. */
int tide_draft_train_step(const tide_draft_config *cfg, tide_draft_tensors *params,
                          tide_draft_tensors *grads, tide_adam_state *adam_state,
                          const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                          float lr, float *loss_out,
                          void *workspace, size_t workspace_bytes, void *stream);

/* The same step with its schedule in DEVICE memory, for callers that capture the step into a HIP graph and replay
 * it (Sec. 3.3 runs many such steps back to back on the accumulated signals): tide_draft_train_step bakes lr and the
 * bias corrections of step adam_state->step + 1 into its launch, so a replay would repeat them; here
 *   lr_dev    DEVICE float: learning rate, read when the enqueued work runs (the caller may change it between replays)
 *   step_dev  DEVICE int64: number of updates applied so far; read for the bias corrections and incremented on the
 *             device by every execution of the enqueued work
 * and adam_state->step (host) is neither read nor changed.  The call enqueues kernels only (no memset, no copy, no
 * allocation, no host synchronisation); call any entry point once on the device before capturing (the first call
 * sets one-time function attributes).  Everything else as in tide_draft_train_step. */
int tide_draft_train_step_dev(const tide_draft_config *cfg, tide_draft_tensors *params,
                              tide_draft_tensors *grads, tide_adam_state *adam_state,
                              const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                              const float *lr_dev, int64_t *step_dev, float *loss_out,
                              void *workspace, size_t workspace_bytes, void *stream);

/* Token-input variant.  Sec. 3.2 names EAGLE-3 as the draft architecture; that architecture joins the
 * projected features with the embedding of the token sampled at the position: both vectors are
 * concatenated and a second fully connected layer brings them back to the model width before the decoder
 * layer.  With this struct the first line of the model above becomes
 *     g = Hcat W_fc^T,  e = embed[input_ids]  (a zero row for an id outside [0, embed_rows)),
 *     x0 = [g ; e] W_in^T
 * and everything after x0 is unchanged.  embed is frozen (no gradient); W_in is one more trainable tensor
 * with its own gradient and Adam state.  The paper restates none of this, so it is a reading of the cited
 * architecture (its multi-step unroll: tide_draft_eval_unroll below).
 *   embed       DEVICE [embed_rows, d], dtype per cfg, read-only
 *   input_ids   DEVICE int32 [B,S]: the token whose embedding joins the features of the position
 *   w_in        DEVICE [d, 2d], dtype per cfg: columns [0, d) act on g, columns [d, 2d) on e
 *   grad_w_in, m_w_in, v_w_in   DEVICE float [d, 2d]; master_w_in likewise, bf16 mode only.  These four are
 *               used by tide_draft_train_step_tok only and may be NULL for tide_draft_forward_tok.
 * Fixed-layout batches only.  Other arguments, ownership and errors as in tide_draft_forward /
 * tide_draft_train_step (top1_out and the AdamW step included); TIDE_ERR_NULL for a NULL member that the
 * call needs, TIDE_ERR_CONFIG for embed_rows < 1. */
typedef struct tide_token_input {
  const void *embed;
  int32_t embed_rows;
  const int32_t *input_ids;
  void *w_in;
  void *grad_w_in, *m_w_in, *v_w_in, *master_w_in;
} tide_token_input;
int tide_draft_forward_tok(const tide_draft_config *cfg, const tide_draft_tensors *params,
                           const tide_token_input *tok,
                           const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                           float *loss_out, int32_t *top1_out,
                           void *workspace, size_t workspace_bytes, void *stream);
int tide_draft_train_step_tok(const tide_draft_config *cfg, tide_draft_tensors *params,
                              tide_draft_tensors *grads, tide_adam_state *adam_state,
                              const tide_token_input *tok,
                              const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                              float lr, float *loss_out,
                              void *workspace, size_t workspace_bytes, void *stream);

/* Multi-step evaluation unroll (forward only).  Sec. 3.2 names EAGLE-3 as the draft architecture and Sec. 5.1
 * fixes gamma = 3 draft tokens per round: only the first draft token of a round sees a captured feature, each
 * later one is fed the draft layer's own output of the step before.  This call runs n_steps such steps over the
 * whole batch with the true tokens as inputs and labels, and reports how well step s predicts the s-th token of
 * a round.  Step 1 is tide_draft_eval (tide_draft_forward_tok's model if tok is given).  Step s >= 2, for row
 * i of a sequence, which then stands for position i + s - 1 (rows whose position leaves the sequence carry
 * no loss):
 *     feature   x2 of step s-1 at row i, in place of Hcat W_fc^T (joined with embed[input_ids[i + s - 1]]
 *               through W_in if tok is given)
 *     RoPE      position i + s - 1
 *     attention one softmax over the step-1 keys/values of rows 0..i and the key/value pair the row itself
 *               produced at each of the steps 2..s
 *     label     tokens[i + s - 1], loss_mask[i + s - 1]
 * The paper restates none of this: it is a reading of the cited architecture.
 *   tok           may be NULL (feature-only model); else as in tide_draft_forward_tok
 *   n_steps       1 .. 8
 *   loss_out      DEVICE float [n_steps]: mean cross-entropy of every step over its loss-carrying rows
 *   accuracy_out  DEVICE float [n_steps]: top-1 accuracy of every step over the same rows
 *   workspace     DEVICE, 256-byte aligned, at least tide_draft_unroll_workspace_bytes(cfg, n_steps) bytes
 *                 (0 = invalid config or n_steps): one workspace of the single-step call per step plus the
 *                 shifted inputs and own key/value pairs
 * Fixed-layout batches (packed ones: the _packed forms below).  Enqueues kernels on `stream` and nothing else;
 * errors as in tide_draft_forward, TIDE_ERR_CONFIG for n_steps outside [1, 8]. */
size_t tide_draft_unroll_workspace_bytes(const tide_draft_config *cfg, int32_t n_steps);
/* For tests and profiling: byte offset, inside the unroll workspace of n_steps steps, of intermediate `name` of
 * step `step` (0-based).  Names: those of tide_draft_workspace_offset (the step's own single-step workspace),
 * and "tokens_s", "mask_s", "sel_s", "ids_s" (the step's shifted inputs and row selection), "own_kv" ([B*S,
 * 2*n_kv_heads*head_dim]: the step's own keys then values), "own_grad", "dfeat", "acc_kv1".  -1 if unknown. */
int64_t tide_draft_unroll_workspace_offset(const tide_draft_config *cfg, int32_t n_steps, int32_t step,
                                           const char *name);
int tide_draft_eval_unroll(const tide_draft_config *cfg, const tide_draft_tensors *params,
                           const tide_token_input *tok,
                           const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                           int32_t n_steps, float *loss_out, float *accuracy_out,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Training step over the multi-step unroll above: minimises L = sum_s step_weights[s] * loss_s.  The gradient
 * flows through the whole chain: the feature of step s is the layer output of step s-1, and the keys/values of a
 * step are read by every later step.  One AdamW update at the end, exactly as in tide_draft_train_step.
 *   tok           may be NULL (feature-only model); else as in tide_draft_train_step_tok (W_in is trained)
 *   step_weights  HOST float [n_steps], finite and >= 0, or NULL for all ones (the paper gives none)
 *   loss_out      DEVICE float [n_steps]: the unweighted mean cross-entropy of every step, before the update
 *   grads         out: gradients of L, overwritten
 *   workspace     as in tide_draft_eval_unroll (the same size query covers both calls)
 * Errors as in tide_draft_train_step, TIDE_ERR_CONFIG for a bad n_steps or weight. */
int tide_draft_train_step_unroll(const tide_draft_config *cfg, tide_draft_tensors *params,
                                 tide_draft_tensors *grads, tide_adam_state *adam_state,
                                 const tide_token_input *tok,
                                 const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                                 int32_t n_steps, const float *step_weights, float lr, float *loss_out,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* The two unroll calls on PACKED (variable-length) batches: cu_seqlens, n_seqs, max_seqlen as in
 * tide_draft_forward_packed; every sequence is unrolled by itself (a row's position i + s - 1 must stay inside its
 * own sequence), padding rows carry nothing, and every step's loss is the mean over that step's loss-carrying
 * rows of the whole batch.  With n_steps = 1 and tok given this is the token-input model on a packed batch.
 * Errors as in the fixed-layout calls plus those of tide_draft_forward_packed (malformed offsets: status word). */
int tide_draft_eval_unroll_packed(const tide_draft_config *cfg, const tide_draft_tensors *params,
                                  const tide_token_input *tok,
                                  const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                                  const int32_t *cu_seqlens, int32_t n_seqs, int32_t max_seqlen,
                                  int32_t n_steps, float *loss_out, float *accuracy_out,
                                  void *workspace, size_t workspace_bytes, void *stream);
int tide_draft_train_step_unroll_packed(const tide_draft_config *cfg, tide_draft_tensors *params,
                                        tide_draft_tensors *grads, tide_adam_state *adam_state,
                                        const tide_token_input *tok,
                                        const void *hidden_buf, const int32_t *tokens, const uint8_t *loss_mask,
                                        const int32_t *cu_seqlens, int32_t n_seqs, int32_t max_seqlen,
                                        int32_t n_steps, const float *step_weights, float lr, float *loss_out,
                                        void *workspace, size_t workspace_bytes, void *stream);

/* Message of the last error on the calling thread (static storage, never NULL). */
const char *tide_last_error(void);

/* Byte offset, inside the workspace, of a named intermediate of the last call
 * with this config ("x0", "a", "qkv", "A", "x1", "bn", "gt", "u", "h", "x2",
 * "yhat", "lse", "dyhat", "dx2", "dx1", "dx0", "dqkv", ...; activations have the
 * config's dtype, "lse"/"r1"/"r2"/"r3" are float); "lm_rows" returns the number
 * of rows per logits block instead.  -1 if the name or config is unknown.  After
 * a training step "gt"/"u" hold their gradients.  For tests and profiling.
 * Rows: a position without loss acts on the result only through its key and value, so everything after the
 * attention runs on the selected positions alone (those with loss; every position when top1_out is given).
 * "x0", "a", "qkv", "A", "dA", "dx1", "dx0", "dqkv", "da" have one row per position; "x1", "bn", "gt", "u", "h",
 * "x2", "yhat", "dyhat", "dx2", "dh", "dbn", "A_c", "x0_c", "dx1_c", "dA_c" hold the selected positions densely,
 * row i being position "kept_idx"[i] (int32, "cnt" of them; "row_pos" is the inverse, -1 where not selected).
 *
 * "status" names a device int32 that every forward / eval / train call rewrites: 0 when all is well, else
 * bit 0 (value 1) = the loss came out NaN or infinite, bit 1 (value 2) = packed batch whose cu_seqlens is not
 * ascending inside [0, batch*seq] or holds a sequence longer than max_seqlen (the kernels clamp such offsets
 * so that no access leaves the buffers; the numbers are then meaningless).  Read it after synchronising. */
int64_t tide_draft_workspace_offset(const tide_draft_config *cfg, const char *name);

/* ---- Building blocks, exported for per-kernel parity tests and profiling ----
 * Each runs the same kernels the two calls above use.  Same conventions. */

/* C[M,N] = alpha * op(A) op(B)^T-style product in the three layouts the step uses
 * (Sec. 3.3 training: forward Y = X W^T, input gradient dX = dY W, weight
 * gradient dW = dY^T X):
 *   layout 0 ("NT"): C = A[M,K] * B[N,K]^T
 *   layout 1 ("NN"): C = A[M,K] * B[K,N]
 *   layout 2 ("TN"): C = A[K,M]^T * B[K,N]
 * in_dtype: dtype of A and B; out_dtype: dtype of C (TIDE_DTYPE_*).  accumulate
 * != 0 adds to C instead of overwriting.  residual (may be NULL) is a [M,N]
 * matrix of out_dtype added to the result.
 * workspace (DEVICE, 16-byte aligned, optional): scratch for the split of a partly filled last round of tiles.
 * A product whose 256 x 256 tiles leave the last round of the 256 compute units at most half full (and whose
 * result is float, without residual) can have those tiles split over K; the partial sums go to the workspace
 * and are added to C in a fixed order by a second small kernel (deterministic).  tide_gemm_workspace_bytes
 * gives the bytes that takes (0: the call is never split; bf16 inputs are assumed); with workspace NULL or
 * smaller than that, nothing is split and the result is the same up to the order of the fp32 additions. */
size_t tide_gemm_workspace_bytes(int layout, int64_t M, int64_t N, int64_t K, int out_dtype);
int tide_gemm(int layout, int64_t M, int64_t N, int64_t K, float alpha,
              const void *A, const void *B, void *C, const void *residual,
              int in_dtype, int out_dtype, int accumulate,
              void *workspace, size_t workspace_bytes, void *stream);

/* y = g * x * rsqrt(mean(x^2) + eps) over rows of x [rows, d]; rstd_out [rows] float. */
int tide_rmsnorm_fwd(int64_t rows, int64_t d, const void *x, const void *g, float eps,
                     void *y, float *rstd_out, int dtype, void *stream);
/* dx = (residual_grad or 0) + rmsnorm input gradient; dg [d] float (overwritten).
 * dg_partial: DEVICE float scratch of tide_rmsnorm_bwd_scratch_bytes(rows, d). */
size_t tide_rmsnorm_bwd_scratch_bytes(int64_t rows, int64_t d);
int tide_rmsnorm_bwd(int64_t rows, int64_t d, const void *dy, const void *x, const void *g,
                     const float *rstd, const void *residual_grad, void *dx, float *dg,
                     void *dg_partial, int dtype, void *stream);
/* tide_rmsnorm_bwd for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same kernels and the same results, but the per-block
 * partial sums of dg live in a fixed array inside the library (TIDE_RMSNORM_STATIC_SCRATCH_BYTES of device
 * memory per GPU, held until the process ends) instead of a caller buffer.  The call allocates and frees
 * nothing.  It fails with TIDE_ERR_WORKSPACE when tide_rmsnorm_bwd_scratch_bytes(rows, d) exceeds that size
 * (it does not for any shape tide_rmsnorm_bwd accepts: at most 512 blocks x 8192 columns).  Every call on a
 * GPU shares that GPU's array and every element a call reads it has written itself first, so nothing needs
 * clearing; two calls that overlap on one GPU (different streams, or different host threads) race. */
#define TIDE_RMSNORM_STATIC_SCRATCH_BYTES (16u << 20)
int tide_rmsnorm_bwd_static(int64_t rows, int64_t d, const void *dy, const void *x, const void *g,
                            const float *rstd, const void *residual_grad, void *dx, float *dg,
                            int dtype, void *stream);

/* Causal grouped-query attention on a packed activation qkv [B*S, (n_heads+2*n_kv_heads)*head_dim]
 * (q heads, then k heads, then v heads; RoPE already applied).  out [B*S, n_heads*head_dim];
 * lse [B, n_heads, S] float = log-sum-exp of the scaled scores of each query row. */
int tide_attention_fwd(int B, int S, int n_heads, int n_kv_heads, int head_dim,
                       const void *qkv, void *out, float *lse, int dtype, void *stream);
/* dqkv has the layout of qkv.  delta: DEVICE float scratch [B, n_heads, S]. */
int tide_attention_bwd(int B, int S, int n_heads, int n_kv_heads, int head_dim,
                       const void *qkv, const void *out, const void *dout, const float *lse,
                       float *delta, void *dqkv, int dtype, void *stream);

/* In-place rotate-half RoPE of the q and k heads of a packed qkv activation;
 * inverse != 0 rotates by the negative angle (the backward pass).
 * table: DEVICE float scratch of S*head_dim elements (cos/sin table, overwritten). */
int tide_rope(int B, int S, int n_heads, int n_kv_heads, int head_dim, float theta,
              void *qkv, float *table, int inverse, int dtype, void *stream);

/* Cross-entropy pass of a training call over a block of logits (Sec. 3.3: the draft is
 * trained on the target's emitted tokens; mean CE over the loss-carrying rows):
 * z [rows, ldz] (DEVICE, dtype TIDE_DTYPE_*, ldz a multiple of 8 and >= vocab, rows 16-byte
 * aligned) holds the logits on entry and, on return,
 *     dz[r, c] = keep_r * (exp(z[r, c] - lse_r) - [c == tokens[r]])   for c < vocab, 0 for c in [vocab, ldz)
 * (not divided by the number of loss rows), with keep_r = mask[r] != 0 and 0 <= tokens[r] < vocab.
 * lse [rows] and loss_rows [rows] (DEVICE floats) receive the log-sum-exp of every row and
 * keep_r * (lse_r - z[r, tokens[r]]).  Everything is caller-owned; nothing is allocated. */
int tide_ce_train(int64_t rows, int32_t vocab, void *z, int64_t ldz, const int32_t *tokens,
                  const uint8_t *mask, float *lse, float *loss_rows, int dtype, void *stream);

/* ---- Measurement support ----
 * Between tide_profile_start and tide_profile_stop every kernel the library
 * enqueues is bracketed by a pair of HIP events recorded on the caller's stream
 * (a few microseconds of host time per launch; off by default).  tide_profile_stop
 * waits for the recorded events and writes a JSON array to `report` (HOST buffer):
 * one object per kernel with its launch count, summed duration in ms and summed
 * algorithmic flops and bytes.  Returns TIDE_ERR_WORKSPACE if the buffer is too
 * small (64 KiB is ample).  Not thread-safe against concurrent library calls. */
int tide_profile_start(void);
int tide_profile_stop(char *report, size_t report_bytes);

/* Measurement aid: enqueues a kernel that does nothing but bf16 MFMAs from registers (`blocks` work-groups of
 * 8 wavefronts, each issuing iters x 8 independent v_mfma_f32_32x32x16_bf16 on random operands, a different pair
 * per instruction), so that the caller can time the rate the matrix pipes sustain on this chip under its power
 * limit (time a few hundred milliseconds of launches): the practical ceiling next to the nominal 2516.6 TFLOP/s.  sink: DEVICE buffer of blocks*512 floats (written, so that the
 * work is not optimised away); *flops_out (HOST, optional) receives the flop count of the launch. */
int tide_mfma_probe(int32_t blocks, int32_t iters, float *sink, double *flops_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TIDE_DRAFT_H */
