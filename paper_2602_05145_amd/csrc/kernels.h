// Host-side launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace tide {

enum : int { kF32 = 0, kBF16 = 1 };
enum : int { kNT = 0, kNN = 1, kTN = 2 };

inline size_t dtype_size(int dt) { return dt == kBF16 ? 2 : 4; }

// ---- gemm_mfma.hip / gemm_simple.hip ---------------------------------------------------------
// C[M,N] (ldc) = alpha * sum over operand pairs of op(A) op(B)  (+ residual) (+ C if accumulate)
// layout NT: A[M,K] lda, B[N,K] ldb.  NN: A[M,K], B[K,N].  TN: A[K,M], B[K,N].
// A second operand pair (A2,B2,K2; same layout and leading dims) extends the contraction.
struct GemmArgs {
  int layout;
  int64_t M, N, K;
  const void* A; int64_t lda;
  const void* B; int64_t ldb;
  const void* A2; const void* B2; int64_t K2;
  void* C; int64_t ldc;
  const void* residual; int64_t ldr;
  float alpha;
  const float* alpha_dev;   // optional device scalar multiplied into alpha
  int in_dtype, out_dtype;
  int accumulate;
  // Optional device-side sizes (the LM head works on the rows that carry loss, whose number is only known
  // on the GPU): effective M = clamp(*m_dev - m_off, 0, M), effective K = clamp(*k_dev - k_off, 0, K).
  // M / K above stay the upper bounds the grid is sized for; tiles past the effective size exit at once.
  const int* m_dev; int64_t m_off;
  const int* k_dev; int64_t k_off;
  // Optional device scratch (16-byte aligned) of gemm_splitk_scratch_bytes(args) bytes: with it, a launch whose
  // tiles leave the last round of the 256 CUs at most half full splits those tiles over K (fp32 results only;
  // the partial sums are added in a fixed order by a second small kernel).  Without it nothing is split.
  void* scratch; size_t scratch_bytes;
};
bool gemm_mfma_supported(const GemmArgs& a);
size_t gemm_splitk_scratch_bytes(const GemmArgs& a);   // 0 when the launch would not be split
hipError_t launch_gemm_mfma(const GemmArgs& a, hipStream_t s);
hipError_t launch_gemm_simple(const GemmArgs& a, hipStream_t s);
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);  // picks the MFMA path when supported

// ---- elementwise.hip ------------------------------------------------------------------------
// Row plan of the LM head.  keep_t = mask_t != 0 and 0 <= token_t < V.  scal[0] = N = max(1, #keep),
// scal[1] = 1/N.  The rows the LM head processes are the kept ones (or all of them if select_all):
// kept_idx[0..cnt[0]) lists them in ascending order, row_pos[t] is the position of row t in that list or -1.
size_t plan_rows_scratch_bytes(int64_t T);   // blk_counts below
// sel_mask (optional, device, one byte per row) replaces the rule above for WHICH rows are selected (the
// unroll selects the rows that carry loss at the current or a later step); N still counts the kept rows.
hipError_t launch_plan_rows(const int32_t* tokens, const uint8_t* mask, int64_t T, int V, int select_all,
                            float* scal, int* cnt, int32_t* kept_idx, int32_t* row_pos, const int* cu, int nseq,
                            int max_len, uint8_t* mask_eff, int* status, int* blk_counts, const uint8_t* sel_mask,
                            hipStream_t s);
// packed batches (cu = device offsets of nseq sequences): position of each row in its sequence, and zeroing
// of the rows of a [T, row_bytes] array that no sequence owns
hipError_t launch_seq_pos(const int* cu, int nseq, int64_t T, int max_len, int32_t* pos, hipStream_t s);
hipError_t launch_zero_padding_rows(void* p, const int* cu, int nseq, int64_t T, int64_t row_bytes, hipStream_t s);
// out[t] = embed[ids[t]] for 0 <= ids[t] < rows, else a zero row (rows of width d)
hipError_t launch_embed_rows(int64_t T, int d, const void* embed, int rows, const int32_t* ids, void* out, int dtype,
                             hipStream_t s);
// dst0[i] = src0[kept_idx[i]] for i < *cnt (rows of width d0), likewise src1 -> dst1 (width d1; src1 may be
// NULL), tokens and mask
hipError_t launch_gather_rows(int64_t T, int d0, const void* src0, void* dst0, int d1, const void* src1, void* dst1,
                              const int32_t* tokens, const uint8_t* mask, const int32_t* kept_idx, const int* cnt,
                              int32_t* tokens_c, uint8_t* mask_c, int dtype, hipStream_t s);
// dst0[t] = row_pos[t] >= 0 ? src0[row_pos[t]] : 0, likewise src1 -> dst1 (src1 may be NULL)
hipError_t launch_scatter_rows(int64_t T, int d0, const void* src0, void* dst0, int d1, const void* src1, void* dst1,
                               const int32_t* row_pos, int dtype, hipStream_t s);
// rows_dev (optional, device): only the first min(rows, *rows_dev) rows are processed
hipError_t launch_rmsnorm_fwd(int64_t rows, int d, const void* x, const void* g, float eps, void* y,
                              float* rstd, int dtype, const int* rows_dev, hipStream_t s);
size_t rmsnorm_bwd_scratch_bytes(int64_t rows, int d);
hipError_t launch_rmsnorm_bwd(int64_t rows, int d, const void* dy, const void* x, const void* g,
                              const float* rstd, const void* res, void* dx, float* dg,
                              float* dg_partial, int dtype, const int* rows_dev, hipStream_t s,
                              int accumulate = 0);   // accumulate: dg += instead of dg =
hipError_t launch_rope_table(int S, int dh, float theta, float* cs, hipStream_t s);  // cs [S, dh/2, 2]
// row_pos (optional, device): position of every row in its sequence; NULL = row % S.  pos_offset is added to
// every position (the table must reach that far).
hipError_t launch_rope(int B, int S, int nh, int nkv, int dh, const float* cs, void* qkv, int inverse,
                       int dtype, const int32_t* row_pos, int pos_offset, hipStream_t s);
// n = rows * per_row elements; rows_dev (optional, device): only the first *rows_dev rows are processed
hipError_t launch_swiglu_fwd(int64_t n, const void* gt, const void* u, void* h, int dtype, int64_t per_row,
                             const int* rows_dev, hipStream_t s);
hipError_t launch_swiglu_bwd(int64_t n, const void* dh, const void* gt, const void* u, void* dgt,
                             void* du, int dtype, int64_t per_row, const int* rows_dev, hipStream_t s);
// z [rows, ldz]: per-row log-sum-exp, loss term keep*(lse - z[label]) and optional arg-max
// rows is an upper bound; rows_dev/rows_off (optional) give the effective count clamp(*rows_dev - rows_off, 0, rows).
// top1 (optional) is written through top1_idx: top1[top1_idx[row]] = arg-max of row; hit_rows (optional)
// gets 1 where a kept row's arg-max equals its label, else 0.
hipError_t launch_ce_stats(int64_t rows, int V, const void* z, int64_t ldz, const int32_t* tokens,
                           const uint8_t* mask, float* lse, float* loss_rows, int32_t* top1,
                           const int32_t* top1_idx, float* hit_rows, const int* rows_dev, int64_t rows_off,
                           int dtype, hipStream_t s);
// training pass: the outputs of ce_stats (without arg-max) and dz = keep * (exp(z - lse) - onehot(label)) written
// over z (unscaled by 1/N), in one kernel
hipError_t launch_ce_train(int64_t rows, int V, void* z, int64_t ldz, const int32_t* tokens, const uint8_t* mask,
                           float* lse, float* loss_rows, const int* rows_dev, int64_t rows_off, int dtype,
                           hipStream_t s);
// loss = scal[1] * sum of loss_rows[0 .. *cnt); optionally accuracy = scal[1] * sum of hit_rows[0 .. *cnt)
hipError_t launch_loss_reduce(const float* loss_rows, const float* hit_rows, const int* cnt, const float* scal,
                              float* loss_out, float* acc_out, int* status, hipStream_t s);

// b^t for an integer t >= 0 by repeated squaring, in IEEE double multiplications only: the host and the device
// get the same bits (the bias corrections of AdamW are computed on either side).
__host__ __device__ inline double pow_int(double b, long long t) {
  double r = 1.0;
  while (t > 0) {
    if (t & 1) r *= b;
    b *= b;
    t >>= 1;
  }
  return r;
}

struct AdamTensor { void* p; const float* g; float* m; float* v; float* master; int64_t n; };
constexpr int kMaxAdamTensors = 11;   // the ten tensors of the draft and W_in of the token-input variant
struct AdamArgs {
  AdamTensor t[kMaxAdamTensors];
  int nt;
  float lr, beta1, beta2, eps, wd, inv_bc1, inv_sqrt_bc2;
  int dtype;
  // optional (device): {lr, 1 - lr * wd, 1 / (1 - beta1^t), 1 / sqrt(1 - beta2^t)} written by launch_adam_schedule;
  // when set, the kernel takes these four from device memory instead of the host values above
  const float* dyn;
};
hipError_t launch_adamw(const AdamArgs& a, hipStream_t s);
// t = *step_dev + 1; dyn[0..3] = {*lr_dev, 1 - *lr_dev * wd, 1 / (1 - beta1^t), 1 / sqrt(1 - beta2^t)}; *step_dev = t
hipError_t launch_adam_schedule(const float* lr_dev, int64_t* step_dev, float beta1, float beta2, float wd, float* dyn,
                                hipStream_t s);

// ---- attention_simple.hip / attention_mfma.hip ----------------------------------------------
// bits of the device status word of a step (written by plan_rows, OR-ed by loss_reduce)
constexpr int kStatusLossNotFinite = 1;   // the loss came out NaN or infinite
constexpr int kStatusBadSeqlens = 2;      // packed batch: cu_seqlens not ascending inside [0, T] or a sequence longer than max_seqlen

struct AttnArgs {
  int B, S, nh, nkv, dh;
  const void* qkv; void* out; float* lse;           // forward
  const void* dout; float* delta; void* dqkv;       // backward
  int dtype;
  // packed batches: device offsets of the B sequences (B+1 ascending values, the last <= total_rows) and
  // the row count of the activations; S is then the longest sequence allowed.  NULL = B x S fixed layout.
  // lse / delta are [B, nh, S] in the fixed layout and [nh, total_rows] when packed.
  const int* cu_seqlens = nullptr;
  int64_t total_rows = 0;
};
bool attn_mfma_supported(const AttnArgs& a);
hipError_t launch_attn_delta(const AttnArgs& a, hipStream_t s);  // delta = rowsum(dO * O)
hipError_t launch_attn_fwd_simple(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_bwd_simple(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_fwd_mfma(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_bwd_mfma(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_fwd(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_bwd(const AttnArgs& a, hipStream_t s);

// ---- unroll.hip: the multi-step unroll (the draft fed its own output) ------------------------------
constexpr int kMaxUnroll = 8;
// tokens / mask / input ids (ids, ids_s optional) moved left by `shift` inside every sequence (S rows each, or
// the packed sequences given by the device offsets cu[0..nseq]; padding rows carry nothing), and sel_s[t] = 1
// where row t carries loss at a step in (shift, n_steps]
hipError_t launch_shift_inputs(const int32_t* tokens, const uint8_t* mask, const int32_t* ids, int64_t T, int S, int V,
                               int shift, int n_steps, int32_t* tokens_s, uint8_t* mask_s, uint8_t* sel_s,
                               int32_t* ids_s, const int* cu, int nseq, hipStream_t s);
// own[T, 2 nk] = key/value columns of qkv (rows of nq + 2 nk), which then receive those of qkv1
hipError_t launch_kv_swap(int64_t T, int nq, int nk, void* qkv, const void* qkv1, void* own, int dtype, hipStream_t s);
struct OwnKV { const void* kv[kMaxUnroll]; };   // per later step: [T, 2 nk], keys then values
// merges the n_own own key/value pairs of every row into the causal attention result (out, lse) over step 1
// T rows; lse / delta are [T / S, nh, S], or [nh, T] if packed
hipError_t launch_own_kv_merge_fwd(int64_t T, int S, int nh, int nkv, int dh, const void* qkv, void* out, float* lse,
                                   const OwnKV& own, int n_own, int packed, int dtype, hipStream_t s);
struct OwnKVGrad { void* kv[kMaxUnroll]; };   // gradient buffers of the same pairs, same layout
// backward of the merge: adds the pairs' share to the query gradients in dqkv and writes (first) or adds the
// pairs' own gradients; lse / delta are those of the merged result
hipError_t launch_own_kv_merge_bwd(int64_t T, int S, int nh, int nkv, int dh, const void* qkv, const void* dout,
                                   const float* lse, const float* delta, const OwnKV& own, const OwnKVGrad& grad,
                                   int n_own, int first, void* dqkv, int packed, int dtype, hipStream_t s);
// key/value columns of dqkv <-> the running step-1 key/value gradient acc1 [T, 2 nk]: mode 0 acc1 = columns,
// mode 1 acc1 += columns (both then put own_grad [T, 2 nk] into the columns), mode 2 columns += acc1
hipError_t launch_kv_grad_route(int64_t T, int nq, int nk, void* dqkv, void* acc1, const void* own_grad, int mode,
                                int dtype, hipStream_t s);

// pure-MFMA rate probe: blocks x 8 waves x iters x 8 MFMAs of 2*32*32*16 flop; sink holds blocks*512 floats
hipError_t launch_mfma_probe(int blocks, int iters, float* sink, hipStream_t s);

}  // namespace tide
