// C ABI of the TIDE draft-training step (see include/tide_draft.h): argument validation, workspace
// carving and the order in which the gfx950 kernels are enqueued.  Host code only; every arithmetic
// step runs in the kernels of this directory.
#include "../../include/tide_draft.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include <mutex>
#include <string>
#include <vector>

#include "kernels.h"
#include "prof.h"

using namespace tide;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int hip_fail(hipError_t e, const char* what) {
  return fail(TIDE_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define TIDE_HIP(call, what)                          \
  do {                                                \
    hipError_t e__ = (call);                          \
    if (e__ != hipSuccess) return hip_fail(e__, what); \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool check_config(const tide_draft_config* c) {
  if (!c) { fail(TIDE_ERR_NULL, "config is NULL"); return false; }
  if (c->batch <= 0 || c->seq <= 0 || c->n_capture <= 0 || c->target_hidden <= 0 || c->hidden <= 0 ||
      c->n_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 || c->ffn <= 0 || c->vocab <= 0) {
    fail(TIDE_ERR_CONFIG, "all sizes must be positive");
    return false;
  }
  if (c->lm_block_rows < 0) { fail(TIDE_ERR_CONFIG, "lm_block_rows must be >= 0"); return false; }
  if (c->dtype != TIDE_DTYPE_FP32 && c->dtype != TIDE_DTYPE_BF16) { fail(TIDE_ERR_CONFIG, "dtype must be TIDE_DTYPE_FP32 or TIDE_DTYPE_BF16"); return false; }
  if (c->n_heads % c->n_kv_heads) { fail(TIDE_ERR_CONFIG, "n_heads (%d) must be a multiple of n_kv_heads (%d)", c->n_heads, c->n_kv_heads); return false; }
  if ((int64_t)c->n_heads * c->head_dim != c->hidden) { fail(TIDE_ERR_CONFIG, "hidden (%d) must equal n_heads*head_dim (%d*%d)", c->hidden, c->n_heads, c->head_dim); return false; }
  if (c->head_dim % 2) { fail(TIDE_ERR_CONFIG, "head_dim must be even"); return false; }
  if (c->head_dim > 256) { fail(TIDE_ERR_CONFIG, "head_dim must be <= 256"); return false; }
  if (!(c->rms_eps > 0.f) || !(c->rope_theta > 0.f)) { fail(TIDE_ERR_CONFIG, "rms_eps and rope_theta must be > 0"); return false; }
  if (!(c->beta1 >= 0.f && c->beta1 < 1.f && c->beta2 >= 0.f && c->beta2 < 1.f) || !(c->adam_eps >= 0.f) || !(c->weight_decay >= 0.f)) { fail(TIDE_ERR_CONFIG, "invalid AdamW constants"); return false; }
  const bool norm_ok = (c->hidden % 8 == 0 && c->hidden <= 8192) || c->hidden <= 1024;
  if (!norm_ok) { fail(TIDE_ERR_CONFIG, "hidden must be <= 1024, or a multiple of 8 that is <= 8192"); return false; }
  const int64_t T = (int64_t)c->batch * c->seq;
  if (T > ((int64_t)1 << 22) || c->batch > 65535) { fail(TIDE_ERR_CONFIG, "batch*seq must be <= 2^22 and batch <= 65535"); return false; }
  const int64_t lim = (int64_t)1 << 21;
  if (c->vocab >= lim || c->ffn >= lim || (int64_t)c->n_capture * c->target_hidden >= lim) { fail(TIDE_ERR_CONFIG, "vocab, ffn and n_capture*target_hidden must be < 2^21"); return false; }
  return true;
}

// ---- workspace plan ----------------------------------------------------------------------------
struct Plan {
  int64_t T, KH, d, nq, nk, nqkv, F, V, ldz, lm_rows, z_rows;
  size_t es;  // activation element size
  // offsets (bytes)
  size_t scal, adam_dyn, cnt, status, plan_cnt, kept_idx, row_pos, tokens_c, mask_c, mask_eff, seq_pos, rope_cs, x0, r1, a, qkv, attn_lse, A, A_c, x0_c, x1, r2, bn, gt, u, h, x2, r3, yhat, lse, loss_rows, hit_rows, z;
  size_t fwd_end;
  size_t dyhat, dx2, dx1_c, dx1, dx0, dh, dbn, dA_c, dA, dqkv, da, delta, dg_partial;
  size_t splitk; size_t splitk_bytes;   // scratch of the weight-gradient products whose last tile round is split over K
  size_t g0, e0, dg0;   // token-input variant: projected features, looked-up embeddings, gradient of the features
  size_t total;
};

struct Bump {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  }
};

Plan make_plan(const tide_draft_config* c) {
  Plan p;
  p.T = (int64_t)c->batch * c->seq;
  p.KH = (int64_t)c->n_capture * c->target_hidden;
  p.d = c->hidden;
  p.nq = (int64_t)c->n_heads * c->head_dim;
  p.nk = (int64_t)c->n_kv_heads * c->head_dim;
  p.nqkv = p.nq + 2 * p.nk;
  p.F = c->ffn;
  p.V = c->vocab;
  p.ldz = (int64_t)align_up((size_t)p.V, 64);
  p.es = c->dtype == TIDE_DTYPE_BF16 ? 2 : 4;
  // The LM head works by blocks of lm_rows rows: half of the batch, at most 16384 rows (the forward and the
  // input-gradient products measured faster at that height than over all rows at once) and 6 GiB of logits,
  // but not fewer than 4096 rows (a batch that small is one block: a second block would cost another pass
  // over dW_lm and another set of launches for a few hundred rows).
  // The logit buffer holds ONE block: logits never exist for more rows than that, and dW_lm accumulates block
  // by block.  With cfg->lm_keep_all_rows it holds all rows instead: the logit gradients of every block are
  // then still there after the loop and dW_lm is one product over all of them.
  int64_t rows = c->lm_block_rows > 0 ? (int64_t)c->lm_block_rows : std::max<int64_t>((p.T + 1) / 2, std::min<int64_t>(p.T, 4096));
  rows = (int64_t)align_up((size_t)rows, 64);
  if (c->lm_block_rows <= 0) {
    if (rows > 16384) rows = 16384;
    while (rows > 256 && (size_t)rows * p.ldz * p.es > ((size_t)6 << 30)) rows /= 2;
  }
  if (rows > p.T) rows = p.T;
  p.z_rows = c->lm_keep_all_rows ? p.T : rows;
  p.lm_rows = rows;
  const size_t T = (size_t)p.T, es = p.es;
  Bump b;
  p.scal = b.take(64);
  p.adam_dyn = b.take(64);
  p.cnt = b.take(64);
  p.status = b.take(64);
  p.plan_cnt = b.take(plan_rows_scratch_bytes(p.T));
  p.kept_idx = b.take(T * 4);
  p.row_pos = b.take(T * 4);
  p.tokens_c = b.take(T * 4);
  p.mask_c = b.take(T);
  p.mask_eff = b.take(T);
  p.seq_pos = b.take(T * 4);
  p.rope_cs = b.take((T + kMaxUnroll) * c->head_dim * sizeof(float));   // up to T positions (one packed sequence may fill the batch), plus the unroll's shift
  p.x0 = b.take(T * p.d * es);
  p.r1 = b.take(T * 4);
  p.a = b.take(T * p.d * es);
  p.qkv = b.take(T * p.nqkv * es);
  p.attn_lse = b.take((size_t)c->batch * c->n_heads * c->seq * 4);
  p.A = b.take(T * p.nq * es);
  // from here to the LM head the arrays hold the selected rows only, densely (at most T of them)
  p.A_c = b.take(T * p.nq * es);
  p.x0_c = b.take(T * p.d * es);
  p.x1 = b.take(T * p.d * es);
  p.r2 = b.take(T * 4);
  p.bn = b.take(T * p.d * es);
  p.gt = b.take(T * p.F * es);
  p.u = b.take(T * p.F * es);
  p.h = b.take(T * p.F * es);
  p.x2 = b.take(T * p.d * es);
  p.r3 = b.take(T * 4);
  p.yhat = b.take(T * p.d * es);
  p.lse = b.take(T * 4);
  p.loss_rows = b.take(T * 4);
  p.hit_rows = b.take(T * 4);
  const size_t z_bytes = (size_t)p.z_rows * p.ldz * es;
  p.z = b.take(z_bytes);
  p.fwd_end = b.off;
  p.dyhat = b.take(T * p.d * es);
  // What only the layer's backward pass touches lives INSIDE the logit buffer as far as that reaches: the
  // backward pass starts after the LM head has finished (in the unroll: after the LM heads of all steps, each in
  // its own workspace), and the last block of logit gradients is dead by then.
  Bump zb;
  zb.off = p.z;
  auto bwd_take = [&](size_t bytes) {
    if (align_up(zb.off + bytes, 256) <= p.z + z_bytes) return zb.take(bytes);
    return b.take(bytes);
  };
  p.dh = bwd_take(T * p.F * es);
  p.dx2 = bwd_take(T * p.d * es);
  p.dx1_c = bwd_take(T * p.d * es);
  p.dx1 = bwd_take(T * p.d * es);
  p.dx0 = bwd_take(T * p.d * es);
  p.dbn = bwd_take(T * p.d * es);
  p.dA_c = bwd_take(T * p.nq * es);
  p.dA = bwd_take(T * p.nq * es);
  p.dqkv = bwd_take(T * p.nqkv * es);
  p.da = bwd_take(T * p.d * es);
  p.dg0 = bwd_take(T * p.d * es);
  p.delta = bwd_take((size_t)c->batch * c->n_heads * c->seq * 4);
  p.dg_partial = bwd_take(rmsnorm_bwd_scratch_bytes(p.T, (int)p.d));
  {
    // the largest split-K scratch any weight-gradient product of this configuration asks for
    const int64_t shapes[7][2] = {{p.V, p.d}, {p.d, p.F}, {p.F, p.d}, {p.d, p.nq}, {p.nqkv, p.d}, {p.d, p.KH}, {p.d, 2 * p.d}};
    size_t need = 0;
    for (auto& sh : shapes) {
      GemmArgs g;
      std::memset(&g, 0, sizeof(g));
      g.layout = kTN; g.M = sh[0]; g.N = sh[1]; g.K = p.T; g.lda = sh[0]; g.ldb = sh[1]; g.ldc = sh[1];
      g.in_dtype = c->dtype == TIDE_DTYPE_BF16 ? kBF16 : kF32; g.out_dtype = kF32;
      g.A = g.B = g.C = (void*)256;   // alignment only
      const size_t n = gemm_splitk_scratch_bytes(g);
      if (n > need) need = n;
    }
    p.splitk_bytes = need;
    p.splitk = b.take(need ? need : 16);
  }
  p.g0 = b.take(T * p.d * es);
  p.e0 = b.take(T * p.d * es);
  p.total = b.off;
  return p;
}

bool tensors_ok(const tide_draft_tensors* t, const char* what) {
  if (!t) { fail(TIDE_ERR_NULL, "%s is NULL", what); return false; }
  const void* ptrs[10] = {t->w_fc, t->g1, t->w_qkv, t->w_o, t->g2, t->w_gate, t->w_up, t->w_down, t->g3, t->w_lm};
  for (int i = 0; i < 10; ++i)
    if (!ptrs[i]) { fail(TIDE_ERR_NULL, "%s has a NULL tensor (index %d)", what, i); return false; }
  return true;
}

int check_token_input(const tide_token_input* tok, bool train, int dtype) {
  if (!tok) return fail(TIDE_ERR_NULL, "tok is NULL");
  if (!tok->embed || !tok->input_ids || !tok->w_in) return fail(TIDE_ERR_NULL, "tok.embed, tok.input_ids and tok.w_in must not be NULL");
  if (tok->embed_rows < 1) return fail(TIDE_ERR_CONFIG, "tok.embed_rows must be >= 1");
  if (train) {
    if (!tok->grad_w_in || !tok->m_w_in || !tok->v_w_in) return fail(TIDE_ERR_NULL, "tok.grad_w_in, tok.m_w_in and tok.v_w_in must not be NULL for a training step");
    if (dtype == TIDE_DTYPE_BF16 && !tok->master_w_in) return fail(TIDE_ERR_NULL, "tok.master_w_in must not be NULL in bf16 mode");
  }
  return TIDE_OK;
}

int check_common(const tide_draft_config* cfg, const tide_draft_tensors* params, const void* hidden_buf,
                 const int32_t* tokens, const uint8_t* loss_mask, float* loss_out, void* workspace,
                 size_t workspace_bytes, const Plan& p) {
  if (!tensors_ok(params, "params")) return TIDE_ERR_NULL;
  if (!hidden_buf || !tokens || !loss_mask || !loss_out) return fail(TIDE_ERR_NULL, "hidden_buf, tokens, loss_mask and loss_out must not be NULL");
  if (!workspace) return fail(TIDE_ERR_NULL, "workspace is NULL");
  if (((uintptr_t)workspace & 255) != 0) return fail(TIDE_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (workspace_bytes < p.total) return fail(TIDE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, p.total);
  (void)cfg;
  return TIDE_OK;
}

GemmArgs gemm_args(int layout, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                   int64_t ldb, void* C, int64_t ldc, int in_dt, int out_dt) {
  GemmArgs g;
  std::memset(&g, 0, sizeof(g));
  g.layout = layout; g.M = M; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
  g.alpha = 1.0f; g.in_dtype = in_dt; g.out_dtype = out_dt;
  return g;
}

// How the T = batch * seq rows split into sequences: the fixed layout (cu == nullptr: `n` sequences of
// `max_len` rows each) or a packed batch (cu = device offsets of n sequences, none longer than max_len;
// rows outside [cu[0], cu[n]) are padding).
struct Seqs {
  const int* cu;
  int n, max_len;
};

Seqs fixed_seqs(const tide_draft_config* c) { return Seqs{nullptr, c->batch, c->seq}; }

int check_packed(const tide_draft_config* c, const int32_t* cu_seqlens, int32_t n_seqs, int32_t max_seqlen) {
  if (!cu_seqlens) return fail(TIDE_ERR_NULL, "cu_seqlens is NULL");
  const int64_t T = (int64_t)c->batch * c->seq;
  if (n_seqs < 1 || n_seqs > 65535) return fail(TIDE_ERR_CONFIG, "n_seqs must be in [1, 65535]");
  if (max_seqlen < 1 || max_seqlen > T) return fail(TIDE_ERR_CONFIG, "max_seqlen must be in [1, batch*seq]");
  return TIDE_OK;
}

AttnArgs attn_args(const tide_draft_config* c, const Seqs& q, char* ws, const Plan& p) {
  AttnArgs at;
  std::memset(&at, 0, sizeof(at));
  at.B = q.n; at.S = q.max_len; at.nh = c->n_heads; at.nkv = c->n_kv_heads; at.dh = c->head_dim;
  at.qkv = ws + p.qkv; at.out = ws + p.A; at.lse = (float*)(ws + p.attn_lse); at.dtype = c->dtype;
  at.cu_seqlens = q.cu; at.total_rows = p.T;
  return at;
}

// RoPE over all T rows: position = row % seq in the fixed layout, the planned per-row position when packed
int enqueue_rope(const tide_draft_config* c, const Seqs& q, char* ws, const Plan& p, void* qkv, int inverse, int pos_offset, hipStream_t s) {
  const float* cs = (const float*)(ws + p.rope_cs);
  if (q.cu) TIDE_HIP(launch_rope(1, (int)p.T, c->n_heads, c->n_kv_heads, c->head_dim, cs, qkv, inverse, c->dtype, (const int32_t*)(ws + p.seq_pos), pos_offset, s), "rope");
  else TIDE_HIP(launch_rope(c->batch, c->seq, c->n_heads, c->n_kv_heads, c->head_dim, cs, qkv, inverse, c->dtype, nullptr, pos_offset, s), "rope");
  return TIDE_OK;
}

// One step of the multi-step unroll (fixed layout only).  Step `shift + 1` works in its own workspace; tokens,
// mask and the token input handed to enqueue_trunk are already the shifted ones.
struct UnrollStep {
  int shift;                    // 0 for the first step
  int n_steps;
  const uint8_t* sel;           // rows that carry loss at this or a later step
  const char* prev_ws;          // workspace of the step before (its x2 and row_pos feed this step); shift > 0
  const char* first_ws;         // workspace of step 1 (its keys and values); shift > 0
  char* own_kv[kMaxUnroll];     // [T, 2 nk] own key/value pairs of steps 2 .. shift + 1 (the last one is written here)
};

// Forward pass up to the final RMSNorm (everything except the LM head).
int enqueue_trunk(const tide_draft_config* c, const tide_draft_tensors* P, const tide_token_input* tok,
                  const void* hidden_buf, const int32_t* tokens, const uint8_t* mask, int select_all, const Seqs& q,
                  char* ws, const Plan& p, hipStream_t s, const UnrollStep* ur = nullptr) {
  const int dt = c->dtype;
  const int64_t T = p.T;
  float* scal = (float*)(ws + p.scal);
  const int shift = ur ? ur->shift : 0;
  TIDE_HIP(launch_plan_rows(tokens, mask, T, c->vocab, select_all, scal, (int*)(ws + p.cnt), (int32_t*)(ws + p.kept_idx), (int32_t*)(ws + p.row_pos), q.cu, q.n, q.max_len, (uint8_t*)(ws + p.mask_eff), (int*)(ws + p.status), (int*)(ws + p.plan_cnt), ur ? ur->sel : nullptr, s), "plan_rows");
  if (q.cu) TIDE_HIP(launch_seq_pos(q.cu, q.n, T, q.max_len, (int32_t*)(ws + p.seq_pos), s), "sequence positions");
  if (shift > 0) {
    // the feature of a later step is the layer output of the step before (dense over that step's selected
    // rows; rows it did not select carry no loss from here on and get zeros)
    void* feat = tok ? ws + p.g0 : ws + p.x0;
    TIDE_HIP(launch_scatter_rows(T, (int)p.d, ur->prev_ws + p.x2, feat, 0, nullptr, nullptr, (const int32_t*)(ur->prev_ws + p.row_pos), dt, s), "scatter features");
    if (tok) {
      TIDE_HIP(launch_embed_rows(T, (int)p.d, tok->embed, tok->embed_rows, tok->input_ids, ws + p.e0, dt, s), "embed rows");
      GemmArgs g = gemm_args(kNT, T, p.d, p.d, ws + p.g0, p.d, tok->w_in, 2 * p.d, ws + p.x0, p.d, dt, dt);
      g.A2 = ws + p.e0; g.B2 = (const char*)tok->w_in + (size_t)p.d * p.es; g.K2 = p.d;
      TIDE_HIP(launch_gemm(g, s), "gemm in");
    }
  } else if (!tok) {
    // x0 = Hcat W_fc^T
    TIDE_HIP(launch_gemm(gemm_args(kNT, T, p.d, p.KH, hidden_buf, p.KH, P->w_fc, p.KH, ws + p.x0, p.d, dt, dt), s), "gemm fc");
  } else {
    // token-input variant: g = Hcat W_fc^T, e = embed[input_ids], x0 = [g ; e] W_in^T as ONE contraction over
    // the two operand pairs (g, W_in[:, :d]) and (e, W_in[:, d:]); W_in's row stride is 2d for both halves
    TIDE_HIP(launch_gemm(gemm_args(kNT, T, p.d, p.KH, hidden_buf, p.KH, P->w_fc, p.KH, ws + p.g0, p.d, dt, dt), s), "gemm fc");
    TIDE_HIP(launch_embed_rows(T, (int)p.d, tok->embed, tok->embed_rows, tok->input_ids, ws + p.e0, dt, s), "embed rows");
    GemmArgs g = gemm_args(kNT, T, p.d, p.d, ws + p.g0, p.d, tok->w_in, 2 * p.d, ws + p.x0, p.d, dt, dt);
    g.A2 = ws + p.e0; g.B2 = (const char*)tok->w_in + (size_t)p.d * p.es; g.K2 = p.d;
    TIDE_HIP(launch_gemm(g, s), "gemm in");
  }
  TIDE_HIP(launch_rmsnorm_fwd(T, (int)p.d, ws + p.x0, P->g1, c->rms_eps, ws + p.a, (float*)(ws + p.r1), dt, nullptr, s), "rmsnorm1");
  TIDE_HIP(launch_gemm(gemm_args(kNT, T, p.nqkv, p.d, ws + p.a, p.d, P->w_qkv, p.d, ws + p.qkv, p.nqkv, dt, dt), s), "gemm qkv");
  TIDE_HIP(launch_rope_table(q.max_len + shift, c->head_dim, c->rope_theta, (float*)(ws + p.rope_cs), s), "rope table");
  { const int rc = enqueue_rope(c, q, ws, p, ws + p.qkv, 0, shift, s); if (rc) return rc; }
  // later step of the unroll: keep the step's own key/value pair aside and attend to the step-1 keys/values
  if (shift > 0) TIDE_HIP(launch_kv_swap(T, (int)p.nq, (int)p.nk, ws + p.qkv, ur->first_ws + p.qkv, ur->own_kv[shift - 1], dt, s), "kv swap");
  {
    const AttnArgs at = attn_args(c, q, ws, p);
    TIDE_HIP(launch_attn_fwd(at, s), "attention fwd");
    if (shift > 0) {
      OwnKV own;
      for (int j = 0; j < kMaxUnroll; ++j) own.kv[j] = j < shift ? ur->own_kv[j] : nullptr;
      TIDE_HIP(launch_own_kv_merge_fwd(T, c->seq, c->n_heads, c->n_kv_heads, c->head_dim, ws + p.qkv, ws + p.A, (float*)(ws + p.attn_lse), own, shift, q.cu != nullptr, dt, s), "own kv merge");
    }
    // padding rows are written by no sequence: make them finite (they enter weight-gradient contractions)
    if (q.cu) TIDE_HIP(launch_zero_padding_rows(ws + p.A, q.cu, q.n, T, (int64_t)(p.nq * p.es), s), "zero padding rows");
  }
  // Only the selected rows go on (see gather_rows): their number *cnt is known on the device alone, so every
  // launch below is sized for T rows and trims itself.
  const int* cnt = (const int*)(ws + p.cnt);
  TIDE_HIP(launch_gather_rows(T, (int)p.nq, ws + p.A, ws + p.A_c, (int)p.d, ws + p.x0, ws + p.x0_c, tokens, (const uint8_t*)(ws + p.mask_eff),
                              (const int32_t*)(ws + p.kept_idx), cnt, (int32_t*)(ws + p.tokens_c), (uint8_t*)(ws + p.mask_c), dt, s), "gather rows");
  auto rows_gemm = [&](int layout, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc) {
    GemmArgs g = gemm_args(layout, T, N, K, A, lda, B, ldb, C, ldc, dt, dt);
    g.m_dev = cnt;
    return g;
  };
  // x1 = x0 + A W_o^T
  {
    GemmArgs g = rows_gemm(kNT, p.d, p.nq, ws + p.A_c, p.nq, P->w_o, p.nq, ws + p.x1, p.d);
    g.residual = ws + p.x0_c; g.ldr = p.d;
    TIDE_HIP(launch_gemm(g, s), "gemm o");
  }
  TIDE_HIP(launch_rmsnorm_fwd(T, (int)p.d, ws + p.x1, P->g2, c->rms_eps, ws + p.bn, (float*)(ws + p.r2), dt, cnt, s), "rmsnorm2");
  TIDE_HIP(launch_gemm(rows_gemm(kNT, p.F, p.d, ws + p.bn, p.d, P->w_gate, p.d, ws + p.gt, p.F), s), "gemm gate");
  TIDE_HIP(launch_gemm(rows_gemm(kNT, p.F, p.d, ws + p.bn, p.d, P->w_up, p.d, ws + p.u, p.F), s), "gemm up");
  TIDE_HIP(launch_swiglu_fwd(T * p.F, ws + p.gt, ws + p.u, ws + p.h, dt, p.F, cnt, s), "swiglu");
  {
    GemmArgs g = rows_gemm(kNT, p.d, p.F, ws + p.h, p.F, P->w_down, p.F, ws + p.x2, p.d);
    g.residual = ws + p.x1; g.ldr = p.d;
    TIDE_HIP(launch_gemm(g, s), "gemm down");
  }
  TIDE_HIP(launch_rmsnorm_fwd(T, (int)p.d, ws + p.x2, P->g3, c->rms_eps, ws + p.yhat, (float*)(ws + p.r3), dt, cnt, s), "rmsnorm3");
  return TIDE_OK;
}

// LM head by row blocks over the selected rows (those that carry loss; every row when arg-max ids are wanted):
// logits of one block (bf16), row statistics, and (training) the logit gradient written over them and the
// product dyhat that consumes it.  Logits exist for one block at a time: a forward-only call reuses one block
// region; a training call turns each block into its gradient before the next block's logits are computed, and
// keeps those bf16 gradients of all blocks (when the buffer may hold them) so that dW_lm is ONE product over
// all rows afterwards.  fp32 logits or probabilities of [rows, V] never exist.  The number of compacted rows
// lives on the device, so every launch is sized for the worst case and trims itself.
int enqueue_lm_head(const tide_draft_config* c, const tide_draft_tensors* P, tide_draft_tensors* G,
                    const int32_t* tokens, const uint8_t* mask, int32_t* top1, float* loss_out, float* acc_out,
                    char* ws, const Plan& p, bool train, hipStream_t s, float grad_weight = 1.f, bool add_to_dw = false) {
  const int dt = c->dtype;
  float* scal = (float*)(ws + p.scal);
  const int* cnt = (const int*)(ws + p.cnt);
  const int32_t* kept_idx = (const int32_t*)(ws + p.kept_idx);
  const int32_t* tokens_c = (const int32_t*)(ws + p.tokens_c);
  const uint8_t* mask_c = (const uint8_t*)(ws + p.mask_c);
  float* lse = (float*)(ws + p.lse);
  float* loss_rows = (float*)(ws + p.loss_rows);
  float* hit_rows = acc_out ? (float*)(ws + p.hit_rows) : nullptr;
  char* yhat_c = ws + p.yhat;   // dense over the selected rows, as everything after the attention
  (void)tokens; (void)mask;
  const bool all_rows = p.z_rows >= p.T;   // the logit buffer holds every row (see make_plan)
  int blk = 0;
  for (int64_t r0 = 0; r0 < p.T; r0 += p.lm_rows, ++blk) {
    const int64_t rows = (p.T - r0 < p.lm_rows) ? (p.T - r0) : p.lm_rows;
    const char* yb = yhat_c + (size_t)r0 * p.d * p.es;
    char* z = ws + p.z + ((all_rows && train) ? (size_t)r0 * p.ldz * p.es : 0);
    {
      GemmArgs g = gemm_args(kNT, rows, p.V, p.d, yb, p.d, P->w_lm, p.d, z, p.ldz, dt, dt);
      g.m_dev = cnt; g.m_off = r0;
      TIDE_HIP(launch_gemm(g, s), "gemm lm_head");
    }
    if (train) {
      TIDE_HIP(launch_ce_train(rows, (int)p.V, z, p.ldz, tokens_c + r0, mask_c + r0, lse + r0, loss_rows + r0, cnt, r0, dt, s), "ce train");
    } else {
      TIDE_HIP(launch_ce_stats(rows, (int)p.V, z, p.ldz, tokens_c + r0, mask_c + r0, lse + r0, loss_rows + r0, top1, top1 ? kept_idx + r0 : nullptr, hit_rows ? hit_rows + r0 : nullptr, cnt, r0, dt, s), "ce stats");
      continue;
    }
    {
      // dyhat = (1/N) dZ W_lm
      GemmArgs g = gemm_args(kNN, rows, p.d, p.V, z, p.ldz, P->w_lm, p.d, ws + p.dyhat + (size_t)r0 * p.d * p.es, p.d, dt, dt);
      g.alpha = grad_weight; g.alpha_dev = scal + 1;
      g.m_dev = cnt; g.m_off = r0;
      TIDE_HIP(launch_gemm(g, s), "gemm dyhat");
    }
    if (!all_rows) {
      // dW_lm (+)= (1/N) dZ^T yhat of this block
      GemmArgs g = gemm_args(kTN, p.V, p.d, rows, z, p.ldz, yb, p.d, G->w_lm, p.d, dt, kF32);
      g.alpha = grad_weight; g.alpha_dev = scal + 1;
      g.accumulate = blk > 0 || add_to_dw;
      g.k_dev = cnt; g.k_off = r0;
      g.scratch = ws + p.splitk; g.scratch_bytes = p.splitk_bytes;
      TIDE_HIP(launch_gemm(g, s), "gemm dW_lm");
    }
  }
  if (train && all_rows) {
    // dW_lm = (1/N) dZ^T yhat over all selected rows at once
    GemmArgs g = gemm_args(kTN, p.V, p.d, p.T, ws + p.z, p.ldz, yhat_c, p.d, G->w_lm, p.d, dt, kF32);
    g.alpha = grad_weight; g.alpha_dev = scal + 1;
    g.accumulate = add_to_dw;
    g.k_dev = cnt; g.k_off = 0;
    g.scratch = ws + p.splitk; g.scratch_bytes = p.splitk_bytes;
    TIDE_HIP(launch_gemm(g, s), "gemm dW_lm");
  }
  TIDE_HIP(launch_loss_reduce(loss_rows, hit_rows, cnt, scal, loss_out, acc_out, (int*)(ws + p.status), s), "loss reduce");
  return TIDE_OK;
}

}  // namespace

extern "C" {

const char* tide_last_error(void) { return g_err; }

size_t tide_draft_workspace_bytes(const tide_draft_config* cfg) {
  if (!check_config(cfg)) return 0;
  return make_plan(cfg).total;
}

// Byte offset of a named intermediate inside the workspace (for tests and profiling); -1 if unknown.
int64_t tide_draft_workspace_offset(const tide_draft_config* cfg, const char* name) {
  if (!check_config(cfg) || !name) return -1;
  const Plan p = make_plan(cfg);
  struct { const char* n; size_t o; } tab[] = {
      {"scal", p.scal}, {"status", p.status}, {"x0", p.x0}, {"r1", p.r1}, {"a", p.a}, {"qkv", p.qkv}, {"attn_lse", p.attn_lse},
      {"A", p.A}, {"x1", p.x1}, {"r2", p.r2}, {"bn", p.bn}, {"gt", p.gt}, {"u", p.u}, {"h", p.h},
      {"x2", p.x2}, {"r3", p.r3}, {"yhat", p.yhat}, {"lse", p.lse}, {"loss_rows", p.loss_rows}, {"z", p.z},
      {"dyhat", p.dyhat}, {"A_c", p.A_c}, {"x0_c", p.x0_c}, {"dx1_c", p.dx1_c}, {"dA_c", p.dA_c}, {"row_pos", p.row_pos}, {"cnt", p.cnt}, {"kept_idx", p.kept_idx}, {"dx2", p.dx2}, {"dx1", p.dx1}, {"dx0", p.dx0}, {"dh", p.dh}, {"dbn", p.dbn},
      {"dA", p.dA}, {"dqkv", p.dqkv}, {"da", p.da}, {"g0", p.g0}, {"e0", p.e0}, {"dg0", p.dg0}};
  for (auto& e : tab)
    if (std::strcmp(e.n, name) == 0) return (int64_t)e.o;
  if (std::strcmp(name, "lm_rows") == 0) return p.lm_rows;
  return -1;
}

static int forward_impl(const tide_draft_config* cfg, const tide_draft_tensors* params, const tide_token_input* tok,
                        const void* hidden_buf,
                        const int32_t* tokens, const uint8_t* loss_mask, const Seqs* packed, float* loss_out,
                        int32_t* top1_out, float* accuracy_out, void* workspace, size_t workspace_bytes, void* stream) {
  const Plan p = make_plan(cfg);
  int rc = check_common(cfg, params, hidden_buf, tokens, loss_mask, loss_out, workspace, workspace_bytes, p);
  if (rc) return rc;
  const Seqs q = packed ? *packed : fixed_seqs(cfg);
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  rc = enqueue_trunk(cfg, params, tok, hidden_buf, tokens, loss_mask, top1_out != nullptr, q, ws, p, s);
  if (rc) return rc;
  return enqueue_lm_head(cfg, params, nullptr, tokens, loss_mask, top1_out, loss_out, accuracy_out, ws, p, false, s);
}

int tide_draft_forward(const tide_draft_config* cfg, const tide_draft_tensors* params, const void* hidden_buf,
                       const int32_t* tokens, const uint8_t* loss_mask, float* loss_out, int32_t* top1_out,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  return forward_impl(cfg, params, nullptr, hidden_buf, tokens, loss_mask, nullptr, loss_out, top1_out, nullptr, workspace, workspace_bytes, stream);
}

int tide_draft_forward_packed(const tide_draft_config* cfg, const tide_draft_tensors* params, const void* hidden_buf,
                              const int32_t* tokens, const uint8_t* loss_mask, const int32_t* cu_seqlens,
                              int32_t n_seqs, int32_t max_seqlen, float* loss_out, int32_t* top1_out,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  const int rc = check_packed(cfg, cu_seqlens, n_seqs, max_seqlen);
  if (rc) return rc;
  const Seqs q{cu_seqlens, n_seqs, max_seqlen};
  return forward_impl(cfg, params, nullptr, hidden_buf, tokens, loss_mask, &q, loss_out, top1_out, nullptr, workspace, workspace_bytes, stream);
}

int tide_draft_eval(const tide_draft_config* cfg, const tide_draft_tensors* params, const void* hidden_buf,
                    const int32_t* tokens, const uint8_t* loss_mask, float* loss_out, float* accuracy_out,
                    void* workspace, size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  if (!accuracy_out) return fail(TIDE_ERR_NULL, "accuracy_out is NULL");
  return forward_impl(cfg, params, nullptr, hidden_buf, tokens, loss_mask, nullptr, loss_out, nullptr, accuracy_out, workspace, workspace_bytes, stream);
}

// ---- multi-step evaluation unroll -----------------------------------------------------------------
namespace {
struct UnrollPlan {
  size_t step_bytes;                    // one workspace per step
  size_t tokens_s, mask_s, sel_s, ids_s, own_kv, own_grad, dfeat, acc_kv1;   // per-step extras (offset of step 0; stride extra_stride)
  size_t extra_stride, total;
};
UnrollPlan make_unroll_plan(const Plan& p, int n_steps) {
  UnrollPlan u;
  u.step_bytes = align_up(p.total, 256);
  Bump b;
  const size_t T = (size_t)p.T;
  u.tokens_s = b.take(T * 4);
  u.mask_s = b.take(T);
  u.sel_s = b.take(T);
  u.ids_s = b.take(T * 4);
  u.own_kv = b.take(T * 2 * (size_t)p.nk * p.es);
  u.own_grad = b.take(T * 2 * (size_t)p.nk * p.es);   // training: gradient of the step's own key/value pair
  u.dfeat = b.take(T * (size_t)p.d * p.es);           // training: gradient reaching x2 from the step after
  u.acc_kv1 = b.take(T * 2 * (size_t)p.nk * p.es);    // training: running step-1 key/value gradient (step 0's is used)
  u.extra_stride = b.off;
  u.total = (u.step_bytes + u.extra_stride) * (size_t)n_steps;
  return u;
}
}  // namespace

size_t tide_draft_unroll_workspace_bytes(const tide_draft_config* cfg, int32_t n_steps) {
  if (!check_config(cfg)) return 0;
  if (n_steps < 1 || n_steps > kMaxUnroll) { fail(TIDE_ERR_CONFIG, "n_steps must be in [1, %d]", kMaxUnroll); return 0; }
  return make_unroll_plan(make_plan(cfg), n_steps).total;
}

// Byte offset inside the unroll workspace: of a single-step intermediate of step `step` (names as in
// tide_draft_workspace_offset), or of one of the step's extras; -1 if unknown.
int64_t tide_draft_unroll_workspace_offset(const tide_draft_config* cfg, int32_t n_steps, int32_t step, const char* name) {
  if (!check_config(cfg) || !name || n_steps < 1 || n_steps > kMaxUnroll || step < 0 || step >= n_steps) return -1;
  const UnrollPlan u = make_unroll_plan(make_plan(cfg), n_steps);
  const size_t extra = u.step_bytes * (size_t)n_steps + u.extra_stride * (size_t)step;
  struct { const char* n; size_t o; } tab[] = {{"tokens_s", u.tokens_s}, {"mask_s", u.mask_s}, {"sel_s", u.sel_s}, {"ids_s", u.ids_s},
                                               {"own_kv", u.own_kv}, {"own_grad", u.own_grad}, {"dfeat", u.dfeat}, {"acc_kv1", u.acc_kv1}};
  for (auto& e : tab)
    if (std::strcmp(e.n, name) == 0) return (int64_t)(extra + e.o);
  const int64_t o = tide_draft_workspace_offset(cfg, name);
  return o < 0 ? -1 : (int64_t)(u.step_bytes * (size_t)step) + o;
}

static int eval_unroll_impl(const tide_draft_config* cfg, const tide_draft_tensors* params, const tide_token_input* tok,
                            const void* hidden_buf, const int32_t* tokens, const uint8_t* loss_mask, const Seqs* packed,
                            int32_t n_steps, float* loss_out, float* accuracy_out, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (n_steps < 1 || n_steps > kMaxUnroll) return fail(TIDE_ERR_CONFIG, "n_steps must be in [1, %d]", kMaxUnroll);
  if (!accuracy_out) return fail(TIDE_ERR_NULL, "accuracy_out is NULL");
  if (tok) { const int rc = check_token_input(tok, false, cfg->dtype); if (rc) return rc; }
  const Plan p = make_plan(cfg);
  const UnrollPlan u = make_unroll_plan(p, n_steps);
  {
    const int rc = check_common(cfg, params, hidden_buf, tokens, loss_mask, loss_out, workspace, u.step_bytes, p);
    if (rc) return rc;
  }
  if (workspace_bytes < u.total) return fail(TIDE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, u.total);
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  char* extra = ws + u.step_bytes * (size_t)n_steps;
  const Seqs q = packed ? *packed : fixed_seqs(cfg);
  UnrollStep ur;
  std::memset(&ur, 0, sizeof(ur));
  ur.n_steps = n_steps;
  for (int k = 0; k < n_steps; ++k) {
    char* wk = ws + u.step_bytes * (size_t)k;
    char* ek = extra + u.extra_stride * (size_t)k;
    int32_t* tokens_s = (int32_t*)(ek + u.tokens_s);
    uint8_t* mask_s = (uint8_t*)(ek + u.mask_s);
    uint8_t* sel_s = (uint8_t*)(ek + u.sel_s);
    int32_t* ids_s = tok ? (int32_t*)(ek + u.ids_s) : nullptr;
    TIDE_HIP(launch_shift_inputs(tokens, loss_mask, tok ? tok->input_ids : nullptr, p.T, cfg->seq, cfg->vocab, k, n_steps, tokens_s, mask_s, sel_s, ids_s, q.cu, q.n, s), "shift inputs");
    tide_token_input tk;
    if (tok) { tk = *tok; tk.input_ids = ids_s; }
    ur.shift = k;
    ur.sel = sel_s;
    ur.prev_ws = k ? ws + u.step_bytes * (size_t)(k - 1) : nullptr;
    ur.first_ws = ws;
    if (k) ur.own_kv[k - 1] = ek + u.own_kv;
    int rc = enqueue_trunk(cfg, params, tok ? &tk : nullptr, hidden_buf, tokens_s, mask_s, 0, q, wk, p, s, &ur);
    if (rc) return rc;
    rc = enqueue_lm_head(cfg, params, nullptr, tokens_s, mask_s, nullptr, loss_out + k, accuracy_out + k, wk, p, false, s);
    if (rc) return rc;
  }
  return TIDE_OK;
}

// What the backward pass of one step of the multi-step unroll needs beyond the single-step one.
struct BwdOpts {
  int accumulate = 0;               // weight and gain gradients are added to what the buffers hold
  const UnrollStep* ur = nullptr;   // nullptr: the ordinary single step
  const void* dx2_extra = nullptr;  // dense over the selected rows: gradient reaching x2 from the step after
  OwnKVGrad own_grad{};             // gradient buffers of the own key/value pairs of steps 2 .. n
  char* acc_kv1 = nullptr;          // running gradient of the step-1 keys/values [T, 2 nk]
  // shift > 0: where the gradient of this step's input feature goes (dense over the selected rows of the step
  // before, whose workspace and shifted tokens are given)
  void* dfeat_out = nullptr;
  char* prev_ws = nullptr;
  const int32_t* prev_tokens = nullptr;
};

// Backward pass of one step from dyhat (left by the LM head) to the weight gradients.
static int enqueue_backward(const tide_draft_config* cfg, const tide_draft_tensors* P, tide_draft_tensors* G,
                            const tide_token_input* tok, const void* hidden_buf, const Seqs& q, char* ws, const Plan& p,
                            hipStream_t s, const BwdOpts& o) {
  const int dt = cfg->dtype;
  const int64_t T = p.T;
  const int acc = o.accumulate;
  const int shift = o.ur ? o.ur->shift : 0;
  float* dgp = (float*)(ws + p.dg_partial);
  const int* cnt = (const int*)(ws + p.cnt);
  // Backward over the selected rows (dense, *cnt of them) down to the attention output.  dX products trim
  // their M, dW products their K.
  auto rows_dx = [&](int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc) {
    GemmArgs g = gemm_args(kNN, T, N, K, A, lda, B, ldb, C, ldc, dt, dt);
    g.m_dev = cnt;
    return g;
  };
  auto rows_dw = [&](int64_t M, int64_t N, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc) {
    GemmArgs g = gemm_args(kTN, M, N, T, A, lda, B, ldb, C, ldc, dt, kF32);
    g.k_dev = cnt;
    g.accumulate = acc;
    g.scratch = ws + p.splitk; g.scratch_bytes = p.splitk_bytes;
    return g;
  };
  auto full_dw = [&](int64_t M, int64_t N, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc, int add) {
    GemmArgs g = gemm_args(kTN, M, N, T, A, lda, B, ldb, C, ldc, dt, kF32);
    g.accumulate = add;
    g.scratch = ws + p.splitk; g.scratch_bytes = p.splitk_bytes;
    return g;
  };
  // final norm (plus, in the unroll, what the step after sends back into x2)
  TIDE_HIP(launch_rmsnorm_bwd(T, (int)p.d, ws + p.dyhat, ws + p.x2, P->g3, (const float*)(ws + p.r3), o.dx2_extra, ws + p.dx2, (float*)G->g3, dgp, dt, cnt, s, acc), "rmsnorm3 bwd");
  // x2 = x1 + h W_down^T
  TIDE_HIP(launch_gemm(rows_dx(p.F, p.d, ws + p.dx2, p.d, P->w_down, p.F, ws + p.dh, p.F), s), "gemm dh");
  TIDE_HIP(launch_gemm(rows_dw(p.d, p.F, ws + p.dx2, p.d, ws + p.h, p.F, G->w_down, p.F), s), "gemm dW_down");
  TIDE_HIP(launch_swiglu_bwd(T * p.F, ws + p.dh, ws + p.gt, ws + p.u, ws + p.gt, ws + p.u, dt, p.F, cnt, s), "swiglu bwd");
  {
    // d bn = dGate W_gate + dUp W_up: one contraction over both operand pairs
    GemmArgs g = rows_dx(p.d, p.F, ws + p.gt, p.F, P->w_gate, p.d, ws + p.dbn, p.d);
    g.A2 = ws + p.u; g.B2 = P->w_up; g.K2 = p.F;
    TIDE_HIP(launch_gemm(g, s), "gemm dbn");
  }
  TIDE_HIP(launch_gemm(rows_dw(p.F, p.d, ws + p.gt, p.F, ws + p.bn, p.d, G->w_gate, p.d), s), "gemm dW_gate");
  TIDE_HIP(launch_gemm(rows_dw(p.F, p.d, ws + p.u, p.F, ws + p.bn, p.d, G->w_up, p.d), s), "gemm dW_up");
  TIDE_HIP(launch_rmsnorm_bwd(T, (int)p.d, ws + p.dbn, ws + p.x1, P->g2, (const float*)(ws + p.r2), ws + p.dx2, ws + p.dx1_c, (float*)G->g2, dgp, dt, cnt, s, acc), "rmsnorm2 bwd");
  // x1 = x0 + A W_o^T
  TIDE_HIP(launch_gemm(rows_dx(p.nq, p.d, ws + p.dx1_c, p.d, P->w_o, p.nq, ws + p.dA_c, p.nq), s), "gemm dA");
  TIDE_HIP(launch_gemm(rows_dw(p.d, p.nq, ws + p.dx1_c, p.d, ws + p.A_c, p.nq, G->w_o, p.nq), s), "gemm dW_o");
  // back to one row per position: rows that were not selected get no gradient from above (only, through
  // the attention, from the later rows that read their key and value)
  TIDE_HIP(launch_scatter_rows(T, (int)p.nq, ws + p.dA_c, ws + p.dA, (int)p.d, ws + p.dx1_c, ws + p.dx1, (const int32_t*)(ws + p.row_pos), dt, s), "scatter rows");
  {
    AttnArgs at = attn_args(cfg, q, ws, p);
    at.dout = ws + p.dA; at.delta = (float*)(ws + p.delta); at.dqkv = ws + p.dqkv;
    TIDE_HIP(launch_attn_bwd(at, s), "attention bwd");
  }
  if (o.ur && shift > 0) {
    // later step of the unroll: the flash backward saw the step's queries beside the STEP-1 keys/values.  Add the
    // own pairs' share, move the step-1 share to its running sum and put this step's own pair gradient (complete
    // now: every later step ran before) in its place.
    OwnKV own;
    for (int j = 0; j < kMaxUnroll; ++j) own.kv[j] = j < shift ? o.ur->own_kv[j] : nullptr;
    const int last = shift == o.ur->n_steps - 1;
    TIDE_HIP(launch_own_kv_merge_bwd(T, cfg->seq, cfg->n_heads, cfg->n_kv_heads, cfg->head_dim, ws + p.qkv, ws + p.dA, (const float*)(ws + p.attn_lse), (const float*)(ws + p.delta), own, o.own_grad, shift, last, ws + p.dqkv, q.cu != nullptr, dt, s), "own kv merge bwd");
    TIDE_HIP(launch_kv_grad_route(T, (int)p.nq, (int)p.nk, ws + p.dqkv, o.acc_kv1, o.own_grad.kv[shift - 1], last ? 0 : 1, dt, s), "kv grad route");
  } else if (o.ur && o.ur->n_steps > 1) {
    TIDE_HIP(launch_kv_grad_route(T, (int)p.nq, (int)p.nk, ws + p.dqkv, o.acc_kv1, nullptr, 2, dt, s), "kv grad route");
  }
  // padding rows of a packed batch are written by no sequence (or hold whatever the merge made of them): make
  // them zero before the contractions over all rows
  if (q.cu) TIDE_HIP(launch_zero_padding_rows(ws + p.dqkv, q.cu, q.n, T, (int64_t)(p.nqkv * p.es), s), "zero padding rows");
  { const int rc2 = enqueue_rope(cfg, q, ws, p, ws + p.dqkv, 1, shift, s); if (rc2) return rc2; }
  TIDE_HIP(launch_gemm(gemm_args(kNN, T, p.d, p.nqkv, ws + p.dqkv, p.nqkv, P->w_qkv, p.d, ws + p.da, p.d, dt, dt), s), "gemm da");
  TIDE_HIP(launch_gemm(full_dw(p.nqkv, p.d, ws + p.dqkv, p.nqkv, ws + p.a, p.d, G->w_qkv, p.d, acc), s), "gemm dW_qkv");
  TIDE_HIP(launch_rmsnorm_bwd(T, (int)p.d, ws + p.da, ws + p.x0, P->g1, (const float*)(ws + p.r1), ws + p.dx1, ws + p.dx0, (float*)G->g1, dgp, dt, nullptr, s, acc), "rmsnorm1 bwd");
  const void* dfeat = ws + p.dx0;   // gradient of the step's input feature (feature-only model: x0 is the feature)
  if (tok) {
    // x0 = [g ; e] W_in^T: dW_in = dx0^T [g ; e] (two products into the column halves of dW_in), dg = dx0 W_in[:, :d]
    // (the embedding table is frozen)
    float* dwin = (float*)tok->grad_w_in;
    TIDE_HIP(launch_gemm(full_dw(p.d, p.d, ws + p.dx0, p.d, ws + p.g0, p.d, dwin, 2 * p.d, acc), s), "gemm dW_in (features)");
    TIDE_HIP(launch_gemm(full_dw(p.d, p.d, ws + p.dx0, p.d, ws + p.e0, p.d, dwin + p.d, 2 * p.d, acc), s), "gemm dW_in (embeddings)");
    TIDE_HIP(launch_gemm(gemm_args(kNN, T, p.d, p.d, ws + p.dx0, p.d, tok->w_in, 2 * p.d, ws + p.dg0, p.d, dt, dt), s), "gemm dg");
    dfeat = ws + p.dg0;
  }
  if (shift == 0) {
    // the feature is Hcat W_fc^T: weight gradient only, the captured states are data (step 1 is the only one
    // that reads W_fc, so this is never an accumulation)
    TIDE_HIP(launch_gemm(full_dw(p.d, p.KH, dfeat, p.d, hidden_buf, p.KH, G->w_fc, p.KH, 0), s), "gemm dW_fc");
  } else {
    // the feature is the layer output of the step before: hand its gradient over, dense over that step's rows
    TIDE_HIP(launch_gather_rows(T, (int)p.d, dfeat, o.dfeat_out, 0, nullptr, nullptr, o.prev_tokens, (const uint8_t*)(o.prev_ws + p.mask_eff),
                                (const int32_t*)(o.prev_ws + p.kept_idx), (const int*)(o.prev_ws + p.cnt), (int32_t*)(o.prev_ws + p.tokens_c),
                                (uint8_t*)(o.prev_ws + p.mask_c), dt, s), "gather feature gradient");
  }
  return TIDE_OK;
}

// AdamW over all tensors in one launch
// Device-resident schedule of a training step (the graph-capturable form): learning rate and step count live in
// device memory, are read by the kernels of the launch, and the count is advanced on the device.
struct DevSchedule { const float* lr; int64_t* step; float* dyn; };

static int enqueue_adamw(const tide_draft_config* cfg, tide_draft_tensors* params, tide_draft_tensors* G, tide_adam_state* st,
                         const tide_token_input* tok, float lr, const Plan& p, hipStream_t s,
                         const DevSchedule* dev = nullptr) {
  const int dt = cfg->dtype;
  AdamArgs a;
  std::memset(&a, 0, sizeof(a));
  void* pp[10] = {params->w_fc, params->g1, params->w_qkv, params->w_o, params->g2, params->w_gate, params->w_up, params->w_down, params->g3, params->w_lm};
  void* gg[10] = {G->w_fc, G->g1, G->w_qkv, G->w_o, G->g2, G->w_gate, G->w_up, G->w_down, G->g3, G->w_lm};
  void* mm[10] = {st->m.w_fc, st->m.g1, st->m.w_qkv, st->m.w_o, st->m.g2, st->m.w_gate, st->m.w_up, st->m.w_down, st->m.g3, st->m.w_lm};
  void* vv[10] = {st->v.w_fc, st->v.g1, st->v.w_qkv, st->v.w_o, st->v.g2, st->v.w_gate, st->v.w_up, st->v.w_down, st->v.g3, st->v.w_lm};
  void* ms[10] = {st->master.w_fc, st->master.g1, st->master.w_qkv, st->master.w_o, st->master.g2, st->master.w_gate, st->master.w_up, st->master.w_down, st->master.g3, st->master.w_lm};
  const int64_t nn[10] = {p.d * p.KH, p.d, p.nqkv * p.d, p.d * p.nq, p.d, p.F * p.d, p.F * p.d, p.d * p.F, p.d, p.V * p.d};
  for (int i = 0; i < 10; ++i) a.t[i] = AdamTensor{pp[i], (const float*)gg[i], (float*)mm[i], (float*)vv[i], dt == TIDE_DTYPE_BF16 ? (float*)ms[i] : nullptr, nn[i]};
  a.nt = 10;
  if (tok) {
    a.t[10] = AdamTensor{tok->w_in, (const float*)tok->grad_w_in, (float*)tok->m_w_in, (float*)tok->v_w_in,
                         dt == TIDE_DTYPE_BF16 ? (float*)tok->master_w_in : nullptr, 2 * p.d * p.d};
    a.nt = 11;
  }
  a.beta1 = cfg->beta1; a.beta2 = cfg->beta2; a.eps = cfg->adam_eps; a.wd = cfg->weight_decay;
  a.dtype = dt;
  if (dev) {
    TIDE_HIP(launch_adam_schedule(dev->lr, dev->step, cfg->beta1, cfg->beta2, cfg->weight_decay, dev->dyn, s), "adam schedule");
    a.dyn = dev->dyn;
    TIDE_HIP(launch_adamw(a, s), "adamw");
    return TIDE_OK;
  }
  const long long t = (long long)(st->step + 1);
  a.lr = lr;
  a.inv_bc1 = (float)(1.0 / (1.0 - pow_int((double)cfg->beta1, t)));
  a.inv_sqrt_bc2 = (float)(1.0 / std::sqrt(1.0 - pow_int((double)cfg->beta2, t)));
  TIDE_HIP(launch_adamw(a, s), "adamw");
  st->step += 1;
  return TIDE_OK;
}

static int check_train_args(const tide_draft_config* cfg, tide_draft_tensors* grads, tide_adam_state* st, float lr) {
  if (!tensors_ok(grads, "grads")) return TIDE_ERR_NULL;
  if (!st) return fail(TIDE_ERR_NULL, "adam_state is NULL");
  if (!tensors_ok(&st->m, "adam_state.m") || !tensors_ok(&st->v, "adam_state.v")) return TIDE_ERR_NULL;
  if (cfg->dtype == TIDE_DTYPE_BF16 && !tensors_ok(&st->master, "adam_state.master")) return TIDE_ERR_NULL;
  if (st->step < 0) return fail(TIDE_ERR_CONFIG, "adam_state.step must be >= 0");
  if (!(lr >= 0.f)) return fail(TIDE_ERR_CONFIG, "lr must be >= 0");
  return TIDE_OK;
}

static int train_impl(const tide_draft_config* cfg, tide_draft_tensors* params, tide_draft_tensors* grads,
                      tide_adam_state* st, const tide_token_input* tok, const void* hidden_buf, const int32_t* tokens,
                      const uint8_t* loss_mask, const Seqs* packed, float lr, float* loss_out, void* workspace,
                      size_t workspace_bytes, void* stream, const float* lr_dev = nullptr, int64_t* step_dev = nullptr) {
  const Plan p = make_plan(cfg);
  const Seqs q = packed ? *packed : fixed_seqs(cfg);
  int rc = check_common(cfg, params, hidden_buf, tokens, loss_mask, loss_out, workspace, workspace_bytes, p);
  if (rc) return rc;
  rc = check_train_args(cfg, grads, st, lr);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  rc = enqueue_trunk(cfg, params, tok, hidden_buf, tokens, loss_mask, 0, q, ws, p, s);
  if (rc) return rc;
  rc = enqueue_lm_head(cfg, params, grads, tokens, loss_mask, nullptr, loss_out, nullptr, ws, p, true, s);
  if (rc) return rc;
  rc = enqueue_backward(cfg, params, grads, tok, hidden_buf, q, ws, p, s, BwdOpts{});
  if (rc) return rc;
  if (lr_dev) {
    const DevSchedule dev{lr_dev, step_dev, (float*)(ws + p.adam_dyn)};
    return enqueue_adamw(cfg, params, grads, st, tok, 0.f, p, s, &dev);
  }
  return enqueue_adamw(cfg, params, grads, st, tok, lr, p, s);
}

static int train_unroll_impl(const tide_draft_config* cfg, tide_draft_tensors* params, tide_draft_tensors* grads,
                             tide_adam_state* st, const tide_token_input* tok, const void* hidden_buf,
                             const int32_t* tokens, const uint8_t* loss_mask, const Seqs* packed, int32_t n_steps,
                             const float* step_weights, float lr, float* loss_out, void* workspace,
                             size_t workspace_bytes, void* stream) {
  if (n_steps < 1 || n_steps > kMaxUnroll) return fail(TIDE_ERR_CONFIG, "n_steps must be in [1, %d]", kMaxUnroll);
  if (tok) { const int rc = check_token_input(tok, true, cfg->dtype); if (rc) return rc; }
  if (step_weights)
    for (int k = 0; k < n_steps; ++k)
      if (!(step_weights[k] >= 0.f) || !std::isfinite(step_weights[k])) return fail(TIDE_ERR_CONFIG, "step_weights must be finite and >= 0");
  const Plan p = make_plan(cfg);
  const UnrollPlan u = make_unroll_plan(p, n_steps);
  int rc = check_common(cfg, params, hidden_buf, tokens, loss_mask, loss_out, workspace, u.step_bytes, p);
  if (rc) return rc;
  if (workspace_bytes < u.total) return fail(TIDE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, u.total);
  rc = check_train_args(cfg, grads, st, lr);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  char* extra = ws + u.step_bytes * (size_t)n_steps;
  const Seqs q = packed ? *packed : fixed_seqs(cfg);
  UnrollStep ur[kMaxUnroll];
  tide_token_input tk[kMaxUnroll];
  std::memset(ur, 0, sizeof(ur));
  // forward, step by step; the LM head of every step leaves dyhat in the step's workspace and adds its share of dW_lm
  for (int k = 0; k < n_steps; ++k) {
    char* wk = ws + u.step_bytes * (size_t)k;
    char* ek = extra + u.extra_stride * (size_t)k;
    int32_t* tokens_s = (int32_t*)(ek + u.tokens_s);
    uint8_t* mask_s = (uint8_t*)(ek + u.mask_s);
    uint8_t* sel_s = (uint8_t*)(ek + u.sel_s);
    int32_t* ids_s = tok ? (int32_t*)(ek + u.ids_s) : nullptr;
    TIDE_HIP(launch_shift_inputs(tokens, loss_mask, tok ? tok->input_ids : nullptr, p.T, cfg->seq, cfg->vocab, k, n_steps, tokens_s, mask_s, sel_s, ids_s, q.cu, q.n, s), "shift inputs");
    if (tok) { tk[k] = *tok; tk[k].input_ids = ids_s; }
    if (k) ur[k] = ur[k - 1];          // the own pairs of the steps before
    ur[k].shift = k;
    ur[k].n_steps = n_steps;
    ur[k].sel = sel_s;
    ur[k].prev_ws = k ? ws + u.step_bytes * (size_t)(k - 1) : nullptr;
    ur[k].first_ws = ws;
    if (k) ur[k].own_kv[k - 1] = ek + u.own_kv;
    rc = enqueue_trunk(cfg, params, tok ? &tk[k] : nullptr, hidden_buf, tokens_s, mask_s, 0, q, wk, p, s, &ur[k]);
    if (rc) return rc;
    rc = enqueue_lm_head(cfg, params, grads, tokens_s, mask_s, nullptr, loss_out + k, nullptr, wk, p, true, s,
                         step_weights ? step_weights[k] : 1.f, k > 0);
    if (rc) return rc;
  }
  // backward, last step first: a step's backward needs what every later step sends back into its output and
  // into its keys and values
  for (int k = n_steps - 1; k >= 0; --k) {
    char* wk = ws + u.step_bytes * (size_t)k;
    BwdOpts o;
    o.accumulate = k != n_steps - 1;
    o.ur = &ur[k];
    o.dx2_extra = k < n_steps - 1 ? extra + u.extra_stride * (size_t)k + u.dfeat : nullptr;
    for (int j = 0; j < kMaxUnroll; ++j) o.own_grad.kv[j] = j + 1 < n_steps ? extra + u.extra_stride * (size_t)(j + 1) + u.own_grad : nullptr;
    o.acc_kv1 = extra + u.acc_kv1;
    if (k) {
      char* ep = extra + u.extra_stride * (size_t)(k - 1);
      o.dfeat_out = ep + u.dfeat;
      o.prev_ws = ws + u.step_bytes * (size_t)(k - 1);
      o.prev_tokens = (const int32_t*)(ep + u.tokens_s);
    }
    rc = enqueue_backward(cfg, params, grads, tok ? &tk[k] : nullptr, hidden_buf, q, wk, p, s, o);
    if (rc) return rc;
  }
  return enqueue_adamw(cfg, params, grads, st, tok, lr, p, s);
}

int tide_draft_eval_unroll(const tide_draft_config* cfg, const tide_draft_tensors* params, const tide_token_input* tok,
                           const void* hidden_buf, const int32_t* tokens, const uint8_t* loss_mask, int32_t n_steps,
                           float* loss_out, float* accuracy_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  return eval_unroll_impl(cfg, params, tok, hidden_buf, tokens, loss_mask, nullptr, n_steps, loss_out, accuracy_out, workspace, workspace_bytes, stream);
}

int tide_draft_eval_unroll_packed(const tide_draft_config* cfg, const tide_draft_tensors* params, const tide_token_input* tok,
                                  const void* hidden_buf, const int32_t* tokens, const uint8_t* loss_mask,
                                  const int32_t* cu_seqlens, int32_t n_seqs, int32_t max_seqlen, int32_t n_steps,
                                  float* loss_out, float* accuracy_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  const int rc = check_packed(cfg, cu_seqlens, n_seqs, max_seqlen);
  if (rc) return rc;
  const Seqs q{cu_seqlens, n_seqs, max_seqlen};
  return eval_unroll_impl(cfg, params, tok, hidden_buf, tokens, loss_mask, &q, n_steps, loss_out, accuracy_out, workspace, workspace_bytes, stream);
}

int tide_draft_train_step_unroll(const tide_draft_config* cfg, tide_draft_tensors* params, tide_draft_tensors* grads,
                                 tide_adam_state* st, const tide_token_input* tok, const void* hidden_buf,
                                 const int32_t* tokens, const uint8_t* loss_mask, int32_t n_steps,
                                 const float* step_weights, float lr, float* loss_out, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  return train_unroll_impl(cfg, params, grads, st, tok, hidden_buf, tokens, loss_mask, nullptr, n_steps, step_weights, lr, loss_out, workspace, workspace_bytes, stream);
}

int tide_draft_train_step_unroll_packed(const tide_draft_config* cfg, tide_draft_tensors* params, tide_draft_tensors* grads,
                                        tide_adam_state* st, const tide_token_input* tok, const void* hidden_buf,
                                        const int32_t* tokens, const uint8_t* loss_mask, const int32_t* cu_seqlens,
                                        int32_t n_seqs, int32_t max_seqlen, int32_t n_steps, const float* step_weights,
                                        float lr, float* loss_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  const int rc = check_packed(cfg, cu_seqlens, n_seqs, max_seqlen);
  if (rc) return rc;
  const Seqs q{cu_seqlens, n_seqs, max_seqlen};
  return train_unroll_impl(cfg, params, grads, st, tok, hidden_buf, tokens, loss_mask, &q, n_steps, step_weights, lr, loss_out, workspace, workspace_bytes, stream);
}

int tide_draft_train_step(const tide_draft_config* cfg, tide_draft_tensors* params, tide_draft_tensors* grads,
                          tide_adam_state* st, const void* hidden_buf, const int32_t* tokens,
                          const uint8_t* loss_mask, float lr, float* loss_out, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  return train_impl(cfg, params, grads, st, nullptr, hidden_buf, tokens, loss_mask, nullptr, lr, loss_out, workspace, workspace_bytes, stream);
}

int tide_draft_train_step_dev(const tide_draft_config* cfg, tide_draft_tensors* params, tide_draft_tensors* grads,
                              tide_adam_state* st, const void* hidden_buf, const int32_t* tokens,
                              const uint8_t* loss_mask, const float* lr_dev, int64_t* step_dev, float* loss_out,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  if (!lr_dev || !step_dev) return fail(TIDE_ERR_NULL, "lr_dev and step_dev must not be NULL");
  return train_impl(cfg, params, grads, st, nullptr, hidden_buf, tokens, loss_mask, nullptr, 0.f, loss_out, workspace, workspace_bytes, stream, lr_dev, step_dev);
}

int tide_draft_forward_tok(const tide_draft_config* cfg, const tide_draft_tensors* params, const tide_token_input* tok,
                           const void* hidden_buf, const int32_t* tokens, const uint8_t* loss_mask, float* loss_out,
                           int32_t* top1_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  const int rc = check_token_input(tok, false, cfg->dtype);
  if (rc) return rc;
  return forward_impl(cfg, params, tok, hidden_buf, tokens, loss_mask, nullptr, loss_out, top1_out, nullptr, workspace, workspace_bytes, stream);
}

int tide_draft_train_step_tok(const tide_draft_config* cfg, tide_draft_tensors* params, tide_draft_tensors* grads,
                              tide_adam_state* st, const tide_token_input* tok, const void* hidden_buf,
                              const int32_t* tokens, const uint8_t* loss_mask, float lr, float* loss_out,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  const int rc = check_token_input(tok, true, cfg->dtype);
  if (rc) return rc;
  return train_impl(cfg, params, grads, st, tok, hidden_buf, tokens, loss_mask, nullptr, lr, loss_out, workspace, workspace_bytes, stream);
}

int tide_draft_train_step_packed(const tide_draft_config* cfg, tide_draft_tensors* params, tide_draft_tensors* grads,
                                 tide_adam_state* st, const void* hidden_buf, const int32_t* tokens,
                                 const uint8_t* loss_mask, const int32_t* cu_seqlens, int32_t n_seqs,
                                 int32_t max_seqlen, float lr, float* loss_out, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  if (!check_config(cfg)) return cfg ? TIDE_ERR_CONFIG : TIDE_ERR_NULL;
  const int rc = check_packed(cfg, cu_seqlens, n_seqs, max_seqlen);
  if (rc) return rc;
  const Seqs q{cu_seqlens, n_seqs, max_seqlen};
  return train_impl(cfg, params, grads, st, nullptr, hidden_buf, tokens, loss_mask, &q, lr, loss_out, workspace, workspace_bytes, stream);
}

// ---- building blocks ---------------------------------------------------------------------------
size_t tide_gemm_workspace_bytes(int layout, int64_t M, int64_t N, int64_t K, int out_dtype) {
  if (layout < 0 || layout > 2 || M <= 0 || N <= 0 || K <= 0) return 0;
  const int64_t lda = layout == kTN ? M : K, ldb = layout == kNT ? K : N;
  GemmArgs g = gemm_args(layout, M, N, K, (void*)256, lda, (void*)256, ldb, (void*)256, N, kBF16, out_dtype);
  return gemm_splitk_scratch_bytes(g);
}

int tide_gemm(int layout, int64_t M, int64_t N, int64_t K, float alpha, const void* A, const void* B, void* C,
              const void* residual, int in_dtype, int out_dtype, int accumulate, void* workspace,
              size_t workspace_bytes, void* stream) {
  if (!A || !B || !C) return fail(TIDE_ERR_NULL, "A, B and C must not be NULL");
  if (layout < 0 || layout > 2 || M <= 0 || N <= 0 || K <= 0) return fail(TIDE_ERR_CONFIG, "bad layout or sizes");
  if ((in_dtype != 0 && in_dtype != 1) || (out_dtype != 0 && out_dtype != 1) || (in_dtype == 0 && out_dtype == 1))
    return fail(TIDE_ERR_CONFIG, "unsupported dtype combination");
  const int64_t lda = layout == kTN ? M : K, ldb = layout == kNT ? K : N;
  GemmArgs g = gemm_args(layout, M, N, K, A, lda, B, ldb, C, N, in_dtype, out_dtype);
  g.alpha = alpha; g.residual = residual; g.ldr = N; g.accumulate = accumulate;
  if (workspace && (((uintptr_t)workspace) & 15) == 0) { g.scratch = workspace; g.scratch_bytes = workspace_bytes; }
  TIDE_HIP(launch_gemm(g, (hipStream_t)stream), "gemm");
  return TIDE_OK;
}

int tide_rmsnorm_fwd(int64_t rows, int64_t d, const void* x, const void* g, float eps, void* y, float* rstd,
                     int dtype, void* stream) {
  if (!x || !g || !y || !rstd) return fail(TIDE_ERR_NULL, "NULL argument");
  if (rows <= 0 || d <= 0 || d > (1 << 24)) return fail(TIDE_ERR_CONFIG, "bad sizes");
  TIDE_HIP(launch_rmsnorm_fwd(rows, (int)d, x, g, eps, y, rstd, dtype, nullptr, (hipStream_t)stream), "rmsnorm fwd");
  return TIDE_OK;
}

size_t tide_rmsnorm_bwd_scratch_bytes(int64_t rows, int64_t d) { return rmsnorm_bwd_scratch_bytes(rows, (int)d); }

int tide_rmsnorm_bwd(int64_t rows, int64_t d, const void* dy, const void* x, const void* g, const float* rstd,
                     const void* residual_grad, void* dx, float* dg, void* dg_partial, int dtype, void* stream) {
  if (!dy || !x || !g || !rstd || !dx || !dg || !dg_partial) return fail(TIDE_ERR_NULL, "NULL argument");
  const bool ok = (d % 8 == 0 && d <= 8192) || d <= 1024;
  if (rows <= 0 || d <= 0 || !ok) return fail(TIDE_ERR_CONFIG, "bad sizes");
  TIDE_HIP(launch_rmsnorm_bwd(rows, (int)d, dy, x, g, rstd, residual_grad, dx, dg, (float*)dg_partial, dtype, nullptr, (hipStream_t)stream), "rmsnorm bwd");
  return TIDE_OK;
}

}  // extern "C"

// Scratch of tide_rmsnorm_bwd_static: a fixed device array, one copy per GPU.  In host code the array's name is
// only a handle; its device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char g_rmsnorm_static_scratch[TIDE_RMSNORM_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void* g_static_ptr[kMaxDevices] = {};

// device address of the scratch array on the current device (nullptr + error message on failure)
void* static_scratch_ptr() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { hip_fail(e, "hipGetDevice"); return nullptr; }
  if (dev < 0 || dev >= kMaxDevices) { fail(TIDE_ERR_HIP, "device index %d outside [0, %d)", dev, kMaxDevices); return nullptr; }
  std::lock_guard<std::mutex> lk(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_rmsnorm_static_scratch));
    if (e != hipSuccess || !ptr) { hip_fail(e, "hipGetSymbolAddress(static scratch)"); return nullptr; }
    g_static_ptr[dev] = ptr;
  }
  return g_static_ptr[dev];
}
}  // namespace

extern "C" {

int tide_rmsnorm_bwd_static(int64_t rows, int64_t d, const void* dy, const void* x, const void* g, const float* rstd,
                            const void* residual_grad, void* dx, float* dg, int dtype, void* stream) {
  if (!dy || !x || !g || !rstd || !dx || !dg) return fail(TIDE_ERR_NULL, "NULL argument");
  const bool ok = (d % 8 == 0 && d <= 8192) || d <= 1024;
  if (rows <= 0 || d <= 0 || !ok) return fail(TIDE_ERR_CONFIG, "bad sizes");
  if (dtype != TIDE_DTYPE_FP32 && dtype != TIDE_DTYPE_BF16) return fail(TIDE_ERR_CONFIG, "bad dtype");
  const size_t need = rmsnorm_bwd_scratch_bytes(rows, (int)d);
  if (need > (size_t)TIDE_RMSNORM_STATIC_SCRATCH_BYTES)
    return fail(TIDE_ERR_WORKSPACE, "rows=%lld d=%lld need %zu bytes of scratch, the fixed array holds %u",
                (long long)rows, (long long)d, need, (unsigned)TIDE_RMSNORM_STATIC_SCRATCH_BYTES);
  void* scratch = static_scratch_ptr();
  if (!scratch) return TIDE_ERR_HIP;
  TIDE_HIP(launch_rmsnorm_bwd(rows, (int)d, dy, x, g, rstd, residual_grad, dx, dg, (float*)scratch, dtype, nullptr, (hipStream_t)stream), "rmsnorm bwd");
  return TIDE_OK;
}

static int attn_check(int B, int S, int nh, int nkv, int dh) {
  if (B <= 0 || S <= 0 || nh <= 0 || nkv <= 0 || dh <= 0 || nh % nkv || dh > 256 || B > 65535) return fail(TIDE_ERR_CONFIG, "bad attention shape");
  return 0;
}

int tide_attention_fwd(int B, int S, int nh, int nkv, int dh, const void* qkv, void* out, float* lse, int dtype,
                       void* stream) {
  if (!qkv || !out || !lse) return fail(TIDE_ERR_NULL, "NULL argument");
  if (attn_check(B, S, nh, nkv, dh)) return TIDE_ERR_CONFIG;
  AttnArgs at;
  std::memset(&at, 0, sizeof(at));
  at.B = B; at.S = S; at.nh = nh; at.nkv = nkv; at.dh = dh; at.qkv = qkv; at.out = out; at.lse = lse; at.dtype = dtype;
  TIDE_HIP(launch_attn_fwd(at, (hipStream_t)stream), "attention fwd");
  return TIDE_OK;
}

int tide_attention_bwd(int B, int S, int nh, int nkv, int dh, const void* qkv, const void* out, const void* dout,
                       const float* lse, float* delta, void* dqkv, int dtype, void* stream) {
  if (!qkv || !out || !dout || !lse || !delta || !dqkv) return fail(TIDE_ERR_NULL, "NULL argument");
  if (attn_check(B, S, nh, nkv, dh)) return TIDE_ERR_CONFIG;
  AttnArgs at;
  std::memset(&at, 0, sizeof(at));
  at.B = B; at.S = S; at.nh = nh; at.nkv = nkv; at.dh = dh; at.qkv = qkv; at.out = const_cast<void*>(out);
  at.lse = const_cast<float*>(lse); at.dout = dout; at.delta = delta; at.dqkv = dqkv; at.dtype = dtype;
  TIDE_HIP(launch_attn_bwd(at, (hipStream_t)stream), "attention bwd");
  return TIDE_OK;
}

int tide_rope(int B, int S, int nh, int nkv, int dh, float theta, void* qkv, float* table, int inverse, int dtype,
              void* stream) {
  if (!qkv || !table) return fail(TIDE_ERR_NULL, "NULL argument");
  if (B <= 0 || S <= 0 || nh <= 0 || nkv <= 0 || dh <= 0 || dh % 2) return fail(TIDE_ERR_CONFIG, "bad rope shape");
  TIDE_HIP(launch_rope_table(S, dh, theta, table, (hipStream_t)stream), "rope table");
  TIDE_HIP(launch_rope(B, S, nh, nkv, dh, table, qkv, inverse, dtype, nullptr, 0, (hipStream_t)stream), "rope");
  return TIDE_OK;
}

int tide_ce_train(int64_t rows, int32_t vocab, void* z, int64_t ldz, const int32_t* tokens, const uint8_t* mask,
                  float* lse, float* loss_rows, int dtype, void* stream) {
  if (!z || !tokens || !mask || !lse || !loss_rows) return fail(TIDE_ERR_NULL, "NULL argument");
  if (rows < 0 || rows > 0x7fffffff || vocab <= 0 || ldz < vocab || ldz % 8) return fail(TIDE_ERR_CONFIG, "bad logit block shape");
  if (dtype != TIDE_DTYPE_FP32 && dtype != TIDE_DTYPE_BF16) return fail(TIDE_ERR_CONFIG, "bad dtype");
  if (((uintptr_t)z) & 15) return fail(TIDE_ERR_CONFIG, "z must be 16-byte aligned");
  TIDE_HIP(launch_ce_train(rows, vocab, z, ldz, tokens, mask, lse, loss_rows, nullptr, 0,
                           dtype == TIDE_DTYPE_BF16 ? kBF16 : kF32, (hipStream_t)stream), "ce train");
  return TIDE_OK;
}

}  // extern "C"

// ---- optional per-launch profiler (prof.h) --------------------------------------------------------
namespace tide {
namespace {
struct ProfRec { const char* name; double flops, bytes; hipEvent_t e0, e1; const int* dyn; long long dyn_off, dyn_max; };
struct Profiler {
  std::mutex mu;
  bool on = false;
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> pool;
  hipEvent_t get() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};
Profiler g_prof;
}  // namespace

bool prof_enabled() { return g_prof.on; }

void prof_begin(const char* kernel, double flops, double bytes, hipStream_t s) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  ProfRec r{kernel, flops, bytes, g_prof.get(), g_prof.get(), nullptr, 0, 0};
  if (r.e0) (void)hipEventRecord(r.e0, s);
  g_prof.recs.push_back(r);
}

void prof_dynamic(const int* dev, long long off, long long maxv) {
  if (!g_prof.on) return;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  if (g_prof.recs.empty()) return;
  g_prof.recs.back().dyn = dev;
  g_prof.recs.back().dyn_off = off;
  g_prof.recs.back().dyn_max = maxv;
}

void prof_end(hipStream_t s) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  if (!g_prof.recs.empty() && g_prof.recs.back().e1) (void)hipEventRecord(g_prof.recs.back().e1, s);
}
}  // namespace tide

extern "C" {

int tide_mfma_probe(int32_t blocks, int32_t iters, float* sink, double* flops_out, void* stream) {
  if (!sink) return fail(TIDE_ERR_NULL, "sink is NULL");
  if (blocks < 1 || blocks > (1 << 20) || iters < 1 || iters > (1 << 24)) return fail(TIDE_ERR_CONFIG, "blocks must be in [1, 2^20] and iters in [1, 2^24]");
  if (flops_out) *flops_out = (double)blocks * 8.0 * (double)iters * 8.0 * (2.0 * 32 * 32 * 16);
  TIDE_HIP(launch_mfma_probe(blocks, iters, sink, (hipStream_t)stream), "mfma probe");
  return TIDE_OK;
}

int tide_profile_start(void) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  for (auto& r : g_prof.recs) { if (r.e0) g_prof.pool.push_back(r.e0); if (r.e1) g_prof.pool.push_back(r.e1); }
  g_prof.recs.clear();
  g_prof.on = true;
  return TIDE_OK;
}

int tide_profile_stop(char* report, size_t report_bytes) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  g_prof.on = false;
  struct Agg { const char* name; long n; double ms, flops, bytes; };
  std::vector<Agg> agg;
  for (auto& r : g_prof.recs) {
    float ms = 0.f;
    if (r.e0 && r.e1) {
      hipError_t e = hipEventSynchronize(r.e1);
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.e0, r.e1);
      if (e != hipSuccess) return hip_fail(e, "profile events");
    }
    Agg* a = nullptr;
    for (auto& x : agg) if (std::strcmp(x.name, r.name) == 0) { a = &x; break; }
    if (!a) { agg.push_back(Agg{r.name, 0, 0, 0, 0}); a = &agg.back(); }
    double scale = 1.0;
    if (r.dyn && r.dyn_max > 0) {
      // the launch trimmed itself to a device-side size: read it back (events are complete, value is final)
      int v = 0;
      hipError_t e = hipMemcpy(&v, r.dyn, sizeof(int), hipMemcpyDeviceToHost);
      if (e != hipSuccess) return hip_fail(e, "profile size read-back");
      long long eff = (long long)v - r.dyn_off;
      eff = eff < 0 ? 0 : (eff > r.dyn_max ? r.dyn_max : eff);
      scale = (double)eff / (double)r.dyn_max;
    }
    a->n += 1; a->ms += ms; a->flops += r.flops * scale; a->bytes += r.bytes * scale;
    if (r.e0) g_prof.pool.push_back(r.e0);
    if (r.e1) g_prof.pool.push_back(r.e1);
  }
  g_prof.recs.clear();
  std::string out = "[";
  char line[512];
  for (size_t i = 0; i < agg.size(); ++i) {
    snprintf(line, sizeof(line), "%s{\"kernel\": \"%s\", \"launches\": %ld, \"total_ms\": %.6f, \"flops\": %.6e, \"bytes\": %.6e}",
             i ? ", " : "", agg[i].name, agg[i].n, agg[i].ms, agg[i].flops, agg[i].bytes);
    out += line;
  }
  out += "]";
  if (!report || report_bytes < out.size() + 1) return fail(TIDE_ERR_WORKSPACE, "profile report needs %zu bytes", out.size() + 1);
  std::memcpy(report, out.c_str(), out.size() + 1);
  return TIDE_OK;
}

}  // extern "C"

namespace tide {
hipError_t launch_attn_fwd(const AttnArgs& a, hipStream_t s) {
  if (attn_mfma_supported(a)) return launch_attn_fwd_mfma(a, s);
  return launch_attn_fwd_simple(a, s);
}
hipError_t launch_attn_bwd(const AttnArgs& a, hipStream_t s) {
  if (attn_mfma_supported(a)) return launch_attn_bwd_mfma(a, s);
  return launch_attn_bwd_simple(a, s);
}
}  // namespace tide
