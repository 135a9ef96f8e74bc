"""Plain NumPy fp64 oracle of the TIDE online draft-training step.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's cpu_baseline leg; never by the product path.  It shares no code
with the HIP library.

What it computes (paper sections cited per function):

* The draft model is one decoder layer plus an LM head that reads the
  concatenation of three captured target hidden states (Sec. 3.2, "Serving-Time
  Training Signal Extraction"), is fine-tuned on those captured states with only
  the draft resident (Sec. 3.3, "Online Draft Model Adaptation"), and predicts
  over the target's own vocabulary (Sec. 5.1, "Draft Model Configuration").
  What "correct" means is the top-1 match with the tokens the target emitted
  (Fig. 7 caption), so the loss is hard-label softmax cross-entropy on them.
* The paper gives no layer equations.  The block internals are the textbook
  ones: pre-norm RMSNorm, rotate-half RoPE, grouped-query causal softmax
  attention, SwiGLU MLP, residual connections, a final RMSNorm, an untied LM
  head, decoupled-weight-decay Adam (AdamW).  Every such reading is listed in
  the design notes of the repository.

Everything is the plain definition in float64: full [S,S] score matrices, full
[rows,V] logits (row-chunked only to bound memory, which does not change any
value), explicit hand-derived gradients, no autograd, no blocking or fusion.

Parity pins (tests/test_oracle_*.py): central finite differences for every
parameter tensor, softmax-minus-onehot closed form and zero row sums, W_lm = 0
gives ln V, mask / causality / padding invariances, brute-force per-(i,j)
attention, GQA == MHA with replicated K/V rows, RoPE relative-position and
isometry properties, RMSNorm scale invariance, AdamW first-step closed form and
torch.optim.AdamW, and the whole forward/backward against torch CPU fp64
autograd built from library primitives.  No function here is "parity unpinned".

Token-input variant (optional `tok` argument of forward / train_step).  Sec. 3.2
names EAGLE-3 as the draft architecture without restating it.  That
architecture joins the projected features with the embedding of the token
sampled at the position: the two vectors are concatenated and a second fully
connected layer brings them back to the model width before the decoder layer.
Here: g = Hcat W_fc^T, e = E[input_id] (E frozen, an out-of-range id gives a zero
row), x0 = [g ; e] W_in^T with one more trainable tensor W_in [d, 2d].  The TIDE
paper fixes none of this (no equation, no number), so against the paper this
variant is "parity unpinned"; what pins it is mathematics: W_in = [I | 0]
reproduces the base model exactly, W_in = [0 | I] makes the result independent
of the captured states, central finite differences on W_in and W_fc, and torch CPU
fp64 autograd over F.embedding / torch.cat / F.linear.  The
multi-step unroll of that architecture (the draft fed its own output) is in unroll_oracle.py.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64

PARAM_NAMES = ("w_fc", "g1", "w_qkv", "w_o", "g2", "w_gate", "w_up", "w_down", "g3", "w_lm")
TOKEN_PARAM = "w_in"   # [d, 2d], present only in the token-input variant


def param_shapes(cfg):
    """Shapes of the ten parameter tensors, weights stored [out, in] row-major."""
    d = cfg["hidden"]
    nq = cfg["n_heads"] * cfg["head_dim"]
    nkv = cfg["n_kv_heads"] * cfg["head_dim"]
    return {
        "w_fc": (d, cfg["n_capture"] * cfg["target_hidden"]),
        "g1": (d,),
        "w_qkv": (nq + 2 * nkv, d),
        "w_o": (d, nq),
        "g2": (d,),
        "w_gate": (cfg["ffn"], d),
        "w_up": (cfg["ffn"], d),
        "w_down": (d, cfg["ffn"]),
        "g3": (d,),
        "w_lm": (cfg["vocab"], d),
    }


# --------------------------------------------------------------------------
# RMSNorm:  y = g * x * r,  r = (mean(x^2) + eps)^(-1/2)
# --------------------------------------------------------------------------
def rmsnorm_fwd(x, g, eps):
    x = np.asarray(x, F64)
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return g * x * r, r


def rmsnorm_bwd(dy, x, g, r):
    """dx = r*u - x * r^3 * <u,x>/d with u = g*dy ;  dg = sum_rows dy * x * r."""
    d = x.shape[-1]
    u = g * dy
    dot = np.sum(u * x, axis=-1, keepdims=True)
    dx = r * u - x * (r ** 3) * dot / d
    dg = np.sum((dy * x * r).reshape(-1, d), axis=0)
    return dx, dg


# --------------------------------------------------------------------------
# RoPE, rotate-half pairing (i, i + d_h/2); position = index in the sequence.
# --------------------------------------------------------------------------
def rope_angles(seq, head_dim, theta):
    half = head_dim // 2
    inv = np.asarray(theta, F64) ** (-2.0 * np.arange(half, dtype=F64) / head_dim)
    phi = np.arange(seq, dtype=F64)[:, None] * inv[None, :]
    return np.cos(phi), np.sin(phi)  # [S, d_h/2]


def rope_apply(x, cos, sin, inverse=False):
    """x: [B, S, n, d_h].  inverse=True rotates by -phi (this is the backward)."""
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    c = cos[None, :, None, :]
    s = sin[None, :, None, :]
    if inverse:
        s = -s
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


# --------------------------------------------------------------------------
# Causal grouped-query attention, plain definition with full [S,S] matrices.
# q: [B,S,n_h,d_h]; k,v: [B,S,n_kv,d_h]; query head h reads kv head h // G.
# --------------------------------------------------------------------------
def attention_fwd(q, k, v):
    B, S, nh, dh = q.shape
    nkv = k.shape[2]
    G = nh // nkv
    scale = 1.0 / np.sqrt(F64(dh))
    A = np.empty_like(q)
    P = np.empty((B, nh, S, S), F64)
    future = np.triu(np.ones((S, S), bool), 1)
    for b in range(B):
        for h in range(nh):
            kh = h // G
            sc = (q[b, :, h, :] @ k[b, :, kh, :].T) * scale
            sc[future] = -np.inf
            sc = sc - sc.max(axis=-1, keepdims=True)
            e = np.exp(sc)
            p = e / e.sum(axis=-1, keepdims=True)
            P[b, h] = p
            A[b, :, h, :] = p @ v[b, :, kh, :]
    return A, P


def attention_bwd(dA, q, k, v, P):
    B, S, nh, dh = q.shape
    nkv = k.shape[2]
    G = nh // nkv
    scale = 1.0 / np.sqrt(F64(dh))
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for b in range(B):
        for h in range(nh):
            kh = h // G
            p = P[b, h]
            da = dA[b, :, h, :]
            dv[b, :, kh, :] += p.T @ da
            dp = da @ v[b, :, kh, :].T
            dsc = p * (dp - np.sum(p * dp, axis=-1, keepdims=True))
            dq[b, :, h, :] = (dsc @ k[b, :, kh, :]) * scale
            dk[b, :, kh, :] += (dsc.T @ q[b, :, h, :]) * scale
    return dq, dk, dv


# --------------------------------------------------------------------------
# SwiGLU:  h = silu(gt) * u,  silu(x) = x * sigmoid(x)
# --------------------------------------------------------------------------
def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def swiglu_fwd(gt, u):
    return gt * sigmoid(gt) * u


def swiglu_bwd(dh, gt, u):
    s = sigmoid(gt)
    dgt = dh * u * s * (1.0 + gt * (1.0 - s))
    du = dh * gt * s
    return dgt, du


# --------------------------------------------------------------------------
# LM head + softmax cross-entropy against the emitted tokens.
# A label outside [0,V) is treated as masked.  N = max(1, number of rows kept).
# --------------------------------------------------------------------------
def effective_mask(tokens, loss_mask, vocab):
    tokens = np.asarray(tokens).reshape(-1)
    m = np.asarray(loss_mask).reshape(-1) != 0
    return m & (tokens >= 0) & (tokens < vocab)


def lmhead_ce_fwd(yhat, w_lm, tokens, loss_mask, row_chunk=1024, want_top1=False):
    """yhat [T,d], w_lm [V,d] -> loss, lse [T], n_valid, (top1 [T])."""
    T = yhat.shape[0]
    V = w_lm.shape[0]
    tok = np.asarray(tokens).reshape(-1).astype(np.int64)
    keep = effective_mask(tok, loss_mask, V)
    N = max(1, int(keep.sum()))
    lse = np.empty(T, F64)
    zlab = np.zeros(T, F64)
    top1 = np.zeros(T, np.int64)
    for r0 in range(0, T, row_chunk):
        r1 = min(T, r0 + row_chunk)
        z = yhat[r0:r1] @ w_lm.T
        zmax = z.max(axis=-1)
        lse[r0:r1] = zmax + np.log(np.exp(z - zmax[:, None]).sum(axis=-1))
        safe = np.where(keep[r0:r1], tok[r0:r1], 0)
        zlab[r0:r1] = z[np.arange(r1 - r0), safe]
        if want_top1:
            top1[r0:r1] = np.argmax(z, axis=-1)  # first (lowest) index on ties
    loss = float(np.sum(np.where(keep, lse - zlab, 0.0)) / N)
    out = (loss, lse, N)
    return out + (top1,) if want_top1 else out


def top1_accuracy(top1, tokens, loss_mask, vocab):
    """Fraction of the N = max(1, #kept) loss-carrying positions whose arg-max equals the label: the paper's
    training-accuracy metric (Fig. 7 caption) and what Algorithm 1's evaluation step reports."""
    tok = np.asarray(tokens).reshape(-1)
    keep = effective_mask(tok, loss_mask, vocab)
    N = max(1, int(keep.sum()))
    return float(np.sum(keep & (np.asarray(top1).reshape(-1) == tok))) / N


def lmhead_ce_bwd(yhat, w_lm, tokens, loss_mask, lse, row_chunk=1024):
    """dz = (keep/N) (softmax(z) - onehot(y));  dyhat = dz W_lm;  dW_lm = dz^T yhat."""
    T = yhat.shape[0]
    V = w_lm.shape[0]
    tok = np.asarray(tokens).reshape(-1).astype(np.int64)
    keep = effective_mask(tok, loss_mask, V)
    N = max(1, int(keep.sum()))
    dyhat = np.zeros_like(yhat)
    dw = np.zeros_like(w_lm)
    for r0 in range(0, T, row_chunk):
        r1 = min(T, r0 + row_chunk)
        kk = keep[r0:r1]
        if not kk.any():
            continue
        z = yhat[r0:r1] @ w_lm.T
        dz = np.exp(z - lse[r0:r1, None])
        rows = np.nonzero(kk)[0]
        dz[rows, tok[r0:r1][rows]] -= 1.0
        dz *= (kk.astype(F64) / N)[:, None]
        dyhat[r0:r1] = dz @ w_lm
        dw += dz.T @ yhat[r0:r1]
    return dyhat, dw


def ce_dz(z, tokens, loss_mask):
    """Dense dz for small cases: (keep/N)(softmax(z) - onehot(y)), z [T,V]."""
    T, V = z.shape
    tok = np.asarray(tokens).reshape(-1).astype(np.int64)
    keep = effective_mask(tok, loss_mask, V)
    N = max(1, int(keep.sum()))
    zz = z - z.max(axis=-1, keepdims=True)
    p = np.exp(zz)
    p /= p.sum(axis=-1, keepdims=True)
    rows = np.nonzero(keep)[0]
    p[rows, tok[rows]] -= 1.0
    return p * (keep.astype(F64) / N)[:, None]


# --------------------------------------------------------------------------
# Whole step
# --------------------------------------------------------------------------
def _as64(params):
    return {k: np.asarray(v, F64) for k, v in params.items()}


def embed_rows(embed, input_ids):
    """e[t] = E[input_ids[t]]; an id outside [0, rows) gives a zero row."""
    E = np.asarray(embed, F64)
    ids = np.asarray(input_ids).reshape(-1).astype(np.int64)
    ok = (ids >= 0) & (ids < E.shape[0])
    e = np.zeros((ids.shape[0], E.shape[1]), F64)
    e[ok] = E[ids[ok]]
    return e


def forward(cfg, params, hidden_buf, tokens, loss_mask, want_top1=False, tok=None):
    """Forward pass of the draft on captured hidden states (Sec. 3.2, 3.3).

    hidden_buf [B,S,K*H_t]; tokens [B,S] (label already aligned to the
    position); loss_mask [B,S].  tok (optional, token-input variant, see the
    module header): dict(embed [rows, d], input_ids [B,S]); params then holds
    "w_in" [d, 2d].  Returns (loss, cache)."""
    p = _as64(params)
    B, S = cfg["batch"], cfg["seq"]
    d, nh, nkv, dh = cfg["hidden"], cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    eps = cfg["rms_eps"]
    T = B * S
    Hc = np.asarray(hidden_buf, F64).reshape(T, -1)

    g0 = Hc @ p["w_fc"].T
    if tok is None:
        x0, ge = g0, None
    else:
        ge = np.concatenate([g0, embed_rows(tok["embed"], tok["input_ids"])], axis=1)   # [T, 2d]
        x0 = ge @ p[TOKEN_PARAM].T
    a, r1 = rmsnorm_fwd(x0, p["g1"], eps)
    qkv = a @ p["w_qkv"].T
    nq, nk = nh * dh, nkv * dh
    q = qkv[:, :nq].reshape(B, S, nh, dh)
    k = qkv[:, nq:nq + nk].reshape(B, S, nkv, dh)
    v = qkv[:, nq + nk:].reshape(B, S, nkv, dh)
    cos, sin = rope_angles(S, dh, cfg["rope_theta"])
    qr = rope_apply(q, cos, sin)
    kr = rope_apply(k, cos, sin)
    A, P = attention_fwd(qr, kr, v)
    A2 = A.reshape(T, nq)
    x1 = x0 + A2 @ p["w_o"].T
    bn, r2 = rmsnorm_fwd(x1, p["g2"], eps)
    gt = bn @ p["w_gate"].T
    u = bn @ p["w_up"].T
    h = swiglu_fwd(gt, u)
    x2 = x1 + h @ p["w_down"].T
    yhat, r3 = rmsnorm_fwd(x2, p["g3"], eps)
    res = lmhead_ce_fwd(yhat, p["w_lm"], tokens, loss_mask, want_top1=want_top1)
    loss, lse, N = res[:3]
    cache = dict(Hc=Hc, x0=x0, r1=r1, a=a, qr=qr, kr=kr, v=v, P=P, A=A2, x1=x1, r2=r2,
                 bn=bn, gt=gt, u=u, h=h, x2=x2, r3=r3, yhat=yhat, lse=lse, N=N,
                 cos=cos, sin=sin, qkv=qkv, ge=ge)
    if want_top1:
        cache["top1"] = res[3]
    return loss, cache


def backward(cfg, params, cache, tokens, loss_mask):
    """Gradients of the loss w.r.t. the ten parameter tensors (none w.r.t. the
    captured hidden states, which are data)."""
    p = _as64(params)
    B, S = cfg["batch"], cfg["seq"]
    nh, nkv, dh = cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    T = B * S
    nq, nk = nh * dh, nkv * dh
    c = cache
    g = {}

    dyhat, g["w_lm"] = lmhead_ce_bwd(c["yhat"], p["w_lm"], tokens, loss_mask, c["lse"])
    dx2, g["g3"] = rmsnorm_bwd(dyhat, c["x2"], p["g3"], c["r3"])
    # x2 = x1 + h W_d^T
    dh_ = dx2 @ p["w_down"]
    g["w_down"] = dx2.T @ c["h"]
    dgt, du = swiglu_bwd(dh_, c["gt"], c["u"])
    dbn = dgt @ p["w_gate"] + du @ p["w_up"]
    g["w_gate"] = dgt.T @ c["bn"]
    g["w_up"] = du.T @ c["bn"]
    dx1n, g["g2"] = rmsnorm_bwd(dbn, c["x1"], p["g2"], c["r2"])
    dx1 = dx2 + dx1n
    # x1 = x0 + A W_o^T
    dA = (dx1 @ p["w_o"]).reshape(B, S, nh, dh)
    g["w_o"] = dx1.T @ c["A"]
    dqr, dkr, dv = attention_bwd(dA, c["qr"], c["kr"], c["v"], c["P"])
    dq = rope_apply(dqr, c["cos"], c["sin"], inverse=True)
    dk = rope_apply(dkr, c["cos"], c["sin"], inverse=True)
    dqkv = np.concatenate([dq.reshape(T, nq), dk.reshape(T, nk), dv.reshape(T, nk)], axis=1)
    da = dqkv @ p["w_qkv"]
    g["w_qkv"] = dqkv.T @ c["a"]
    dx0n, g["g1"] = rmsnorm_bwd(da, c["x0"], p["g1"], c["r1"])
    dx0 = dx1 + dx0n
    if c.get("ge") is None:
        g["w_fc"] = dx0.T @ c["Hc"]
    else:
        # x0 = [g ; e] W_in^T: the embedding table is frozen, the feature half carries on to W_fc
        d = dx0.shape[1]
        g[TOKEN_PARAM] = dx0.T @ c["ge"]
        dg0 = dx0 @ p[TOKEN_PARAM][:, :d]
        g["w_fc"] = dg0.T @ c["Hc"]
    return g


def adamw_step(cfg, params, grads, m, v, step, lr):
    """One decoupled-weight-decay Adam update; `step` is the count BEFORE the
    update.  Returns new (params, m, v, step+1); inputs are not modified."""
    b1, b2 = F64(cfg["beta1"]), F64(cfg["beta2"])
    eps, wd = F64(cfg["adam_eps"]), F64(cfg["weight_decay"])
    t = step + 1
    bc1 = 1.0 - b1 ** t
    bc2 = 1.0 - b2 ** t
    np_, nm, nv = {}, {}, {}
    for k in params:
        g = np.asarray(grads[k], F64)
        nm[k] = b1 * np.asarray(m[k], F64) + (1.0 - b1) * g
        nv[k] = b2 * np.asarray(v[k], F64) + (1.0 - b2) * g * g
        th = np.asarray(params[k], F64) * (1.0 - lr * wd)
        np_[k] = th - lr * (nm[k] / bc1) / (np.sqrt(nv[k] / bc2) + eps)
    return np_, nm, nv, t


def train_step(cfg, params, m, v, step, hidden_buf, tokens, loss_mask, lr, tok=None):
    """forward + backward + AdamW.  Returns loss, grads, new params, m, v, step."""
    loss, cache = forward(cfg, params, hidden_buf, tokens, loss_mask, tok=tok)
    grads = backward(cfg, params, cache, tokens, loss_mask)
    np_, nm, nv, t = adamw_step(cfg, params, grads, m, v, step, lr)
    return loss, grads, np_, nm, nv, t


def train_quantities_packed(cfg, params, hidden_rows, tokens, loss_mask, cu_seqlens, want_top1=False):
    """Loss and gradients of a PACKED batch: row t of hidden_rows [T, K*H_t] / tokens [T] / loss_mask [T]
    belongs to sequence i iff cu_seqlens[i] <= t < cu_seqlens[i+1]; rows outside [cu[0], cu[-1]) are padding.

    Sequences are independent samples (attention and RoPE positions never cross a boundary), and the loss
    is the mean over the loss-carrying positions of the whole batch (Sec. 3.2, 3.3: the signals are
    per-request segments of accepted tokens).  So this runs the single-sequence definition above on every
    sequence by itself and combines them with their share keep_i / N of the N loss positions.
    Returns (loss, grads, top1 [T] or None); top1 of padding rows is -1."""
    cu = [int(c) for c in cu_seqlens]
    T = np.asarray(tokens).reshape(-1).shape[0]
    hidden_rows = np.asarray(hidden_rows, F64).reshape(T, -1)
    tokens = np.asarray(tokens).reshape(-1)
    mask = np.asarray(loss_mask).reshape(-1).copy()
    inside = np.zeros(T, bool)
    inside[cu[0]:cu[-1]] = True
    keep = effective_mask(tokens, mask, cfg["vocab"]) & inside
    N = max(1, int(keep.sum()))
    loss = 0.0
    grads = {k: np.zeros(np.asarray(v).shape, F64) for k, v in params.items()}
    top1 = np.full(T, -1, np.int64) if want_top1 else None
    for i in range(len(cu) - 1):
        a, b = cu[i], cu[i + 1]
        if b <= a:
            continue
        sub = dict(cfg, batch=1, seq=b - a)
        l_i, cache = forward(sub, params, hidden_rows[a:b][None], tokens[a:b][None], mask[a:b][None], want_top1=want_top1)
        if want_top1:
            top1[a:b] = cache["top1"]
        n_i = int(keep[a:b].sum())
        if n_i == 0:
            continue
        g_i = backward(sub, params, cache, tokens[a:b][None], mask[a:b][None])
        loss += l_i * n_i / N
        for k in grads:
            grads[k] += g_i[k] * (n_i / N)
    return float(loss), grads, top1
