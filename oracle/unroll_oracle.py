"""Plain NumPy fp64 oracle of the multi-step evaluation unroll of the draft (forward only).

TEST INFRASTRUCTURE ONLY, like the rest of this package: imported by tests, never by the product path.

What it computes.  Sec. 3.2 names EAGLE-3 as the draft architecture and Sec. 5.1 fixes gamma = 3 draft
tokens per round; neither restates how the draft runs past its first token.  While drafting, only the first
draft token of a round sees a feature captured from the target; every later one is fed the draft layer's own
output of the step before, in place of that feature.  The unroll repeats this on a whole batch at once, with the
true tokens as inputs and labels (teacher forcing), so that step s measures how well the draft predicts the
s-th token of a round.

Step 1 is the ordinary forward pass.  Step s >= 2, written for row i of a sequence (the row then stands for the
position i + s - 1, which must still lie inside the sequence; other rows carry no loss):

    feature      f_i   = x2 of step s-1 at row i (the layer output before the final norm)
    input        x0_i  = f_i                                   (feature-only model)
                 x0_i  = W_in [f_i ; E[input_ids[i + s - 1]]]  (token-input model)
    RoPE         q, k of the row are rotated for position i + s - 1
    attention    over the step-1 keys/values of rows 0..i, plus, for j = 2..s, the one key/value the row
                 itself produced at step j (one softmax over all of them)
    label, mask  tokens[i + s - 1], loss_mask[i + s - 1]

Every step reports its mean cross-entropy and top-1 accuracy over its own loss-carrying rows.

Against the TIDE paper this is "parity unpinned" (it prints no equation or number for it).  It is pinned by
mathematics in tests/test_oracle_unroll.py: one step equals the ordinary forward; and, for any start
position, every step equals a key/value-cache simulation of chain drafting written independently in the
test (process the prefix once, then append one position per draft step), which is the process the unroll
stands for.
"""
from __future__ import annotations

import numpy as np

from . import tide_oracle as O

F64 = np.float64


def shifted(x, shift, fill):
    """[B,S] array moved left by `shift` inside every sequence; the vacated tail holds `fill`."""
    x = np.asarray(x)
    out = np.full_like(x, fill)
    if shift < x.shape[1]:
        out[:, :x.shape[1] - shift] = x[:, shift:]
    return out


def attention_with_own_keys(q, k1, v1, own_k, own_v):
    """q [B,S,n_h,d_h]; k1, v1 [B,S,n_kv,d_h]: step-1 keys/values, causal (rows 0..i for row i);
    own_k, own_v: lists of [B,S,n_kv,d_h], one entry per later step, of which row i sees row i alone."""
    B, S, nh, dh = q.shape
    G = nh // k1.shape[2]
    scale = 1.0 / np.sqrt(F64(dh))
    A = np.empty_like(q)
    future = np.triu(np.ones((S, S), bool), 1)
    for b in range(B):
        for h in range(nh):
            kh = h // G
            sc = (q[b, :, h, :] @ k1[b, :, kh, :].T) * scale
            sc[future] = -np.inf
            own = [np.sum(q[b, :, h, :] * kj[b, :, kh, :], axis=-1) * scale for kj in own_k]   # each [S]
            full = np.concatenate([sc] + [o[:, None] for o in own], axis=1)                    # [S, S + n_own]
            full = full - full.max(axis=-1, keepdims=True)
            e = np.exp(full)
            p = e / e.sum(axis=-1, keepdims=True)
            out = p[:, :S] @ v1[b, :, kh, :]
            for j, vj in enumerate(own_v):
                out = out + p[:, S + j:S + j + 1] * vj[b, :, kh, :]
            A[b, :, h, :] = out
    return A


def unroll_forward(cfg, params, hidden_buf, tokens, loss_mask, n_steps, tok=None):
    """Returns a list with one dict per step: loss, accuracy, n (loss-carrying rows), top1 [B*S], x2 [B*S, d],
    tokens / mask (the step's shifted labels and mask, [B,S])."""
    p = {k: np.asarray(v, F64) for k, v in params.items()}
    B, S = cfg["batch"], cfg["seq"]
    d, nh, nkv, dh = cfg["hidden"], cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    eps = cfg["rms_eps"]
    T = B * S
    nq, nk = nh * dh, nkv * dh
    tokens = np.asarray(tokens).reshape(B, S)
    loss_mask = np.asarray(loss_mask).reshape(B, S)
    cos_all, sin_all = O.rope_angles(S + n_steps - 1, dh, cfg["rope_theta"])
    feat = np.asarray(hidden_buf, F64).reshape(T, -1) @ p["w_fc"].T
    k1 = v1 = None
    own_k, own_v = [], []
    steps = []
    for s in range(1, n_steps + 1):
        sh = s - 1
        tok_s = shifted(tokens, sh, -1)
        mask_s = shifted(loss_mask, sh, 0)
        if tok is None:
            x0 = feat
        else:
            ids_s = shifted(np.asarray(tok["input_ids"]).reshape(B, S), sh, -1)
            x0 = np.concatenate([feat, O.embed_rows(tok["embed"], ids_s)], axis=1) @ p[O.TOKEN_PARAM].T
        a, _ = O.rmsnorm_fwd(x0, p["g1"], eps)
        qkv = a @ p["w_qkv"].T
        cos, sin = cos_all[sh:sh + S], sin_all[sh:sh + S]
        q = O.rope_apply(qkv[:, :nq].reshape(B, S, nh, dh), cos, sin)
        k = O.rope_apply(qkv[:, nq:nq + nk].reshape(B, S, nkv, dh), cos, sin)
        v = qkv[:, nq + nk:].reshape(B, S, nkv, dh)
        if s == 1:
            k1, v1 = k, v
        else:
            own_k.append(k)
            own_v.append(v)
        A = attention_with_own_keys(q, k1, v1, own_k, own_v).reshape(T, nq)
        x1 = x0 + A @ p["w_o"].T
        bn, _ = O.rmsnorm_fwd(x1, p["g2"], eps)
        x2 = x1 + O.swiglu_fwd(bn @ p["w_gate"].T, bn @ p["w_up"].T) @ p["w_down"].T
        yhat, _ = O.rmsnorm_fwd(x2, p["g3"], eps)
        loss, _, n, top1 = O.lmhead_ce_fwd(yhat, p["w_lm"], tok_s, mask_s, want_top1=True)
        steps.append(dict(loss=loss, accuracy=O.top1_accuracy(top1, tok_s, mask_s, cfg["vocab"]), n=n, top1=top1,
                          x2=x2, tokens=tok_s, mask=mask_s))
        feat = x2
    return steps
