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

unroll_backward differentiates L = sum_s w_s loss_s through the whole chain (the feature of step s is the output
of step s-1; the keys/values of a step are read by every later step), with hand-derived gradients as in the
single-step oracle; it is pinned by central finite differences on every tensor, for both input variants and
unequal step weights, by reducing to the single-step gradients for one step, and by torch CPU fp64 autograd over
a different formulation (all steps' keys concatenated under a block mask, F.scaled_dot_product_attention).

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


def attention_with_own_keys(q, k1, v1, own_k, own_v, want_probs=False):
    """q [B,S,n_h,d_h]; k1, v1 [B,S,n_kv,d_h]: step-1 keys/values, causal (rows 0..i for row i);
    own_k, own_v: lists of [B,S,n_kv,d_h], one entry per later step, of which row i sees row i alone.
    want_probs: also returns the softmax weights [B, n_h, S, S + n_own] (prefix columns, then one per own pair)."""
    B, S, nh, dh = q.shape
    G = nh // k1.shape[2]
    scale = 1.0 / np.sqrt(F64(dh))
    A = np.empty_like(q)
    P = np.empty((B, nh, S, S + len(own_k)), F64) if want_probs else None
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
            if want_probs:
                P[b, h] = p
    return (A, P) if want_probs else A


def attention_with_own_keys_bwd(dA, q, k1, v1, own_k, own_v, P):
    """Gradients of attention_with_own_keys: dq, dk1, dv1 and one (dk, dv) per own pair.
    With p the joint softmax and dp = dA . v:  ds = p * (dp - sum(p * dp)),  then every score's two factors."""
    B, S, nh, dh = q.shape
    G = nh // k1.shape[2]
    scale = 1.0 / np.sqrt(F64(dh))
    dq = np.zeros_like(q)
    dk1, dv1 = np.zeros_like(k1), np.zeros_like(v1)
    d_own_k = [np.zeros_like(k) for k in own_k]
    d_own_v = [np.zeros_like(v) for v in own_v]
    for b in range(B):
        for h in range(nh):
            kh = h // G
            p = P[b, h]
            da = dA[b, :, h, :]
            dp = np.concatenate([da @ v1[b, :, kh, :].T] + [np.sum(da * vj[b, :, kh, :], axis=-1)[:, None] for vj in own_v], axis=1)
            ds = p * (dp - np.sum(p * dp, axis=-1, keepdims=True))
            dv1[b, :, kh, :] += p[:, :S].T @ da
            dq[b, :, h, :] = (ds[:, :S] @ k1[b, :, kh, :]) * scale
            dk1[b, :, kh, :] += (ds[:, :S].T @ q[b, :, h, :]) * scale
            for j in range(len(own_k)):
                dq[b, :, h, :] += ds[:, S + j:S + j + 1] * own_k[j][b, :, kh, :] * scale
                d_own_k[j][b, :, kh, :] += ds[:, S + j:S + j + 1] * q[b, :, h, :] * scale
                d_own_v[j][b, :, kh, :] += p[:, S + j:S + j + 1] * da
    return dq, dk1, dv1, d_own_k, d_own_v


def unroll_forward(cfg, params, hidden_buf, tokens, loss_mask, n_steps, tok=None, keep_cache=False):
    """Returns a list with one dict per step: loss, accuracy, n (loss-carrying rows), top1 [B*S], x2 [B*S, d],
    tokens / mask (the step's shifted labels and mask, [B,S]); keep_cache adds what unroll_backward needs."""
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
        a, r1 = O.rmsnorm_fwd(x0, p["g1"], eps)
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
        A, P = attention_with_own_keys(q, k1, v1, list(own_k), list(own_v), want_probs=True)
        A = A.reshape(T, nq)
        x1 = x0 + A @ p["w_o"].T
        bn, r2 = O.rmsnorm_fwd(x1, p["g2"], eps)
        gt, u = bn @ p["w_gate"].T, bn @ p["w_up"].T
        h = O.swiglu_fwd(gt, u)
        x2 = x1 + h @ p["w_down"].T
        yhat, r3 = O.rmsnorm_fwd(x2, p["g3"], eps)
        loss, lse, n, top1 = O.lmhead_ce_fwd(yhat, p["w_lm"], tok_s, mask_s, want_top1=True)
        st = dict(loss=loss, accuracy=O.top1_accuracy(top1, tok_s, mask_s, cfg["vocab"]), n=n, top1=top1,
                  x2=x2, tokens=tok_s, mask=mask_s)
        if keep_cache:
            st.update(feat=feat, ge=None if tok is None else np.concatenate([feat, O.embed_rows(tok["embed"], ids_s)], axis=1),
                      x0=x0, r1=r1, a=a, q=q, P=P, n_own=len(own_k), cos=cos, sin=sin, A=A, x1=x1, r2=r2, bn=bn, gt=gt, u=u, h=h,
                      r3=r3, yhat=yhat, lse=lse)
        steps.append(st)
        feat = x2
    if keep_cache:
        steps[0]["shared"] = dict(Hc=np.asarray(hidden_buf, F64).reshape(T, -1), k1=k1, v1=v1, own_k=own_k, own_v=own_v)
    return steps


def unroll_backward(cfg, params, steps, step_weights=None):
    """Gradients of L = sum_s step_weights[s] * loss_s w.r.t. every parameter tensor (W_in included when the
    steps were run with a token input), for `steps` = unroll_forward(..., keep_cache=True).  The gradient of a
    step's input feature flows into the layer output of the step before; key/value gradients of step j collect
    the contributions of every step that read them before step j's own projection is differentiated."""
    p = {k: np.asarray(v, F64) for k, v in params.items()}
    B, S = cfg["batch"], cfg["seq"]
    d, nh, nkv, dh = cfg["hidden"], cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    T = B * S
    nq, nk = nh * dh, nkv * dh
    n_steps = len(steps)
    w = np.ones(n_steps, F64) if step_weights is None else np.asarray(step_weights, F64)
    sh = steps[0]["shared"]
    g = {k: np.zeros_like(v) for k, v in p.items()}
    dk1, dv1 = np.zeros_like(sh["k1"]), np.zeros_like(sh["v1"])
    d_own_k = [np.zeros_like(k) for k in sh["own_k"]]
    d_own_v = [np.zeros_like(v) for v in sh["own_v"]]
    dx2_next = np.zeros((T, d), F64)          # gradient reaching x2 of the current step from the step after it
    for s in range(n_steps, 0, -1):
        c = steps[s - 1]
        dyhat, dw_lm = O.lmhead_ce_bwd(c["yhat"], p["w_lm"], c["tokens"], c["mask"], c["lse"])
        g["w_lm"] += w[s - 1] * dw_lm
        dx2, dg3 = O.rmsnorm_bwd(w[s - 1] * dyhat, c["x2"], p["g3"], c["r3"])
        g["g3"] += dg3
        dx2 = dx2 + dx2_next
        g["w_down"] += dx2.T @ c["h"]
        dgt, du = O.swiglu_bwd(dx2 @ p["w_down"], c["gt"], c["u"])
        g["w_gate"] += dgt.T @ c["bn"]
        g["w_up"] += du.T @ c["bn"]
        dx1n, dg2 = O.rmsnorm_bwd(dgt @ p["w_gate"] + du @ p["w_up"], c["x1"], p["g2"], c["r2"])
        g["g2"] += dg2
        dx1 = dx2 + dx1n
        g["w_o"] += dx1.T @ c["A"]
        dA = (dx1 @ p["w_o"]).reshape(B, S, nh, dh)
        n_own = c["n_own"]
        dq, a_dk1, a_dv1, a_dok, a_dov = attention_with_own_keys_bwd(dA, c["q"], sh["k1"], sh["v1"], sh["own_k"][:n_own],
                                                                     sh["own_v"][:n_own], c["P"])
        dk1 += a_dk1
        dv1 += a_dv1
        for j in range(n_own):
            d_own_k[j] += a_dok[j]
            d_own_v[j] += a_dov[j]
        # this step's own key/value: every later step has added its share by now
        dk_s, dv_s = (dk1, dv1) if s == 1 else (d_own_k[s - 2], d_own_v[s - 2])
        dq_ = O.rope_apply(dq, c["cos"], c["sin"], inverse=True)
        dk_ = O.rope_apply(dk_s, c["cos"], c["sin"], inverse=True)
        dqkv = np.concatenate([dq_.reshape(T, nq), dk_.reshape(T, nk), dv_s.reshape(T, nk)], axis=1)
        g["w_qkv"] += dqkv.T @ c["a"]
        dx0n, dg1 = O.rmsnorm_bwd(dqkv @ p["w_qkv"], c["x0"], p["g1"], c["r1"])
        g["g1"] += dg1
        dx0 = dx1 + dx0n
        if c["ge"] is None:
            dfeat = dx0
        else:
            g[O.TOKEN_PARAM] += dx0.T @ c["ge"]
            dfeat = dx0 @ p[O.TOKEN_PARAM][:, :d]
        if s == 1:
            g["w_fc"] += dfeat.T @ sh["Hc"]
        else:
            dx2_next = dfeat
    return g


def unroll_train_quantities_packed(cfg, params, hidden_rows, tokens, loss_mask, cu_seqlens, n_steps, tok=None,
                                   step_weights=None):
    """Per-step losses and the gradients of L = sum_s w_s loss_s for a PACKED batch (row t belongs to sequence i iff
    cu_seqlens[i] <= t < cu_seqlens[i+1]; other rows are padding).  Sequences are independent samples and every
    step's loss is the mean over that step's loss-carrying rows of the whole batch, so each sequence runs the
    single-sequence unroll above and enters step s with its share n_is / N_s of that step's loss rows.
    tok: dict(embed, input_ids [T]).  Returns (losses [n_steps], grads)."""
    cu = [int(c) for c in cu_seqlens]
    tokens = np.asarray(tokens).reshape(-1)
    T = tokens.shape[0]
    hidden_rows = np.asarray(hidden_rows, F64).reshape(T, -1)
    mask = np.asarray(loss_mask).reshape(-1)
    w = np.ones(n_steps, F64) if step_weights is None else np.asarray(step_weights, F64)
    runs = []
    for i in range(len(cu) - 1):
        a, b = cu[i], cu[i + 1]
        if b <= a:
            continue
        sub = dict(cfg, batch=1, seq=b - a)
        tk = None if tok is None else dict(embed=tok["embed"], input_ids=np.asarray(tok["input_ids"]).reshape(-1)[a:b][None])
        steps = unroll_forward(sub, params, hidden_rows[a:b][None], tokens[a:b][None], mask[a:b][None], n_steps, tok=tk, keep_cache=True)
        counts = [int(O.effective_mask(st["tokens"], st["mask"], cfg["vocab"]).sum()) for st in steps]
        runs.append((sub, steps, counts))
    N = [max(1, sum(r[2][s] for r in runs)) for s in range(n_steps)]
    losses = [sum(r[1][s]["loss"] * r[2][s] / N[s] for r in runs) for s in range(n_steps)]
    grads = {k: np.zeros(np.asarray(v).shape, F64) for k, v in params.items()}
    for sub, steps, counts in runs:
        if not any(counts):
            continue
        g = unroll_backward(sub, params, steps, step_weights=[w[s] * counts[s] / N[s] for s in range(n_steps)])
        for k in grads:
            grads[k] += g[k]
    return [float(x) for x in losses], grads
