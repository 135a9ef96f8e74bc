"""Pins for the CPU oracle: each test checks it against something other than
itself (finite differences, closed forms, invariants, brute force, library
routines), so that a dropped term, wrong sign or transposed operand fails."""
import copy

import numpy as np
import pytest
import torch

from oracle import tide_oracle as O
from paper_2602_05145_amd import workloads as W
from tests.helpers import micro_cfg, micro_workload


# ------------------------------------------------------------------ whole step
def _loss_of(cfg, params, wl):
    return O.forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"])[0]


@pytest.mark.parametrize("kw", [
    dict(),                                            # GQA, G=2
    dict(n_heads=2, n_kv_heads=2),                     # MHA, G=1
    dict(seq=1, mask="none"),                          # single position
    dict(batch=2, seq=4, n_heads=4, n_kv_heads=2, hidden=16, ffn=10, vocab=13),
])
def test_finite_differences_every_tensor(kw):
    cfg = micro_cfg(**kw)
    wl = micro_workload(cfg)
    params = wl["params"]
    loss, cache = O.forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"])
    grads = O.backward(cfg, params, cache, wl["tokens"], wl["mask"])
    rng = np.random.default_rng(0)
    h = 1e-6
    for name in O.PARAM_NAMES:
        g = grads[name]
        assert g.shape == params[name].shape
        flat = params[name].reshape(-1)
        idx = rng.choice(flat.size, size=min(12, flat.size), replace=False)
        for i in idx:
            pp = copy.deepcopy(params)
            pp[name].reshape(-1)[i] += h
            lp = _loss_of(cfg, pp, wl)
            pp[name].reshape(-1)[i] -= 2 * h
            lm = _loss_of(cfg, pp, wl)
            fd = (lp - lm) / (2 * h)
            an = g.reshape(-1)[i]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)) + 2e-8, (name, i, fd, an)


def _torch_reference(cfg, params, wl, tok_in=None):
    """Same model composed from torch CPU fp64 library primitives + autograd (tok_in: the token-input variant's
    embedding table and ids, joined through F.embedding, torch.cat and F.linear)."""
    import torch.nn.functional as F
    B, S = cfg["batch"], cfg["seq"]
    nh, nkv, dh = cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    P = {k: torch.tensor(np.asarray(v, np.float64), requires_grad=True) for k, v in params.items()}
    Hc = torch.tensor(wl["hidden"], dtype=torch.float64).reshape(B * S, -1)

    def rms(x, g):
        return g * x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + cfg["rms_eps"])

    x0 = F.linear(Hc, P["w_fc"])
    if tok_in is not None:
        E = torch.tensor(np.asarray(tok_in["embed"], np.float64))
        ids = torch.tensor(np.asarray(tok_in["input_ids"]).reshape(-1).astype(np.int64))
        x0 = F.linear(torch.cat([x0, F.embedding(ids, E)], dim=1), P["w_in"])
    a = rms(x0, P["g1"])
    qkv = F.linear(a, P["w_qkv"])
    nq, nk = nh * dh, nkv * dh
    q = qkv[:, :nq].reshape(B, S, nh, dh)
    k = qkv[:, nq:nq + nk].reshape(B, S, nkv, dh)
    v = qkv[:, nq + nk:].reshape(B, S, nkv, dh)
    half = dh // 2
    inv = torch.tensor(cfg["rope_theta"], dtype=torch.float64) ** (
        -torch.arange(0, dh, 2, dtype=torch.float64) / dh)
    ang = torch.arange(S, dtype=torch.float64)[:, None] * inv[None]
    cos = torch.cat([ang.cos(), ang.cos()], -1)[None, :, None, :]
    sin = torch.cat([ang.sin(), ang.sin()], -1)[None, :, None, :]

    def rot(x):
        return torch.cat([-x[..., half:], x[..., :half]], -1)

    q = q * cos + rot(q) * sin
    k = k * cos + rot(k) * sin
    G = nh // nkv
    kk = k.repeat_interleave(G, dim=2)
    vv = v.repeat_interleave(G, dim=2)
    A = F.scaled_dot_product_attention(q.transpose(1, 2), kk.transpose(1, 2), vv.transpose(1, 2),
                                       is_causal=True)
    A = A.transpose(1, 2).reshape(B * S, nq)
    x1 = x0 + F.linear(A, P["w_o"])
    b = rms(x1, P["g2"])
    hmid = F.silu(F.linear(b, P["w_gate"])) * F.linear(b, P["w_up"])
    x2 = x1 + F.linear(hmid, P["w_down"])
    y = rms(x2, P["g3"])
    z = F.linear(y, P["w_lm"])
    tok = torch.tensor(wl["tokens"].reshape(-1).astype(np.int64))
    m = torch.tensor(wl["mask"].reshape(-1).astype(np.float64))
    per = F.cross_entropy(z, tok, reduction="none")
    loss = (per * m).sum() / max(1.0, float(m.sum()))
    loss.backward()
    return float(loss.detach()), {k: t.grad.numpy() for k, t in P.items()}, z.detach().numpy()


@pytest.mark.parametrize("kw", [dict(), dict(batch=2, seq=9, n_heads=4, n_kv_heads=2, hidden=16,
                                             head_dim=4, ffn=12, vocab=37)])
def test_against_torch_autograd(kw):
    cfg = micro_cfg(**kw)
    wl = micro_workload(cfg)
    loss, cache = O.forward(cfg, wl["params"], wl["hidden"], wl["tokens"], wl["mask"])
    grads = O.backward(cfg, wl["params"], cache, wl["tokens"], wl["mask"])
    tl, tg, _ = _torch_reference(cfg, wl["params"], wl)
    assert abs(loss - tl) <= 1e-12 * abs(tl)
    for k in O.PARAM_NAMES:
        np.testing.assert_allclose(grads[k], tg[k], rtol=1e-9, atol=1e-13, err_msg=k)


# ------------------------------------------------------------------ cross-entropy
def test_ce_closed_forms():
    rng = np.random.default_rng(1)
    T, V = 9, 17
    z = rng.standard_normal((T, V)) * 3
    tok = rng.integers(0, V, T)
    mask = np.array([1, 1, 0, 1, 1, 1, 0, 1, 1], np.uint8)
    dz = O.ce_dz(z, tok, mask)
    N = int(mask.sum())
    # rows of softmax - onehot sum to zero; masked rows are exactly zero
    assert np.all(np.abs(dz.sum(-1)) < 1e-15)
    assert np.all(dz[mask == 0] == 0.0)
    # the label entry is p-1 < 0, all others positive
    for t in np.nonzero(mask)[0]:
        assert dz[t, tok[t]] < 0
        others = np.delete(dz[t], tok[t])
        assert np.all(others > 0)
        p = np.exp(z[t] - np.log(np.sum(np.exp(z[t]))))
        np.testing.assert_allclose(dz[t, tok[t]], (p[tok[t]] - 1) / N, rtol=1e-12)
    # dz from the chunked routine (via identity weights) equals the dense form
    d = V
    yhat, w = z.copy(), np.eye(V)
    loss, lse, n = O.lmhead_ce_fwd(yhat, w, tok, mask, row_chunk=4)
    assert n == N
    ref = np.sum([(np.log(np.sum(np.exp(z[t]))) - z[t, tok[t]]) for t in range(T) if mask[t]]) / N
    np.testing.assert_allclose(loss, ref, rtol=1e-13)
    dy, dw = O.lmhead_ce_bwd(yhat, w, tok, mask, lse, row_chunk=4)
    np.testing.assert_allclose(dy, dz, atol=1e-15)          # dz @ I
    np.testing.assert_allclose(dw, dz.T @ yhat, atol=1e-14)


@pytest.mark.parametrize("V", [11, 4096])
def test_zero_lm_head_gives_log_vocab(V):
    cfg = micro_cfg(vocab=V)
    wl = micro_workload(cfg)
    wl["params"]["w_lm"][:] = 0.0
    loss, _ = O.forward(cfg, wl["params"], wl["hidden"], wl["tokens"], wl["mask"])
    assert abs(loss - np.log(V)) < 1e-13


def test_log_vocab_constants():
    # values the method must reproduce for the workload vocabularies
    for V, ref in [(4096, 8.3178), (32000, 10.3735), (128256, 11.7618), (152064, 11.9321)]:
        assert abs(np.log(V) - ref) < 5e-5


# ------------------------------------------------------------------ masking
def test_mask_invariances_and_all_masked():
    cfg = micro_cfg(batch=2, seq=6)
    wl = micro_workload(cfg)
    P = wl["params"]
    loss, cache = O.forward(cfg, P, wl["hidden"], wl["tokens"], wl["mask"])
    grads = O.backward(cfg, P, cache, wl["tokens"], wl["mask"])
    # tokens at masked positions are irrelevant (bit exact)
    tok2 = wl["tokens"].copy()
    tok2[wl["mask"] == 0] = (tok2[wl["mask"] == 0] + 3) % cfg["vocab"]
    loss2, cache2 = O.forward(cfg, P, wl["hidden"], tok2, wl["mask"])
    grads2 = O.backward(cfg, P, cache2, tok2, wl["mask"])
    assert loss2 == loss
    for k in grads:
        assert np.array_equal(grads[k], grads2[k])
    # flipping one mask bit off removes exactly that row's term
    flat = wl["mask"].reshape(-1)
    t = int(np.nonzero(flat)[0][0])
    m3 = wl["mask"].copy()
    m3.reshape(-1)[t] = 0
    loss3, _ = O.forward(cfg, P, wl["hidden"], wl["tokens"], m3)
    N = int(flat.sum())
    z_t = cache["yhat"][t] @ np.asarray(P["w_lm"]).T
    term = np.log(np.sum(np.exp(z_t))) - z_t[wl["tokens"].reshape(-1)[t]]
    np.testing.assert_allclose(loss3 * (N - 1), loss * N - term, rtol=1e-12)
    # an out-of-range label behaves as a masked position
    tok4 = wl["tokens"].copy()
    tok4.reshape(-1)[t] = cfg["vocab"] + 5
    loss4, cache4 = O.forward(cfg, P, wl["hidden"], tok4, wl["mask"])
    assert loss4 == loss3
    tok5 = wl["tokens"].copy()
    tok5.reshape(-1)[t] = -1
    assert O.forward(cfg, P, wl["hidden"], tok5, wl["mask"])[0] == loss3
    # all masked: loss 0 and every gradient exactly 0
    m0 = np.zeros_like(wl["mask"])
    loss0, cache0 = O.forward(cfg, P, wl["hidden"], wl["tokens"], m0)
    grads0 = O.backward(cfg, P, cache0, wl["tokens"], m0)
    assert loss0 == 0.0
    for k in grads0:
        assert not np.any(grads0[k]), k


# ------------------------------------------------------------------ causality / padding / batch
def test_causality_and_batch_independence():
    cfg = micro_cfg(batch=2, seq=7, mask="none")
    wl = micro_workload(cfg)
    P = wl["params"]
    _, c0 = O.forward(cfg, P, wl["hidden"], wl["tokens"], wl["mask"])
    h2 = wl["hidden"].copy()
    tp = 4
    h2[0, tp, :] += 1.7
    _, c1 = O.forward(cfg, P, h2, wl["tokens"], wl["mask"])
    S = cfg["seq"]
    y0 = c0["yhat"].reshape(2, S, -1)
    y1 = c1["yhat"].reshape(2, S, -1)
    assert np.array_equal(y0[0, :tp], y1[0, :tp])          # earlier positions untouched
    assert np.array_equal(c0["lse"].reshape(2, S)[0, :tp], c1["lse"].reshape(2, S)[0, :tp])
    assert not np.allclose(y0[0, tp:], y1[0, tp:])         # later ones do change
    assert np.array_equal(y0[1], y1[1])                    # other sequence untouched


def test_right_padding_changes_nothing():
    cfg = micro_cfg(batch=1, seq=5, mask="none")
    wl = micro_workload(cfg)
    P = wl["params"]
    loss, cache = O.forward(cfg, P, wl["hidden"], wl["tokens"], wl["mask"])
    grads = O.backward(cfg, P, cache, wl["tokens"], wl["mask"])
    cfgp = dict(cfg, seq=8)
    hp = np.zeros((1, 8, wl["hidden"].shape[-1]))
    hp[:, :5] = wl["hidden"]
    tp = np.zeros((1, 8), np.int32)
    tp[:, :5] = wl["tokens"]
    mp = np.zeros((1, 8), np.uint8)
    mp[:, :5] = 1
    lossp, cachep = O.forward(cfgp, P, hp, tp, mp)
    gradsp = O.backward(cfgp, P, cachep, tp, mp)
    np.testing.assert_allclose(lossp, loss, rtol=1e-14)
    assert np.all(np.isfinite(cachep["yhat"]))
    for k in grads:
        np.testing.assert_allclose(gradsp[k], grads[k], rtol=1e-11, atol=1e-15, err_msg=k)


# ------------------------------------------------------------------ attention
def _attention_bruteforce(q, k, v):
    B, S, nh, dh = q.shape
    G = nh // k.shape[2]
    A = np.zeros_like(q)
    for b in range(B):
        for h in range(nh):
            for i in range(S):
                w = [np.exp(sum(q[b, i, h, c] * k[b, j, h // G, c] for c in range(dh)) / np.sqrt(dh))
                     for j in range(i + 1)]
                tot = sum(w)
                for j in range(i + 1):
                    A[b, i, h, :] += (w[j] / tot) * v[b, j, h // G, :]
    return A


def test_attention_special_cases_and_bruteforce():
    rng = np.random.default_rng(3)
    B, S, nh, nkv, dh = 2, 6, 4, 2, 4
    q = rng.standard_normal((B, S, nh, dh))
    k = rng.standard_normal((B, S, nkv, dh))
    v = rng.standard_normal((B, S, nkv, dh))
    A, P = O.attention_fwd(q, k, v)
    np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-15)
    assert np.all(P[:, :, np.triu(np.ones((S, S), bool), 1)] == 0.0)
    np.testing.assert_allclose(A, _attention_bruteforce(q, k, v), atol=1e-14)
    # q = 0: uniform weights, output is the running mean of v
    A0, _ = O.attention_fwd(np.zeros_like(q), k, v)
    run = np.cumsum(v, axis=1) / np.arange(1, S + 1)[None, :, None, None]
    np.testing.assert_allclose(A0, np.repeat(run, nh // nkv, axis=2), atol=1e-15)
    # S = 1: output is v of the matching kv head
    A1, _ = O.attention_fwd(q[:, :1], k[:, :1], v[:, :1])
    np.testing.assert_allclose(A1, np.repeat(v[:, :1], nh // nkv, axis=2), atol=1e-16)


def test_attention_backward_finite_differences():
    rng = np.random.default_rng(4)
    B, S, nh, nkv, dh = 1, 5, 2, 1, 3
    q = rng.standard_normal((B, S, nh, dh))
    k = rng.standard_normal((B, S, nkv, dh))
    v = rng.standard_normal((B, S, nkv, dh))
    w = rng.standard_normal((B, S, nh, dh))

    def f(q, k, v):
        return float(np.sum(O.attention_fwd(q, k, v)[0] * w))

    A, P = O.attention_fwd(q, k, v)
    dq, dk, dv = O.attention_bwd(w, q, k, v, P)
    h = 1e-6
    for arr, gr in ((q, dq), (k, dk), (v, dv)):
        for i in range(arr.size):
            old = arr.reshape(-1)[i]
            arr.reshape(-1)[i] = old + h
            fp = f(q, k, v)
            arr.reshape(-1)[i] = old - h
            fm = f(q, k, v)
            arr.reshape(-1)[i] = old
            assert abs((fp - fm) / (2 * h) - gr.reshape(-1)[i]) < 1e-7


def test_gqa_equals_mha_with_replicated_kv():
    cfg = micro_cfg(batch=1, seq=6, n_heads=4, n_kv_heads=2, hidden=16, head_dim=4, ffn=10)
    wl = micro_workload(cfg)
    P = wl["params"]
    loss, cache = O.forward(cfg, P, wl["hidden"], wl["tokens"], wl["mask"])
    grads = O.backward(cfg, P, cache, wl["tokens"], wl["mask"])
    nh, nkv, dh = 4, 2, 4
    G = nh // nkv
    nq, nk = nh * dh, nkv * dh
    wq, wk, wv = P["w_qkv"][:nq], P["w_qkv"][nq:nq + nk], P["w_qkv"][nq + nk:]
    rep = lambda w: np.repeat(w.reshape(nkv, dh, -1), G, axis=0).reshape(nh * dh, -1)
    P2 = dict(P, w_qkv=np.concatenate([wq, rep(wk), rep(wv)], 0))
    cfg2 = dict(cfg, n_kv_heads=nh)
    loss2, cache2 = O.forward(cfg2, P2, wl["hidden"], wl["tokens"], wl["mask"])
    grads2 = O.backward(cfg2, P2, cache2, wl["tokens"], wl["mask"])
    np.testing.assert_allclose(loss2, loss, rtol=1e-14)
    fold = lambda g: g.reshape(nkv, G, dh, -1).sum(1).reshape(nk, -1)
    g2 = grads2["w_qkv"]
    np.testing.assert_allclose(grads["w_qkv"][:nq], g2[:nq], rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(grads["w_qkv"][nq:nq + nk], fold(g2[nq:nq + nq]), rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(grads["w_qkv"][nq + nk:], fold(g2[nq + nq:]), rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(grads["w_fc"], grads2["w_fc"], rtol=1e-11, atol=1e-15)


# ------------------------------------------------------------------ RoPE
def test_rope_properties():
    rng = np.random.default_rng(5)
    S, dh = 9, 8
    cos, sin = O.rope_angles(S + 5, dh, 1e4)
    x = rng.standard_normal((1, S, 2, dh))
    y = rng.standard_normal((1, S, 2, dh))
    rx = O.rope_apply(x, cos[:S], sin[:S])
    # position 0 is the identity; rotation preserves norms
    assert np.array_equal(rx[:, 0], x[:, 0])
    np.testing.assert_allclose(np.linalg.norm(rx, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-14)
    # explicit pairing (i, i + d_h/2) with angle pos * theta^(-2i/d_h)
    pos, i = 3, 1
    ang = pos * 1e4 ** (-2 * i / dh)
    np.testing.assert_allclose(rx[0, pos, 0, i], x[0, pos, 0, i] * np.cos(ang) - x[0, pos, 0, i + dh // 2] * np.sin(ang), rtol=1e-13)
    np.testing.assert_allclose(rx[0, pos, 0, i + dh // 2], x[0, pos, 0, i + dh // 2] * np.cos(ang) + x[0, pos, 0, i] * np.sin(ang), rtol=1e-13)
    # scores depend only on the relative position: shift every position by 5
    ry = O.rope_apply(y, cos[:S], sin[:S])
    rx5 = O.rope_apply(x, cos[5:5 + S], sin[5:5 + S])
    ry5 = O.rope_apply(y, cos[5:5 + S], sin[5:5 + S])
    s0 = np.einsum("bihd,bjhd->bhij", rx, ry)
    s5 = np.einsum("bihd,bjhd->bhij", rx5, ry5)
    np.testing.assert_allclose(s0, s5, atol=1e-12)
    # the inverse rotation is the transpose: <R x, y> = <x, R^T y>
    rty = O.rope_apply(y, cos[:S], sin[:S], inverse=True)
    np.testing.assert_allclose(np.sum(rx * y), np.sum(x * rty), rtol=1e-13)
    np.testing.assert_allclose(O.rope_apply(rx, cos[:S], sin[:S], inverse=True), x, atol=1e-14)


# ------------------------------------------------------------------ RMSNorm
def test_rmsnorm_properties():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((7, 12))
    g = 1.0 + 0.2 * rng.standard_normal(12)
    y, r = O.rmsnorm_fwd(x, np.ones(12), 0.0)
    np.testing.assert_allclose(np.sqrt(np.mean(y * y, -1)), 1.0, rtol=1e-14)
    y3, _ = O.rmsnorm_fwd(3.5 * x, g, 0.0)
    y1, r1 = O.rmsnorm_fwd(x, g, 0.0)
    np.testing.assert_allclose(y3, y1, rtol=1e-13)
    dy = rng.standard_normal((7, 12))
    dx, dg = O.rmsnorm_bwd(dy, x, g, r1)
    # scale invariance => gradient orthogonal to x (eps = 0)
    assert np.all(np.abs(np.sum(dx * x, -1)) < 1e-13)
    # finite differences incl. eps
    eps = 1e-2
    y, r = O.rmsnorm_fwd(x, g, eps)
    dx, dg = O.rmsnorm_bwd(dy, x, g, r)
    h = 1e-6
    for i in range(0, x.size, 5):
        xp = x.copy(); xp.reshape(-1)[i] += h
        xm = x.copy(); xm.reshape(-1)[i] -= h
        fd = (np.sum(O.rmsnorm_fwd(xp, g, eps)[0] * dy) - np.sum(O.rmsnorm_fwd(xm, g, eps)[0] * dy)) / (2 * h)
        assert abs(fd - dx.reshape(-1)[i]) < 1e-8
    for j in range(12):
        gp = g.copy(); gp[j] += h
        gm = g.copy(); gm[j] -= h
        fd = (np.sum(O.rmsnorm_fwd(x, gp, eps)[0] * dy) - np.sum(O.rmsnorm_fwd(x, gm, eps)[0] * dy)) / (2 * h)
        assert abs(fd - dg[j]) < 1e-8
    # zero rows stay finite and zero (eps > 0)
    y0, _ = O.rmsnorm_fwd(np.zeros((2, 12)), g, 1e-5)
    assert np.all(y0 == 0)


# ------------------------------------------------------------------ SwiGLU
def test_swiglu_derivatives():
    gt = np.linspace(-6, 6, 25)
    u = np.linspace(1.5, -2.0, 25)
    dh = np.ones(25)
    dgt, du = O.swiglu_bwd(dh, gt, u)
    h = 1e-6
    fd_g = (O.swiglu_fwd(gt + h, u) - O.swiglu_fwd(gt - h, u)) / (2 * h)
    fd_u = (O.swiglu_fwd(gt, u + h) - O.swiglu_fwd(gt, u - h)) / (2 * h)
    np.testing.assert_allclose(dgt, fd_g, atol=1e-8)
    np.testing.assert_allclose(du, fd_u, atol=1e-8)
    # silu'(0) = 1/2 ; silu(x) -> x for large x ; silu(0) = 0
    d0, _ = O.swiglu_bwd(np.ones(1), np.zeros(1), np.ones(1))
    assert d0[0] == 0.5
    assert O.swiglu_fwd(np.zeros(1), np.ones(1))[0] == 0.0
    np.testing.assert_allclose(O.swiglu_fwd(np.array([40.0]), np.array([2.0])), [80.0], rtol=1e-15)
    np.testing.assert_allclose(O.swiglu_fwd(gt, u), torch.nn.functional.silu(torch.tensor(gt)).numpy() * u, rtol=1e-14)


# ------------------------------------------------------------------ AdamW
def test_adamw_closed_forms_and_torch():
    cfg = micro_cfg()
    rng = np.random.default_rng(8)
    P = {"a": rng.standard_normal((5, 3)), "b": rng.standard_normal(4)}
    G = {"a": rng.standard_normal((5, 3)), "b": np.zeros(4)}
    Z = {k: np.zeros_like(v) for k, v in P.items()}
    lr, wd, eps = 1e-2, cfg["weight_decay"], cfg["adam_eps"]
    p1, m1, v1, t1 = O.adamw_step(cfg, P, G, Z, Z, 0, lr)
    assert t1 == 1
    # first step: bias-corrected moments are g and g^2
    np.testing.assert_allclose(p1["a"], P["a"] * (1 - lr * wd) - lr * G["a"] / (np.abs(G["a"]) + eps), rtol=1e-13)
    # zero gradient: pure decay, moments stay zero
    np.testing.assert_allclose(p1["b"], P["b"] * (1 - lr * wd), rtol=1e-15)
    assert not np.any(m1["b"]) and not np.any(v1["b"])
    # constant gradient keeps the corrected moments at g, g^2
    p, m, v, t = P, Z, Z, 0
    for _ in range(5):
        p, m, v, t = O.adamw_step(cfg, p, G, m, v, t, lr)
    np.testing.assert_allclose(m["a"] / (1 - cfg["beta1"] ** 5), G["a"], rtol=1e-13)
    np.testing.assert_allclose(v["a"] / (1 - cfg["beta2"] ** 5), G["a"] ** 2, rtol=1e-12)
    # library routine, several steps with varying gradients
    tp = {k: torch.tensor(v.copy(), requires_grad=True) for k, v in P.items()}
    opt = torch.optim.AdamW(list(tp.values()), lr=lr, betas=(cfg["beta1"], cfg["beta2"]), eps=eps,
                            weight_decay=wd)
    p, m, v, t = P, Z, Z, 0
    for s in range(4):
        Gs = {k: rng.standard_normal(P[k].shape) for k in P}
        for k in tp:
            tp[k].grad = torch.tensor(Gs[k])
        opt.step()
        p, m, v, t = O.adamw_step(cfg, p, Gs, m, v, t, lr)
    for k in P:
        np.testing.assert_allclose(p[k], tp[k].detach().numpy(), rtol=1e-12, atol=1e-15)


def test_train_step_moves_weights_by_lr_and_lowers_loss():
    cfg = micro_cfg(batch=2, seq=6)
    wl = micro_workload(cfg)
    P = wl["params"]
    Z = {k: np.zeros_like(v) for k, v in P.items()}
    lr = 1e-3
    loss, grads, p1, m1, v1, t1 = O.train_step(cfg, P, Z, Z, 0, wl["hidden"], wl["tokens"], wl["mask"], lr)
    for k in P:
        big = np.abs(grads[k]) > 1e-5
        step = p1[k] - P[k] * (1 - lr * cfg["weight_decay"])
        np.testing.assert_allclose(step[big], -lr * np.sign(grads[k][big]), rtol=2e-3)
    loss1, _ = O.forward(cfg, p1, wl["hidden"], wl["tokens"], wl["mask"])
    assert loss1 < loss


def test_top1_lowest_index_on_ties():
    rng = np.random.default_rng(9)
    yhat = rng.standard_normal((6, 5))
    w = rng.standard_normal((9, 5))
    w[7] = w[2]                      # duplicated row -> exact tie
    loss, lse, n, top1 = O.lmhead_ce_fwd(yhat, w, np.zeros(6, int), np.ones(6), want_top1=True)
    z = yhat @ w.T
    for t in range(6):
        best = max(range(9), key=lambda j: (z[t, j], -j))
        assert top1[t] == best
        assert top1[t] != 7


def test_top1_accuracy_definition():
    # brute force on a tiny case, and the two extremes
    rng = np.random.default_rng(10)
    T, V = 12, 7
    z = rng.standard_normal((T, V))
    tok = rng.integers(0, V, T)
    mask = (rng.random(T) > 0.3).astype(np.uint8)
    top1 = np.array([max(range(V), key=lambda j: (z[t, j], -j)) for t in range(T)])
    hits = sum(1 for t in range(T) if mask[t] and top1[t] == tok[t])
    assert O.top1_accuracy(top1, tok, mask, V) == hits / max(1, int(mask.sum()))
    assert O.top1_accuracy(tok.copy(), tok, mask, V) == 1.0
    assert O.top1_accuracy((tok + 1) % V, tok, mask, V) == 0.0
    assert O.top1_accuracy(tok, tok, np.zeros(T, np.uint8), V) == 0.0        # N = max(1, 0): no position counts
    bad = tok.copy(); bad[0] = V + 3                                          # out-of-range label never counts
    m1 = np.ones(T, np.uint8)
    assert O.top1_accuracy(bad, bad, m1, V) == (T - 1) / (T - 1)


def _tiny_ragged(seed=21):
    """A small fp64 problem with ragged sequences: (cfg, params, per-sequence lists)."""
    cfg = dict(W.get_config("tiny"), hidden=32, n_heads=4, n_kv_heads=2, head_dim=8, ffn=48, vocab=50,
               target_hidden=12, n_capture=3)
    rng = np.random.default_rng(seed)
    params = W.make_params(cfg, rng)
    params = {k: np.asarray(v, np.float64) for k, v in params.items()}
    lens = [5, 1, 7, 3]
    KH = cfg["n_capture"] * cfg["target_hidden"]
    hid = [rng.standard_normal((n, KH)) for n in lens]
    tok = [rng.integers(0, cfg["vocab"], n) for n in lens]
    msk = [(rng.random(n) > 0.3).astype(np.uint8) for n in lens]
    msk[1][:] = 0                      # a sequence without any loss position
    return cfg, params, lens, hid, tok, msk


def test_packed_equals_fixed_batch_when_lengths_are_equal():
    cfg = dict(W.get_config("tiny"), hidden=32, n_heads=4, n_kv_heads=2, head_dim=8, ffn=48, vocab=50,
               target_hidden=12, n_capture=3, batch=3, seq=6)
    rng = np.random.default_rng(5)
    params = {k: np.asarray(v, np.float64) for k, v in W.make_params(cfg, rng).items()}
    KH = cfg["n_capture"] * cfg["target_hidden"]
    hid = rng.standard_normal((3, 6, KH))
    tok = rng.integers(0, cfg["vocab"], (3, 6))
    msk = (rng.random((3, 6)) > 0.25).astype(np.uint8)
    loss, cache = O.forward(cfg, params, hid, tok, msk)
    g = O.backward(cfg, params, cache, tok, msk)
    loss_p, g_p, _ = O.train_quantities_packed(cfg, params, hid.reshape(18, KH), tok.reshape(-1), msk.reshape(-1), [0, 6, 12, 18])
    assert loss_p == pytest.approx(loss, rel=1e-13)
    for k in g:
        assert np.max(np.abs(g_p[k] - g[k])) <= 1e-13 * max(1.0, np.max(np.abs(g[k]))), k


def test_packed_equals_right_padded_batch():
    # the same ragged sequences, once packed back to back and once right-padded to the longest with the pads
    # masked: causality keeps the pads from reaching any real position, so loss and gradients agree
    cfg, params, lens, hid, tok, msk = _tiny_ragged()
    S, B, KH = max(lens), len(lens), hid[0].shape[1]
    hp = np.zeros((B, S, KH)); tp = np.zeros((B, S), np.int64); mp = np.zeros((B, S), np.uint8)
    for i, n in enumerate(lens):
        hp[i, :n], tp[i, :n], mp[i, :n] = hid[i], tok[i], msk[i]
    cpad = dict(cfg, batch=B, seq=S)
    loss, cache = O.forward(cpad, params, hp, tp, mp)
    g = O.backward(cpad, params, cache, tp, mp)
    cu = np.concatenate([[0], np.cumsum(lens)])
    T = int(cu[-1]) + 3                                   # three padding rows at the end of the packed buffer
    hr = np.concatenate(hid + [np.full((3, KH), 7.0)]); tr = np.concatenate(tok + [np.array([1, 2, 3])])
    mr = np.concatenate(msk + [np.ones(3, np.uint8)])     # the caller left the mask set on padding rows: ignored
    loss_p, g_p, top1 = O.train_quantities_packed(dict(cfg, batch=1, seq=T), params, hr, tr, mr, cu, want_top1=True)
    assert loss_p == pytest.approx(loss, rel=1e-12)
    for k in g:
        assert np.max(np.abs(g_p[k] - g[k])) <= 1e-12 * max(1.0, np.max(np.abs(g[k]))), k
    assert np.all(top1[int(cu[-1]):] == -1) and np.all(top1[:int(cu[-1])] >= 0)
    # an empty sequence in the middle changes nothing
    cu2 = [0, 5, 5, 6, 13, 16]
    loss_q, g_q, _ = O.train_quantities_packed(dict(cfg, batch=1, seq=T), params, hr, tr, mr, cu2)
    assert loss_q == pytest.approx(loss_p, rel=1e-14)
    # moving a boundary does change the result (the attention span of the moved rows differs)
    loss_r, _, _ = O.train_quantities_packed(dict(cfg, batch=1, seq=T), params, hr, tr, mr, [0, 4, 6, 13, 16])
    assert abs(loss_r - loss_p) > 1e-6


# ------------------------------------------------------------------ token-input variant
def test_token_input_against_torch_autograd():
    cfg, wl, params, tok = _tok_setup(batch=2, seq=9, n_heads=4, n_kv_heads=2, hidden=16, head_dim=4, ffn=12, vocab=37)
    loss, cache = O.forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"], tok=tok)
    grads = O.backward(cfg, params, cache, wl["tokens"], wl["mask"])
    tl, tg, _ = _torch_reference(cfg, params, wl, tok_in=tok)
    assert abs(loss - tl) <= 1e-12 * abs(tl)
    for k in O.PARAM_NAMES + ("w_in",):
        np.testing.assert_allclose(grads[k], tg[k], rtol=1e-9, atol=1e-13, err_msg=k)


def _tok_setup(**kw):
    cfg = micro_cfg(**kw)
    wl = micro_workload(cfg)
    ti = W.make_token_input(cfg, embed_rows=9)
    ti = {k: np.asarray(v, np.float64) if k != "input_ids" else v for k, v in ti.items()}
    params = dict(wl["params"], w_in=ti["w_in"])
    tok = dict(embed=ti["embed"], input_ids=ti["input_ids"])
    return cfg, wl, params, tok


def test_token_input_identity_projection_is_the_base_model():
    """W_in = [I | 0] passes the projected features through unchanged: loss and the ten base gradients are
    those of the model without token input (an independent code path of the oracle)."""
    cfg, wl, params, tok = _tok_setup()
    d = cfg["hidden"]
    params["w_in"] = np.concatenate([np.eye(d), np.zeros((d, d))], axis=1)
    base = {k: params[k] for k in O.PARAM_NAMES}
    l0, c0 = O.forward(cfg, base, wl["hidden"], wl["tokens"], wl["mask"])
    g0 = O.backward(cfg, base, c0, wl["tokens"], wl["mask"])
    l1, c1 = O.forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"], tok=tok)
    g1 = O.backward(cfg, params, c1, wl["tokens"], wl["mask"])
    assert abs(l1 - l0) <= 1e-13 * abs(l0)
    for k in O.PARAM_NAMES:
        assert np.max(np.abs(g1[k] - g0[k])) <= 1e-12 * max(1.0, np.max(np.abs(g0[k]))), k
    assert g1["w_in"].shape == (d, 2 * d) and np.max(np.abs(g1["w_in"])) > 0


def test_token_input_embedding_only_ignores_the_captured_states():
    """W_in = [0 | I]: the layer sees the embeddings alone, so the captured states cannot matter: changing
    them leaves the loss unchanged and dW_fc is exactly zero.  An out-of-range id is a zero embedding."""
    cfg, wl, params, tok = _tok_setup()
    d = cfg["hidden"]
    params["w_in"] = np.concatenate([np.zeros((d, d)), np.eye(d)], axis=1)
    l1, c1 = O.forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"], tok=tok)
    l2, _ = O.forward(cfg, params, wl["hidden"] * -3.0 + 1.0, wl["tokens"], wl["mask"], tok=tok)
    assert l1 == l2
    g = O.backward(cfg, params, c1, wl["tokens"], wl["mask"])
    assert not np.any(g["w_fc"] != 0)
    assert np.allclose(c1["x0"], O.embed_rows(tok["embed"], tok["input_ids"]), rtol=0, atol=0)
    bad = dict(tok, input_ids=tok["input_ids"].copy())
    bad["input_ids"][0, 0], bad["input_ids"][-1, -1] = -1, tok["embed"].shape[0]
    e = O.embed_rows(bad["embed"], bad["input_ids"])
    assert not np.any(e[0] != 0) and not np.any(e[-1] != 0) and np.any(e[1] != 0)


def test_token_input_finite_differences():
    cfg, wl, params, tok = _tok_setup(batch=2, seq=4, n_heads=4, n_kv_heads=2, hidden=16, ffn=10, vocab=13)
    loss, cache = O.forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"], tok=tok)
    grads = O.backward(cfg, params, cache, wl["tokens"], wl["mask"])
    rng = np.random.default_rng(1)
    h = 1e-6
    for name in ("w_in", "w_fc", "w_qkv", "g1", "w_lm"):
        flat = params[name].reshape(-1)
        for i in rng.choice(flat.size, size=min(16, flat.size), replace=False):
            pp = copy.deepcopy(params)
            pp[name].reshape(-1)[i] += h
            lp = O.forward(cfg, pp, wl["hidden"], wl["tokens"], wl["mask"], tok=tok)[0]
            pp[name].reshape(-1)[i] -= 2 * h
            lm = O.forward(cfg, pp, wl["hidden"], wl["tokens"], wl["mask"], tok=tok)[0]
            fd, an = (lp - lm) / (2 * h), grads[name].reshape(-1)[i]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)) + 2e-8, (name, i, fd, an)
