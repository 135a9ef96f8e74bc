"""Pins for the multi-step unroll oracle (forward).  The unroll stands for chain drafting with the true tokens
as inputs: process the verified prefix once, then append one position per draft step, each fed the layer output
of the step before.  That process is written here on its own, with a growing key/value cache, one start position
at a time and from plain NumPy (none of the oracle's functions), and every step of the oracle's batched unroll
must reproduce it row by row."""
import copy

import numpy as np
import pytest

from oracle import tide_oracle as O
from oracle import unroll_oracle as U
from tests.helpers import micro_cfg, micro_workload


def _token_input(cfg, seed=3):
    rng = np.random.default_rng(seed)
    d = cfg["hidden"]
    return dict(embed=rng.standard_normal((cfg["vocab"], d)), input_ids=rng.integers(0, cfg["vocab"], (cfg["batch"], cfg["seq"])),
                w_in=0.3 * rng.standard_normal((d, 2 * d)))


class ChainDrafter:
    """One sequence, one start position: the layer as a key/value-cache decoder."""

    def __init__(self, cfg, p, w_in=None, embed=None):
        self.c, self.p, self.w_in, self.embed = cfg, p, w_in, embed
        self.K, self.V = [], []   # one [n_kv, d_h] entry per cached position

    def _norm(self, x, g):
        return g * x / np.sqrt(np.mean(x * x) + self.c["rms_eps"])

    def _rot(self, x, pos):
        dh = self.c["head_dim"]
        half = dh // 2
        ang = pos * self.c["rope_theta"] ** (-2.0 * np.arange(half) / dh)
        x1, x2 = x[:, :half], x[:, half:]
        return np.concatenate([x1 * np.cos(ang) - x2 * np.sin(ang), x2 * np.cos(ang) + x1 * np.sin(ang)], axis=1)

    def step(self, feat, token_id, pos):
        """Appends position `pos` (feature vector, id of its input token) and returns (layer output, logits)."""
        c, p = self.c, self.p
        nh, nkv, dh = c["n_heads"], c["n_kv_heads"], c["head_dim"]
        x0 = feat if self.w_in is None else self.w_in @ np.concatenate([feat, self.embed[token_id]])
        qkv = p["w_qkv"] @ self._norm(x0, p["g1"])
        q = self._rot(qkv[:nh * dh].reshape(nh, dh), pos)
        k = self._rot(qkv[nh * dh:(nh + nkv) * dh].reshape(nkv, dh), pos)
        v = qkv[(nh + nkv) * dh:].reshape(nkv, dh)
        self.K.append(k)
        self.V.append(v)
        out = np.zeros((nh, dh))
        for h in range(nh):
            kh = h // (nh // nkv)
            sc = np.array([q[h] @ kk[kh] for kk in self.K]) / np.sqrt(dh)
            w = np.exp(sc - sc.max())
            w /= w.sum()
            out[h] = sum(wi * vv[kh] for wi, vv in zip(w, self.V))
        x1 = x0 + p["w_o"] @ out.reshape(-1)
        bn = self._norm(x1, p["g2"])
        gt = p["w_gate"] @ bn
        x2 = x1 + p["w_down"] @ (gt / (1.0 + np.exp(-gt)) * (p["w_up"] @ bn))
        return x2, p["w_lm"] @ self._norm(x2, p["g3"])


@pytest.mark.parametrize("token_input", [False, True])
@pytest.mark.parametrize("kw", [dict(seq=7), dict(seq=9, n_heads=4, n_kv_heads=2, hidden=16, head_dim=4, ffn=10, vocab=13)])
def test_unroll_equals_chain_drafting_with_a_key_value_cache(kw, token_input):
    cfg = micro_cfg(mask="none", **kw)
    wl = micro_workload(cfg)
    p = {k: np.asarray(v, np.float64) for k, v in wl["params"].items()}
    tok = _token_input(cfg) if token_input else None
    params = dict(wl["params"], **({O.TOKEN_PARAM: tok["w_in"]} if tok else {}))
    n_steps, S = 3, cfg["seq"]
    steps = U.unroll_forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"], n_steps, tok=tok)
    feats = wl["hidden"].reshape(S, -1) @ p["w_fc"].T
    ids = tok["input_ids"].reshape(-1) if tok else np.zeros(S, int)
    labels = wl["tokens"].reshape(-1)
    nll = [[] for _ in range(n_steps)]
    for t0 in range(S):
        dr = ChainDrafter(cfg, p, tok["w_in"] if tok else None, tok["embed"] if tok else None)
        for pos in range(t0 + 1):                       # the verified prefix, captured features
            out, z = dr.step(feats[pos], ids[pos], pos)
        for s in range(1, n_steps + 1):
            pos = t0 + s - 1
            if pos >= S:
                break
            if s > 1:
                out, z = dr.step(out, ids[pos], pos)    # fed its own output, the true token as input
            np.testing.assert_allclose(steps[s - 1]["x2"][t0], out, rtol=1e-10, atol=1e-12)
            assert steps[s - 1]["top1"][t0] == int(np.argmax(z))
            nll[s - 1].append(np.log(np.sum(np.exp(z - z.max()))) + z.max() - z[labels[pos]])
    for s in range(n_steps):
        assert steps[s]["n"] == S - s == len(nll[s])
        assert abs(steps[s]["loss"] - np.mean(nll[s])) <= 1e-12 * max(1.0, abs(steps[s]["loss"]))


def test_one_step_is_the_ordinary_forward_and_masks_shift_with_the_labels():
    cfg = micro_cfg(batch=2, seq=6, mask="bernoulli", mask_p=0.4)
    wl = micro_workload(cfg)
    loss, cache = O.forward(cfg, wl["params"], wl["hidden"], wl["tokens"], wl["mask"], want_top1=True)
    steps = U.unroll_forward(cfg, wl["params"], wl["hidden"], wl["tokens"], wl["mask"], 3)
    assert steps[0]["loss"] == loss and np.array_equal(steps[0]["top1"], cache["top1"])
    np.testing.assert_array_equal(steps[0]["x2"], cache["x2"])
    for s, st in enumerate(steps):
        assert np.array_equal(st["mask"][:, :cfg["seq"] - s], wl["mask"][:, s:])
        assert not st["mask"][:, cfg["seq"] - s:].any()           # rows whose position left the sequence
        assert np.array_equal(st["tokens"][:, :cfg["seq"] - s], wl["tokens"][:, s:])
        assert st["n"] == max(1, int((st["mask"] != 0).sum()))


def test_later_steps_do_not_see_other_rows_later_keys():
    """Changing the captured states of the last row changes no other row at any step (causality carries over)."""
    cfg = micro_cfg(seq=6, mask="none")
    wl = micro_workload(cfg)
    a = U.unroll_forward(cfg, wl["params"], wl["hidden"], wl["tokens"], wl["mask"], 3)
    h2 = wl["hidden"].copy()
    h2[0, -1] += 1.0
    b = U.unroll_forward(cfg, wl["params"], h2, wl["tokens"], wl["mask"], 3)
    for s in range(3):
        np.testing.assert_array_equal(a[s]["x2"][:-1], b[s]["x2"][:-1])
        assert np.abs(a[s]["x2"][-1] - b[s]["x2"][-1]).max() > 1e-6


def _weighted_loss(cfg, params, wl, tok, w):
    steps = U.unroll_forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"], len(w), tok=tok)
    return sum(wi * st["loss"] for wi, st in zip(w, steps))


@pytest.mark.parametrize("token_input", [False, True])
@pytest.mark.parametrize("kw", [dict(seq=6), dict(batch=2, seq=5, n_heads=4, n_kv_heads=2, hidden=16, head_dim=4, ffn=10, vocab=13)])
def test_unroll_gradients_by_finite_differences(kw, token_input):
    cfg = micro_cfg(mask="bernoulli", mask_p=0.3, **kw)
    wl = micro_workload(cfg)
    tok = _token_input(cfg) if token_input else None
    params = {k: np.asarray(v, np.float64) for k, v in wl["params"].items()}
    if tok:
        params[O.TOKEN_PARAM] = tok["w_in"]
    w = [1.0, 0.7, 0.45]
    steps = U.unroll_forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"], 3, tok=tok, keep_cache=True)
    grads = U.unroll_backward(cfg, params, steps, step_weights=w)
    rng = np.random.default_rng(1)
    h = 1e-6
    for name, g in grads.items():
        assert g.shape == params[name].shape
        idx = rng.choice(g.size, size=min(10, g.size), replace=False)
        for i in idx:
            pp = copy.deepcopy(params)
            pp[name].reshape(-1)[i] += h
            lp = _weighted_loss(cfg, pp, wl, tok, w)
            pp[name].reshape(-1)[i] -= 2 * h
            lm = _weighted_loss(cfg, pp, wl, tok, w)
            fd = (lp - lm) / (2 * h)
            an = g.reshape(-1)[i]
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(fd)) + 5e-8, (name, i, fd, an)


def test_one_step_gradients_are_the_single_step_gradients():
    cfg = micro_cfg(batch=2, seq=6, mask="bernoulli", mask_p=0.3)
    wl = micro_workload(cfg)
    tok = _token_input(cfg)
    params = dict({k: np.asarray(v, np.float64) for k, v in wl["params"].items()}, **{O.TOKEN_PARAM: tok["w_in"]})
    _, cache = O.forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"], tok=tok)
    ref = O.backward(cfg, params, cache, wl["tokens"], wl["mask"])
    got = U.unroll_backward(cfg, params, U.unroll_forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"], 1, tok=tok, keep_cache=True))
    for k in ref:
        np.testing.assert_allclose(got[k], ref[k], rtol=1e-12, atol=1e-14)


def test_packed_unroll_of_equal_lengths_is_the_batched_unroll():
    """The per-sequence combination (shares n_is / N_s) reproduces the batched definition when all sequences have
    the batch's length, losses and gradients alike."""
    cfg = micro_cfg(batch=3, seq=5, mask="bernoulli", mask_p=0.4)
    wl = micro_workload(cfg)
    tok = _token_input(cfg)
    params = dict({k: np.asarray(v, np.float64) for k, v in wl["params"].items()}, **{O.TOKEN_PARAM: tok["w_in"]})
    w = [1.0, 0.6, 0.3]
    steps = U.unroll_forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"], 3, tok=tok, keep_cache=True)
    g_ref = U.unroll_backward(cfg, params, steps, step_weights=w)
    T = cfg["batch"] * cfg["seq"]
    losses, g = U.unroll_train_quantities_packed(cfg, params, wl["hidden"].reshape(T, -1), wl["tokens"].reshape(-1),
                                                 wl["mask"].reshape(-1), [0, 5, 10, 15], 3,
                                                 tok=dict(embed=tok["embed"], input_ids=tok["input_ids"].reshape(-1)), step_weights=w)
    for s in range(3):
        assert abs(losses[s] - steps[s]["loss"]) <= 1e-12 * max(1.0, abs(losses[s]))
    for k in g_ref:
        np.testing.assert_allclose(g[k], g_ref[k], rtol=1e-10, atol=1e-13)


def _torch_unroll(cfg, params, wl, tok, n_steps, w):
    """The unroll composed from torch CPU fp64 library primitives + autograd.  Attention of step s: the keys and
    values of ALL steps so far concatenated along the sequence ([s * S] of them) under a mask that is causal on the
    step-1 block and the identity on every later block, through F.scaled_dot_product_attention."""
    import torch
    import torch.nn.functional as F
    B, S = cfg["batch"], cfg["seq"]
    nh, nkv, dh = cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    G = nh // nkv
    P = {k: torch.tensor(np.asarray(v, np.float64), requires_grad=True) for k, v in params.items()}
    feat = F.linear(torch.tensor(wl["hidden"], dtype=torch.float64).reshape(B * S, -1), P["w_fc"])
    tokens = torch.tensor(wl["tokens"].astype(np.int64))
    mask = torch.tensor(wl["mask"].astype(np.float64))
    ids = torch.tensor(np.asarray(tok["input_ids"]).astype(np.int64)) if tok else None
    E = torch.tensor(np.asarray(tok["embed"], np.float64)) if tok else None
    half = dh // 2
    inv = torch.tensor(cfg["rope_theta"], dtype=torch.float64) ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)

    def rms(x, g):
        return g * x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + cfg["rms_eps"])

    def rope(x, shift):
        ang = (torch.arange(S, dtype=torch.float64) + shift)[:, None] * inv[None]
        cos = torch.cat([ang.cos(), ang.cos()], -1)[None, :, None, :]
        sin = torch.cat([ang.sin(), ang.sin()], -1)[None, :, None, :]
        return x * cos + torch.cat([-x[..., half:], x[..., :half]], -1) * sin

    keys, vals, losses = [], [], []
    total = 0.0
    for s in range(n_steps):
        valid = torch.zeros(B, S, dtype=torch.float64)
        valid[:, :S - s] = 1.0 if S - s > 0 else 0.0
        lab = torch.roll(tokens, -s, dims=1)
        m = torch.roll(mask, -s, dims=1) * valid
        if tok:
            e = F.embedding(torch.roll(ids, -s, dims=1).reshape(-1), E) * valid.reshape(-1, 1)
            x0 = F.linear(torch.cat([feat, e], dim=1), P["w_in"])
        else:
            x0 = feat
        qkv = F.linear(rms(x0, P["g1"]), P["w_qkv"])
        q = rope(qkv[:, :nh * dh].reshape(B, S, nh, dh), s)
        k = rope(qkv[:, nh * dh:(nh + nkv) * dh].reshape(B, S, nkv, dh), s)
        v = qkv[:, (nh + nkv) * dh:].reshape(B, S, nkv, dh)
        keys.append(k.repeat_interleave(G, dim=2).transpose(1, 2))
        vals.append(v.repeat_interleave(G, dim=2).transpose(1, 2))
        allow = torch.cat([torch.tril(torch.ones(S, S, dtype=torch.bool))] + [torch.eye(S, dtype=torch.bool)] * s, dim=1)
        A = F.scaled_dot_product_attention(q.transpose(1, 2), torch.cat(keys, dim=2), torch.cat(vals, dim=2), attn_mask=allow)
        x1 = x0 + F.linear(A.transpose(1, 2).reshape(B * S, nh * dh), P["w_o"])
        b = rms(x1, P["g2"])
        x2 = x1 + F.linear(F.silu(F.linear(b, P["w_gate"])) * F.linear(b, P["w_up"]), P["w_down"])
        z = F.linear(rms(x2, P["g3"]), P["w_lm"])
        per = F.cross_entropy(z, lab.reshape(-1), reduction="none")
        loss = (per * m.reshape(-1)).sum() / max(1.0, float(m.sum()))
        losses.append(float(loss.detach()))
        total = total + w[s] * loss
        feat = x2
    total.backward()
    return losses, {k: t.grad.numpy() for k, t in P.items()}


@pytest.mark.parametrize("token_input", [False, True])
def test_unroll_against_torch_autograd(token_input):
    cfg = micro_cfg(batch=2, seq=7, n_heads=4, n_kv_heads=2, hidden=16, head_dim=4, ffn=12, vocab=37, mask="bernoulli", mask_p=0.3)
    wl = micro_workload(cfg)
    tok = _token_input(cfg) if token_input else None
    params = {k: np.asarray(v, np.float64) for k, v in wl["params"].items()}
    if tok:
        params[O.TOKEN_PARAM] = tok["w_in"]
    w = [1.0, 0.7, 0.45]
    steps = U.unroll_forward(cfg, params, wl["hidden"], wl["tokens"], wl["mask"], 3, tok=tok, keep_cache=True)
    grads = U.unroll_backward(cfg, params, steps, step_weights=w)
    t_losses, t_grads = _torch_unroll(cfg, params, wl, tok, 3, w)
    for s in range(3):
        assert abs(steps[s]["loss"] - t_losses[s]) <= 1e-12 * max(1.0, abs(t_losses[s])), s
    for k in grads:
        np.testing.assert_allclose(grads[k], t_grads[k], rtol=1e-9, atol=1e-13, err_msg=k)
