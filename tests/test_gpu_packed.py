"""Packed (variable-length) batches: tide_draft_forward_packed / tide_draft_train_step_packed through the
C ABI against the oracle's per-sequence definition, and against the library's own fixed-layout entry points
on the same sequences right-padded.  Covers ragged lengths, a length-1 and an empty sequence, sequences that
straddle the 128-row attention blocks, padding rows at the end of the buffer (with the mask left set and
non-zero hidden states there), and the error codes of the two entry points."""
import numpy as np
import pytest
import torch

from oracle import tide_oracle as O
from paper_2602_05145_amd import workloads as W
from tests.gpu_util import cosine, rel_max, sync

pytestmark = pytest.mark.gpu


def ragged_workload(cfg, lens, tail, seed):
    """Rows = the sequences back to back + `tail` padding rows.  Same distributions as workloads.make_inputs."""
    T = sum(lens) + tail
    c = dict(cfg, batch=1, seq=T)
    wl = W.make_workload(dict(c, seed=seed))
    rng = np.random.default_rng(seed + 1)
    mask = (rng.random(T) > 0.2).astype(np.uint8)       # independent of sequence boundaries
    if tail:
        mask[-tail:] = 1                                 # left set on purpose: padding rows must be ignored
    wl["mask"] = mask.reshape(1, T)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return c, wl, cu


def run_packed(c, wl, cu, lr):
    from paper_2602_05145_amd import runtime
    tr = runtime.trainer_from_workload(c, wl)
    tr.set_packed(cu)
    loss_f, top1 = tr.forward_packed(want_top1=True)
    sync()
    lf = float(loss_f.item())
    tr.train_step_packed(lr)
    sync()
    return tr, lf, top1.cpu().numpy(), float(tr.loss.item())


def test_packed_fp32_against_oracle():
    cfg = W.get_config("tiny")
    lens = [37, 1, 0, 64, 19, 5]
    c, wl, cu = ragged_workload(cfg, lens, tail=6, seed=77)
    lr = cfg["lr"]
    p0 = {k: np.asarray(v, np.float64) for k, v in wl["params"].items()}
    T = c["seq"]
    loss_ref, g_ref, top1_ref = O.train_quantities_packed(c, p0, wl["hidden"].astype(np.float64).reshape(T, -1), wl["tokens"].reshape(-1),
                                                          wl["mask"].reshape(-1), cu, want_top1=True)
    tr, loss_fwd, top1, loss = run_packed(c, wl, cu, lr)
    assert abs(loss - loss_ref) <= 1e-4 * abs(loss_ref), (loss, loss_ref)
    assert abs(loss_fwd - loss_ref) <= 1e-4 * abs(loss_ref)
    g = tr.host(tr.grads)
    for k in O.PARAM_NAMES:
        assert np.all(np.isfinite(g[k])), k
        assert rel_max(g[k], g_ref[k]) <= 1e-4, (k, rel_max(g[k], g_ref[k]))
    n_real = int(cu[-1])
    # arg-max ids of the real rows (fp32: equal wherever the oracle's top-2 margin is not rounding-sized)
    same = top1[:n_real] == top1_ref[:n_real]
    assert same.mean() > 0.98
    # AdamW consumed these gradients: parameters moved by at most lr
    p = tr.host(tr.params)
    for k in O.PARAM_NAMES:
        assert np.max(np.abs(p[k] - p0[k] * (1 - lr * cfg["weight_decay"]))) <= lr * (1 + 1e-3), k


@pytest.mark.parametrize("lens,tail", [([200, 56, 128, 129, 3], 12), ([516], 12), ([1] * 40 + [250, 238], 0)])
def test_packed_bf16_against_oracle(lens, tail):
    cfg = W.get_config("small", batch=1, seq=64, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    c, wl, cu = ragged_workload(cfg, lens, tail, seed=91)
    lr = cfg["lr"]
    p0 = {k: np.asarray(v, np.float64) for k, v in wl["params"].items()}
    T = c["seq"]
    loss_ref, g_ref, _ = O.train_quantities_packed(c, p0, wl["hidden"].astype(np.float64).reshape(T, -1), wl["tokens"].reshape(-1),
                                                   wl["mask"].reshape(-1), cu)
    tr, loss_fwd, top1, loss = run_packed(c, wl, cu, lr)
    assert abs(loss - loss_ref) <= 1e-2 * abs(loss_ref), (loss, loss_ref)
    assert abs(loss_fwd - loss) <= 1e-5 * abs(loss)
    g = tr.host(tr.grads)
    for k in O.PARAM_NAMES:
        assert np.all(np.isfinite(g[k])), k
        assert cosine(g[k], g_ref[k]) >= 0.999, (k, cosine(g[k], g_ref[k]))


@pytest.mark.parametrize("seed", range(6))
def test_packed_random_segmentations_bf16(seed):
    """Seeded random segmentations: 1 to 24 sequences of 0 to 300 rows (several empty ones, runs of length 1,
    batch x kv heads sometimes a multiple of 8, which switches the attention's block numbering), random tail."""
    rng = np.random.default_rng(300 + seed)
    n = int(rng.choice([1, 3, 8, 16, 24]))
    lens = [int(x) for x in rng.integers(0, 301, size=n)]
    for i in rng.choice(n, size=max(1, n // 4), replace=False):
        lens[int(i)] = int(rng.choice([0, 1, 2]))
    if sum(lens) == 0:
        lens[0] = 17
    tail = int(rng.integers(0, 20))
    nkv = int(rng.choice([1, 2]))
    cfg = W.get_config("small", batch=1, seq=64, target_hidden=48, hidden=256, n_heads=2, n_kv_heads=nkv,
                       head_dim=128, ffn=200, vocab=777)
    print(f"seed {seed}: {n} sequences, {sum(lens)} rows + {tail} padding, n_kv_heads {nkv}", flush=True)
    c, wl, cu = ragged_workload(cfg, lens, tail, seed=400 + seed)
    p0 = {k: np.asarray(v, np.float64) for k, v in wl["params"].items()}
    T = c["seq"]
    loss_ref, g_ref, _ = O.train_quantities_packed(c, p0, wl["hidden"].astype(np.float64).reshape(T, -1), wl["tokens"].reshape(-1),
                                                   wl["mask"].reshape(-1), cu)
    tr, loss_fwd, top1, loss = run_packed(c, wl, cu, cfg["lr"])
    assert tr.status() == 0
    assert abs(loss - loss_ref) <= 1e-2 * abs(loss_ref), (loss, loss_ref)
    g = tr.host(tr.grads)
    for k in O.PARAM_NAMES:
        assert np.all(np.isfinite(g[k])), k
        assert cosine(g[k], g_ref[k]) >= 0.999, (k, cosine(g[k], g_ref[k]))


def test_packed_equals_right_padded_fixed_batch_on_the_gpu():
    """The same sequences through the fixed-layout entry point (right-padded, pads masked) and packed."""
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("small", batch=1, seq=64, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    lens = [130, 64, 7, 160]
    c, wl, cu = ragged_workload(cfg, lens, tail=0, seed=33)
    S, B, KH = max(lens), len(lens), wl["hidden"].shape[-1]
    hid = wl["hidden"].reshape(-1, KH); tok = wl["tokens"].reshape(-1); msk = wl["mask"].reshape(-1)
    hp = np.zeros((B, S, KH), hid.dtype); tp = np.zeros((B, S), tok.dtype); mp = np.zeros((B, S), np.uint8)
    for i, n in enumerate(lens):
        a = int(cu[i])
        hp[i, :n], tp[i, :n], mp[i, :n] = hid[a:a + n], tok[a:a + n], msk[a:a + n]
    cpad = dict(c, batch=B, seq=S)
    tr_pad = runtime.trainer_from_workload(cpad, dict(params=wl["params"], hidden=hp, tokens=tp, mask=mp))
    tr_pad.train_step(cfg["lr"])
    tr, _, _, loss = run_packed(c, wl, cu, cfg["lr"])
    sync()
    assert abs(loss - float(tr_pad.loss.item())) <= 2e-3 * abs(loss)
    g, gp = tr.host(tr.grads), tr_pad.host(tr_pad.grads)
    for k in O.PARAM_NAMES:
        assert cosine(g[k], gp[k]) >= 0.9995, (k, cosine(g[k], gp[k]))


def test_packed_with_equal_lengths_is_the_fixed_layout():
    """cu_seqlens = multiples of seq reproduces the fixed-layout result bit for bit (same kernels, same order)."""
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("small", batch=3, seq=160, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    wl = W.make_workload(cfg)
    a = runtime.trainer_from_workload(cfg, wl)
    a.train_step(cfg["lr"])
    b = runtime.trainer_from_workload(cfg, wl)
    b.set_packed([0, 160, 320, 480])
    b.train_step_packed(cfg["lr"])
    sync()
    assert float(a.loss.item()) == float(b.loss.item())
    for k in O.PARAM_NAMES:
        assert torch.equal(a.grads[k], b.grads[k]), k
        assert torch.equal(a.params[k], b.params[k]), k


def test_packed_argument_errors():
    from paper_2602_05145_amd import binding as B, runtime
    cfg = W.get_config("tiny")
    wl = W.make_workload(cfg)
    tr = runtime.trainer_from_workload(cfg, wl)
    tr.set_packed([0, 10, 128])
    T = cfg["batch"] * cfg["seq"]
    s = tr._stream()
    def fwd(cu, n, m):
        return B.tide_draft_forward_packed(tr.ccfg, tr.c_params, tr.hidden, tr.tokens, tr.mask, cu, n, m, tr.loss, None,
                                           tr.workspace, tr.ws_bytes, s, check=False)
    assert fwd(None, 2, 118) == B.TIDE_ERR_NULL
    assert fwd(tr.cu, 0, 118) == B.TIDE_ERR_CONFIG and fwd(tr.cu, 70000, 118) == B.TIDE_ERR_CONFIG
    assert fwd(tr.cu, 2, 0) == B.TIDE_ERR_CONFIG and fwd(tr.cu, 2, T + 1) == B.TIDE_ERR_CONFIG
    assert "max_seqlen" in B.tide_last_error()
    assert fwd(tr.cu, 2, 118) == 0
    rc = B.tide_draft_train_step_packed(tr.ccfg, tr.c_params, tr.c_grads, tr.c_adam, tr.hidden, tr.tokens, tr.mask, None, 2, 118,
                                        1e-3, tr.loss, tr.workspace, tr.ws_bytes, s, check=False)
    assert rc == B.TIDE_ERR_NULL and tr.step == 0
    sync()
