"""Multi-step unroll (and, with one step, the token-input model) on PACKED batches through the C ABI against the
oracle's per-sequence definition: ragged lengths, a length-1 and an empty sequence, sequences shorter than the
number of steps, padding rows at the end of the buffer with the mask left set.  Tolerances of the single step."""
import numpy as np
import pytest
import torch

from oracle import tide_oracle as O
from oracle import unroll_oracle as U
from paper_2602_05145_amd import workloads as W
from tests.gpu_util import cosine, rel_max, sync
from tests.test_gpu_packed import ragged_workload

pytestmark = pytest.mark.gpu


def _setup(cfg, lens, tail, seed, token_input):
    from paper_2602_05145_amd import runtime
    c, wl, cu = ragged_workload(cfg, lens, tail, seed)
    tr = runtime.trainer_from_workload(c, wl)
    tr.set_packed(cu)
    params = {k: np.asarray(v, np.float64) for k, v in wl["params"].items()}
    tok = None
    if token_input:
        ti = W.make_token_input(c, embed_rows=min(c["vocab"], 301))
        tr.set_token_input(ti["embed"], ti["input_ids"], ti["w_in"])
        params["w_in"] = np.asarray(ti["w_in"], np.float64)
        tok = dict(embed=np.asarray(ti["embed"], np.float64), input_ids=ti["input_ids"].reshape(-1))
    return c, wl, cu, tr, params, tok


def _reference(c, wl, cu, params, tok, n_steps, w):
    T = c["seq"]
    return U.unroll_train_quantities_packed(c, params, wl["hidden"].astype(np.float64).reshape(T, -1), wl["tokens"].reshape(-1),
                                            wl["mask"].reshape(-1), cu, n_steps, tok=tok, step_weights=w)


def _grads(tr, token_input):
    g = tr.host(tr.grads)
    if token_input:
        g["w_in"] = tr.grad_w_in.cpu().numpy().astype(np.float64)
    return g


@pytest.mark.parametrize("token_input", [False, True])
def test_packed_unroll_fp32(token_input):
    cfg = W.get_config("tiny")
    lens = [37, 1, 0, 64, 2, 19, 5]
    c, wl, cu, tr, params, tok = _setup(cfg, lens, 6, 91, token_input)
    w = [1.0, 0.7, 0.45]
    loss_ref, g_ref = _reference(c, wl, cu, params, tok, 3, w)
    ev_loss, ev_acc = tr.eval_unroll(3, token_input=token_input, packed=True)
    loss = tr.train_step_unroll(c["lr"], 3, step_weights=w, token_input=token_input, packed=True)
    sync()
    for s in range(3):
        assert abs(float(loss[s].item()) - loss_ref[s]) <= 1e-4 * abs(loss_ref[s]), (s, float(loss[s].item()), loss_ref[s])
        assert abs(float(ev_loss[s].item()) - loss_ref[s]) <= 1e-4 * abs(loss_ref[s]), s
        assert 0.0 <= float(ev_acc[s].item()) <= 1.0
    g = _grads(tr, token_input)
    for k in g_ref:
        assert np.all(np.isfinite(g[k])), k
        assert rel_max(g[k], g_ref[k]) <= 1e-4, (k, rel_max(g[k], g_ref[k]))


def test_packed_token_input_single_step_fp32():
    """One step of the unroll with a token input: the token-input model on a packed batch."""
    cfg = W.get_config("tiny")
    c, wl, cu, tr, params, tok = _setup(cfg, [20, 33, 1, 40], 3, 17, True)
    loss_ref, g_ref = _reference(c, wl, cu, params, tok, 1, None)
    loss = tr.train_step_unroll(c["lr"], 1, token_input=True, packed=True)
    sync()
    assert abs(float(loss[0].item()) - loss_ref[0]) <= 1e-4 * abs(loss_ref[0])
    g = _grads(tr, True)
    for k in g_ref:
        assert rel_max(g[k], g_ref[k]) <= 1e-4, (k, rel_max(g[k], g_ref[k]))


def test_packed_unroll_without_token_input_one_step_is_the_packed_training_step():
    cfg = W.get_config("small", batch=1, seq=8, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128, ffn=256, vocab=512)
    from paper_2602_05145_amd import runtime
    c, wl, cu = ragged_workload(cfg, [130, 0, 1, 259], 10, 5)
    a = runtime.trainer_from_workload(c, wl)
    b = runtime.trainer_from_workload(c, wl)
    a.set_packed(cu)
    b.set_packed(cu)
    la = a.train_step_unroll(c["lr"], 1, packed=True)
    b.train_step_packed(c["lr"])
    sync()
    assert float(la[0].item()) == float(b.loss.item())
    for k in O.PARAM_NAMES:
        assert torch.equal(a.grads[k], b.grads[k]) and torch.equal(a.params[k], b.params[k]), k


@pytest.mark.parametrize("lens,tail", [([130, 1, 259], 10), ([64, 128, 3, 200, 5], 0)])
def test_packed_unroll_bf16(lens, tail):
    cfg = W.get_config("small", batch=1, seq=8, target_hidden=64, hidden=512, n_heads=4, n_kv_heads=2, head_dim=128, ffn=256, vocab=512)
    c, wl, cu, tr, params, tok = _setup(cfg, lens, tail, 23, True)
    w = [1.0, 0.8, 0.64]
    loss_ref, g_ref = _reference(c, wl, cu, params, tok, 3, w)
    zeros = {k: np.zeros_like(v) for k, v in params.items()}
    p1_ref, *_ = O.adamw_step(c, params, g_ref, zeros, zeros, 0, c["lr"])
    loss = tr.train_step_unroll(c["lr"], 3, step_weights=w, token_input=True, packed=True)
    sync()
    for s in range(3):
        assert abs(float(loss[s].item()) - loss_ref[s]) <= 1e-2 * abs(loss_ref[s]), s
    g = _grads(tr, True)
    for k in g_ref:
        assert np.all(np.isfinite(g[k])), k
        assert cosine(g[k], g_ref[k]) >= 0.999, (k, cosine(g[k], g_ref[k]))
    p = tr.host(tr.master)
    for k in O.PARAM_NAMES:
        assert np.max(np.abs(p[k] - p1_ref[k])) <= 2e-3, k


def test_packed_unroll_poisoned_workspace_and_padding_rows():
    """Padding rows hold unwritten statistics (NaN bit patterns here): whatever the merge kernels make of them must
    be gone before the contractions over all rows."""
    from paper_2602_05145_amd import binding as B
    cfg = W.get_config("small", batch=1, seq=8, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128, ffn=256, vocab=512)
    out = []
    for poison in (False, True):
        c, wl, cu, tr, params, tok = _setup(cfg, [130, 0, 1, 200], 20, 3, True)
        need = B.tide_draft_unroll_workspace_bytes(tr.ccfg, 3)
        tr.unroll_ws = torch.full((need,), 0xFF if poison else 0, dtype=torch.uint8, device=tr.device)
        if poison:
            for g_ in tr.grads.values():
                g_.fill_(float("nan"))
            tr.grad_w_in.fill_(float("nan"))
        loss = tr.train_step_unroll(c["lr"], 3, token_input=True, packed=True).clone()
        sync()
        out.append((tr, loss))
    (a, la), (b, lb) = out
    assert torch.equal(la, lb) and bool(torch.isfinite(lb).all())
    for k in O.PARAM_NAMES:
        assert bool(torch.isfinite(b.grads[k]).all()), k
        assert torch.equal(a.grads[k], b.grads[k]), k
    assert torch.equal(a.grad_w_in, b.grad_w_in)


def test_packed_unroll_malformed_offsets_are_reported_not_followed():
    """Offsets that the host cannot check are clamped by the kernels that use them (every access stays inside the
    buffers) and reported through the status word of the first step's workspace."""
    from paper_2602_05145_amd import binding as B
    cfg = W.get_config("small", batch=1, seq=8, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128, ffn=256, vocab=512)
    c, wl, cu, tr, params, tok = _setup(cfg, [130, 1, 259], 10, 5, True)

    def status():
        off = B.tide_draft_unroll_workspace_offset(tr.ccfg, 3, 0, "status")
        return int(tr.unroll_ws[off:off + 4].view(torch.int32).item())
    tr.eval_unroll(3, token_input=True, packed=True)
    sync()
    assert status() == 0
    for bad in ([0, 200, 100, 390], [-5, 100, 390], [0, 100, 500], [0, 10, 390]):
        tr.set_packed(bad, max_seqlen=260)
        tr.eval_unroll(3, token_input=True, packed=True)
        sync()
        assert status() == 2, bad
    tr.set_packed(cu)
    loss, _ = tr.eval_unroll(3, token_input=True, packed=True)
    sync()
    assert status() == 0 and bool(torch.isfinite(loss).all())
