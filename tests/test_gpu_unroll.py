"""Multi-step evaluation unroll (the draft fed its own output from the second step on) through the C ABI against
the fp64 oracle: per-step loss within 1e-4 (fp32) / 1e-2 (bf16) relative, per-step accuracy within a few rows
(an arg-max can flip on a near tie), and the layer output of every step on the rows it selected."""
import numpy as np
import pytest
import torch

from oracle import tide_oracle as O
from oracle import unroll_oracle as U
from paper_2602_05145_amd import binding as B
from paper_2602_05145_amd import workloads as W
from tests.gpu_util import rel_max, sync

pytestmark = pytest.mark.gpu


def _setup(cfg, token_input):
    from paper_2602_05145_amd import runtime
    wl = W.make_workload(cfg)
    tr = runtime.trainer_from_workload(cfg, wl)
    params = {k: np.asarray(v, np.float64) for k, v in wl["params"].items()}
    tok = None
    if token_input:
        ti = W.make_token_input(cfg, embed_rows=min(cfg["vocab"], 301))
        ti["input_ids"][0, 1] = -3                      # out of range: zero embedding on both sides
        tr.set_token_input(ti["embed"], ti["input_ids"], ti["w_in"])
        params["w_in"] = np.asarray(ti["w_in"], np.float64)
        tok = dict(embed=np.asarray(ti["embed"], np.float64), input_ids=ti["input_ids"])
    return wl, tr, params, tok


def _step_rows(tr, step, name, width):
    """Dense rows of a named intermediate of one step, and the row indices they belong to."""
    base = step * ((tr.ws_bytes + 255) // 256 * 256)
    ws = tr.unroll_ws

    def view(nm, nbytes, dt):
        off = base + B.tide_draft_workspace_offset(tr.ccfg, nm)
        return ws[off:off + nbytes].view(dt)
    cnt = int(view("cnt", 4, torch.int32).item())
    idx = view("kept_idx", 4 * cnt, torch.int32).cpu().numpy()
    dt = torch.float32 if tr.dtype == "fp32" else torch.bfloat16
    x = view(name, cnt * width * (4 if tr.dtype == "fp32" else 2), dt).view(cnt, width)
    return idx, x.float().cpu().numpy().astype(np.float64)


def _check(cfg, token_input, n_steps, tol, x_tol):
    wl, tr, params, tok = _setup(cfg, token_input)
    ref = U.unroll_forward(cfg, params, wl["hidden"].astype(np.float64), wl["tokens"], wl["mask"], n_steps, tok=tok)
    loss, acc = tr.eval_unroll(n_steps, token_input=token_input)
    sync()
    loss, acc = loss.cpu().numpy(), acc.cpu().numpy()
    T = cfg["batch"] * cfg["seq"]
    for s in range(n_steps):
        assert abs(loss[s] - ref[s]["loss"]) <= tol * abs(ref[s]["loss"]), (s, loss[s], ref[s]["loss"])
        assert abs(acc[s] - ref[s]["accuracy"]) <= max(2.0, 0.01 * ref[s]["n"]) / ref[s]["n"] + 1e-6, (s, acc[s], ref[s]["accuracy"])
        idx, x2 = _step_rows(tr, s, "x2", cfg["hidden"])
        # the rows a step selects: those that carry loss at this or a later step
        need = np.zeros(T, bool)
        for j in range(s, n_steps):
            need |= O.effective_mask(ref[j]["tokens"], ref[j]["mask"], cfg["vocab"])
        assert np.array_equal(idx, np.nonzero(need)[0])
        assert rel_max(x2, ref[s]["x2"][idx]) <= x_tol, (s, rel_max(x2, ref[s]["x2"][idx]))
    return tr, loss, acc


@pytest.mark.parametrize("token_input", [False, True])
@pytest.mark.parametrize("kw", [dict(), dict(batch=3, seq=37, target_hidden=24, hidden=48, n_heads=6, n_kv_heads=2,
                                             head_dim=8, ffn=100, vocab=203)])
def test_unroll_fp32(kw, token_input):
    _check(W.get_config("tiny", **kw), token_input, 3, 1e-4, 1e-4)


def test_unroll_fp32_wide_heads_and_five_steps():
    cfg = W.get_config("small", batch=2, seq=200, target_hidden=64, hidden=512, n_heads=4, n_kv_heads=2, head_dim=128,
                       ffn=264, vocab=1000, dtype="fp32")
    _check(cfg, True, 5, 1e-4, 1e-4)


@pytest.mark.parametrize("token_input", [False, True])
def test_unroll_bf16(token_input):
    cfg = W.get_config("small", batch=2, seq=160, target_hidden=64, hidden=512, n_heads=4, n_kv_heads=2, head_dim=128,
                       ffn=256, vocab=512)
    _check(cfg, token_input, 3, 1e-2, 3e-2)


def test_first_step_equals_the_single_step_evaluation():
    """One step selects the same rows as the plain evaluation: the same bits.  With more steps the first one also
    carries rows that only later steps need, so its sums run in another order."""
    cfg = W.get_config("small", batch=2, seq=96, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    wl, tr, _, _ = _setup(cfg, False)
    loss, acc = tr.eval_unroll(3)
    l1, a1 = tr.eval()
    sync()
    assert abs(float(loss[0].item()) - float(l1.item())) <= 1e-6 * float(l1.item())
    assert abs(float(acc[0].item()) - float(a1.item())) <= 1e-6
    one_l, one_a = tr.eval_unroll(1)
    sync()
    assert float(one_l[0].item()) == float(l1.item()) and float(one_a[0].item()) == float(a1.item())


def test_argument_errors():
    cfg = W.get_config("tiny")
    wl, tr, _, _ = _setup(cfg, False)
    assert B.tide_draft_unroll_workspace_bytes(tr.ccfg, 0) == 0
    assert B.tide_draft_unroll_workspace_bytes(tr.ccfg, 9) == 0
    need = B.tide_draft_unroll_workspace_bytes(tr.ccfg, 3)
    assert need >= 3 * tr.ws_bytes
    ws = torch.empty(need, dtype=torch.uint8, device=tr.device)
    out = torch.zeros(3, device=tr.device)
    stream = torch.cuda.current_stream().cuda_stream
    args = (tr.ccfg, tr.c_params, None, tr.hidden, tr.tokens, tr.mask)
    assert B.tide_draft_eval_unroll(*args, 3, out, out, ws, need - 1, stream, check=False) == B.TIDE_ERR_WORKSPACE
    assert B.tide_draft_eval_unroll(*args, 0, out, out, ws, need, stream, check=False) == B.TIDE_ERR_CONFIG
    assert B.tide_draft_eval_unroll(*args, 3, out, None, ws, need, stream, check=False) == B.TIDE_ERR_NULL
    assert B.tide_draft_eval_unroll(*args, 3, out, out, ws, need, stream, check=False) == B.TIDE_OK
    sync()
