"""Multi-step unroll (the draft fed its own output from the second step on) through the C ABI against the fp64
oracle.  Evaluation: per-step loss within 1e-4 (fp32) / 1e-2 (bf16) relative, per-step accuracy within a few rows
(an arg-max can flip on a near tie), and the layer output of every step on the rows it selected.  Training:
the tolerances of the single step (fp32 1e-4 relative on losses and gradients; bf16 1e-2 on the losses, gradient
cosine >= 0.999, parameters after the AdamW update within 2e-3)."""
import numpy as np
import pytest
import torch

from oracle import tide_oracle as O
from oracle import unroll_oracle as U
from paper_2602_05145_amd import binding as B
from paper_2602_05145_amd import workloads as W
from tests.gpu_util import cosine, rel_max, sync

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


def _step_rows(tr, n_steps, step, name, width):
    """Dense rows of a named intermediate of one step, and the row indices they belong to."""
    ws = tr.unroll_ws

    def view(nm, nbytes, dt):
        off = B.tide_draft_unroll_workspace_offset(tr.ccfg, n_steps, step, nm)
        assert off >= 0
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
        idx, x2 = _step_rows(tr, n_steps, s, "x2", cfg["hidden"])
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


def _train_reference(cfg, wl, params, tok, n_steps, w, lr):
    steps = U.unroll_forward(cfg, params, wl["hidden"].astype(np.float64), wl["tokens"], wl["mask"], n_steps, tok=tok, keep_cache=True)
    grads = U.unroll_backward(cfg, params, steps, step_weights=w)
    zeros = {k: np.zeros_like(v) for k, v in params.items()}
    new_p, m, v, _ = O.adamw_step(cfg, params, grads, zeros, zeros, 0, lr)
    return [st["loss"] for st in steps], grads, new_p


def _device_grads(tr, token_input):
    g = tr.host(tr.grads)
    if token_input:
        g["w_in"] = tr.grad_w_in.cpu().numpy().astype(np.float64)
    return g


@pytest.mark.parametrize("token_input", [False, True])
@pytest.mark.parametrize("kw", [dict(), dict(batch=3, seq=37, target_hidden=24, hidden=48, n_heads=6, n_kv_heads=2,
                                             head_dim=8, ffn=100, vocab=203)])
def test_train_unroll_fp32(kw, token_input):
    cfg = W.get_config("tiny", **kw)
    wl, tr, params, tok = _setup(cfg, token_input)
    w = [1.0, 0.7, 0.45]
    loss_ref, g_ref, p1_ref = _train_reference(cfg, wl, params, tok, 3, w, cfg["lr"])
    loss = tr.train_step_unroll(cfg["lr"], 3, step_weights=w, token_input=token_input)
    sync()
    assert tr.step == 1
    for s in range(3):
        assert abs(float(loss[s].item()) - loss_ref[s]) <= 1e-4 * abs(loss_ref[s]), s
    g = _device_grads(tr, token_input)
    for k in g_ref:
        assert rel_max(g[k], g_ref[k]) <= 1e-4, (k, rel_max(g[k], g_ref[k]))
    p = tr.host(tr.params)
    for k in O.PARAM_NAMES:
        solid = np.abs(g_ref[k]) >= 1e-4 * np.max(np.abs(g_ref[k]))
        assert np.max(np.abs(p[k] - p1_ref[k])[solid]) <= 0.01 * cfg["lr"], k


def test_train_unroll_fp32_two_and_five_steps_default_weights():
    cfg = W.get_config("tiny", batch=2, seq=41, target_hidden=24, hidden=64, n_heads=4, n_kv_heads=2, head_dim=16, ffn=72, vocab=157)
    for n in (2, 5):
        wl, tr, params, tok = _setup(cfg, True)
        loss_ref, g_ref, _ = _train_reference(cfg, wl, params, tok, n, None, cfg["lr"])
        loss = tr.train_step_unroll(cfg["lr"], n, token_input=True)
        sync()
        g = _device_grads(tr, True)
        for s in range(n):
            assert abs(float(loss[s].item()) - loss_ref[s]) <= 1e-4 * abs(loss_ref[s]), (n, s)
        for k in g_ref:
            assert rel_max(g[k], g_ref[k]) <= 1e-4, (n, k, rel_max(g[k], g_ref[k]))


def test_train_unroll_one_step_is_the_ordinary_training_step():
    cfg = W.get_config("small", batch=2, seq=96, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    wl, a, _, _ = _setup(cfg, True)
    _, b, _, _ = _setup(cfg, True)
    la = a.train_step_unroll(cfg["lr"], 1, token_input=True)
    b.train_step_tok(cfg["lr"])
    sync()
    assert float(la[0].item()) == float(b.loss.item())
    for k in O.PARAM_NAMES:
        assert torch.equal(a.grads[k], b.grads[k]) and torch.equal(a.params[k], b.params[k]), k
    assert torch.equal(a.grad_w_in, b.grad_w_in) and torch.equal(a.w_in, b.w_in)


@pytest.mark.parametrize("token_input", [False, True])
def test_train_unroll_bf16(token_input):
    cfg = W.get_config("small", batch=2, seq=160, target_hidden=64, hidden=512, n_heads=4, n_kv_heads=2, head_dim=128,
                       ffn=256, vocab=512)
    wl, tr, params, tok = _setup(cfg, token_input)
    w = [1.0, 0.8, 0.64]
    loss_ref, g_ref, p1_ref = _train_reference(cfg, wl, params, tok, 3, w, cfg["lr"])
    loss = tr.train_step_unroll(cfg["lr"], 3, step_weights=w, token_input=token_input)
    sync()
    for s in range(3):
        assert abs(float(loss[s].item()) - loss_ref[s]) <= 1e-2 * abs(loss_ref[s]), s
    g = _device_grads(tr, token_input)
    for k in g_ref:
        assert cosine(g[k], g_ref[k]) >= 0.999, (k, cosine(g[k], g_ref[k]))
    p = tr.host(tr.master)
    for k in O.PARAM_NAMES:
        assert np.max(np.abs(p[k] - p1_ref[k])) <= 2e-3, k


def test_more_steps_than_positions_and_an_all_masked_batch():
    """Steps whose positions have all left the sequence carry no loss: loss 0, and they add nothing to the
    gradients.  A batch without any loss row gives zero losses and exactly zero gradients at every step."""
    cfg = W.get_config("tiny", batch=3, seq=2, target_hidden=24, hidden=48, n_heads=6, n_kv_heads=2, head_dim=8, ffn=100,
                       vocab=203, mask="none")
    wl, tr, params, tok = _setup(cfg, True)
    loss_ref, g_ref, _ = _train_reference(cfg, wl, params, tok, 4, None, cfg["lr"])
    assert loss_ref[2] == 0.0 and loss_ref[3] == 0.0
    loss = tr.train_step_unroll(cfg["lr"], 4, token_input=True)
    sync()
    assert float(loss[2].item()) == 0.0 and float(loss[3].item()) == 0.0
    for s in range(2):
        assert abs(float(loss[s].item()) - loss_ref[s]) <= 1e-4 * abs(loss_ref[s]), s
    g = _device_grads(tr, True)
    for k in g_ref:
        assert rel_max(g[k], g_ref[k]) <= 1e-4, (k, rel_max(g[k], g_ref[k]))
    # nothing carries loss
    cfg2 = W.get_config("tiny")
    wl2, tr2, _, _ = _setup(cfg2, False)
    tr2.mask.zero_()
    for g_ in tr2.grads.values():
        g_.fill_(7.0)
    loss2 = tr2.train_step_unroll(cfg2["lr"], 3)
    ev_loss, ev_acc = tr2.eval_unroll(3)
    sync()
    assert bool((loss2 == 0).all()) and bool((ev_loss == 0).all()) and bool((ev_acc == 0).all())
    for k in O.PARAM_NAMES:
        assert bool((tr2.grads[k] == 0).all()), k


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
    targs = (tr.ccfg, tr.c_params, tr.c_grads, tr.c_adam, None, tr.hidden, tr.tokens, tr.mask)
    assert B.tide_draft_train_step_unroll(*targs, 3, [1.0, -1.0, 1.0], 1e-4, out, ws, need, stream, check=False) == B.TIDE_ERR_CONFIG
    assert B.tide_draft_train_step_unroll(*targs, 3, [1.0, float("nan"), 1.0], 1e-4, out, ws, need, stream, check=False) == B.TIDE_ERR_CONFIG
    assert B.tide_draft_train_step_unroll(*targs, 9, None, 1e-4, out, ws, need, stream, check=False) == B.TIDE_ERR_CONFIG
    assert B.tide_draft_train_step_unroll(*targs, 3, None, 1e-4, out, ws, need - 1, stream, check=False) == B.TIDE_ERR_WORKSPACE
    assert tr.step == 0


def test_unroll_at_the_benchmarked_size_prefix_of_one_sequence_against_oracle():
    """8B-shaped batch in bf16, 3 steps.  By causality the first rows of a sequence depend on that prefix alone at
    every step (step s row i needs the step-1 keys of rows 0..i and the labels up to i + s - 1), so an oracle unroll
    over the prefix gives their layer outputs and loss terms exactly."""
    import bench
    cfg = W.get_config("8b")
    dev = torch.device("cuda:0")
    print("generating the 8b workload on the device", flush=True)
    params, hidden, tokens, mask = bench.device_workload(cfg, dev, cfg["seed"])
    tr = bench.DeviceTrainer(cfg, params, hidden, tokens, mask)
    n_steps = 3
    print("3-step evaluation unroll at full size", flush=True)
    loss, acc = tr.eval_unroll(n_steps)
    l1, a1 = tr.eval()
    sync()
    assert bool(torch.isfinite(loss).all()) and bool(((acc >= 0) & (acc <= 1)).all())
    assert abs(float(loss[0].item()) - float(l1.item())) <= 1e-5 * float(l1.item())
    b, S, d = cfg["batch"] - 1, cfg["seq"], cfg["hidden"]
    first_loss = int(torch.nonzero(tr.mask[b] != 0)[0].item())
    L = first_loss + 48
    sub = dict(cfg, batch=1, seq=L)
    params64 = {k: v.float().cpu().numpy().astype(np.float64) for k, v in params.items()}
    hid = tr.hidden[b, :L].float().cpu().numpy().astype(np.float64)[None]
    tok = tr.tokens[b, :L].cpu().numpy()[None]
    msk = tr.mask[b, :L].cpu().numpy()[None]
    print(f"oracle unroll over the {L}-position prefix", flush=True)
    ref = U.unroll_forward(sub, params64, hid, tok, msk, n_steps)
    for s in range(n_steps):
        idx, x2 = _step_rows(tr, n_steps, s, "x2", d)
        sel = (idx >= b * S) & (idx < b * S + L - (n_steps - 1))        # rows whose whole chain lies inside the prefix
        assert sel.sum() >= 40
        local = idx[sel] - b * S
        x_ref = ref[s]["x2"][local]
        assert cosine(x2[sel], x_ref) > 0.9995, (s, cosine(x2[sel], x_ref))
        assert np.max(np.abs(x2[sel] - x_ref)) <= 3e-2 * np.max(np.abs(x_ref)), s
        # loss terms of the same rows: lse - z[label] where the step's shifted mask is set
        off = B.tide_draft_unroll_workspace_offset(tr.ccfg, n_steps, s, "loss_rows")
        terms = tr.unroll_ws[off:off + 4 * len(idx)].view(torch.float32).cpu().numpy()[sel]
        yhat, _ = O.rmsnorm_fwd(x_ref, params64["g3"], cfg["rms_eps"])
        z = yhat @ params64["w_lm"].T
        lab = ref[s]["tokens"].reshape(-1)[local]
        keep = O.effective_mask(lab, ref[s]["mask"].reshape(-1)[local], cfg["vocab"])
        zmax = z.max(axis=-1)
        t_ref = np.where(keep, zmax + np.log(np.exp(z - zmax[:, None]).sum(-1)) - z[np.arange(len(lab)), np.where(keep, lab, 0)], 0.0)
        assert np.all(terms[~keep] == 0.0)
        assert abs(terms.sum() - t_ref.sum()) <= 1e-2 * abs(t_ref.sum()), (s, terms.sum(), t_ref.sum())


def test_unroll_training_raises_held_out_accuracy_at_every_step():
    """A property of the whole loop, no stored values: the label of a position is the index of the largest of the
    first 16 channels of its newest captured state, and the input token of a position is a fixed permutation of
    its label, so step 1 can learn the label from the features and later steps (fed the draft's own output) from
    the token embedding.  After 80 bf16 unroll steps on fresh batches the held-out loss of all three steps must
    have dropped and their top-1 accuracy risen far above chance."""
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("tiny", dtype="bf16", vocab=64, batch=4)
    perm = np.random.default_rng(5).permutation(64).astype(np.int32)
    ti = W.make_token_input(cfg, embed_rows=64)

    def batch(seed):
        wl = W.make_workload(cfg, seed=seed)
        newest = wl["hidden"][..., -cfg["target_hidden"]:]
        wl["tokens"] = np.argmax(newest[..., :16], axis=-1).astype(np.int32)
        wl["ids"] = perm[wl["tokens"]]
        return wl

    def load(tr, wl):
        tr.set_batch(wl["hidden"], wl["tokens"], wl["mask"])
        tr.input_ids.copy_(torch.from_numpy(wl["ids"]).to(tr.device))

    held_out = batch(999)
    tr = runtime.trainer_from_workload(cfg, held_out)
    tr.set_token_input(ti["embed"], held_out["ids"], ti["w_in"])
    loss0, acc0 = (x.cpu().numpy() for x in tr.eval_unroll(3, token_input=True))
    for step in range(80):
        load(tr, batch(100 + step))
        tr.train_step_unroll(3e-3, 3, step_weights=[1.0, 0.8, 0.64], token_input=True)
    sync()
    assert tr.step == 80
    load(tr, held_out)
    loss1, acc1 = (x.cpu().numpy() for x in tr.eval_unroll(3, token_input=True))
    print(f"held-out loss {loss0} -> {loss1}, top-1 {acc0} -> {acc1}", flush=True)
    for s in range(3):
        assert np.isfinite(loss1[s]) and loss1[s] < 0.7 * loss0[s], (s, loss0, loss1)
        assert acc0[s] < 0.08 and acc1[s] > 0.15, (s, acc0, acc1)


def test_unroll_training_at_the_benchmarked_size_lm_head_gradient_rows_and_properties():
    """8B-shaped batch in bf16, 3 steps with unequal weights.  dW_lm sums the three steps' shares; a few of its rows
    are recomputed in fp64 from what every step left in its workspace (final-norm output, log-sum-exp, shifted labels
    of the rows it selected) and the initial W_lm.  Properties that hold at any size: finite gradients, zero column
    sums of dW_lm (every logit-gradient row sums to zero), loss of step 1 equal to the single step's."""
    import bench
    cfg = W.get_config("8b")
    dev = torch.device("cuda:0")
    print("generating the 8b workload on the device", flush=True)
    params, hidden, tokens, mask = bench.device_workload(cfg, dev, cfg["seed"])
    w_lm0 = params["w_lm"].clone()
    tr = bench.DeviceTrainer(cfg, params, hidden, tokens, mask)
    n_steps, w = 3, [1.0, 0.7, 0.45]
    l1, _ = tr.eval()
    print("3-step training unroll at full size", flush=True)
    loss = tr.train_step_unroll(cfg["lr"], n_steps, step_weights=w)
    sync()
    assert bool(torch.isfinite(loss).all())
    assert abs(float(loss[0].item()) - float(l1.item())) <= 1e-5 * float(l1.item())
    for k in O.PARAM_NAMES:
        assert bool(torch.isfinite(tr.grads[k]).all()), k
    d, V = cfg["hidden"], cfg["vocab"]
    g = tr.grads["w_lm"]
    assert float(g.sum(0).abs().max()) <= 2e-3 * float(g.abs().sum(0).max())

    def view(step, name, nbytes, dt):
        off = B.tide_draft_unroll_workspace_offset(tr.ccfg, n_steps, step, name)
        assert off >= 0
        return tr.unroll_ws[off:off + nbytes].view(dt)
    picks = [0, V - 1, 12345 % V, int(torch.bincount(tr.tokens.reshape(-1)[tr.mask.reshape(-1) != 0].long(), minlength=V).argmax().item())]
    ref = {v: torch.zeros(d, dtype=torch.float64, device=dev) for v in picks}
    for s in range(n_steps):
        cnt = int(view(s, "cnt", 4, torch.int32).item())
        y = view(s, "yhat", cnt * d * 2, torch.bfloat16).view(cnt, d).double()
        lse = view(s, "lse", cnt * 4, torch.float32).double()
        idx = view(s, "kept_idx", cnt * 4, torch.int32).long()
        labels = view(s, "tokens_s", cfg["batch"] * cfg["seq"] * 4, torch.int32).long()[idx]
        keep = (view(s, "mask_s", cfg["batch"] * cfg["seq"], torch.uint8)[idx] != 0) & (labels >= 0) & (labels < V)
        n = max(1, int(keep.sum().item()))
        for v in picks:
            z = y @ w_lm0[v].double()
            p = (torch.exp(z - lse) - (labels == v).double()) * keep.double()
            ref[v] += (w[s] / n) * (p[:, None] * y).sum(0)
    for v in picks:
        got = g[v].double()
        cos = float((ref[v] * got).sum() / (ref[v].norm() * got.norm()))
        err = float((ref[v] - got).abs().max() / ref[v].abs().max())
        print(f"dW_lm[{v}]: cosine {cos:.6f}, max rel err {err:.2e}", flush=True)
        assert cos >= 0.9999 and err <= 1e-2, (v, cos, err)


@pytest.mark.parametrize("seed", range(8))
def test_unroll_random_shapes_fp32(seed):
    """Seeded random small shapes (odd widths, every GQA ratio, every head_dim path of the merge kernels, all mask
    kinds, 2-4 steps, with and without token input): losses and all gradients against the oracle."""
    from tests.test_gpu_step import _random_cfg
    rng = np.random.default_rng(3000 + seed)
    kw = _random_cfg(rng, "fp32")
    kw["seq"] = min(kw["seq"], 48)                      # the oracle keeps every step's [S, S] weights
    n_steps = int(rng.integers(2, 5))
    token_input = bool(rng.integers(0, 2))
    print(kw, n_steps, token_input, flush=True)
    cfg = W.get_config("tiny", **kw)
    wl, tr, params, tok = _setup(cfg, token_input)
    w = [float(x) for x in rng.uniform(0.2, 1.0, n_steps)]
    loss_ref, g_ref, _ = _train_reference(cfg, wl, params, tok, n_steps, w, cfg["lr"])
    loss = tr.train_step_unroll(cfg["lr"], n_steps, step_weights=w, token_input=token_input)
    sync()
    for s in range(n_steps):
        assert abs(float(loss[s].item()) - loss_ref[s]) <= 1e-4 * abs(loss_ref[s]) + 1e-7, (s, float(loss[s].item()), loss_ref[s])
    g = _device_grads(tr, token_input)
    for k in g_ref:
        assert np.all(np.isfinite(g[k])), k
        den = float(np.max(np.abs(g_ref[k])))
        assert float(np.max(np.abs(g[k] - g_ref[k]))) <= 1e-4 * den + 1e-9, (k, rel_max(g[k], g_ref[k]))
