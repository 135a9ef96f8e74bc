"""Robustness of the step around its memory: a workspace and gradient buffers poisoned with NaN bit patterns
must not change any result (nothing reads what it did not write, gradients are overwritten and not
accumulated), guard bands on both sides of the workspace must stay untouched (nothing is written outside it),
and the optimizer state round-trips through a checkpoint (two steps == step, save, restore, step)."""
import numpy as np
import pytest
import torch

from oracle import tide_oracle as O
from paper_2602_05145_amd import workloads as W
from tests.gpu_util import sync

pytestmark = pytest.mark.gpu

GUARD = 1 << 16


def poisoned(tr):
    """Replaces the trainer's workspace by the middle of a 0xFF-filled buffer and poisons the gradients."""
    big = torch.full((tr.ws_bytes + 2 * GUARD,), 0xFF, dtype=torch.uint8, device=tr.device)
    tr.workspace = big[GUARD:GUARD + tr.ws_bytes]
    assert tr.workspace.data_ptr() % 256 == 0
    for g in tr.grads.values():
        g.fill_(float("nan"))
    return big


def guards_intact(big, ws_bytes):
    return bool((big[:GUARD] == 0xFF).all()) and bool((big[GUARD + ws_bytes:] == 0xFF).all())


CASES = [
    ("tiny", {}),
    ("tiny", dict(batch=3, seq=37, hidden=192, n_heads=3, n_kv_heads=1, head_dim=64, ffn=200, vocab=1001, target_hidden=40)),
    ("small", dict(batch=2, seq=200, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128, ffn=264, vocab=1000)),
]


@pytest.mark.parametrize("name,kw", CASES)
def test_poisoned_workspace_and_guard_bands(name, kw):
    from paper_2602_05145_amd import runtime
    cfg = W.get_config(name, **kw)
    wl = W.make_workload(cfg)
    clean = runtime.trainer_from_workload(cfg, wl)
    lf_clean, top1_clean = clean.forward(want_top1=True)
    lf_clean = float(lf_clean.item())
    clean.train_step(cfg["lr"])
    sync()

    tr = runtime.trainer_from_workload(cfg, wl)
    big = poisoned(tr)
    lf, top1 = tr.forward(want_top1=True)
    sync()
    assert float(lf.item()) == lf_clean
    assert torch.equal(top1, top1_clean)
    assert guards_intact(big, tr.ws_bytes)
    big.fill_(0xFF)                                   # poison again: the training step must not rely on the forward call
    tr.train_step(cfg["lr"])
    sync()
    assert float(tr.loss.item()) == float(clean.loss.item())
    for k in O.PARAM_NAMES:
        assert bool(torch.isfinite(tr.grads[k]).all()), k
        assert torch.equal(tr.grads[k], clean.grads[k]), k
        assert torch.equal(tr.params[k], clean.params[k]), k
    assert guards_intact(big, tr.ws_bytes)


def test_poisoned_workspace_packed():
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("small", batch=1, seq=400, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    wl = W.make_workload(cfg)
    cu = [0, 130, 130, 131, 390]                      # an empty sequence, a length-1 sequence, 10 padding rows
    clean = runtime.trainer_from_workload(cfg, wl)
    clean.set_packed(cu)
    clean.train_step_packed(cfg["lr"])
    sync()
    tr = runtime.trainer_from_workload(cfg, wl)
    tr.set_packed(cu)
    big = poisoned(tr)
    tr.train_step_packed(cfg["lr"])
    sync()
    assert float(tr.loss.item()) == float(clean.loss.item())
    for k in O.PARAM_NAMES:
        assert bool(torch.isfinite(tr.grads[k]).all()), k
        assert torch.equal(tr.grads[k], clean.grads[k]), k
    assert guards_intact(big, tr.ws_bytes)


def test_poisoned_workspace_token_input():
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("small", batch=2, seq=120, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    wl = W.make_workload(cfg)
    ti = W.make_token_input(cfg)
    trainers = []
    for poison in (False, True):
        tr = runtime.trainer_from_workload(cfg, wl)
        tr.set_token_input(ti["embed"], ti["input_ids"], ti["w_in"])
        big = poisoned(tr) if poison else None
        if poison:
            tr.grad_w_in.fill_(float("nan"))
        tr.train_step_tok(cfg["lr"])
        sync()
        trainers.append((tr, big))
    (clean, _), (tr, big) = trainers
    assert float(tr.loss.item()) == float(clean.loss.item())
    for k in O.PARAM_NAMES:
        assert torch.equal(tr.grads[k], clean.grads[k]), k
    assert bool(torch.isfinite(tr.grad_w_in).all()) and torch.equal(tr.grad_w_in, clean.grad_w_in)
    assert torch.equal(tr.w_in, clean.w_in)
    assert guards_intact(big, tr.ws_bytes)


def test_poisoned_workspace_unroll():
    """The unroll's workspace holds sums that later steps add to (own key/value gradients, the step-1 key/value
    gradient, weight gradients): every one of them must be written before it is added to."""
    from paper_2602_05145_amd import binding as B
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("small", batch=2, seq=120, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    wl = W.make_workload(cfg)
    ti = W.make_token_input(cfg)
    results = []
    for poison in (False, True):
        tr = runtime.trainer_from_workload(cfg, wl)
        tr.set_token_input(ti["embed"], ti["input_ids"], ti["w_in"])
        need = B.tide_draft_unroll_workspace_bytes(tr.ccfg, 3)
        big = torch.full((need + 2 * GUARD,), 0xFF if poison else 0, dtype=torch.uint8, device=tr.device)
        tr.unroll_ws = big[GUARD:GUARD + need]
        if poison:
            for g in tr.grads.values():
                g.fill_(float("nan"))
            tr.grad_w_in.fill_(float("nan"))
        ev = tr.eval_unroll(3, token_input=True)
        sync()
        ev = [x.clone() for x in ev]
        if poison:
            assert bool((big[:GUARD] == 0xFF).all()) and bool((big[GUARD + need:] == 0xFF).all())
            big.fill_(0xFF)
        loss = tr.train_step_unroll(cfg["lr"], 3, step_weights=[1.0, 0.5, 0.25], token_input=True).clone()
        sync()
        if poison:
            assert bool((big[:GUARD] == 0xFF).all()) and bool((big[GUARD + need:] == 0xFF).all())
        results.append((tr, ev, loss))
    (a, ev_a, loss_a), (b, ev_b, loss_b) = results
    assert torch.equal(ev_a[0], ev_b[0]) and torch.equal(ev_a[1], ev_b[1]) and torch.equal(loss_a, loss_b)
    assert bool(torch.isfinite(loss_b).all())
    for k in O.PARAM_NAMES:
        assert bool(torch.isfinite(b.grads[k]).all()), k
        assert torch.equal(a.grads[k], b.grads[k]) and torch.equal(a.params[k], b.params[k]), k
    assert torch.equal(a.grad_w_in, b.grad_w_in) and torch.equal(a.w_in, b.w_in)


def test_checkpoint_resume():
    """Parameters, both moments, the master copy and the step counter are caller-owned: copying them out and
    into a fresh trainer continues the run bit for bit."""
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("small", batch=2, seq=96, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    wl = W.make_workload(cfg)
    a = runtime.trainer_from_workload(cfg, wl)
    a.train_step(cfg["lr"])
    a.train_step(cfg["lr"])
    sync()
    b = runtime.trainer_from_workload(cfg, wl)
    b.train_step(cfg["lr"])
    sync()
    ckpt = dict(params={k: v.clone() for k, v in b.params.items()}, m={k: v.clone() for k, v in b.m.items()},
                v={k: v.clone() for k, v in b.v.items()}, master={k: v.clone() for k, v in b.master.items()}, step=b.step)
    c = runtime.trainer_from_workload(cfg, wl)
    for k in O.PARAM_NAMES:
        c.params[k].copy_(ckpt["params"][k]); c.m[k].copy_(ckpt["m"][k]); c.v[k].copy_(ckpt["v"][k]); c.master[k].copy_(ckpt["master"][k])
    c.c_adam.step = ckpt["step"]
    c.train_step(cfg["lr"])
    sync()
    assert c.step == 2 and float(c.loss.item()) == float(a.loss.item())
    for k in O.PARAM_NAMES:
        assert torch.equal(c.params[k], a.params[k]), k
        assert torch.equal(c.m[k], a.m[k]) and torch.equal(c.v[k], a.v[k]) and torch.equal(c.master[k], a.master[k]), k


def test_status_word_flags_malformed_offsets_and_non_finite_loss():
    """What the host cannot check is checked on the device and reported; malformed offsets are clamped so that
    every access stays inside the buffers (the results are then meaningless, but nothing faults)."""
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("small", batch=1, seq=400, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    wl = W.make_workload(cfg)
    tr = runtime.trainer_from_workload(cfg, wl)
    tr.set_packed([0, 130, 131, 390])
    tr.forward_packed()
    sync()
    assert tr.status() == 0
    for bad in ([0, 200, 100, 390], [-5, 100, 390], [0, 100, 500], [0, 10, 390]):
        tr.set_packed(bad, max_seqlen=260)           # the last list is ascending but holds a 380-row sequence
        tr.forward_packed()
        sync()
        assert tr.status() == 2, bad
    tr.set_packed([0, 130, 131, 390])
    tr.forward_packed()
    sync()
    assert tr.status() == 0                          # rewritten by every call
    # fixed layout: a NaN in the captured states reaches the loss and raises bit 0
    tr.forward()
    sync()
    assert tr.status() == 0
    tr.hidden[0, 5, 7] = float("nan")
    tr.forward()
    sync()
    assert tr.status() == 1 and not np.isfinite(float(tr.loss.item()))


def test_forward_and_eval_replay_from_a_hip_graph():
    """The forward-only entry points enqueue kernels and nothing else (no allocation, no memset, no host
    synchronisation), so a caller can capture them into a HIP graph.  The replays (with eager work and
    synchronisations in between, and new inputs written into the captured buffers) must match eager calls."""
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("small", batch=2, seq=160, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=264, vocab=1000)
    wl = W.make_workload(cfg)
    tr = runtime.trainer_from_workload(cfg, wl)
    eager = runtime.trainer_from_workload(cfg, wl)
    tr.eval()                                              # warm-up: one-time function attributes are set outside the capture
    sync()
    acc = torch.zeros(1, dtype=torch.float32, device=tr.device)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            from paper_2602_05145_amd import binding as B
            B.tide_draft_eval(tr.ccfg, tr.c_params, tr.hidden, tr.tokens, tr.mask, tr.loss, acc, tr.workspace, tr.ws_bytes,
                              torch.cuda.current_stream().cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    for i in range(3):
        wl_i = W.make_workload(cfg, seed=500 + i)
        for dst, src in ((tr.hidden, wl_i["hidden"]), (eager.hidden, wl_i["hidden"])):
            dst.copy_(torch.from_numpy(src).to(dst.device).to(dst.dtype))
        for t in (tr, eager):
            t.tokens.copy_(torch.from_numpy(wl_i["tokens"]).to(t.device))
            t.mask.copy_(torch.from_numpy(wl_i["mask"]).to(t.device))
        tr.loss.fill_(-1.0)
        acc.fill_(-1.0)
        sync()
        graph.replay()
        sync()
        loss_e, acc_e = eager.eval()
        sync()
        assert float(tr.loss.item()) == float(loss_e.item()), i
        assert float(acc.item()) == float(acc_e.item()), i
        assert tr.status() == 0


def test_train_step_with_a_device_schedule_replays_from_a_hip_graph():
    """tide_draft_train_step_dev keeps the learning rate and the step count in device memory, so the whole training
    step (forward, backward, AdamW with its bias corrections) can be captured once and replayed: four replays on
    four different batches, with a learning-rate change and eager work in between, must leave bit-identical
    parameters, moments and losses to four eager tide_draft_train_step calls, and the device count must read 4."""
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("small", batch=2, seq=160, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=264, vocab=1000)
    wl = W.make_workload(cfg)
    tr = runtime.trainer_from_workload(cfg, wl)
    eager = runtime.trainer_from_workload(cfg, wl)
    tr.forward()                                           # warm-up: one-time function attributes, outside the capture
    sync()
    lr_dev = torch.full((1,), 1e-3, dtype=torch.float32, device=tr.device)
    step_dev = torch.zeros(1, dtype=torch.int64, device=tr.device)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            tr.train_step_dev(lr_dev, step_dev)
    torch.cuda.current_stream().wait_stream(side)
    sync()
    assert int(step_dev.item()) == 0 and tr.step == 0      # capturing runs nothing
    lrs = [1e-3, 1e-3, 4e-4, 2e-3]
    for i, lr in enumerate(lrs):
        wl_i = W.make_workload(cfg, seed=700 + i)
        for t in (tr, eager):
            t.hidden.copy_(torch.from_numpy(wl_i["hidden"]).to(t.device).to(t.hidden.dtype))
            t.tokens.copy_(torch.from_numpy(wl_i["tokens"]).to(t.device))
            t.mask.copy_(torch.from_numpy(wl_i["mask"]).to(t.device))
        lr_dev.fill_(lr)
        tr.loss.fill_(-1.0)
        sync()
        graph.replay()
        sync()
        eager.train_step(lr)
        sync()
        assert float(tr.loss.item()) == float(eager.loss.item()), i
        assert int(step_dev.item()) == i + 1
        for k in tr.params:
            assert torch.equal(tr.params[k], eager.params[k]), (i, k)
            assert torch.equal(tr.m[k], eager.m[k]) and torch.equal(tr.v[k], eager.v[k]), (i, k)
            assert torch.equal(tr.master[k], eager.master[k]), (i, k)
    assert tr.step == 0 and eager.step == 4
    # eager calls of the device-schedule entry point continue the same sequence
    tr.train_step_dev(lr_dev, step_dev)
    eager.train_step(lrs[-1])
    sync()
    assert int(step_dev.item()) == 5
    for k in tr.params:
        assert torch.equal(tr.params[k], eager.params[k]), k
    from paper_2602_05145_amd import binding as B
    rc = B.tide_draft_train_step_dev(tr.ccfg, tr.c_params, tr.c_grads, tr.c_adam, tr.hidden, tr.tokens, tr.mask, None, step_dev,
                                     tr.loss, tr.workspace, tr.ws_bytes, torch.cuda.current_stream().cuda_stream, check=False)
    assert rc == B.TIDE_ERR_NULL


def test_eval_unroll_replays_from_a_hip_graph():
    """The evaluation unroll too enqueues kernels and nothing else: captured once, replayed on new inputs written
    into the captured buffers, every replay must match an eager call bit for bit."""
    from paper_2602_05145_amd import binding as B
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("small", batch=2, seq=160, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=264, vocab=1000)
    wl = W.make_workload(cfg)
    ti = W.make_token_input(cfg)
    tr, eager = (runtime.trainer_from_workload(cfg, wl) for _ in range(2))
    for t in (tr, eager):
        t.set_token_input(ti["embed"], ti["input_ids"], ti["w_in"])
    tr.eval_unroll(3, token_input=True)                    # warm-up outside the capture; allocates the unroll workspace
    sync()
    loss = torch.zeros(3, dtype=torch.float32, device=tr.device)
    acc = torch.zeros(3, dtype=torch.float32, device=tr.device)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            B.tide_draft_eval_unroll(tr.ccfg, tr.c_params, tr.c_tok, tr.hidden, tr.tokens, tr.mask, 3, loss, acc, tr.unroll_ws,
                                     tr.unroll_ws.numel(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    for i in range(3):
        wl_i = W.make_workload(cfg, seed=700 + i)
        for t in (tr, eager):
            t.hidden.copy_(torch.from_numpy(wl_i["hidden"]).to(t.device).to(t.hidden.dtype))
            t.tokens.copy_(torch.from_numpy(wl_i["tokens"]).to(t.device))
            t.mask.copy_(torch.from_numpy(wl_i["mask"]).to(t.device))
        loss.fill_(-1.0)
        acc.fill_(-1.0)
        sync()
        graph.replay()
        sync()
        loss_e, acc_e = eager.eval_unroll(3, token_input=True)
        sync()
        assert torch.equal(loss, loss_e) and torch.equal(acc, acc_e), i
