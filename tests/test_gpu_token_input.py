"""Token-input variant (features joined with the sampled token's embedding through a second projection) through
the C ABI against the fp64 oracle, same tolerances as the base step: fp32 1e-4 relative on loss and gradients,
bf16 1e-2 on the loss, gradient cosine >= 0.999, parameters after one AdamW step within 2e-3."""
import numpy as np
import pytest
import torch

from oracle import tide_oracle as O
from paper_2602_05145_amd import workloads as W
from tests.gpu_util import cosine, rel_max, sync

pytestmark = pytest.mark.gpu


def _setup(cfg, embed_rows=None):
    from paper_2602_05145_amd import runtime
    wl = W.make_workload(cfg)
    ti = W.make_token_input(cfg, embed_rows=embed_rows)
    tr = runtime.trainer_from_workload(cfg, wl)
    tr.set_token_input(ti["embed"], ti["input_ids"], ti["w_in"])
    p0 = {k: np.asarray(v, np.float64) for k, v in wl["params"].items()}
    p0["w_in"] = np.asarray(ti["w_in"], np.float64)
    tok = dict(embed=np.asarray(ti["embed"], np.float64), input_ids=ti["input_ids"])
    return wl, ti, tr, p0, tok


def _reference(cfg, wl, p0, tok, lr):
    zeros = {k: np.zeros_like(v) for k, v in p0.items()}
    return O.train_step(cfg, p0, zeros, zeros, 0, wl["hidden"].astype(np.float64), wl["tokens"], wl["mask"], lr, tok=tok)


@pytest.mark.parametrize("kw", [dict(), dict(batch=3, seq=33, target_hidden=24, hidden=48, n_heads=6, n_kv_heads=2,
                                             head_dim=8, ffn=100, vocab=203)])
def test_token_input_fp32(kw):
    cfg = W.get_config("tiny", **kw)
    wl, ti, tr, p0, tok = _setup(cfg, embed_rows=57)
    ti["input_ids"][0, 0] = -4            # out of range: zero embedding on both sides
    ti["input_ids"][-1, -1] = 57
    tr.set_token_input(ti["embed"], ti["input_ids"], ti["w_in"])
    tok["input_ids"] = ti["input_ids"]
    lr = cfg["lr"]
    loss_ref, g_ref, p1_ref, m_ref, v_ref, _ = _reference(cfg, wl, p0, tok, lr)
    loss_f, top1 = tr.forward_tok(want_top1=True)
    sync()
    assert abs(float(loss_f.item()) - loss_ref) <= 1e-4 * abs(loss_ref)
    tr.train_step_tok(lr)
    sync()
    assert tr.step == 1 and tr.status() == 0
    assert abs(float(tr.loss.item()) - loss_ref) <= 1e-4 * abs(loss_ref)
    g = tr.host(tr.grads)
    g["w_in"] = tr.grad_w_in.cpu().numpy().astype(np.float64)
    for k in O.PARAM_NAMES + ("w_in",):
        assert rel_max(g[k], g_ref[k]) <= 1e-4, (k, rel_max(g[k], g_ref[k]))
    w_in = tr.w_in.float().cpu().numpy().astype(np.float64)
    solid = np.abs(g_ref["w_in"]) >= 1e-4 * np.max(np.abs(g_ref["w_in"]))
    assert np.max(np.abs(w_in - p1_ref["w_in"])[solid]) <= 0.01 * lr
    assert rel_max(tr.m_w_in.cpu().numpy().astype(np.float64), m_ref["w_in"]) <= 1e-4
    # arg-max ids of the forward entry point
    _, cache = O.forward(cfg, p0, wl["hidden"].astype(np.float64), wl["tokens"], wl["mask"], want_top1=True, tok=tok)
    assert np.mean(top1.cpu().numpy() == cache["top1"]) > 0.99


def test_token_input_bf16():
    cfg = W.get_config("small", batch=2, seq=96, target_hidden=64, hidden=256, n_heads=2, n_kv_heads=1, head_dim=128,
                       ffn=256, vocab=512)
    wl, ti, tr, p0, tok = _setup(cfg)
    lr = cfg["lr"]
    loss_ref, g_ref, p1_ref, *_ = _reference(cfg, wl, p0, tok, lr)
    tr.train_step_tok(lr)
    sync()
    assert abs(float(tr.loss.item()) - loss_ref) <= 1e-2 * abs(loss_ref)
    g = tr.host(tr.grads)
    g["w_in"] = tr.grad_w_in.cpu().numpy().astype(np.float64)
    for k in O.PARAM_NAMES + ("w_in",):
        assert cosine(g[k], g_ref[k]) >= 0.999, (k, cosine(g[k], g_ref[k]))
    p = tr.host(tr.master)
    p["w_in"] = tr.master_w_in.cpu().numpy().astype(np.float64)
    for k in O.PARAM_NAMES + ("w_in",):
        assert np.max(np.abs(p[k] - p1_ref[k])) <= 2e-3, k
    assert np.max(np.abs(tr.w_in.float().cpu().numpy() - p1_ref["w_in"])) <= 2e-3


def test_identity_projection_equals_the_base_entry_point_on_the_gpu():
    """W_in = [I | 0]: the token-input step must give the base step's loss and gradients (two different
    launch sequences of the library; the extra GEMM rounds x0 once more in bf16, hence fp32 here)."""
    from paper_2602_05145_amd import runtime
    cfg = W.get_config("tiny")
    wl, ti, tr, p0, tok = _setup(cfg)
    d = cfg["hidden"]
    eye = np.concatenate([np.eye(d, dtype=np.float32), np.zeros((d, d), np.float32)], axis=1)
    tr.set_token_input(ti["embed"], ti["input_ids"], eye)
    base = runtime.trainer_from_workload(cfg, wl)
    tr.train_step_tok(cfg["lr"])
    base.train_step(cfg["lr"])
    sync()
    assert abs(float(tr.loss.item()) - float(base.loss.item())) <= 1e-6 * abs(float(base.loss.item()))
    for k in tr.grads:
        a, b = tr.grads[k].double().cpu().numpy(), base.grads[k].double().cpu().numpy()
        assert rel_max(a, b) <= 1e-5, k


def test_token_input_argument_errors():
    from paper_2602_05145_amd import binding as B
    cfg = W.get_config("tiny", batch=1, seq=8)
    wl, ti, tr, p0, tok = _setup(cfg)
    s = torch.cuda.current_stream().cuda_stream
    rc = B.tide_draft_train_step_tok(tr.ccfg, tr.c_params, tr.c_grads, tr.c_adam, None, tr.hidden, tr.tokens, tr.mask, 1e-4,
                                     tr.loss, tr.workspace, tr.ws_bytes, s, check=False)
    assert rc == B.TIDE_ERR_NULL
    bad = B.make_token_input(tr.embed, tr.input_ids, tr.w_in)          # no gradient / Adam buffers
    rc = B.tide_draft_train_step_tok(tr.ccfg, tr.c_params, tr.c_grads, tr.c_adam, bad, tr.hidden, tr.tokens, tr.mask, 1e-4,
                                     tr.loss, tr.workspace, tr.ws_bytes, s, check=False)
    assert rc == B.TIDE_ERR_NULL and "grad_w_in" in B.tide_last_error()
    B.tide_draft_forward_tok(tr.ccfg, tr.c_params, bad, tr.hidden, tr.tokens, tr.mask, tr.loss, None, tr.workspace,
                             tr.ws_bytes, s)                           # forward needs none of them
    bad.embed_rows = 0
    rc = B.tide_draft_forward_tok(tr.ccfg, tr.c_params, bad, tr.hidden, tr.tokens, tr.mask, tr.loss, None, tr.workspace,
                                  tr.ws_bytes, s, check=False)
    assert rc == B.TIDE_ERR_CONFIG
    assert tr.step == 0
    sync()


def test_large_tiles_identity_projection_is_bit_identical_to_the_base_step():
    """8B-shaped widths (d 4096, 32/8 heads, FFN 14336) with a reduced vocabulary, so that the projections of
    the variant run the 256x256-tile MFMA kernels with two operand pairs and a row stride of 2d.  In bf16,
    W_in = [I | 0] reproduces x0 bit for bit (a bf16 value times one, accumulated in fp32), so loss and the ten
    base gradients must be IDENTICAL to those of the base entry point; dW_in is checked against a plain matrix
    product of the workspace buffers."""
    import bench
    from paper_2602_05145_amd import binding as B
    cfg = W.get_config("8b", batch=8, vocab=8192)
    dev = torch.device("cuda:0")
    params, hidden, tokens, mask = bench.device_workload(cfg, dev, cfg["seed"])
    base = bench.DeviceTrainer(cfg, {k: v.clone() for k, v in params.items()}, hidden, tokens, mask)
    tr = bench.DeviceTrainer(cfg, {k: v.clone() for k, v in params.items()}, hidden, tokens, mask)
    d, T = cfg["hidden"], cfg["batch"] * cfg["seq"]
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    tr.embed = (torch.randn((4096, d), device=dev, generator=g) * 0.5).to(torch.bfloat16)
    tr.input_ids = torch.randint(0, 4096, (cfg["batch"], cfg["seq"]), device=dev, generator=g, dtype=torch.int32)
    tr.w_in = torch.cat([torch.eye(d, device=dev), torch.zeros((d, d), device=dev)], dim=1).to(torch.bfloat16).contiguous()
    f32 = dict(dtype=torch.float32, device=dev)
    tr.grad_w_in, tr.m_w_in, tr.v_w_in = (torch.zeros((d, 2 * d), **f32) for _ in range(3))
    tr.master_w_in = tr.w_in.float()
    tr.c_tok = B.make_token_input(tr.embed, tr.input_ids, tr.w_in, tr.grad_w_in, tr.m_w_in, tr.v_w_in, tr.master_w_in)
    print("base step", flush=True)
    base.train_step(cfg["lr"])
    print("token-input step", flush=True)
    tr.train_step_tok(cfg["lr"])
    sync()
    assert tr.status() == 0
    assert float(tr.loss.item()) == float(base.loss.item())
    for k in tr.grads:
        assert torch.equal(tr.grads[k], base.grads[k]), k
    dx0 = tr.intermediate("dx0", (T, d)).float()
    g0 = tr.intermediate("g0", (T, d)).float()
    e0 = tr.intermediate("e0", (T, d)).float()
    assert torch.equal(e0, tr.embed[tr.input_ids.reshape(-1).long()].float())
    for half, src in ((0, g0), (1, e0)):
        ref = dx0.T @ src
        got = tr.grad_w_in[:, half * d:(half + 1) * d]
        err = float((got - ref).abs().max()) / float(ref.abs().max())
        assert err <= 2e-3, (half, err)
    # W_in moved by at most lr per entry, and only where its gradient is non-zero
    step = (tr.master_w_in - torch.cat([torch.eye(d, device=dev), torch.zeros((d, d), device=dev)], dim=1) * (1 - cfg["lr"] * cfg["weight_decay"])).abs()
    assert float(step.max()) <= cfg["lr"] * (1 + 1e-3)
