"""Per-kernel parity: each HIP building block, called through the C ABI, against the matching
function of the CPU oracle on the same seeded inputs.  Shapes span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

from oracle import tide_oracle as O
from tests.gpu_util import DEV, cosine, quantize, rel_max, stream, sync, to_dev, to_host

pytestmark = pytest.mark.gpu

DT = {"fp32": 0, "bf16": 1}


@pytest.fixture(scope="module")
def B():
    from paper_2602_05145_amd import binding
    return binding


# ------------------------------------------------------------------ GEMM
def _gemm_case(B, layout, M, N, K, in_dt, out_dt, seed, residual=False, accumulate=False, alpha=1.0):
    rng = np.random.default_rng(seed)
    shapeA = (K, M) if layout == B.LAYOUT_TN else (M, K)
    shapeB = (N, K) if layout == B.LAYOUT_NT else (K, N)
    A = quantize(rng.standard_normal(shapeA), in_dt)
    Bm = quantize(rng.standard_normal(shapeB), in_dt)
    C0 = quantize(rng.standard_normal((M, N)), out_dt)
    R = quantize(rng.standard_normal((M, N)), out_dt)
    opA = A.T if layout == B.LAYOUT_TN else A
    opB = Bm.T if layout == B.LAYOUT_NT else Bm
    ref = alpha * (opA @ opB)
    if residual:
        ref = ref + R
    if accumulate:
        ref = ref + C0
    dA, dB = to_dev(A, in_dt), to_dev(Bm, in_dt)
    dC, dR = to_dev(C0, out_dt), to_dev(R, out_dt)
    print(f"gemm layout={layout} M={M} N={N} K={K} {in_dt}->{out_dt} res={residual} acc={accumulate}", flush=True)
    B.tide_gemm(layout, M, N, K, alpha, dA, dB, dC, dR if residual else None, DT[in_dt], DT[out_dt],
                accumulate, stream())
    sync()
    return to_host(dC), ref


@pytest.mark.parametrize("layout", [0, 1, 2])
@pytest.mark.parametrize("shape", [(300, 520, 136), (64, 72, 64), (8, 8, 8), (1000, 264, 1096)])
def test_gemm_bf16_small_tiles(B, layout, shape):
    M, N, K = shape
    got, ref = _gemm_case(B, layout, M, N, K, "bf16", "fp32", seed=11 + layout)
    assert rel_max(got, ref) < 2e-5
    got, ref = _gemm_case(B, layout, M, N, K, "bf16", "bf16", seed=21 + layout, residual=True, alpha=0.5)
    assert rel_max(got, ref) < 6e-3      # bf16 output rounding (2^-9 relative)
    assert cosine(got, ref) > 0.99999


@pytest.mark.parametrize("layout", [0, 1, 2])
@pytest.mark.parametrize("K", [200, 192, 448])
def test_gemm_bf16_large_tiles_ragged(B, layout, K):
    # >= 200 tiles of 256x256 selects the large-tile kernel; M and N ragged w.r.t. 256, K ragged w.r.t. the slab
    # depth of 64 (200) or a whole number of slabs (192, 448: the path with loop-constant load offsets; 3 slabs
    # and 7 slabs end in different positions of the ring)
    M, N = 3720, 3656
    got, ref = _gemm_case(B, layout, M, N, K, "bf16", "fp32", seed=31 + layout, accumulate=True)
    assert rel_max(got, ref) < 2e-5
    got, ref = _gemm_case(B, layout, M, N, K, "bf16", "bf16", seed=41 + layout)
    assert rel_max(got, ref) < 6e-3
    assert cosine(got, ref) > 0.99999


@pytest.mark.parametrize("K", [4408, 4416])
@pytest.mark.parametrize("layout,accumulate", [(2, False), (2, True), (0, False), (1, True)])
def test_gemm_split_of_the_last_tile_round(B, layout, accumulate, K):
    """fp32 results whose tiles leave the last round of the 256 compute units at most half full: with a workspace
    those tiles are split over K and a second kernel adds the partial sums.  Against the oracle product, and
    against the unsplit launch (same tiles, different order of the fp32 additions).  17 x 16 tiles of 256 =
    272 = one round + 16 tiles, split four ways (a part keeps at least 1024 of K); ragged M and N; K ragged (4408)
    or a whole number of 64-deep slabs (4416: the launches whose loads take loop-constant offsets)."""
    M, N = 17 * 256 - 40, 16 * 256 - 8
    need = B.tide_gemm_workspace_bytes(layout, M, N, K, DT["fp32"])
    assert need == 3 * 16 * 256 * 256 * 4
    assert B.tide_gemm_workspace_bytes(layout, M, N, K, DT["bf16"]) == 0             # bf16 results are never split
    assert B.tide_gemm_workspace_bytes(layout, 16 * 256, 16 * 256, K, DT["fp32"]) == 0   # a full round
    rng = np.random.default_rng(71 + layout)
    shapeA = (K, M) if layout == B.LAYOUT_TN else (M, K)
    shapeB = (N, K) if layout == B.LAYOUT_NT else (K, N)
    A, Bm = quantize(rng.standard_normal(shapeA), "bf16"), quantize(rng.standard_normal(shapeB), "bf16")
    C0 = rng.standard_normal((M, N)).astype(np.float32).astype(np.float64)
    opA = A.T if layout == B.LAYOUT_TN else A
    opB = Bm.T if layout == B.LAYOUT_NT else Bm
    ref = 0.5 * (opA @ opB) + (C0 if accumulate else 0.0)
    dA, dB = to_dev(A, "bf16"), to_dev(Bm, "bf16")
    out = []
    for ws_bytes in (need, 0):
        dC = to_dev(C0, "fp32")
        ws = torch.full((max(ws_bytes, 16),), 0xFF, dtype=torch.uint8, device=DEV)       # NaN patterns: every partial must be written
        print(f"gemm split layout={layout} acc={accumulate} workspace={ws_bytes}", flush=True)
        B.tide_gemm(layout, M, N, K, 0.5, dA, dB, dC, None, DT["bf16"], DT["fp32"], accumulate, stream(),
                    workspace=ws if ws_bytes else None, workspace_bytes=ws_bytes)
        sync()
        out.append(to_host(dC))
    assert rel_max(out[0], ref) < 2e-5 and rel_max(out[1], ref) < 2e-5
    assert rel_max(out[0], out[1]) < 5e-6
    assert not np.array_equal(out[0], out[1])          # the split really happened (another summation order)


@pytest.mark.parametrize("layout", [0, 1, 2])
def test_gemm_unaligned_falls_back(B, layout):
    # K, M, N not multiples of 8: the shape-agnostic kernel takes over
    got, ref = _gemm_case(B, layout, 77, 53, 101, "bf16", "fp32", seed=51 + layout)
    assert rel_max(got, ref) < 2e-5
    got, ref = _gemm_case(B, layout, 77, 53, 101, "fp32", "fp32", seed=61 + layout, residual=True, accumulate=True, alpha=-1.5)
    assert rel_max(got, ref) < 2e-6


def test_gemm_bad_arguments(B):
    a = torch.zeros(64, device=DEV)
    assert B.tide_gemm(0, 8, 8, 8, 1.0, None, a, a, None, 0, 0, 0, stream(), check=False) == B.TIDE_ERR_NULL
    assert B.tide_gemm(5, 8, 8, 8, 1.0, a, a, a, None, 0, 0, 0, stream(), check=False) == B.TIDE_ERR_CONFIG
    assert B.tide_gemm(0, 0, 8, 8, 1.0, a, a, a, None, 0, 0, 0, stream(), check=False) == B.TIDE_ERR_CONFIG
    assert "layout" in B.tide_last_error() or "size" in B.tide_last_error()


# ------------------------------------------------------------------ cross-entropy pass
@pytest.mark.parametrize("dtype,vocab", [
    ("bf16", 11), ("bf16", 4093), ("bf16", 9001), ("bf16", 16391), ("bf16", 40003), ("bf16", 70001),
    ("bf16", 128256), ("bf16", 131080), ("bf16", 152064), ("bf16", 250007), ("fp32", 9001)])
def test_cross_entropy_pass_of_a_logit_block(B, dtype, vocab):
    """tide_ce_train on a block of logits against the oracle's ce_dz on the same (storage-rounded) logits: lse and
    the loss terms to fp32 accuracy, every gradient element to the rounding of its storage type, padded columns
    exactly zero, masked rows and rows with an out-of-range label exactly zero.  The bf16 kernel keeps a row in the
    registers and LDS of a 512-thread block (16-byte chunks 4096 columns apart): the vocabulary sizes end inside a
    chunk, are no multiple of 8, leave whole chunks past the end of the row, need one block per CU (152064), or do
    not fit at all and take the two-read kernel (250007)."""
    rng = np.random.default_rng(vocab)
    rows = 37
    ldz = (vocab + 63) // 64 * 64
    z = quantize(rng.standard_normal((rows, vocab)) * 3.0, dtype)
    z[5, :] += 40.0 * (rng.random(vocab) < 1e-3)              # a row dominated by a few large logits
    z[6, :] = quantize(-30.0 + rng.standard_normal(vocab), dtype)
    z = quantize(z, dtype)
    tokens = rng.integers(0, vocab, rows).astype(np.int32)
    tokens[0], tokens[1], tokens[2] = vocab - 1, 0, min(vocab - 1, 4096)
    tokens[3], tokens[4] = vocab + 3, -1                      # out of range: the row keeps no loss
    mask = np.ones(rows, np.uint8)
    mask[7] = 0
    zp = np.full((rows, ldz), 7.0)                            # the padding holds garbage on entry
    zp[:, :vocab] = z
    dz_d = to_dev(zp, dtype)
    tok_d = torch.from_numpy(tokens).to(DEV)
    mask_d = torch.from_numpy(mask).to(DEV)
    lse_d = torch.empty(rows, dtype=torch.float32, device=DEV)
    loss_d = torch.empty(rows, dtype=torch.float32, device=DEV)
    print(f"ce pass {dtype} rows={rows} vocab={vocab} ldz={ldz}", flush=True)
    B.tide_ce_train(rows, vocab, dz_d, ldz, tok_d, mask_d, lse_d, loss_d, DT[dtype], stream())
    sync()
    dz, lse, loss = to_host(dz_d), to_host(lse_d), to_host(loss_d)
    keep = O.effective_mask(tokens, mask, vocab)
    assert int(keep.sum()) == rows - 3
    ref = O.ce_dz(z, tokens, mask) * int(keep.sum())          # the pass leaves the 1/N to the products that read dz
    zmax = z.max(-1)
    lse_ref = np.log(np.sum(np.exp(z - zmax[:, None]), -1)) + zmax
    assert np.max(np.abs(lse - lse_ref)) <= 1e-5 * np.max(np.abs(lse_ref)) + 1e-5
    loss_ref = np.where(keep, lse_ref - z[np.arange(rows), np.clip(tokens, 0, vocab - 1)], 0.0)
    assert np.max(np.abs(loss - loss_ref)) <= 1e-4
    assert not np.any(dz[:, vocab:] != 0)
    assert not np.any(dz[~keep] != 0)
    ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -16        # storage rounding plus the fp32 exponential of |z - lse| <= 64
    assert np.all(np.abs(dz[:, :vocab] - ref) <= ulp * np.abs(ref) + 1e-9)


def test_cross_entropy_pass_rejects_bad_arguments(B):
    t = torch.zeros(64, dtype=torch.float32, device=DEV)
    i = torch.zeros(4, dtype=torch.int32, device=DEV)
    m = torch.ones(4, dtype=torch.uint8, device=DEV)
    assert B.tide_ce_train(1, 16, None, 16, i, m, t, t, 0, stream(), check=False) == B.TIDE_ERR_NULL
    assert B.tide_ce_train(1, 16, t, 8, i, m, t, t, 0, stream(), check=False) == B.TIDE_ERR_CONFIG     # ldz < vocab
    assert B.tide_ce_train(1, 12, t, 12, i, m, t, t, 0, stream(), check=False) == B.TIDE_ERR_CONFIG    # ldz % 8
    assert B.tide_ce_train(1, 16, t, 16, i, m, t, t, 5, stream(), check=False) == B.TIDE_ERR_CONFIG    # dtype
    assert B.tide_ce_train(0, 16, t, 16, i, m, t, t, 0, stream()) == 0                                  # no rows: nothing to do


# ------------------------------------------------------------------ RMSNorm
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("rows,d", [(70, 256), (33, 4096), (5, 24), (40, 100)])
def test_rmsnorm_fwd_bwd(B, dtype, rows, d):
    rng = np.random.default_rng(rows * 1000 + d)
    x = quantize(rng.standard_normal((rows, d)) * 3, dtype)
    x[rows // 2] = 0.0  # a pad row: finite output, zero gradient contribution
    g = quantize(1 + 0.2 * rng.standard_normal(d), dtype)
    dy = quantize(rng.standard_normal((rows, d)), dtype)
    res = quantize(rng.standard_normal((rows, d)), dtype)
    eps = 1e-5
    y_ref, r_ref = O.rmsnorm_fwd(x, g, eps)
    dx_ref, dg_ref = O.rmsnorm_bwd(dy, x, g, r_ref)
    dx_ref = dx_ref + res
    dx_, dg_, y_ = to_dev(np.zeros_like(x), dtype), torch.zeros(d, device=DEV), to_dev(np.zeros_like(x), dtype)
    rstd = torch.zeros(rows, device=DEV)
    xd, gd, dyd, resd = to_dev(x, dtype), to_dev(g, dtype), to_dev(dy, dtype), to_dev(res, dtype)
    print(f"rmsnorm rows={rows} d={d} {dtype}", flush=True)
    B.tide_rmsnorm_fwd(rows, d, xd, gd, eps, y_, rstd, DT[dtype], stream())
    scratch = torch.empty(B.tide_rmsnorm_bwd_scratch_bytes(rows, d), dtype=torch.uint8, device=DEV)
    B.tide_rmsnorm_bwd(rows, d, dyd, xd, gd, rstd, resd, dx_, dg_, scratch, DT[dtype], stream())
    sync()
    tol = 1e-5 if dtype == "fp32" else 8e-3
    assert rel_max(to_host(rstd), r_ref[:, 0]) < 1e-5
    assert rel_max(to_host(y_), y_ref) < tol
    assert rel_max(to_host(dx_), dx_ref) < tol
    assert rel_max(to_host(dg_), dg_ref) < 1e-5
    assert np.all(to_host(y_)[rows // 2] == 0.0)


# ------------------------------------------------------------------ RoPE
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_rope_forward_and_inverse(B, dtype):
    Bn, S, nh, nkv, dh, theta = 2, 300, 4, 2, 64, 5e5
    rng = np.random.default_rng(5)
    ld = (nh + 2 * nkv) * dh
    qkv = quantize(rng.standard_normal((Bn * S, ld)), dtype)
    cos, sin = O.rope_angles(S, dh, theta)
    q = qkv[:, :nh * dh].reshape(Bn, S, nh, dh)
    k = qkv[:, nh * dh:(nh + nkv) * dh].reshape(Bn, S, nkv, dh)
    ref = qkv.copy()
    ref[:, :nh * dh] = O.rope_apply(q, cos, sin).reshape(Bn * S, -1)
    ref[:, nh * dh:(nh + nkv) * dh] = O.rope_apply(k, cos, sin).reshape(Bn * S, -1)
    d = to_dev(qkv, dtype)
    table = torch.empty(S * dh, device=DEV)
    B.tide_rope(Bn, S, nh, nkv, dh, theta, d, table, 0, DT[dtype], stream())
    sync()
    got = to_host(d)
    tol = 2e-6 if dtype == "fp32" else 8e-3
    assert rel_max(got, ref) < tol
    assert np.array_equal(got[:, (nh + nkv) * dh:], qkv[:, (nh + nkv) * dh:])  # v untouched
    # inverse rotation = the backward pass
    refi = qkv.copy()
    refi[:, :nh * dh] = O.rope_apply(q, cos, sin, inverse=True).reshape(Bn * S, -1)
    refi[:, nh * dh:(nh + nkv) * dh] = O.rope_apply(k, cos, sin, inverse=True).reshape(Bn * S, -1)
    d = to_dev(qkv, dtype)
    B.tide_rope(Bn, S, nh, nkv, dh, theta, d, table, 1, DT[dtype], stream())
    sync()
    assert rel_max(to_host(d), refi) < tol


# ------------------------------------------------------------------ attention
def _attn_case(B, dtype, Bn, S, nh, nkv, dh, seed):
    rng = np.random.default_rng(seed)
    ld = (nh + 2 * nkv) * dh
    qkv = quantize(rng.standard_normal((Bn * S, ld)), dtype)
    dout = quantize(rng.standard_normal((Bn * S, nh * dh)), dtype)
    q = qkv[:, :nh * dh].reshape(Bn, S, nh, dh)
    k = qkv[:, nh * dh:(nh + nkv) * dh].reshape(Bn, S, nkv, dh)
    v = qkv[:, (nh + nkv) * dh:].reshape(Bn, S, nkv, dh)
    A, P = O.attention_fwd(q, k, v)
    qd = to_dev(qkv, dtype)
    out = to_dev(np.zeros((Bn * S, nh * dh)), dtype)
    lse = torch.zeros(Bn * nh * S, device=DEV)
    print(f"attention {dtype} B={Bn} S={S} nh={nh} nkv={nkv} dh={dh}", flush=True)
    B.tide_attention_fwd(Bn, S, nh, nkv, dh, qd, out, lse, DT[dtype], stream())
    sync()
    # backward consumes the forward's own (rounded) output, like the training step does
    A_dev = to_host(out).reshape(Bn, S, nh, dh)
    dq, dk, dv = O.attention_bwd(dout.reshape(Bn, S, nh, dh), q, k, v, P)
    dref = np.concatenate([dq.reshape(Bn * S, -1), dk.reshape(Bn * S, -1), dv.reshape(Bn * S, -1)], 1)
    dqkv = to_dev(np.zeros_like(qkv), dtype)
    delta = torch.zeros(Bn * nh * S, device=DEV)
    B.tide_attention_bwd(Bn, S, nh, nkv, dh, qd, out, to_dev(dout, dtype), lse, delta, dqkv, DT[dtype], stream())
    sync()
    # lse reference from the scores
    scale = 1 / np.sqrt(dh)
    G = nh // nkv
    lse_ref = np.empty((Bn, nh, S))
    for b in range(Bn):
        for h in range(nh):
            sc = (q[b, :, h] @ k[b, :, h // G].T) * scale
            sc[np.triu(np.ones((S, S), bool), 1)] = -np.inf
            m = sc.max(-1)
            lse_ref[b, h] = m + np.log(np.exp(sc - m[:, None]).sum(-1))
    return (A_dev.reshape(Bn * S, -1), A.reshape(Bn * S, -1), to_host(lse).reshape(Bn, nh, S), lse_ref,
            to_host(dqkv), dref, (nh * dh, nkv * dh))


@pytest.mark.parametrize("dtype,shape", [
    ("fp32", (2, 70, 4, 2, 64)), ("fp32", (1, 1, 2, 1, 8)), ("fp32", (1, 130, 2, 2, 16)),
    ("bf16", (2, 70, 4, 2, 64)), ("bf16", (1, 200, 4, 1, 128)), ("bf16", (2, 333, 4, 2, 128)),
    # batch * kv heads a multiple of 8: the blocks of a kv head are then numbered so that they share an XCD
    ("bf16", (4, 300, 4, 2, 128)), ("bf16", (8, 129, 2, 1, 128)), ("bf16", (16, 40, 3, 3, 128)),
])
def test_attention_fwd_bwd(B, dtype, shape):
    got, ref, lse, lse_ref, dgot, dref, (nq, nk) = _attn_case(B, dtype, *shape, seed=sum(shape))
    if dtype == "fp32":
        assert rel_max(got, ref) < 1e-5
        assert np.max(np.abs(lse - lse_ref)) < 1e-5
        for sl in (slice(0, nq), slice(nq, nq + nk), slice(nq + nk, None)):
            assert rel_max(dgot[:, sl], dref[:, sl]) < 2e-5
    else:
        assert rel_max(got, ref) < 1e-2
        assert np.max(np.abs(lse - lse_ref)) < 2e-2
        for sl in (slice(0, nq), slice(nq, nq + nk), slice(nq + nk, None)):
            assert cosine(dgot[:, sl], dref[:, sl]) > 0.9995
            assert rel_max(dgot[:, sl], dref[:, sl]) < 3e-2


def test_mfma_probe_runs_and_counts(B):
    """The pure-MFMA probe: flop count, finite output within the bound its operands allow, argument checks."""
    sink = torch.zeros(4 * 512, dtype=torch.float32, device="cuda:0")
    s = torch.cuda.current_stream().cuda_stream
    fl = B.tide_mfma_probe(4, 10, sink, s)
    sync()
    assert fl == 4 * 8 * 10 * 8 * 2 * 32 * 32 * 16
    assert bool(torch.isfinite(sink).all())
    # operands have magnitude below 2: every accumulator element gains at most 16 products of 4 per MFMA, so
    # |value| <= 8 acc x 16 elem x 10 it x 64; random signs keep the sums far from zero as well as from the bound
    assert 0.0 < float(sink.abs().max()) <= 8 * 16 * 10 * 64
    import ctypes
    assert B.lib().tide_mfma_probe(0, 10, ctypes.c_void_p(sink.data_ptr()), None, s) == B.TIDE_ERR_CONFIG
    assert B.lib().tide_mfma_probe(4, 10, None, None, s) == B.TIDE_ERR_NULL


@pytest.mark.parametrize("shape", [(16, 2048, 32, 8), (2, 8192, 32, 8)])
def test_attention_at_benchmark_shapes_against_library_attention(B, shape):
    """Forward and backward of the flash kernels at the benchmark's head layout and sequence lengths against the
    framework's scaled_dot_product_attention (fp32 math on the same bf16 inputs, autograd for the gradients):
    an independent implementation at sizes the CPU oracle cannot reach."""
    import torch.nn.functional as F
    Bn, S, nh, nkv = shape
    dh, G = 128, nh // nkv
    g = torch.Generator(device=DEV)
    g.manual_seed(S)
    ld = (nh + 2 * nkv) * dh
    qkv = torch.randn((Bn * S, ld), device=DEV, generator=g).to(torch.bfloat16)
    dout = torch.randn((Bn * S, nh * dh), device=DEV, generator=g).to(torch.bfloat16)
    out = torch.empty((Bn * S, nh * dh), device=DEV, dtype=torch.bfloat16)
    lse = torch.empty(Bn * nh * S, device=DEV)
    delta = torch.empty(Bn * nh * S, device=DEV)
    dqkv = torch.empty_like(qkv)
    print(f"attention at B={Bn} S={S} nh={nh} nkv={nkv}", flush=True)
    B.tide_attention_fwd(Bn, S, nh, nkv, dh, qkv, out, lse, DT["bf16"], stream())
    B.tide_attention_bwd(Bn, S, nh, nkv, dh, qkv, out, dout, lse, delta, dqkv, DT["bf16"], stream())
    sync()
    # reference: one batch element at a time to bound memory (fp32 scores of 32 heads x S x S)
    worst = {}
    for b in range(0, Bn, max(1, Bn // 2)):                      # two batch elements are enough
        rows = slice(b * S, (b + 1) * S)
        x = qkv[rows].float().requires_grad_(True)
        q = x[:, :nh * dh].reshape(S, nh, dh).transpose(0, 1)
        k = x[:, nh * dh:(nh + nkv) * dh].reshape(S, nkv, dh).transpose(0, 1).repeat_interleave(G, dim=0)
        v = x[:, (nh + nkv) * dh:].reshape(S, nkv, dh).transpose(0, 1).repeat_interleave(G, dim=0)
        chunks = []
        for h0 in range(0, nh, 8):                               # 8 heads at a time
            chunks.append(F.scaled_dot_product_attention(q[h0:h0 + 8][None], k[h0:h0 + 8][None], v[h0:h0 + 8][None],
                                                         is_causal=True)[0])
        ref = torch.cat(chunks, 0).transpose(0, 1).reshape(S, nh * dh)
        ref.backward(dout[rows].float())
        for name, got, want in (("out", out[rows].float(), ref.detach()), ("dq", dqkv[rows, :nh * dh].float(), x.grad[:, :nh * dh]),
                                ("dk", dqkv[rows, nh * dh:(nh + nkv) * dh].float(), x.grad[:, nh * dh:(nh + nkv) * dh]),
                                ("dv", dqkv[rows, (nh + nkv) * dh:].float(), x.grad[:, (nh + nkv) * dh:])):
            cos = float((got * want).sum() / (got.norm() * want.norm()))
            err = float((got - want).abs().max() / want.abs().max())
            worst[name] = (min(cos, worst.get(name, (1.0, 0.0))[0]), max(err, worst.get(name, (1.0, 0.0))[1]))
        del x, q, k, v, ref, chunks
    print(worst, flush=True)
    for name, (cos, err) in worst.items():
        assert cos >= 0.9999 and err <= 1e-2, (name, cos, err)
