"""tide_rmsnorm_bwd_static (the entry point for callers that cannot allocate: its per-block partial sums live in a
fixed array inside the library) against tide_rmsnorm_bwd with a caller buffer: same kernels, same grid, so the
results must be bit-identical.  Two calls in a row share the array, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2602_05145_amd import binding as B
from tests.gpu_util import DEV, stream, sync

pytestmark = pytest.mark.gpu


def _case(rows, d, dtype, seed, with_residual):
    tdt = torch.bfloat16 if dtype == B.TIDE_DTYPE_BF16 else torch.float32
    g = torch.Generator(device="cpu").manual_seed(seed)
    mk = lambda *shape: torch.randn(*shape, generator=g, dtype=torch.float32).to(DEV).to(tdt)
    x, dy, gain = mk(rows, d), mk(rows, d), (1.0 + 0.1 * mk(d).float()).to(tdt)
    res = mk(rows, d) if with_residual else None
    rstd = torch.rsqrt(x.float().pow(2).mean(-1) + 1e-5).contiguous()
    out = []
    for static in (False, True):
        dx = torch.full((rows, d), float("nan"), dtype=tdt, device=DEV)
        dg = torch.full((d,), float("nan"), dtype=torch.float32, device=DEV)
        print(f"rmsnorm bwd rows={rows} d={d} dtype={dtype} residual={with_residual} static={static}", flush=True)
        if static:
            B.tide_rmsnorm_bwd_static(rows, d, dy, x, gain, rstd, res, dx, dg, dtype, stream())
        else:
            scratch = torch.empty(B.tide_rmsnorm_bwd_scratch_bytes(rows, d), dtype=torch.uint8, device=DEV)
            B.tide_rmsnorm_bwd(rows, d, dy, x, gain, rstd, res, dx, dg, scratch, dtype, stream())
        sync()
        out.append((dx, dg))
    (dx0, dg0), (dx1, dg1) = out
    assert bool(torch.isfinite(dg1).all()) and bool(torch.isfinite(dx1.float()).all())
    assert torch.equal(dx0, dx1)
    assert torch.equal(dg0, dg1)


def test_static_scratch_matches_caller_scratch_on_two_calls_in_a_row():
    # the larger call first: it leaves its partial sums in the shared array; the smaller one must not see them
    _case(5000, 4096, B.TIDE_DTYPE_BF16, 1, True)
    _case(37, 4096, B.TIDE_DTYPE_BF16, 2, False)
    _case(700, 8192, B.TIDE_DTYPE_BF16, 3, True)      # the shape that fills the array exactly (512 blocks x 8192)
    _case(9, 264, B.TIDE_DTYPE_FP32, 4, False)
    _case(300, 1000, B.TIDE_DTYPE_FP32, 5, True)      # scalar path (d not a multiple of 8)


def test_static_scratch_argument_errors():
    x = torch.zeros(8, 16, device=DEV)
    r = torch.ones(8, device=DEV)
    dg = torch.zeros(16, device=DEV)
    s = stream()
    assert B.tide_rmsnorm_bwd_static(8, 16, x, x, dg, r, None, None, dg, 0, s, check=False) == B.TIDE_ERR_NULL
    assert B.tide_rmsnorm_bwd_static(8, 9000, x, x, dg, r, None, x, dg, 0, s, check=False) == B.TIDE_ERR_CONFIG
    assert B.tide_rmsnorm_bwd_static(0, 16, x, x, dg, r, None, x, dg, 0, s, check=False) == B.TIDE_ERR_CONFIG
    assert B.tide_rmsnorm_bwd_scratch_bytes(1 << 20, 8192) <= 16 << 20
