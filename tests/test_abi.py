"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header
declares, and validates configurations before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2602_05145_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2602_05145_amd import binding
    return binding


def _declared_symbols():
    """Every function declared by the two headers that libtide_draft.so implements (tide_control.h belongs
    to the host-only libtide_control.so and is checked in test_control_parity.py)."""
    names = set()
    for hdr in ("tide_draft.h", "tide_ingest.h"):
        text = open(os.path.join(ROOT, "include", hdr)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(tide_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol(B):
    lib = ctypes.CDLL(B.LIB_PATH)
    names = _declared_symbols()
    assert "tide_draft_forward" in names and "tide_draft_train_step" in names and "tide_ingest_submit" in names
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(B.EXPORTED)


def test_workspace_sizes_and_config_validation(B):
    for name in W.CONFIGS:
        c = B.make_config(W.get_config(name))
        assert B.tide_draft_workspace_bytes(c) > 0, name
    c = B.make_config(W.get_config("8b"))
    assert B.tide_draft_workspace_offset(c, "lm_rows") == 16384       # the LM head works by blocks of half the rows
    assert B.tide_draft_workspace_offset(B.make_config(W.get_config("small")), "lm_rows") == 4096   # ... of at least 4096
    assert B.tide_draft_workspace_offset(B.make_config(W.get_config("small", batch=12)), "lm_rows") == 4096
    assert B.tide_draft_workspace_offset(B.make_config(W.get_config("small", batch=20)), "lm_rows") == 5120
    assert B.tide_draft_workspace_offset(c, "nonsense") == -1
    bad = [("n_heads", 3, "multiple"), ("hidden", 250, "hidden"), ("head_dim", 63, "hidden"),
           ("vocab", 0, "positive"), ("dtype", 7, "dtype"), ("rms_eps", 0.0, "rms_eps"), ("batch", -1, "positive")]
    for field, val, word in bad:
        c = B.make_config(W.get_config("tiny"))
        setattr(c, field, val)
        assert B.tide_draft_workspace_bytes(c) == 0, field
        assert word in B.tide_last_error(), (field, B.tide_last_error())


def test_split_plan_of_a_partly_filled_last_tile_round(B):
    """Host logic of the split over K (no device call): only float results whose 256 x 256 tiles leave the last round
    of the 256 compute units at most half full are split, into as many parts as fit that round (at most 8, each at
    least 32 slabs of 32 long); the workspace is one 256 x 256 float tile per further part and split tile."""
    TN, F32, BF16 = 2, B.TIDE_DTYPE_FP32, B.TIDE_DTYPE_BF16
    tile = 256 * 256 * 4
    need = B.tide_gemm_workspace_bytes
    assert need(TN, 14336, 4096, 27856, F32) == 1 * 128 * tile        # 896 tiles = 3.5 rounds: 128 tiles in two parts
    assert need(TN, 6144, 4096, 32768, F32) == 1 * 128 * tile         # 384 tiles = 1.5 rounds
    assert need(TN, 128256, 4096, 16384, F32) == 2 * 80 * tile        # 8016 tiles = 31 rounds + 80: three parts each
    assert need(TN, 4096, 4096, 27856, F32) == 0                      # 256 tiles: the round is full
    assert need(TN, 4096 + 256 * 9, 4096, 27856, F32) == 0            # 400 tiles: 144 left, more than half a round
    assert need(TN, 14336, 4096, 27856, BF16) == 0                    # bf16 results are never split
    assert need(TN, 2048, 4096, 27856, F32) == 0                      # 128 tiles: the small-tile kernel takes those
    assert need(TN, 14336, 4096, 1024, F32) == 0                      # K too short for two parts of 32 slabs
    assert need(TN, 4096 + 256, 4096, 1 << 20, F32) == 7 * 16 * tile  # 16 tiles left: 8 parts at most
    assert need(0, 14336 + 128, 4096, 27856, F32) == need(TN, 14336 + 128, 4096, 27856, F32)   # any layout


def test_calls_reject_bad_arguments_before_touching_the_device(B):
    c = B.make_config(W.get_config("tiny"))
    t = B.make_tensors(None)
    rc = B.tide_draft_forward(c, t, 256, 256, 256, 256, None, 256, 1 << 40, None, check=False)
    assert rc == B.TIDE_ERR_NULL and "params" in B.tide_last_error()
    rc = B.tide_draft_forward(None, t, 256, 256, 256, 256, None, 256, 1 << 40, None, check=False)
    assert rc == B.TIDE_ERR_NULL
    c.n_kv_heads = 3
    rc = B.tide_draft_train_step(c, t, t, B.TideAdamState(), 256, 256, 256, 1e-4, 256, 256, 1 << 40, None, check=False)
    assert rc == B.TIDE_ERR_CONFIG
    with pytest.raises(B.TideError):
        B.tide_draft_train_step(c, t, t, B.TideAdamState(), 256, 256, 256, 1e-4, 256, 256, 1 << 40, None)


def test_unroll_calls_validate_before_touching_the_device(B):
    c = B.make_config(W.get_config("8b"))
    one = B.tide_draft_workspace_bytes(c)
    for n in (1, 3, 8):
        need = B.tide_draft_unroll_workspace_bytes(c, n)
        assert need >= n * one
        assert B.tide_draft_unroll_workspace_offset(c, n, n - 1, "x2") >= (n - 1) * one
        assert B.tide_draft_unroll_workspace_offset(c, n, n - 1, "own_kv") >= n * one
        assert B.tide_draft_unroll_workspace_offset(c, n, n, "x2") == -1
    assert B.tide_draft_unroll_workspace_bytes(c, 0) == 0 and B.tide_draft_unroll_workspace_bytes(c, 9) == 0
    assert B.tide_draft_unroll_workspace_offset(c, 3, 0, "nonsense") == -1
    t = B.make_tensors(None)
    assert B.tide_draft_eval_unroll(c, t, None, 256, 256, 256, 3, 256, 256, 256, 1 << 40, None, check=False) == B.TIDE_ERR_NULL
    assert B.tide_draft_eval_unroll(c, t, None, 256, 256, 256, 0, 256, 256, 256, 1 << 40, None, check=False) == B.TIDE_ERR_CONFIG
    assert B.tide_draft_train_step_unroll(c, t, t, B.TideAdamState(), None, 256, 256, 256, 9, None, 1e-4, 256, 256, 1 << 40,
                                          None, check=False) == B.TIDE_ERR_CONFIG
    assert B.tide_draft_train_step_unroll(c, t, t, B.TideAdamState(), None, 256, 256, 256, 2, [1.0, -1.0], 1e-4, 256, 256,
                                          1 << 40, None, check=False) == B.TIDE_ERR_CONFIG
    assert B.tide_draft_eval_unroll_packed(c, t, None, 256, 256, 256, None, 2, 100, 3, 256, 256, 256, 1 << 40, None,
                                           check=False) == B.TIDE_ERR_NULL
    assert B.tide_draft_train_step_unroll_packed(c, t, t, B.TideAdamState(), None, 256, 256, 256, 256, 0, 100, 3, None, 1e-4,
                                                 256, 256, 1 << 40, None, check=False) == B.TIDE_ERR_CONFIG


def test_every_header_in_include_is_covered():
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["tide_control.h", "tide_draft.h", "tide_ingest.h"]


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py says so and exits before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
    env = dict(os.environ, WORLD_SIZE="4")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
