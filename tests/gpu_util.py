"""Helpers for GPU parity tests: device upload / download and error metrics."""
import numpy as np
import torch

from paper_2602_05145_amd import workloads as W

DEV = "cuda:0"


def to_dev(x, dtype):
    """numpy fp32/fp64 -> device tensor of the mode's storage dtype."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DEV)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def to_host(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def quantize(x, dtype):
    """What the device will actually hold, as fp64."""
    x = np.asarray(x, np.float32)
    return (W.round_to_bf16(x) if dtype == "bf16" else x).astype(np.float64)


def rel_max(a, b):
    """max |a-b| / max |b|"""
    den = float(np.max(np.abs(b)))
    return float(np.max(np.abs(a - b))) / (den if den > 0 else 1.0)


def cosine(a, b):
    a = a.reshape(-1)
    b = b.reshape(-1)
    na, nb = np.linalg.norm(a), np.linalg.norm(b)
    if na == 0 and nb == 0:
        return 1.0
    return float(a @ b / (na * nb))


def stream():
    return torch.cuda.current_stream().cuda_stream


def sync():
    torch.cuda.synchronize()
