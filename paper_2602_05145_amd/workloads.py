"""Seeded synthetic workloads for the TIDE draft-training step.

Holds no arithmetic of the method: only configuration tables, random input
generation and dtype packing.  Both the HIP path's tests/benchmark and the CPU
oracle's tests draw their inputs from here.

The paper trains the draft on hidden states captured while serving real
conversation / science / math / code traffic (Sec. 5.1); none of that data is
available, so these generators stand in for it with tensors of the same shape
and gross statistics: three concatenated residual-stream captures with a few
massive-activation channels, Zipf-distributed next-token ids, and prompt / pad
masking.
"""
from __future__ import annotations

import numpy as np

PARAM_NAMES = ("w_fc", "g1", "w_qkv", "w_o", "g2", "w_gate", "w_up", "w_down", "g3", "w_lm")

_COMMON = dict(n_capture=3, rms_eps=1e-5, beta1=0.9, beta2=0.999, adam_eps=1e-8,
               weight_decay=0.01, lr=1e-4)

CONFIGS = {
    # name: model/shape config + input recipe
    "tiny": dict(_COMMON, batch=2, seq=64, target_hidden=256, hidden=256, n_heads=4,
                 n_kv_heads=2, head_dim=64, ffn=688, vocab=4096, rope_theta=1e4, dtype="fp32",
                 seed=1001, outlier_frac=0.02, outlier_scale=8.0, zipf_s=1.1,
                 mask="bernoulli", mask_p=0.10),
    "small": dict(_COMMON, batch=8, seq=512, target_hidden=2048, hidden=2048, n_heads=16,
                  n_kv_heads=8, head_dim=128, ffn=5632, vocab=32000, rope_theta=1e4, dtype="bf16",
                  seed=1002, outlier_frac=0.01, outlier_scale=20.0, zipf_s=1.1,
                  mask="lengths", len_lo=128, len_hi=512),
    "8b": dict(_COMMON, batch=16, seq=2048, target_hidden=4096, hidden=4096, n_heads=32,
               n_kv_heads=8, head_dim=128, ffn=14336, vocab=128256, rope_theta=5e5, dtype="bf16",
               seed=1003, outlier_frac=0.01, outlier_scale=20.0, zipf_s=1.05,
               mask="prefix", mask_p=0.15),
    "longctx": dict(_COMMON, batch=2, seq=16384, target_hidden=4096, hidden=4096, n_heads=32,
                    n_kv_heads=8, head_dim=128, ffn=14336, vocab=128256, rope_theta=5e5,
                    dtype="bf16", seed=1004, outlier_frac=0.01, outlier_scale=20.0, zipf_s=1.05,
                    mask="prefix", mask_p=0.15),
    "32b": dict(_COMMON, batch=8, seq=4096, target_hidden=5120, hidden=5120, n_heads=40,
                n_kv_heads=8, head_dim=128, ffn=25600, vocab=152064, rope_theta=5e5, dtype="bf16",
                seed=1005, outlier_frac=0.01, outlier_scale=20.0, zipf_s=1.05,
                mask="prefix", mask_p=0.15),
}


def get_config(name, **overrides):
    cfg = dict(CONFIGS[name])
    cfg["name"] = name
    cfg.update(overrides)
    return cfg


def param_shapes(cfg):
    d = cfg["hidden"]
    nq = cfg["n_heads"] * cfg["head_dim"]
    nkv = cfg["n_kv_heads"] * cfg["head_dim"]
    return {
        "w_fc": (d, cfg["n_capture"] * cfg["target_hidden"]),
        "g1": (d,),
        "w_qkv": (nq + 2 * nkv, d),
        "w_o": (d, nq),
        "g2": (d,),
        "w_gate": (cfg["ffn"], d),
        "w_up": (cfg["ffn"], d),
        "w_down": (d, cfg["ffn"]),
        "g3": (d,),
        "w_lm": (cfg["vocab"], d),
    }


def n_params(cfg):
    return int(sum(int(np.prod(s)) for s in param_shapes(cfg).values()))


# ---- bf16 packing (round to nearest even), pure bit manipulation ----------
def f32_to_bf16_bits(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x):
    """fp32 array -> the nearest bf16 value, returned as fp32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x)).reshape(np.shape(x))


# ---- generators -----------------------------------------------------------
def make_params(cfg, rng):
    """Matrices N(0, 0.02^2), norm gains 1; fp32."""
    out = {}
    for name, shp in param_shapes(cfg).items():
        if len(shp) == 1:
            out[name] = np.ones(shp, np.float32)
        else:
            out[name] = (rng.standard_normal(shp, dtype=np.float32) * np.float32(0.02))
    return out


def make_inputs(cfg, rng):
    """hidden_buf [B,S,K*H_t] fp32, tokens [B,S] int32, loss_mask [B,S] uint8."""
    B, S = cfg["batch"], cfg["seq"]
    K, Ht, V = cfg["n_capture"], cfg["target_hidden"], cfg["vocab"]
    # outlier channels: fixed per captured layer, for all tokens
    n_out = int(round(cfg["outlier_frac"] * Ht))
    out_idx = [np.sort(rng.choice(Ht, size=n_out, replace=False)) for _ in range(K)]
    hidden = rng.standard_normal((B, S, K * Ht), dtype=np.float32)
    for kk in range(K):
        hidden[:, :, kk * Ht + out_idx[kk]] *= np.float32(cfg["outlier_scale"])
    # Zipf labels through a random permutation of the vocabulary
    perm = rng.permutation(V)
    w = np.arange(1, V + 1, dtype=np.float64) ** (-cfg["zipf_s"])
    cdf = np.cumsum(w / w.sum())
    ranks = np.searchsorted(cdf, rng.random((B, S)), side="right")
    ranks = np.minimum(ranks, V - 1)
    tokens = perm[ranks].astype(np.int32)
    # mask
    kind = cfg["mask"]
    if kind == "bernoulli":
        mask = (rng.random((B, S)) >= cfg["mask_p"]).astype(np.uint8)
    elif kind == "prefix":
        npre = int(np.floor(cfg["mask_p"] * S))
        mask = np.ones((B, S), np.uint8)
        mask[:, :npre] = 0
    elif kind == "lengths":
        lo, hi = min(cfg["len_lo"], S), min(cfg["len_hi"], S)
        L = rng.integers(lo, hi + 1, size=B)
        pos = np.arange(S)[None, :]
        mask = (pos < L[:, None]).astype(np.uint8)
        hidden[mask == 0] = 0.0
        tokens[mask == 0] = 0
    elif kind == "none":
        mask = np.ones((B, S), np.uint8)
    else:
        raise ValueError(f"unknown mask kind {kind!r}")
    return hidden, tokens, mask


def make_token_input(cfg, seed=None, embed_rows=None):
    """Seeded inputs of the token-input variant: a frozen embedding table [rows, d] (N(0, 0.5^2), the
    scale of the projected features), the id of the token sampled at every position (Zipf, like the
    labels) and the second projection W_in [d, 2d] (N(0, 0.02^2) like every matrix).  bf16 mode rounds
    the floats to bf16 values, as make_workload does."""
    rng = np.random.default_rng((cfg["seed"] if seed is None else seed) + 7919)
    d, V = cfg["hidden"], cfg["vocab"]
    rows = V if embed_rows is None else embed_rows
    embed = rng.standard_normal((rows, d), dtype=np.float32) * np.float32(0.5)
    w = np.arange(1, rows + 1, dtype=np.float64) ** (-cfg["zipf_s"])
    cdf = np.cumsum(w / w.sum())
    ranks = np.minimum(np.searchsorted(cdf, rng.random((cfg["batch"], cfg["seq"])), side="right"), rows - 1)
    input_ids = rng.permutation(rows)[ranks].astype(np.int32)
    w_in = rng.standard_normal((d, 2 * d), dtype=np.float32) * np.float32(0.02)
    if cfg["dtype"] == "bf16":
        embed, w_in = round_to_bf16(embed), round_to_bf16(w_in)
    return dict(embed=embed, input_ids=input_ids, w_in=w_in)


def make_workload(cfg, seed=None):
    """Seeded host workload.  In bf16 mode every float tensor is rounded to the
    nearest bf16 value once (still returned as fp32), so the HIP path gets the
    bf16 bits and the oracle the same values widened to fp64."""
    rng = np.random.default_rng(cfg["seed"] if seed is None else seed)
    params = make_params(cfg, rng)
    hidden, tokens, mask = make_inputs(cfg, rng)
    if cfg["dtype"] == "bf16":
        params = {k: round_to_bf16(v) for k, v in params.items()}
        hidden = round_to_bf16(hidden)
    return dict(params=params, hidden=hidden, tokens=tokens, mask=mask)


# ---- algorithmic work (for throughput reporting; not part of the method) --
def flops_per_step(cfg):
    """2 flop/MAC; forward + backward; causal attention at S(S+1)/2; no input
    gradient for the projection; no logits recompute counted."""
    T = cfg["batch"] * cfg["seq"]
    ps = {k: int(np.prod(s)) for k, s in param_shapes(cfg).items()}
    six = ps["w_qkv"] + ps["w_o"] + ps["w_gate"] + ps["w_up"] + ps["w_down"] + ps["w_lm"]
    f_gemm = 6 * six + 4 * ps["w_fc"]
    f_attn = 7 * cfg["n_heads"] * cfg["head_dim"] * (cfg["seq"] + 1)
    return float(T) * (f_gemm + f_attn)
