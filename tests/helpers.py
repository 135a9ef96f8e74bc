"""Shared test helpers (no arithmetic of the method)."""
import numpy as np

from paper_2602_05145_amd import workloads as W


def micro_cfg(**kw):
    """A config small enough for finite differences / brute force."""
    cfg = dict(batch=1, seq=5, n_capture=3, target_hidden=4, hidden=8, n_heads=2, n_kv_heads=1,
               head_dim=4, ffn=6, vocab=11, rope_theta=1e4, rms_eps=1e-5, beta1=0.9, beta2=0.999,
               adam_eps=1e-8, weight_decay=0.01, lr=1e-4, dtype="fp32", seed=7,
               outlier_frac=0.25, outlier_scale=3.0, zipf_s=1.1, mask="bernoulli", mask_p=0.2)
    cfg.update(kw)
    return cfg


def micro_workload(cfg, seed=None, weight_scale=0.3):
    """Like make_workload but with larger weights and non-unit gains so every
    term of every gradient is exercised at a visible magnitude."""
    rng = np.random.default_rng(cfg["seed"] if seed is None else seed)
    params = {}
    for name, shp in W.param_shapes(cfg).items():
        if len(shp) == 1:
            params[name] = 1.0 + 0.3 * rng.standard_normal(shp)
        else:
            params[name] = weight_scale * rng.standard_normal(shp)
    hidden, tokens, mask = W.make_inputs(cfg, rng)
    return dict(params=params, hidden=hidden.astype(np.float64), tokens=tokens, mask=mask)
