#!/usr/bin/env python3
"""Benchmark of the TIDE draft-training step on one MI355X.

A step = one tide_draft_train_step (forward + backward + AdamW) over one batch of synthetic captured
hidden states already resident in HBM.  Prints ONE JSON line: whole-job tokens/s, the MFMA roofline
of the dominant kernel (measured live with HIP events recorded by the library on the stream it
launches on), and the CPU oracle timed on the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # MI355X dense bf16 MFMA: 256 CU x 2.4 GHz x 4096 flop/clk/CU
PEAK_HBM_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "train_step_8b_hbm_traffic.txt")


def measured_traffic(kernel):
    """HBM bytes per launch of a GEMM instantiation at the 8B shape, from the committed rocprofv3 counter summary
    (two --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size).  The summary carries one
    line `traffic_bytes_per_launch <kernel> <bytes>` per kernel; None when the file or the kernel is missing
    (a renamed or new kernel has no counter figure until the summary is regenerated)."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                w = line.split()
                if len(w) == 3 and w[0] == "traffic_bytes_per_launch" and w[1] == kernel:
                    return float(w[2])
    except OSError:
        pass
    return None


def device_workload(cfg, device, seed):
    """Same recipe as workloads.make_workload (distributions, outlier channels, Zipf labels, prefix /
    length masks), drawn on the GPU to avoid ~1.2e9 host normals at the large shapes."""
    import torch
    from paper_2602_05145_amd import workloads as W
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    B, S = cfg["batch"], cfg["seq"]
    K, Ht, V = cfg["n_capture"], cfg["target_hidden"], cfg["vocab"]
    params = {}
    for name, shp in W.param_shapes(cfg).items():
        if len(shp) == 1:
            params[name] = torch.ones(shp, device=device, dtype=torch.float32)
        else:
            params[name] = torch.randn(shp, device=device, dtype=torch.float32, generator=g) * 0.02
    hidden = torch.randn((B, S, K * Ht), device=device, dtype=torch.float32, generator=g)
    n_out = int(round(cfg["outlier_frac"] * Ht))
    for kk in range(K):
        idx = torch.randperm(Ht, device=device, generator=g)[:n_out] + kk * Ht
        hidden[:, :, idx] *= cfg["outlier_scale"]
    perm = torch.randperm(V, device=device, generator=g)
    w = torch.arange(1, V + 1, device=device, dtype=torch.float64) ** (-cfg["zipf_s"])
    cdf = torch.cumsum(w / w.sum(), 0)
    ranks = torch.searchsorted(cdf, torch.rand((B, S), device=device, dtype=torch.float64, generator=g), right=True)
    tokens = perm[ranks.clamp_(max=V - 1)].to(torch.int32)
    kind = cfg["mask"]
    if kind == "prefix":
        mask = torch.ones((B, S), device=device, dtype=torch.uint8)
        mask[:, : int(cfg["mask_p"] * S)] = 0
    elif kind == "bernoulli":
        mask = (torch.rand((B, S), device=device, generator=g) >= cfg["mask_p"]).to(torch.uint8)
    elif kind == "lengths":
        L = torch.randint(min(cfg["len_lo"], S), min(cfg["len_hi"], S) + 1, (B,), device=device, generator=g)
        mask = (torch.arange(S, device=device)[None, :] < L[:, None]).to(torch.uint8)
        hidden[mask == 0] = 0.0
        tokens[mask == 0] = 0
    else:
        mask = torch.ones((B, S), device=device, dtype=torch.uint8)
    if cfg["dtype"] == "bf16":
        params = {k: v.to(torch.bfloat16) for k, v in params.items()}
        hidden = hidden.to(torch.bfloat16)
    return params, hidden, tokens, mask


class DeviceTrainer:
    """runtime.DraftTrainer fed from device tensors (no host round trip)."""

    def __new__(cls, cfg, params, hidden, tokens, mask):
        import torch
        from paper_2602_05145_amd import runtime
        tr = runtime.DraftTrainer.__new__(runtime.DraftTrainer)
        from paper_2602_05145_amd import binding as B
        tr.cfg, tr.device, tr.dtype = dict(cfg), hidden.device, cfg["dtype"]
        tr.ccfg = B.make_config(cfg)
        tr.params = params
        f32 = dict(dtype=torch.float32, device=hidden.device)
        tr.grads = {k: torch.zeros(v.shape, **f32) for k, v in params.items()}
        tr.m = {k: torch.zeros(v.shape, **f32) for k, v in params.items()}
        tr.v = {k: torch.zeros(v.shape, **f32) for k, v in params.items()}
        tr.master = {k: v.to(torch.float32) for k, v in params.items()} if cfg["dtype"] == "bf16" else None
        tr.ws_bytes = B.tide_draft_workspace_bytes(tr.ccfg)
        tr.workspace = torch.empty(tr.ws_bytes, dtype=torch.uint8, device=hidden.device)
        tr.loss = torch.zeros(1, **f32)
        tr.c_params, tr.c_grads = B.make_tensors(tr.params), B.make_tensors(tr.grads)
        tr.c_adam = B.TideAdamState()
        tr.c_adam.m, tr.c_adam.v, tr.c_adam.master = B.make_tensors(tr.m), B.make_tensors(tr.v), B.make_tensors(tr.master)
        tr.c_adam.step = 0
        tr.hidden, tr.tokens, tr.mask = hidden.contiguous(), tokens.contiguous(), mask.contiguous()
        return tr


def cpu_baseline(cfg, sample_batch, sample_seq):
    """The fp64 oracle's train step, as it stands, on a bounded slice of the same workload: one sequence of the
    workload's widths.  Forward + backward scale with the positions, AdamW with the parameters only, so the two
    are timed separately and the full-batch figure is given as a labelled extrapolation next to the measured one."""
    import numpy as np
    from oracle import tide_oracle as O
    from paper_2602_05145_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    sc = dict(cfg, batch=sample_batch, seq=sample_seq)
    wl = W.make_workload(sc)
    zeros = {k: np.zeros(v.shape, np.float64) for k, v in wl["params"].items()}
    t0 = time.perf_counter()
    _, cache = O.forward(sc, wl["params"], wl["hidden"], wl["tokens"], wl["mask"])
    grads = O.backward(sc, wl["params"], cache, wl["tokens"], wl["mask"])
    t1 = time.perf_counter()
    del cache
    O.adamw_step(sc, wl["params"], grads, zeros, zeros, 0, sc["lr"])
    t2 = time.perf_counter()
    n = sample_batch * sample_seq
    dt, fb, adam = t2 - t0, t1 - t0, t2 - t1
    T = cfg["batch"] * cfg["seq"]
    return {"value": n / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{cfg['name']} shape (d, F, V, heads as timed on the GPU) at batch {sample_batch} x seq {sample_seq} "
                      f"= {n} positions: fp64 NumPy forward + backward {fb:.1f} s, AdamW over all "
                      f"{W.n_params(cfg)/1e6:.0f}M parameters {adam:.1f} s",
            "forward_backward_s_per_position": fb / n, "adamw_s": adam,
            "extrapolated_full_batch_tokens_per_s": T / (fb / n * T + adam),
            "extrapolation": f"linear in positions from the sample to batch {cfg['batch']} x seq {cfg['seq']} (attention, "
                             f"quadratic in seq, is under 2 % of the work at this seq), AdamW added once"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="8b", help="tiny | small | 8b | longctx | 32b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", default="1x1024", help="batch x seq of the oracle's timed slice")
    ap.add_argument("--ingest", action="store_true",
                    help="every timed step also brings the NEXT batch's hidden states from pinned host memory to "
                         "the device through the ingest ring (copy stream), and the step after it trains on them: "
                         "the PCIe-inclusive rate.  Reported as an extra field; `value` stays the resident-input rate "
                         "measured by a default run.")
    ap.add_argument("--token-input", action="store_true",
                    help="time the token-input variant (features joined with the sampled token's embedding through "
                         "W_in) instead of the benchmarked north-star path")
    ap.add_argument("--unroll", type=int, default=0,
                    help="time the training step over the multi-step unroll (the draft fed its own output from the "
                         "second step on) with this many steps instead of the benchmarked single-step path; "
                         "combines with --token-input")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not bracket the library's launches with HIP events in the timed region (no per-kernel "
                         "figures and no roofline entry; shows what the events themselves cost)")
    ap.add_argument("--graph", action="store_true",
                    help="capture tide_draft_train_step_dev (learning rate and step count in device memory) into a HIP "
                         "graph once and time its replays: what a launch-bound configuration (small) gains from "
                         "replaying; no per-kernel figures in this mode")
    ap.add_argument("--set", action="append", default=[], metavar="KEY=INT",
                    help="override an integer field of the configuration (e.g. lm_keep_all_rows=1, lm_block_rows=8192)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); run it with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_05145_amd import binding as B, workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg = W.get_config(args.workload, **{k: int(v) for k, v in (kv.split("=", 1) for kv in args.set)})
    params, hidden, tokens, mask = device_workload(cfg, dev, cfg["seed"])
    tr = DeviceTrainer(cfg, params, hidden, tokens, mask)
    lr = cfg["lr"]
    T = cfg["batch"] * cfg["seq"]
    step = tr.train_step
    if args.token_input:
        # frozen embedding table (the target's vocabulary, draft width), the token sampled at every position, W_in
        g = torch.Generator(device=dev)
        g.manual_seed(cfg["seed"] + 7919)
        d = cfg["hidden"]
        adt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
        tr.embed = (torch.randn((cfg["vocab"], d), device=dev, generator=g) * 0.5).to(adt)
        tr.input_ids = torch.randint(0, cfg["vocab"], (cfg["batch"], cfg["seq"]), device=dev, generator=g, dtype=torch.int32)
        tr.w_in = (torch.randn((d, 2 * d), device=dev, generator=g) * 0.02).to(adt)
        f32 = dict(dtype=torch.float32, device=dev)
        tr.grad_w_in, tr.m_w_in, tr.v_w_in = (torch.zeros((d, 2 * d), **f32) for _ in range(3))
        tr.master_w_in = tr.w_in.float() if cfg["dtype"] == "bf16" else None
        tr.c_tok = B.make_token_input(tr.embed, tr.input_ids, tr.w_in, tr.grad_w_in, tr.m_w_in, tr.v_w_in, tr.master_w_in)
        step = tr.train_step_tok
    if args.unroll:
        unroll_loss = []

        def step(lr_):
            unroll_loss[:] = [tr.train_step_unroll(lr_, args.unroll, token_input=args.token_input)]

    if args.graph:
        assert not (args.token_input or args.unroll or args.ingest), "--graph times the base training step"
        lr_dev = torch.full((1,), lr, dtype=torch.float32, device=dev)
        step_dev = torch.zeros(1, dtype=torch.int64, device=dev)
        tr.train_step_dev(lr_dev, step_dev)                      # one-time function attributes, outside the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                tr.train_step_dev(lr_dev, step_dev)
        torch.cuda.current_stream().wait_stream(side)
        args.no_kernel_events = True

        def step(lr_):
            graph.replay()

    for _ in range(args.warmup):
        step(lr)
    torch.cuda.synchronize()

    # timed region: exactly K steps; the library brackets each of its launches with HIP events on the
    # stream it launches on, which gives the live per-kernel durations for the roofline entry
    ring = None
    if args.ingest:
        import ctypes
        nbytes = tr.hidden.numel() * tr.hidden.element_size()
        rc, ring = B.tide_ingest_create(nbytes, 2)
        assert rc == 0, B.tide_ingest_last_error()
        bufs = [tr.hidden, torch.empty_like(tr.hidden)]          # device double buffer
        host_batch = tr.hidden.cpu()                              # the producer's copy of a batch (pageable)
        src_addr, cur = host_batch.data_ptr(), 0
        for _ in range(2):                                        # first touch of every pinned slot, untimed
            rc, slot, addr = B.tide_ingest_acquire(ring)
            assert rc == 0, B.tide_ingest_last_error()
            ctypes.memmove(addr, src_addr, nbytes)
            assert B.tide_ingest_submit(ring, slot, bufs[1], nbytes) == 0
        torch.cuda.synchronize()

    if not args.no_kernel_events:
        B.tide_profile_start()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        if ring is not None:
            # producer: fill a pinned slot, start its copy into the idle device buffer; the copy runs while
            # this step trains on the other buffer
            while True:
                rc, slot, addr = B.tide_ingest_acquire(ring)
                if rc != B.TIDE_INGEST_ERR_BUSY:
                    break
                time.sleep(2e-4)    # back-pressure: every pinned slot still waits for its copy (the host runs ahead of the GPU)
            assert rc == 0, B.tide_ingest_last_error()
            ctypes.memmove(addr, src_addr, nbytes)
            # (the idle buffer was read by the step before this one, which may still be running: the copy is
            # ordered after everything enqueued on the compute stream so far)
            assert B.tide_ingest_submit(ring, slot, bufs[cur ^ 1], nbytes, tr._stream(), True) == 0
        step(lr)
        if ring is not None:
            # the next step reads the freshly copied buffer: order it after the copy on the compute stream
            assert B.tide_ingest_wait(ring, slot, tr._stream()) == 0
            cur ^= 1
            tr.hidden = bufs[cur]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prof = B.tide_profile_stop() if not args.no_kernel_events else []
    if args.no_kernel_events:
        print(json.dumps({"ms_per_step": wall * 1e3 / args.steps, "steps": args.steps, "kernel_events": False,
                          "workload": cfg["name"], "graph_replay": bool(args.graph),
                          "tokens_per_s": T / (wall / args.steps)}))
        return
    if ring is not None:
        B.tide_ingest_destroy(ring)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    loss = float(tr.loss.item()) if not args.unroll else float(unroll_loss[0][0].item())
    assert loss == loss and loss > 0, f"bad loss {loss}"

    # what the matrix pipes sustain on this machine with nothing else going on (registers only): the practical ceiling
    sink = torch.empty(2048 * 512, dtype=torch.float32, device=dev)
    for _ in range(30):                                   # a quarter of a second of it first: the power limit takes that long to settle
        B.tide_mfma_probe(2048, 4000, sink, tr._stream())
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    probe_flops = sum(B.tide_mfma_probe(2048, 4000, sink, tr._stream()) for _ in range(10))
    e1.record()
    torch.cuda.synchronize()
    mfma_probe_tflops = probe_flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    del sink

    ms = wall * 1e3 / args.steps
    # FLOPs.  "all positions" is the algorithmic count of the whole step (2 flop/MAC, causal attention at
    # S(S+1)/2, no projection input gradient, no logits recompute).  A position that carries no loss
    # matters only through its key and value, so the library runs everything after the attention (output
    # projection, MLP, LM head: forward and backward) on the loss positions alone; the "executed" count
    # removes those products, 6 flop per weight, for every other position.  MFU is quoted on the executed count.
    flops_all = W.flops_per_step(cfg)
    n_loss = int(((tr.mask != 0) & (tr.tokens >= 0) & (tr.tokens < cfg["vocab"])).sum().item())
    ps = {k: int(np.prod(v)) for k, v in W.param_shapes(cfg).items()}
    after_attention = ps["w_o"] + ps["w_gate"] + ps["w_up"] + ps["w_down"] + ps["w_lm"]
    flops = flops_all - 6.0 * after_attention * (T - n_loss)
    if args.token_input:
        extra = 6.0 * 2 * cfg["hidden"] * cfg["hidden"] * T   # W_in [d, 2d]: forward, dW_in (both halves) and dg, on every position
        flops_all += extra
        flops += extra
    unroll_info = None
    if args.unroll:
        # step s >= 2 has no W_fc product, runs the layer up to the attention on every row and everything after
        # it on the rows that carry loss at step s or later (their count comes from the shifted masks)
        keep = ((tr.mask != 0) & (tr.tokens >= 0) & (tr.tokens < cfg["vocab"])).view(cfg["batch"], cfg["seq"])
        shifted = [torch.nn.functional.pad(keep[:, j:], (0, j)) for j in range(args.unroll)]
        rows = [int(torch.stack(shifted[j:]).any(dim=0).sum().item()) for j in range(args.unroll)]
        per_step_all = flops_all - (6.0 * 2 * cfg["hidden"] * cfg["hidden"] * T if args.token_input else 0.0)
        fc = 4.0 * ps["w_fc"] * T
        in_proj = 6.0 * 2 * cfg["hidden"] * cfg["hidden"] * T if args.token_input else 0.0
        flops = sum(per_step_all - (fc if j else 0.0) + in_proj - 6.0 * after_attention * (T - rows[j]) for j in range(args.unroll))
        flops_all = args.unroll * (per_step_all + in_proj) - (args.unroll - 1) * fc
        unroll_info = {"steps": args.unroll, "rows_after_attention_per_step": rows,
                       "loss_per_step": [float(x) for x in unroll_loss[0].cpu()],
                       "workspace_GiB": B.tide_draft_unroll_workspace_bytes(tr.ccfg, args.unroll) / 2**30}
    prof.sort(key=lambda r: -r["total_ms"])
    kernel_ms = sum(r["total_ms"] for r in prof)
    dom = max((r for r in prof if r["kernel"].startswith("gemm_mfma")), key=lambda r: r["total_ms"], default=None)
    if dom is None:
        dom = next(r for r in prof if r["flops"] > 0)
    dom_tflops = dom["flops"] / (dom["total_ms"] * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": dom["kernel"], "achieved": dom_tflops, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": dom_tflops / PEAK_BF16_TFLOPS,
                "traffic": (measured_traffic(dom["kernel"])
                            if cfg["name"] == "8b" and not args.unroll and not args.token_input else None),
                "launches_per_step": dom["launches"] / args.steps,
                "avg_launch_ms": dom["total_ms"] / dom["launches"],
                "flops_per_launch": dom["flops"] / dom["launches"],
                "measured_mfma_peak": mfma_probe_tflops, "frac_of_measured_mfma_peak": dom_tflops / mfma_probe_tflops}
    out = {
        "metric": "draft-training tokens/sec (fwd+bwd+AdamW) and % bf16 MFMA peak, 1 MI355X",
        "value": T / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "inputs": ("pinned host -> device through the ingest ring, overlapped with the step"
                                      if args.ingest else "resident in HBM"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": (f"{args.unroll}-step unroll, " if args.unroll else "") + ("token-input variant, " if args.token_input else "") + f"{cfg['name']}: batch {cfg['batch']} x seq {cfg['seq']}, 3x{cfg['target_hidden']} captured "
                               f"states -> d {cfg['hidden']}, {cfg['n_heads']}/{cfg['n_kv_heads']} heads x {cfg['head_dim']}, "
                               f"FFN {cfg['ffn']}, vocab {cfg['vocab']}", "global_batch": cfg["batch"], "seq_len": cfg["seq"],
                   "params_M": W.n_params(cfg) / 1e6, "loss_positions": n_loss, "positions": T},
        "tflops_per_step_executed": flops / 1e12, "tflops_per_step_all_positions": flops_all / 1e12,
        "loss_positions_per_s": n_loss / (ms * 1e-3),
        "achieved_tflops": flops / (ms * 1e-3) / 1e12,
        "mfu_vs_bf16_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "mfu_vs_bf16_peak_all_positions": flops_all / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "loss_last_step": loss,
        "roofline": roofline,
        "kernels": [{"kernel": r["kernel"], "ms_per_step": r["total_ms"] / args.steps,
                     "launches_per_step": r["launches"] / args.steps,
                     "tflops": (r["flops"] / (r["total_ms"] * 1e-3) / 1e12) if r["flops"] > 0 and r["total_ms"] > 0 else None,
                     "gbs": (r["bytes"] / (r["total_ms"] * 1e-3) / 1e9) if r["bytes"] > 0 and r["total_ms"] > 0 else None}
                    for r in prof],
        "kernel_ms_per_step": kernel_ms / args.steps,
    }
    if unroll_info:
        out["unroll"] = unroll_info
    if not args.no_cpu_baseline and not args.unroll:
        del tr
        torch.cuda.empty_cache()
        sb, ss = (int(x) for x in args.cpu_sample.lower().split("x"))
        out["cpu_baseline"] = cpu_baseline(cfg, sb, min(ss, cfg["seq"]))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
