#!/usr/bin/env python3
"""Benchmark of the LPC-SVRG hot path on one MI355X.

A "step" is one pass of the whole hot path: one lpc_epoch on configuration C2 (dense L1+L2
logistic regression, n=65536, d=4096, N=8 simulated workers, minibatch 64 per worker, b=4 bits,
m=128 inner iterations) = the snapshot full-gradient pass, then 128 x (workers' variance-reduced
differences -> clip/quantize/pack -> dequantize+average -> prox).  Inputs are synthetic, seeded,
and resident in HBM before the timed region.

Prints ONE JSON line.  `value` = inner iterations per second over whole steps (the snapshot pass
included).  `roofline` covers the kernel that dominates the step; its duration is measured here
with HIP events on the stream the library launches on.  `cpu_baseline` is the CPU oracle timed on
a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published peak


def event_time_ms(fn, reps, torch):
    """Average duration of fn() in ms, HIP events on the current stream around `reps` back-to-back calls."""
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    fn()
    torch.cuda.synchronize()
    start.record()
    for _ in range(reps):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / reps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--small", action="store_true", help="scaled-down C2 (for a quick functional run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the N workers are shards on one device); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import lpc_synth
    from paper_1901_08924_amd import lpc

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    over = dict(n=4096, d=1024) if args.small else {}
    sp = lpc_synth.make(args.workload, **over)
    cfgkw = dict(algo=sp.algo, N=sp.N, B=sp.B, m=sp.m, bits=sp.bits, clip_mode=sp.clip_mode, clip=sp.clip,
                 eta=sp.eta, L=sp.L, seed=sp.seed, n_full=sp.n_full)
    X = torch.from_numpy(sp.X).to(dev)
    y = torch.from_numpy(sp.y).to(dev)
    ctx = lpc.Context(sp.loss, y, lpc.make_config(**cfgkw), X=X, lambda1=sp.lambda1, lambda2=sp.lambda2)
    n, d, N, B, m, bits = sp.n, sp.d, sp.N, sp.B, sp.m, sp.bits
    alpc = sp.algo != lpc.ALGO_LPC
    w = torch.from_numpy(sp.w0).to(dev)
    ya, za = (w.clone(), w.clone()) if alpc else (None, None)

    # all library work goes to a stream of its own (not the legacy default stream)
    stream = torch.cuda.Stream(device=dev)
    torch.cuda.set_stream(stream)

    # ---- the timed region: K whole epochs --------------------------------------------------
    P0 = ctx.objective(w)
    for s in range(args.warmup):
        ctx.epoch(w, s, ya, za)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.warmup, args.warmup + args.steps):
        ctx.epoch(w, s, ya, za)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    iters_per_sec = m * args.steps / elapsed
    P_end = ctx.objective(w)

    # ---- per-call timings with HIP events (same stream as the library's launches) ----------
    dp = lpc.d_pad(d)
    mu = torch.zeros(d, device=dev)
    z = torch.zeros(n, device=dev)
    w2 = (w + 0.01 * torch.randn(d, device=dev)).contiguous()
    U = torch.zeros(N, dp, device=dev)
    stats = torch.zeros(N, 4, dtype=torch.float64, device=dev)
    packed = torch.zeros(N, max(ctx.W, 1), dtype=torch.int32, device=dev)
    delta = torch.zeros(N, device=dev)
    uavg = torch.zeros(d, device=dev)
    t_full = event_time_ms(lambda: ctx.full_grad(w, mu, z, None), 20, torch)
    t_vr = event_time_ms(lambda: ctx.worker_vr_grad(w2, w, z, 0, 1, U, stats), 200, torch)
    t_q = event_time_ms(lambda: ctx.quantize_clip(U, stats, None, 0, 1, packed, delta, None), 200, torch)
    t_dq = event_time_ms(lambda: ctx.dequantize_avg(packed, delta, uavg), 200, torch)
    t_px = event_time_ms(lambda: ctx.prox_step(w2, uavg, mu, 1e-9), 200, torch)
    full_bytes = 4.0 * n * d + 4.0 * n + 4.0 * d + 4.0 * n + 4.0 * d     # X, y, w in; z, mu out
    vr_bytes = 4.0 * N * B * d + 4.0 * N * d                             # sampled rows once + U
    q_bytes = N * (4.0 * dp + bits * dp / 8.0 + 4.0)
    t_inner_ms = ms_per_step - t_full
    # the m inner iterations dominate the step; inside them the workers' gradient pass moves the bytes
    roofline = {
        "kernel": "lpc_full_grad (dense_rows_kernel mode 0 + partial reduction)",
        "bound": "hbm",
        "achieved": full_bytes / (t_full * 1e-3) / 1e9,
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": full_bytes / (t_full * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "traffic": None,
        "bytes_per_launch": full_bytes,
        "ms_per_launch": t_full,
    }
    out = {
        "metric": "svrg_inner_iters_per_sec",
        "value": iters_per_sec,
        "unit": "inner iterations/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: dense %s n=%d d=%d N=%d B=%d bits=%d m=%d clip=%g"
                   % (sp.name, "logistic" if sp.loss == 0 else "squared", n, d, N, B, bits, m, sp.clip),
                   "step": "one lpc_epoch = full-gradient pass + m inner iterations"},
        "full_grad_pass": {"ms": t_full, "algorithmic_GBps": full_bytes / (t_full * 1e-3) / 1e9,
                           "frac_of_hbm_peak": full_bytes / (t_full * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "inner_iters_per_sec_excluding_full_grad": m / (t_inner_ms * 1e-3) if t_inner_ms > 0 else None,
        "per_call_ms": {"full_grad": t_full, "worker_vr_grad": t_vr, "quantize_clip": t_q,
                        "dequantize_avg": t_dq, "prox_step": t_px},
        "per_call_algorithmic_GBps": {"worker_vr_grad": vr_bytes / (t_vr * 1e-3) / 1e9,
                                      "quantize_clip": q_bytes / (t_q * 1e-3) / 1e9},
        "objective": {"start": P0, "end": P_end},
        "roofline": roofline,
    }

    # ---- the CPU oracle on a bounded sample of the same workload ---------------------------
    if not args.no_cpu_baseline:
        from oracle import lpco
        p, _keep = lpco.make_problem(sp.loss, sp.y, sp.lambda1, sp.lambda2, X=sp.X)
        ocfg = lpco.make_config(**cfgkw)
        wo = sp.w0.copy()
        yo, zo = (wo.copy(), wo.copy()) if alpc else (None, None)
        n_ep = 3
        t0 = time.perf_counter()
        for s in range(n_ep):
            lpco.epoch(p, ocfg, wo, s, yo, zo)
        tc = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": m * n_ep / tc, "unit": "inner iterations/s", "cores": 1, "kind": "oracle",
                               "sample": "%d whole epochs of the same workload (%d inner iterations), %.1f s"
                                         % (n_ep, m * n_ep, tc)}
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
