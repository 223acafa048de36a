#!/usr/bin/env python3
"""Benchmark of the LPC-SVRG hot path on one MI355X.

A "step" is one pass of the whole hot path: one lpc_epoch on configuration C2 (dense L1+L2
logistic regression, n=65536, d=4096, N=8 simulated workers, minibatch 64 per worker, b=4 bits,
m=128 inner iterations) = the snapshot full-gradient pass, then 128 x (workers' variance-reduced
differences -> clip/quantize/pack -> dequantize+average -> prox).  Inputs are synthetic, seeded,
and resident in HBM before the timed region.

Prints ONE JSON line.  `value` = inner iterations per second over whole steps (the snapshot pass
included).  After the timed region the same steps are run once more with the library's event
profiling on (HIP events on the launch stream around each kernel class); `kernels` lists every
class, `roofline` is the class with the largest share of the step.  `cpu_baseline` is the CPU oracle
timed on a bounded sample of the same workload.
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

KERNEL_NAMES = {
    "full_rows": "dense_rows_kernel<mode 0> (lpc_full_grad: z = Xw and X'l' in one read of X)",
    "full_fold": "reduce_parts_kernel x2 (fold of the snapshot pass's partial gradients)",
    "vr_rows": "dense_rows_kernel<mode 1> (lpc_worker_vr_grad, all N workers in one launch)",
    "vr_fold": "reduce_parts_kernel (fold of the workers' partials + statistics)",
    "exchange": "fused_exchange_kernel (eq. 3 + quantize + pack + eq. 4 + prox)",
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--small", action="store_true", help="scaled-down problem (quick functional run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the N workers are shards on one device); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

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
    dp = lpc.d_pad(d)
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

    # ---- the same steps again with HIP events around every kernel class ---------------------
    ctx.profile_enable(True)
    s0 = args.warmup + args.steps
    for s in range(s0, s0 + args.steps):
        ctx.epoch(w, s, ya, za)
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    # algorithmic bytes one launch of each class must move
    algo_bytes = {
        "full_rows": 4.0 * sp.n * d + 4.0 * n + 4.0 * d + 4.0 * n + 4.0 * d,   # X, y, w in; z, mu out
        "vr_rows": 4.0 * N * B * d + 4.0 * N * d,                              # each sampled row once; U out
        "exchange": N * (4.0 * dp + bits * dp / 8.0 + 4.0) + 12.0 * d + 4.0 * d,
    }
    kernels = {}
    for k, (ms, cnt) in prof.items():
        if cnt == 0:
            continue
        avg_ms = ms / cnt
        ent = {"name": KERNEL_NAMES[k], "launches_per_step": cnt / args.steps, "avg_us": 1e3 * avg_ms,
               "share_of_step": (ms / args.steps) / ms_per_step}
        if k in algo_bytes:
            gbps = algo_bytes[k] / (avg_ms * 1e-3) / 1e9
            ent.update({"algorithmic_bytes": algo_bytes[k], "GBps": gbps, "frac_of_hbm_peak": gbps / HBM_PEAK_GBPS})
        kernels[k] = ent
    rated = [k for k in kernels if "GBps" in kernels[k]]
    dom = max(rated, key=lambda k: kernels[k]["share_of_step"])
    roofline = {"kernel": kernels[dom]["name"], "bound": "hbm", "achieved": kernels[dom]["GBps"],
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": kernels[dom]["frac_of_hbm_peak"], "traffic": None,
                "bytes_per_launch": kernels[dom]["algorithmic_bytes"], "us_per_launch": kernels[dom]["avg_us"],
                "note": "a launch moves only 4*N*B*d bytes, so it is bound by launch and dependency latency, "
                        "not by HBM; the HBM-bound kernel of the step is full_rows (see kernels)"
                        if dom == "vr_rows" else ""}
    t_full_ms = (prof["full_rows"][0] + prof["full_fold"][0]) / max(1, prof["full_rows"][1])
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
        "full_grad_pass": {"ms": t_full_ms, "algorithmic_GBps": algo_bytes["full_rows"] / (t_full_ms * 1e-3) / 1e9,
                           "frac_of_hbm_peak": algo_bytes["full_rows"] / (t_full_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                           "note": "rows kernel + fold kernels"},
        "inner_iters_per_sec_excluding_full_grad": m / ((ms_per_step - t_full_ms) * 1e-3),
        "objective": {"start": P0, "end": P_end},
        "kernels": kernels,
        "roofline": roofline,
    }

    # ---- the CPU oracle on a bounded sample of the same workload ---------------------------
    if not args.no_cpu_baseline:
        from oracle import lpco
        p, _keep = lpco.make_problem(sp.loss, sp.y, sp.lambda1, sp.lambda2, X=sp.X)
        ocfg = lpco.make_config(**cfgkw)
        wo = sp.w0.copy()
        yo, zo = (wo.copy(), wo.copy()) if alpc else (None, None)
        n_ep = 16
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
