#!/usr/bin/env python3
"""Benchmark of the LPC-SVRG / ALPC-SVRG hot path on one MI355X.

A "step" is one pass of the whole hot path: one lpc_epoch = the snapshot full-gradient pass, then
m inner iterations of (workers' variance-reduced differences -> clip/quantize/pack ->
dequantize+average -> prox [+ ALPC double sampling]).  With no --workload the headline is configuration
C4, the largest that one GPU holds (ALPC-SVRG on dense ridge least squares, n=262144, d=8192, 8.6 GB, N=16
workers, minibatch 64 per worker, b=3 bits, m=256), and the other single-GPU configurations C2 (dense
logistic, 1 GiB), C3 (CSR logistic, n=d=2^20) and C5 (3-layer MLP, 4.2 M parameters) follow as sub-records
under "workloads", each with its own roofline, snapshot-pass figure and CPU baseline.  --workload cN runs one
configuration alone.  Inputs are synthetic, seeded, and resident in HBM before the timed region.

Prints ONE JSON line.  `value` = inner iterations per second over whole steps (the snapshot pass
included).  After the timed region the same steps are run once more with the library's per-class timing on;
`kernels` lists every class with its algorithmic bytes (or flops) per launch, `roofline` is the class that
carries most of the step's algorithmic work (launches per step x work per launch, weighed by its own peak).
A class that is one kernel is timed by that dispatch's own begin and end (the figure a rocprofv3 kernel trace
gives).  `cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, published peak
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix peak

KERNEL_NAMES = {
    "full_rows": "snapshot pass (lpc_full_grad): rows kernel(s)",
    "full_fold": "snapshot pass: fold of the partial gradient rows",
    "vr_rows": "worker pass (lpc_worker_vr_grad): all workers' sampled rows",
    "vr_fold": "worker pass: fold / statistics of U",
    "exchange": "exchange: eq. (3) + quantize + pack + eq. (4) + prox",
    "resident": "inner loop of an epoch as one resident launch (m iterations: rows, fold, exchange, update)",
}


def algorithmic_work(sp, dp, nnz):
    """Per launch of each kernel class: (amount, 'bytes' | 'flops'), as counted from what the method must move."""
    n, d, N, B, bits = sp.n, sp.d, sp.N, sp.B, sp.bits
    n_full = sp.n_full or n
    msg = N * (4.0 * dp + (bits * dp / 8.0 if bits < 32 else 0.0) + 4.0) + 16.0 * d
    if sp.loss == 2:      # MLP: contractions on the matrix cores
        dims = sp.mlp_dims
        mac = sum(dims[l] * dims[l + 1] for l in range(len(dims) - 1))
        fwd_bwd_w = 2.0 * mac * 3            # forward, weight gradient, data gradient (first layer has none)
        bwd_first = 2.0 * dims[0] * dims[1]
        rows = N * B
        vr = rows * (2 * (fwd_bwd_w - bwd_first)) - rows * 2.0 * dims[0] * dims[1]   # layer-1 weight grad once
        return {"full_rows": (n_full * (fwd_bwd_w - bwd_first), "flops"), "vr_rows": (vr, "flops"),
                "exchange": (msg, "bytes")}
    if sp.csr is not None:
        full = (8.0 * nnz * n_full / n + 4.0 * (n_full + 1) + 8.0 * n_full + 8.0 * d, "bytes")
        entries = float(N) * B * nnz / n
        sparse = (bits < 32 and sp.algo == 0 and getattr(sp, "scheme", 0) == 0 and d >= 4 * 8192
                  and 8.0 * B * nnz / n <= d)
        if sparse:
            # u^i stays sparse: the pairs of the sampled rows in, one contribution per entry out; the exchange
            # must still read every worker's packed message and update all d coordinates (w, mu in; w out)
            return {"full_rows": full, "vr_rows": (12.0 * entries, "bytes"),
                    "exchange": (N * bits * dp / 8.0 + 16.0 * d, "bytes")}
        return {"full_rows": full,
                "vr_rows": (8.0 * entries + 8.0 * N * dp, "bytes"),     # rows + zero and write U
                "exchange": (msg, "bytes")}
    nvec = N + (1 if sp.algo != 0 else 0)   # Alg. 2, 3 also draw the shared batch J
    return {"full_rows": (4.0 * n_full * d + 8.0 * n_full + 8.0 * d, "bytes"),  # X, y, w in; z, mu out
            "vr_rows": (4.0 * nvec * B * d + 4.0 * nvec * d, "bytes"),         # each sampled row once; U out
            "exchange": (msg, "bytes"),
            # one launch = m iterations; on the chip U never reaches HBM: the sampled rows in, the messages out
            "resident": (sp.m * (4.0 * nvec * B * d + 8.0 * nvec * B + N * (bits * dp / 8.0 + 4.0)), "bytes")}


# Vector-unit bound of the dense quantizer (Sec. 3.2 rules (1), (2) with one Philox4x32-10 block per four coordinates).
# Instruction mix of the word-per-thread kernel, per coordinate (b = 4): 4.5 64-bit integer products (v_mad_u64_u32:
# 18 per generator block), 4.5 three-input exclusive-ors (v_bitop3_b32) and 13.25 other vector instructions (0.75
# two-input xor of the generator's first rounds, 10 of the rounding rule, the rest packing and addresses).  Rates measured on
# this chip with saturating kernels of independent instructions (8 wavefronts per SIMD): 33 T lane-instructions/s for
# the 64-bit product with a zero addend, 60 T/s for 32-bit add / xor / fma with vector-register operands (37 T/s when
# an operand is a scalar register).  A register-only loop of one generator block plus the rounding rule of four
# coordinates runs at 1.98 T coordinates/s (317 cycles per wavefront and block at 2.4 GHz), the generator alone at
# 3.2 T/s: the second figure of the record (`alu_loop_us`).
QUANT_MAD64_PER_COORD, QUANT_VALU_PER_COORD = 4.5, 17.75
MAD64_RATE, VALU_RATE = 33.0e12, 60.0e12
QUANT_LOOP_COORDS_PER_S = 1.98e12


def quantizer_rooflines(ctx, sp):
    """lpc_vector_stats, lpc_quantize_clip and lpc_dequantize_avg each timed alone on N Gaussian vectors of the
    workload's length (HIP events around 10 launches): rate against the HBM bound and, for the quantizer, against the
    vector-unit bound derived above; `frac` is against the tighter of the two."""
    import torch
    from paper_1901_08924_amd import lpc
    dev = torch.device("cuda:0")
    N, d, bits = sp.N, sp.d, sp.bits
    dp = lpc.d_pad(d)
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    U = torch.randn(N, dp, device=dev, generator=g)
    U[:, d:] = 0
    stats = torch.zeros(N, 4, dtype=torch.float64, device=dev)
    packed = torch.zeros(N, ctx.W, dtype=torch.int32, device=dev)
    delta = torch.zeros(N, dtype=torch.float32, device=dev)
    u_avg = torch.zeros(d, dtype=torch.float32, device=dev)

    def timed(fn, reps=10):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps   # us per call

    out = {}
    coords = float(N) * dp
    us = timed(lambda: ctx.vector_stats(U, N, stats))
    out["vector_stats"] = {"us": us, "algorithmic_bytes": 4.0 * coords, "hbm_bound_us": 4.0 * coords / (HBM_PEAK_GBPS * 1e3),
                           "frac": 4.0 * coords / (HBM_PEAK_GBPS * 1e3) / us,
                           "note": "two launches (partials, fold); events around both"}
    us = timed(lambda: ctx.quantize_clip(U, stats, None, 0, 1, packed, delta, None))
    qbytes = coords * (4.0 + bits / 8.0)
    hbm_us = qbytes / (HBM_PEAK_GBPS * 1e3)
    alu_us = coords * (QUANT_MAD64_PER_COORD / MAD64_RATE + QUANT_VALU_PER_COORD / VALU_RATE) * 1e6
    out["quantize_pack"] = {"us": us, "algorithmic_bytes": qbytes, "hbm_bound_us": hbm_us, "alu_bound_us": alu_us,
                            "alu_loop_us": coords / QUANT_LOOP_COORDS_PER_S * 1e6,
                            "frac_of_hbm_bound": hbm_us / us, "frac_of_alu_bound": alu_us / us,
                            "frac": max(hbm_us, alu_us) / us, "coordinates_per_s": coords / (us * 1e-6),
                            "note": "parameter launch + quantizer (the epoch's instantiation: no clip counts, unconditional draws)"}
    us = timed(lambda: ctx.dequantize_avg(packed, delta, u_avg))
    rbytes = N * bits * dp / 8.0 + 4.0 * d
    out["dequantize_avg"] = {"us": us, "algorithmic_bytes": rbytes, "hbm_bound_us": rbytes / (HBM_PEAK_GBPS * 1e3),
                             "frac": rbytes / (HBM_PEAK_GBPS * 1e3) / us}
    del U, packed, u_avg
    torch.cuda.empty_cache()
    return out


def measured_traffic(workload):
    """HBM bytes per launch and kernel class from the stored rocprofv3 counter summary of this workload
    (FETCH_SIZE / WRITE_SIZE runs scaled by a copy kernel), or {} when no summary is kept for it."""
    path = os.path.join(ROOT, "profiles", "%s_hbm_traffic.md" % workload)
    out = {}
    if os.path.exists(path):
        for line in open(path):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) == 8 and cells[0] in KERNEL_NAMES:
                out[cells[0]] = float(cells[6])
    return out


def host_cores():
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def cpu_baseline(sp, cfgkw, alpc):
    """The oracle as it stands on a bounded sample of the workload: whole epochs on one host thread (its inner
    loop has no threaded form), and for the linear models the snapshot pass once more on all host cores."""
    from oracle import lpco
    sample = dict(cfgkw)
    scale, note = 1.0, ""
    if sp.name == "c5":       # one inner iteration of the full size is ~1 minute of plain loops: shrink the batch
        sample.update(N=2, B=16, m=1, n_full=32)
        scale = (sample["N"] * sample["B"]) / float(sp.N * sp.B)
        note = " with N=2, B=16, snapshot over 32 rows; rate scaled by sampled rows per iteration"
        epochs = 1
    elif sp.name == "c3":
        sample.update(m=32)
        epochs = 1
    elif sp.name == "c4":
        epochs = 1
    else:
        epochs = 16 if sp.name == "c2" else 200
    if sp.csr is not None:
        p, _keep = lpco.make_problem(sp.loss, sp.y, sp.lambda1, sp.lambda2, csr=(*sp.csr, sp.d))
    else:
        p, _keep = lpco.make_problem(sp.loss, sp.y, sp.lambda1, sp.lambda2, X=sp.X, d=sp.d, mlp_dims=sp.mlp_dims)
    ocfg = lpco.make_config(**sample)
    wo = sp.w0.copy()
    yo, zo = (wo.copy(), wo.copy()) if alpc else (None, None)
    t0 = time.perf_counter()
    for s in range(epochs):
        lpco.epoch(p, ocfg, wo, s, yo, zo)
    tc = time.perf_counter() - t0
    iters = sample["m"] * epochs
    cores = host_cores()
    out = {"value": iters / tc * scale, "unit": "inner iterations/s", "cores": 1, "host_cores": cores,
           "kind": "oracle",
           "sample": "%d epoch(s) of %d inner iterations (snapshot pass included)%s: %.1f s"
                     % (epochs, sample["m"], note, tc)}
    if sp.loss != 2:          # the oracle's snapshot pass has a row-parallel form: time it on one and on all cores
        n_full = sp.n_full or sp.n
        t0 = time.perf_counter()
        lpco.full_grad(p, sp.w0)
        t1 = time.perf_counter() - t0
        lpco.set_threads(cores)
        t0 = time.perf_counter()
        lpco.full_grad(p, sp.w0)
        ta = time.perf_counter() - t0
        lpco.set_threads(1)
        out["full_grad_pass"] = {"seconds_one_core": t1, "seconds_all_cores": ta, "cores": cores, "rows": n_full}
    return out


def contraction_shapes():
    """The products of C5's layers (2048 rows per worker pass, 16 workers, snapshot chunks of 2048 rows) and a
    4096^3 reference, each timed alone with HIP events: M, N, K, transposed operands, time, TFLOP/s."""
    import torch
    from paper_1901_08924_amd import lpc
    fn = lpc.lib.lpc_debug_gemm
    st = torch.cuda.Stream()
    torch.cuda.set_stream(st)
    shapes = [("forward layer 1", 2048, 1024, 3072, 0, 0), ("forward layer 2", 2048, 1024, 1024, 0, 0),
              ("forward layer 3", 2048, 10, 1024, 0, 0), ("data gradient layer 2", 2048, 1024, 1024, 0, 1),
              ("data gradient layer 3", 2048, 1024, 10, 0, 1),
              ("weight gradient layer 1, 2048 rows", 3072, 1024, 2048, 1, 0),
              ("weight gradient layer 2, 2048 rows", 1024, 1024, 2048, 1, 0),
              ("weight gradient layer 3, 2048 rows", 1024, 10, 2048, 1, 0),
              ("weight gradient layer 1, one worker", 3072, 1024, 256, 1, 0),
              ("weight gradient layer 2, one worker", 1024, 1024, 256, 1, 0),
              ("reference", 4096, 4096, 4096, 0, 0)]
    for name, M, N, K, tA, tB in shapes:
        A = torch.randn((K, M) if tA else (M, K), device="cuda:0")
        B = torch.randn((N, K) if tB else (K, N), device="cuda:0")
        Cm = torch.zeros(M, N, device="cuda:0")
        lda, ldb = (M if tA else K), (K if tB else N)

        def run():
            rc = fn(A.data_ptr(), B.data_ptr(), Cm.data_ptr(), M, N, K, lda, ldb, N, tA, tB, 1.0, None, 0, 0,
                    st.cuda_stream)
            assert rc == 0
        for _ in range(3):
            run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            run()
        e1.record()
        e1.synchronize()
        us = e0.elapsed_time(e1) / 20 * 1e3
        print(json.dumps({"product": name, "M": M, "N": N, "K": K, "transA": tA, "transB": tB, "us": round(us, 1),
                          "tflops": round(2.0 * M * N * K / us * 1e-6, 1)}), flush=True)


def copy_calibration():
    """What this machine's HBM delivers to a kernel with no arithmetic: 1 GiB device-to-device copies."""
    import torch
    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(9):  # ten copies in all, the first untimed
        dst.copy_(src)
    t1.record()
    torch.cuda.synchronize()
    us = t0.elapsed_time(t1) * 1000.0 / 9.0  # per copy
    out = {"bytes_read": 4 * src.numel(), "bytes_written": 4 * src.numel(), "launches": 10,
           "us_per_copy": round(us, 1), "achieved_GBps": round(8 * src.numel() / us * 1e-3, 1)}
    del src, dst
    torch.cuda.empty_cache()
    return out


DEFAULT_STEPS = {"c1": (50, 3), "c2": (20, 3), "c3": (3, 1), "c4": (5, 1), "c5": (3, 1)}
SMALL = {"c1": {}, "c2": dict(n=4096, d=1024), "c3": dict(n=1 << 14, d=1 << 14), "c4": dict(n=4096, d=1024),
         "c5": dict(n=2048, dims=(256, 128, 128, 10), n_full=512, m=4)}


def run_workload(name, steps, warmup, args, achievable):
    """K timed epochs of one configuration, then the same epochs with per-class timing; returns its record."""
    import torch
    import lpc_synth
    from paper_1901_08924_amd import lpc

    dev = torch.device("cuda:0")
    sp = lpc_synth.make(name, **(SMALL[name] if args.small else {}))
    cfgkw = dict(algo=sp.algo, N=sp.N, B=sp.B, m=sp.m, bits=sp.bits, clip_mode=sp.clip_mode, clip=sp.clip,
                 eta=sp.eta, L=sp.L, seed=sp.seed, n_full=sp.n_full)
    ctx = lpc.context_from_problem(sp)
    for key, val in ((lpc.TUNE_ITER_FORM, args.iter_form), (lpc.TUNE_ITER_TILE, args.iter_tile),
                     (lpc.TUNE_ITER_THREADS, args.iter_threads)):
        if val is not None and sp.loss != 2 and sp.csr is None:
            ctx.tune(key, val)
    n, d, N, B, m, bits = sp.n, sp.d, sp.N, sp.B, sp.m, sp.bits
    dp = lpc.d_pad(d)
    nnz = int(sp.csr[2].size) if sp.csr is not None else 0
    alpc = sp.algo != lpc.ALGO_LPC
    w = torch.from_numpy(sp.w0).to(dev)
    ya, za = (w.clone(), w.clone()) if alpc else (None, None)

    # ---- the timed region: K whole epochs --------------------------------------------------
    P0 = ctx.objective(w)
    for s in range(warmup):
        ctx.epoch(w, s, ya, za)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(warmup, warmup + steps):
        ctx.epoch(w, s, ya, za)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / steps
    iters_per_sec = m * steps / elapsed
    P_end = ctx.objective(w)
    assert ctx.take_device_flags() == 0

    # ---- the same steps again with HIP events on every kernel class ------------------------
    ctx.profile_enable(True)
    s0 = warmup + steps
    psteps = min(steps, 5)
    for s in range(s0, s0 + psteps):
        ctx.epoch(w, s, ya, za)
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    work = algorithmic_work(sp, dp, nnz)
    kernels = {}
    for k, (ms, cnt, exact) in prof.items():
        if cnt == 0:
            continue
        avg_ms = ms / cnt
        ent = {"name": KERNEL_NAMES[k], "launches_per_step": cnt / psteps, "avg_us": 1e3 * avg_ms,
               "share_of_step": (ms / psteps) / ms_per_step,
               # one kernel timed by its own dispatch (what a kernel trace reports), or several launches between
               # two event records (adds a few microseconds of event handling)
               "timing": "kernel dispatch begin to end" if exact else "event records around the launches"}
        if k in work:
            amount, kind = work[k]
            rate = amount / (avg_ms * 1e-3)
            if kind == "bytes":
                ent.update({"bound": "hbm", "algorithmic_bytes": amount, "achieved": rate / 1e9, "unit": "GB/s",
                            "peak": HBM_PEAK_GBPS, "frac": rate / 1e9 / HBM_PEAK_GBPS})
            else:
                ent.update({"bound": "mfma", "algorithmic_flops": amount, "achieved": rate / 1e12, "unit": "TFLOP/s",
                            "peak": MFMA_FP32_PEAK_TFLOPS, "frac": rate / 1e12 / MFMA_FP32_PEAK_TFLOPS})
        kernels[k] = ent
    traffic = {} if args.small else measured_traffic(name)
    for k in kernels:
        if k in traffic:
            kernels[k]["traffic_bytes"] = traffic[k]
    rated = [k for k in kernels if "frac" in kernels[k]]

    # the dominant class: the one that carries most of the step's algorithmic work, measured as the time it
    # would take at its own roofline (launches per step x bytes or flops per launch / peak); time shares of
    # microsecond-scale launches are within each other's measurement noise and would make the choice flip
    def roofline_seconds(k):
        e = kernels[k]
        amount = e.get("algorithmic_bytes", e.get("algorithmic_flops", 0.0))
        peak = e["peak"] * (1e9 if e["unit"] == "GB/s" else 1e12)
        return e["launches_per_step"] * amount / peak
    dom = max(rated, key=roofline_seconds)
    kd = kernels[dom]
    roofline = {"kernel": kd["name"], "bound": kd["bound"], "achieved": kd["achieved"], "peak": kd["peak"],
                "unit": kd["unit"], "frac": kd["frac"], "traffic": kd.get("traffic_bytes"),
                "traffic_source": ("profiles/%s_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, stored)" % name
                                   if kd.get("traffic_bytes") is not None else None),
                "us_per_launch": kd["avg_us"], "timing": kd["timing"], "launches_per_step": kd["launches_per_step"]}
    if kd["bound"] == "hbm" and achievable:
        roofline["measured_achievable"] = {"GBps": achievable["achieved_GBps"],
                                           "what": "1 GiB device-to-device copy on this machine, read + write",
                                           "frac_of_it": kd["achieved"] / achievable["achieved_GBps"]}
    if dom == "vr_rows" and kd["bound"] == "hbm" and kd["avg_us"] < 20:
        roofline["note"] = ("one launch moves only %.1f MB: it is bound by launch and dependency latency and by the "
                            "rows the busiest compute unit has to pull (its workgroups are sized so that this number "
                            "is as small as the batch allows), not by the chip's HBM; the HBM-bound kernel of the "
                            "step is the snapshot pass (kernels.full_rows)" % (kd["algorithmic_bytes"] / 1e6))
    t_full_ms = (prof["full_rows"][0] + prof["full_fold"][0]) / max(1, prof["full_rows"][1])
    rec = {
        "value": iters_per_sec,
        "unit": "inner iterations/s",
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "config": {"workload": "%s%s: %s n=%d d=%d%s N=%d B=%d bits=%d m=%d clip=%s%g algo=%s"
                   % (sp.name, " (scaled down)" if args.small else "",
                      {0: "logistic", 1: "squared loss", 2: "MLP softmax"}[sp.loss] + (" CSR" if sp.csr else " dense"),
                      n, d, " nnz=%d" % nnz if nnz else "", N, B, bits, m, "c*sigma " if sp.clip_mode else "lambda ",
                      sp.clip, {0: "LPC-SVRG", 1: "ALPC-SVRG (Alg. 2)", 2: "ALPC-SVRG (Alg. 3)"}[sp.algo]),
                   "step": "one lpc_epoch = snapshot full-gradient pass + m inner iterations"},
        "full_grad_pass": {"ms": t_full_ms, "note": "rows kernel(s) + fold"},
        "inner_iters_per_sec_excluding_full_grad": m / ((ms_per_step - t_full_ms) * 1e-3),
        "objective": {"start": P0, "end": P_end},
        "kernels": kernels,
        "roofline": roofline,
    }
    if "frac" in kernels.get("full_rows", {}):
        amount, kind = work["full_rows"]
        rate = amount / (t_full_ms * 1e-3)
        rec["full_grad_pass"].update({"achieved": rate / (1e9 if kind == "bytes" else 1e12),
                                      "unit": "GB/s" if kind == "bytes" else "TFLOP/s",
                                      "frac_of_peak": rate / (1e9 * HBM_PEAK_GBPS if kind == "bytes"
                                                              else 1e12 * MFMA_FP32_PEAK_TFLOPS)})
    if name == "c5" and not args.small:
        rec["exchange_steps"] = quantizer_rooflines(ctx, sp)
    ctx.close()
    del ctx, w, ya, za
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(sp, cfgkw, alpc)
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="all", choices=["all", "c1", "c2", "c3", "c4", "c5"],
                    help="all (default): the headline on c4, the largest configuration, with c2, c3 and c5 as "
                         "sub-records under 'workloads'; or one configuration alone")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--iter-form", type=int, default=None, choices=[0, 1, 2, 3],
                    help="form of the dense inner iteration (lpc_tune LPC_TUNE_ITER_FORM; default: the library's)")
    ap.add_argument("--iter-tile", type=int, default=None, choices=[64, 128])
    ap.add_argument("--iter-threads", type=int, default=None, choices=[256, 512])
    ap.add_argument("--small", action="store_true", help="scaled-down problems (quick functional run)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run ten 1 GiB device-to-device copies (a kernel of known traffic: 1 GiB read, "
                         "1 GiB written) so that rocprofv3's FETCH_SIZE / WRITE_SIZE counters can be scaled")
    ap.add_argument("--contractions", action="store_true",
                    help="only time the MLP workload's matrix products one by one (the contraction kernel's "
                         "unit-test entry point), one line per shape")
    args = ap.parse_args()
    if args.contractions:
        contraction_shapes()
        return
    if args.copy_calibration:
        print(json.dumps({"copy_calibration": copy_calibration()}))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the N workers are shards on one device); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    # all library work goes to a stream of its own (not the legacy default stream)
    stream = torch.cuda.Stream(device=torch.device("cuda:0"))
    torch.cuda.set_stream(stream)
    achievable = copy_calibration()

    head = "c4" if args.workload == "all" else args.workload
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[head][0]
    warmup = args.warmup if args.warmup is not None else DEFAULT_STEPS[head][1]
    rec = run_workload(head, steps, warmup, args, achievable)
    out = {
        "metric": "svrg_inner_iters_per_sec",
        "value": rec["value"],
        "unit": rec["unit"],
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": rec["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
    }
    out.update({k: v for k, v in rec.items() if k not in out})
    out["copy_calibration"] = achievable
    if args.workload == "all":
        # the other single-GPU configurations, each with its own steps (the headline above is the largest one)
        out["workloads"] = {}
        for name in ("c2", "c3", "c5"):
            k, wu = DEFAULT_STEPS[name]
            out["workloads"][name] = run_workload(name, k, wu, args, achievable)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
