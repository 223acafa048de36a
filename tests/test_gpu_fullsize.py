"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (same N, B, d, bits, same context constructor).  Where the oracle cannot afford the whole output
(MLP snapshot gradient over 16384 rows, a full epoch of C3) the comparison is made on a sample the
oracle can compute: fewer snapshot rows, one worker, a few inner iterations."""
import numpy as np
import pytest

import lpc_synth
from oracle import lpco
from _common import batch_grad_inf, oracle_config, oracle_problem, to_dev

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]


def _ctx(sp, **over):
    from paper_1901_08924_amd import lpc
    return lpc.context_from_problem(sp, **over)


def _upload(sp):
    """The dense design matrix and the labels on the device, once, for several contexts."""
    return to_dev(sp.X), to_dev(sp.y)


def _ctx_on(sp, dev_xy, **over):
    from paper_1901_08924_amd import lpc
    from _common import config_kwargs
    X, y = dev_xy
    return lpc.Context(sp.loss, y, lpc.make_config(**config_kwargs(sp, **over)), X=X, d=sp.d, mlp_dims=sp.mlp_dims,
                       lambda1=sp.lambda1, lambda2=sp.lambda2)


def _threads():
    import os
    return max(1, min(16, os.cpu_count() or 1))


def _check_vr(sp, ctx, p, cfg, w, ws, zs, workers, epoch=1, it=7):
    import torch
    dp = lpco.d_pad(sp.d)
    U = torch.zeros(sp.N, dp, device="cuda")
    stats = torch.zeros(sp.N, 4, dtype=torch.float64, device="cuda")
    ctx.worker_vr_grad(to_dev(w), to_dev(ws), zs, epoch, it, U, stats)
    got = U.cpu().numpy()
    for i in workers:
        U_o, _ = lpco.worker_vr_grad(p, cfg, w, ws, epoch, it, worker_begin=i, worker_end=i + 1)
        scale = max(batch_grad_inf(sp, w, epoch, it, lpco.TAG_BATCH, i), np.abs(U_o[i]).max())
        assert np.abs(got[i] - U_o[i]).max() <= 2e-5 * scale
    return got, stats.cpu().numpy()


def test_c2_full_size():
    import torch
    sp = lpc_synth.make("c2")
    assert (sp.n, sp.d, sp.N, sp.B, sp.bits, sp.m) == (65536, 4096, 8, 64, 4, 128)
    ctx = _ctx(sp)
    p, _k = oracle_problem(sp)
    cfg = oracle_config(sp)
    rng = np.random.default_rng(0)
    ws = (rng.standard_normal(sp.d) * 2.0).astype(np.float32)
    w = (ws + 0.2 * rng.standard_normal(sp.d)).astype(np.float32)
    mu = torch.zeros(sp.d, device="cuda")
    zs = torch.zeros(sp.n, device="cuda")
    f = torch.zeros(1, dtype=torch.float64, device="cuda")
    ctx.full_grad(to_dev(ws), mu, zs, f)
    mu_o, z_o, f_o = lpco.full_grad(p, ws)
    assert np.abs(mu.cpu().numpy() - mu_o).max() <= 1e-5 * np.abs(mu_o).max()
    assert np.abs(zs.cpu().numpy() - z_o).max() <= 1e-5 * max(1.0, np.abs(z_o).max())
    assert abs(f.item() - f_o) <= 1e-5 * abs(f_o)
    got, st = _check_vr(sp, ctx, p, cfg, w, ws, zs, workers=range(sp.N))
    # quantize the device's own U: the oracle must produce the same bits from the same floats
    packed = torch.zeros(sp.N, ctx.W, dtype=torch.int32, device="cuda")
    delta = torch.zeros(sp.N, device="cuda")
    avg = torch.zeros(sp.d, device="cuda")
    ctx.exchange(to_dev(got), 1, 7, packed, delta, avg)
    po, do, _, _ = lpco.quantize_clip(got, sp.d, sp.bits, sp.clip_mode, sp.clip, seed=sp.seed, epoch=1, iter_=7)
    assert np.array_equal(packed.cpu().numpy().view(np.uint32), po) and np.array_equal(delta.cpu().numpy(), do)
    assert np.array_equal(avg.cpu().numpy(), lpco.dequantize_avg(po, do, sp.d, sp.bits))
    # two whole epochs
    w_o, w_g = sp.w0.copy(), to_dev(sp.w0)
    for s in range(2):
        lpco.epoch(p, cfg, w_o, s)
        ctx.epoch(w_g, s)
    P_o, P_g = lpco.objective(p, w_o), ctx.objective(w_g)
    assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    assert ctx.take_device_flags() == 0
    ctx.close()
    # the paper's operating point lambda = 0.9 (Sec. 6.1) at full size: one epoch, clipped coordinates on both sides
    ctx = _ctx(sp, clip=0.9)
    cfg9 = oracle_config(sp, clip=0.9)
    w_o, w_g = sp.w0.copy(), to_dev(sp.w0)
    dtr_o, ntr_o = lpco.epoch_traced(p, cfg9, w_o, 0)
    dtr, ntr = ctx.epoch_traced(w_g, 0)
    P_o, P_g = lpco.objective(p, w_o), ctx.objective(w_g)
    assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    dtr, ntr = dtr.cpu().numpy(), ntr.cpu().numpy().view(np.uint32)
    assert ntr_o[1:].sum() > sp.m                             # lambda < 1 clips the few coordinates near the maximum
    assert np.abs(dtr - dtr_o).max() <= 1e-3 * dtr_o.max()
    assert np.abs(ntr.astype(np.int64) - ntr_o.astype(np.int64)).max() <= 2
    # and the untraced epoch (fused launches) from the same start
    w_g2 = to_dev(sp.w0)
    ctx.epoch(w_g2, 0)
    assert abs(ctx.objective(w_g2) - P_o) <= 1e-4 * abs(P_o)
    ctx.close()


def test_c3_full_size():
    import torch
    sp = lpc_synth.make("c3")
    assert (sp.n, sp.d, sp.N, sp.B, sp.bits) == (1 << 20, 1 << 20, 16, 256, 2)
    ctx = _ctx(sp)
    p, _k = oracle_problem(sp)
    cfg = oracle_config(sp)
    rng = np.random.default_rng(0)
    ws = (rng.standard_normal(sp.d) * 2.0).astype(np.float32)
    w = (ws + 0.2 * rng.standard_normal(sp.d)).astype(np.float32)
    mu = torch.zeros(sp.d, device="cuda")
    zs = torch.zeros(sp.n, device="cuda")
    ctx.full_grad(to_dev(ws), mu, zs, None)
    mu_o, z_o, _ = lpco.full_grad(p, ws)
    assert np.abs(mu.cpu().numpy() - mu_o).max() <= 1e-5 * np.abs(mu_o).max()
    assert np.abs(zs.cpu().numpy() - z_o).max() <= 1e-5 * max(1.0, np.abs(z_o).max())
    got, st = _check_vr(sp, ctx, p, cfg, w, ws, zs, workers=(0, 7, 15))
    # bit-exact exchange of the device's own U at d = 2^20 (large-d kernels)
    packed = torch.zeros(sp.N, ctx.W, dtype=torch.int32, device="cuda")
    delta = torch.zeros(sp.N, device="cuda")
    avg = torch.zeros(sp.d, device="cuda")
    ctx.exchange(to_dev(got), 0, 3, packed, delta, avg)
    po, do, _, _ = lpco.quantize_clip(got, sp.d, sp.bits, sp.clip_mode, sp.clip, seed=sp.seed, epoch=0, iter_=3)
    assert np.array_equal(packed.cpu().numpy().view(np.uint32), po) and np.array_equal(delta.cpu().numpy(), do)
    assert np.array_equal(avg.cpu().numpy(), lpco.dequantize_avg(po, do, sp.d, sp.bits))
    ctx.close()
    # an epoch with 4 inner iterations at full n, d, N, B
    ctx = _ctx(sp, m=4)
    cfg4 = oracle_config(sp, m=4)
    w_o, w_g = sp.w0.copy(), to_dev(sp.w0)
    lpco.epoch(p, cfg4, w_o, 0)
    ctx.epoch(w_g, 0)
    P_o, P_g = lpco.objective(p, w_o), ctx.objective(w_g)
    assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    ctx.close()


def test_c4_full_size():
    import torch
    sp = lpc_synth.make("c4")
    assert (sp.n, sp.d, sp.N, sp.B, sp.bits) == (262144, 8192, 16, 64, 3)
    dev_xy = _upload(sp)
    ctx = _ctx_on(sp, dev_xy, m=6)
    p, _k = oracle_problem(sp)
    cfg = oracle_config(sp, m=6)
    rng = np.random.default_rng(0)
    ws = (rng.standard_normal(sp.d) / np.sqrt(sp.d)).astype(np.float32)
    w = (ws + 0.1 * rng.standard_normal(sp.d) / np.sqrt(sp.d)).astype(np.float32)
    mu = torch.zeros(sp.d, device="cuda")
    zs = torch.zeros(sp.n, device="cuda")
    ctx.full_grad(to_dev(ws), mu, zs, None)
    mu_o, z_o, _ = lpco.full_grad(p, ws)
    assert np.abs(mu.cpu().numpy() - mu_o).max() <= 1e-5 * np.abs(mu_o).max()
    _check_vr(sp, ctx, p, cfg, w, ws, zs, workers=(0, 5, 15))
    # one ALPC epoch (Alg. 3) with 6 inner iterations at full n, d, N, B
    w_o, y_o, z_o2 = sp.w0.copy(), sp.w0.copy(), sp.w0.copy()
    w_g, y_g, z_g = to_dev(sp.w0), to_dev(sp.w0), to_dev(sp.w0)
    lpco.epoch(p, cfg, w_o, 0, y_o, z_o2)
    ctx.epoch(w_g, 0, y_g, z_g)
    P_o, P_g = lpco.objective(p, w_o), ctx.objective(w_g)
    assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    assert np.abs(z_g.cpu().numpy() - z_o2).max() <= 1e-3 * max(1e-3, np.abs(z_o2).max())
    ctx.close()
    # the rest of the configuration's clip sweep (c = 1 and 4 times sigma; 2 sigma ran above) and Alg. 2 with
    # Theorem 3's parameter rules, each one epoch of 6 inner iterations at full n, d, N, B
    for over in (dict(clip=1.0), dict(clip=4.0), dict(algo=lpco.ALGO_ALPC_SC), dict(algo=lpco.ALGO_ALPC_SC, clip=1.0)):
        ctx = _ctx_on(sp, dev_xy, m=6, **over)
        cfg_v = oracle_config(sp, m=6, **over)
        w_o, y_o, z_o2 = sp.w0.copy(), sp.w0.copy(), sp.w0.copy()
        w_g, y_g, z_g = to_dev(sp.w0), to_dev(sp.w0), to_dev(sp.w0)
        lpco.epoch(p, cfg_v, w_o, 0, y_o, z_o2)
        ctx.epoch(w_g, 0, y_g, z_g)
        P_o, P_g = lpco.objective(p, w_o), ctx.objective(w_g)
        assert abs(P_g - P_o) <= 1e-4 * abs(P_o), over
        assert np.abs(y_g.cpu().numpy() - y_o).max() <= 1e-3 * max(1e-3, np.abs(y_o).max()), over
        assert ctx.take_device_flags() == 0
        ctx.close()


def test_c5_full_size_sampled():
    import torch
    sp = lpc_synth.make("c5")
    assert (sp.d, sp.N, sp.B, sp.bits) == (4206602, 16, 128, 4)
    # snapshot gradient over a sample of 192 rows (the oracle's plain loops take ~0.05 s per row)
    ctx = _ctx(sp, n_full=192)
    p, _k = oracle_problem(sp)
    rng = np.random.default_rng(0)
    ws = sp.w0.copy()
    w = (ws + 0.01 * rng.standard_normal(sp.d).astype(np.float32) * np.abs(ws).mean()).astype(np.float32)
    mu = torch.zeros(sp.d, device="cuda")
    ctx.full_grad(to_dev(ws), mu, None, None)
    mu_o, _, _ = lpco.full_grad(p, ws, n_rows=192)
    assert np.abs(mu.cpu().numpy() - mu_o).max() <= 1e-5 * np.abs(mu_o).max()
    # worker 11's difference, in the N=16, B=128 launch
    cfg = oracle_config(sp)
    dp = lpco.d_pad(sp.d)
    U = torch.zeros(sp.N, dp, device="cuda")
    stats = torch.zeros(sp.N, 4, dtype=torch.float64, device="cuda")
    ctx.worker_vr_grad(to_dev(w), to_dev(ws), None, 0, 2, U, stats)
    # The gradient of a ReLU network jumps where a hidden pre-activation is zero, and the float path may
    # land on either side of a kink that the double oracle resolves: tight parity is demanded for a worker
    # whose batch stays clear of the kinks (margin far above the rounding of a 3072-term float dot product).
    # A batch has 128 x 2048 x 2 hidden pre-activations of order 1, so its margin is a few 1e-6 at best; the
    # float dot product's rounding is about 3e-7, hence the threshold.  EVERY worker whose batch clears it is
    # compared (the oracle's plain loops run one worker per host thread).
    from concurrent.futures import ThreadPoolExecutor

    def margin_of(cand):
        cidx = lpco.sample_batch(sp.seed, 0, 2, lpco.TAG_BATCH, cand, sp.B, sp.n)
        return min(lpco.mlp_relu_margin(p, w, cidx), lpco.mlp_relu_margin(p, ws, cidx))

    def oracle_u(cand):
        U_o, _ = lpco.worker_vr_grad(p, cfg, w, ws, 0, 2, worker_begin=cand, worker_end=cand + 1)
        idx = lpco.sample_batch(sp.seed, 0, 2, lpco.TAG_BATCH, cand, sp.B, sp.n)
        sub, _ks = lpco.make_problem(sp.loss, sp.y[idx[:32]], X=np.ascontiguousarray(sp.X[idx[:32]]), d=sp.d,
                                     mlp_dims=sp.mlp_dims)
        return U_o[cand], max(np.abs(lpco.full_grad(sub, w)[0]).max(), np.abs(U_o[cand]).max())

    with ThreadPoolExecutor(max_workers=_threads()) as ex:
        margins = list(ex.map(margin_of, range(sp.N)))
        clear = [i for i in range(sp.N) if margins[i] > 3e-6]
        assert clear, "no sampled batch clear of the ReLU kinks among the 16 workers"
        refs = list(ex.map(oracle_u, clear))
    gotU = U.cpu().numpy()
    for i, (u_o, scale) in zip(clear, refs):
        assert np.abs(gotU[i] - u_o).max() <= 2e-5 * scale, (i, margins[i])
    # the others may have a unit on the other side of a kink: whole weight-gradient columns then differ by
    # x*delta/B, which is still small against the gradient itself
    for i in set(range(sp.N)) - set(clear):
        u_o, scale = oracle_u(i)
        assert np.abs(gotU[i] - u_o).max() <= 2e-2 * scale, (i, margins[i])
    # bit-exact exchange of the device's own 16 x 4.2M matrix
    packed = torch.zeros(sp.N, ctx.W, dtype=torch.int32, device="cuda")
    delta = torch.zeros(sp.N, device="cuda")
    avg = torch.zeros(sp.d, device="cuda")
    ctx.exchange(U, 0, 2, packed, delta, avg)
    po, do, _, _ = lpco.quantize_clip(gotU, sp.d, sp.bits, sp.clip_mode, sp.clip, seed=sp.seed, epoch=0, iter_=2)
    assert np.array_equal(delta.cpu().numpy(), do)
    assert np.array_equal(packed.cpu().numpy().view(np.uint32), po)
    assert np.array_equal(avg.cpu().numpy(), lpco.dequantize_avg(po, do, sp.d, sp.bits))
    ctx.close()


def _oracle_mean_grad(sp, w, n_rows, chunk=256):
    """The oracle's snapshot gradient over the first n_rows samples, its plain loops spread over the host's threads:
    the mean gradient of each slice of rows is the oracle's own full gradient of a problem made of that slice."""
    from concurrent.futures import ThreadPoolExecutor

    def part(r0):
        r1 = min(n_rows, r0 + chunk)
        sub, _ks = lpco.make_problem(sp.loss, sp.y[r0:r1], X=sp.X[r0:r1], d=sp.d, mlp_dims=sp.mlp_dims)
        g, _, f = lpco.full_grad(sub, w)
        return g.astype(np.float64) * (r1 - r0), f * (r1 - r0)

    with ThreadPoolExecutor(max_workers=_threads()) as ex:
        parts = list(ex.map(part, range(0, n_rows, chunk)))
    g = np.sum([q[0] for q in parts], axis=0) / n_rows
    return g, sum(q[1] for q in parts) / n_rows


def test_c5_snapshot_pass_in_the_benchmarks_launch_shape():
    """The MLP snapshot pass as bench.py runs it: the first layer at its full input width, 8192-row chunks (two of
    them, the second accumulating into the first's result), 2048-row blocks of the weight-gradient products on
    the matrix cores side by side into the rows of U and folded afterwards, 256-row blocks for the bias sums and
    the last layer's weight gradient on the vector units.  Hidden layers are 256 wide so that the oracle affords
    all 12288 rows."""
    import dataclasses
    import torch
    from concurrent.futures import ThreadPoolExecutor
    dims = (3072, 256, 256, 10)
    sp = lpc_synth.make("c5", n=16384, dims=dims, n_full=12288)
    assert (sp.N, sp.B, sp.n_full) == (16, 128, 12288)
    # 12288 rows x 512 hidden units of order 1: a float dot product of 3072 terms is off by a few 1e-6, so a
    # handful of pre-activations lie close enough to zero for the float pass and the double oracle to take
    # different sides of the ReLU kink, and whole weight-gradient columns then differ by x*delta/n.  Rows with a
    # pre-activation within 2e-5 of zero are left out of the data BEFORE either side sees it (the oracle tells
    # which), so the 1e-5 bar applies to what remains.
    p_all, _ka = oracle_problem(sp)

    def margins(r0):
        return [lpco.mlp_relu_margin(p_all, sp.w0, [r]) for r in range(r0, min(sp.n, r0 + 256))]

    with ThreadPoolExecutor(max_workers=_threads()) as ex:
        margin = np.concatenate(list(ex.map(margins, range(0, sp.n, 256))))
    keep = np.flatnonzero(margin > 2e-5)
    assert keep.size >= 12288 + 1024 and keep.size >= sp.n - 512     # few rows sit on a kink
    sp = dataclasses.replace(sp, X=np.ascontiguousarray(sp.X[keep]), y=np.ascontiguousarray(sp.y[keep]),
                             n=int(keep.size))
    ctx = _ctx(sp)
    mu = torch.zeros(sp.d, device="cuda")
    f = torch.zeros(1, dtype=torch.float64, device="cuda")
    ctx.full_grad(to_dev(sp.w0), mu, None, f)
    mu_o, f_o = _oracle_mean_grad(sp, sp.w0, sp.n_full)
    got = mu.cpu().numpy()
    worst = int(np.abs(got - mu_o).argmax())
    assert np.abs(got - mu_o).max() <= 1e-5 * np.abs(mu_o).max(), (worst, got[worst], mu_o[worst], keep.size)
    assert abs(f.item() - f_o) <= 1e-5 * abs(f_o)
    # a ragged row count: one whole chunk, then 2048 + 300 rows (a block-wise part and a remainder)
    ctx.close()
    n2 = 8192 + 2048 + 300
    ctx = _ctx(sp, n_full=n2)
    ctx.full_grad(to_dev(sp.w0), mu, None, f)
    mu_o, f_o = _oracle_mean_grad(sp, sp.w0, n2)
    assert np.abs(mu.cpu().numpy() - mu_o).max() <= 1e-5 * np.abs(mu_o).max()
    assert abs(f.item() - f_o) <= 1e-5 * abs(f_o)
    ctx.close()


def test_c5_epoch_at_full_layer_widths():
    """One LPC-SVRG epoch of the 3072-1024-1024-10 network (whole 4.2 M-coordinate gradient quantized with one
    scale per worker, taken from the weight-gradient products' epilogues) against the oracle: objective and the
    trace of scale factors.  N, B, m and the sample count are small enough for the oracle's plain loops."""
    sp = lpc_synth.make("c5", n=256, n_full=64, N=2, B=32, m=2)
    assert sp.d == 4206602 and sp.mlp_dims == (3072, 1024, 1024, 10)
    p, _k = oracle_problem(sp)
    cfg = oracle_config(sp)
    ctx = _ctx(sp)
    w_o, w_g = sp.w0.copy(), to_dev(sp.w0)
    dtr_o, ntr_o = lpco.epoch_traced(p, cfg, w_o, 0)
    ctx.epoch(w_g, 0)
    P_o, P_g = lpco.objective(p, w_o), ctx.objective(w_g)
    assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    assert np.abs(w_g.cpu().numpy() - w_o).max() <= 1e-3 * np.abs(w_o).max()
    w_t = to_dev(sp.w0)
    dtr, ntr = ctx.epoch_traced(w_t, 0)
    dtr = dtr.cpu().numpy()
    # t = 0: x_0 equals the snapshot, the oracle's difference is exactly zero while the two parameter sets' weight
    # gradients here cancel to float rounding only
    assert dtr_o[0].max() == 0.0 and dtr[0].max() <= 1e-6 * dtr_o[1].max()
    assert np.abs(dtr[1:] - dtr_o[1:]).max() <= 1e-3 * dtr_o[1:].max()
    assert abs(ctx.objective(w_t) - P_o) <= 1e-4 * abs(P_o)
    assert ctx.take_device_flags() == 0
    ctx.close()
