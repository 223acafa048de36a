"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (same N, B, d, bits, same context constructor).  Where the oracle cannot afford the whole output
(MLP snapshot gradient over 16384 rows, a full epoch of C3) the comparison is made on a sample the
oracle can compute: fewer snapshot rows, one worker, a few inner iterations."""
import numpy as np
import pytest

import lpc_synth
from oracle import lpco
from _common import oracle_config, oracle_problem, to_dev

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]


def _ctx(sp, **over):
    from paper_1901_08924_amd import lpc
    return lpc.context_from_problem(sp, **over)


def _check_vr(sp, ctx, p, cfg, w, ws, zs, workers, epoch=1, it=7):
    import torch
    dp = lpco.d_pad(sp.d)
    U = torch.zeros(sp.N, dp, device="cuda")
    stats = torch.zeros(sp.N, 4, dtype=torch.float64, device="cuda")
    ctx.worker_vr_grad(to_dev(w), to_dev(ws), zs, epoch, it, U, stats)
    got = U.cpu().numpy()
    for i in workers:
        U_o, _ = lpco.worker_vr_grad(p, cfg, w, ws, epoch, it, worker_begin=i, worker_end=i + 1)
        gB, _ = lpco.worker_vr_grad(p, cfg, w, np.zeros_like(ws), epoch, it, worker_begin=i, worker_end=i + 1)
        scale = max(np.abs(gB[i]).max(), np.abs(U_o[i]).max())
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
    ctx = _ctx(sp, m=6)
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
    i, idx = None, None
    # A batch has 128 x 2048 x 2 hidden pre-activations of order 1, so its margin is a few 1e-6 at best; the
    # float dot product's rounding is about 3e-7, hence the threshold.
    for cand in range(sp.N):
        cidx = lpco.sample_batch(sp.seed, 0, 2, lpco.TAG_BATCH, cand, sp.B, sp.n)
        if min(lpco.mlp_relu_margin(p, w, cidx), lpco.mlp_relu_margin(p, ws, cidx)) > 3e-6:
            i, idx = cand, cidx
            break
    assert i is not None, "no sampled batch clear of the ReLU kinks among the 16 workers"
    U_o, _ = lpco.worker_vr_grad(p, cfg, w, ws, 0, 2, worker_begin=i, worker_end=i + 1)
    sub, _ks = lpco.make_problem(sp.loss, sp.y[idx[:32]], X=np.ascontiguousarray(sp.X[idx[:32]]), d=sp.d,
                                 mlp_dims=sp.mlp_dims)
    scale = max(np.abs(lpco.full_grad(sub, w)[0]).max(), np.abs(U_o[i]).max())
    got = U[i].cpu().numpy()
    assert np.abs(got - U_o[i]).max() <= 2e-5 * scale
    # bit-exact exchange of the device's own 16 x 4.2M matrix
    gotU = U.cpu().numpy()
    packed = torch.zeros(sp.N, ctx.W, dtype=torch.int32, device="cuda")
    delta = torch.zeros(sp.N, device="cuda")
    avg = torch.zeros(sp.d, device="cuda")
    ctx.exchange(U, 0, 2, packed, delta, avg)
    po, do, _, _ = lpco.quantize_clip(gotU, sp.d, sp.bits, sp.clip_mode, sp.clip, seed=sp.seed, epoch=0, iter_=2)
    assert np.array_equal(delta.cpu().numpy(), do)
    assert np.array_equal(packed.cpu().numpy().view(np.uint32), po)
    assert np.array_equal(avg.cpu().numpy(), lpco.dequantize_avg(po, do, sp.d, sp.bits))
    ctx.close()
