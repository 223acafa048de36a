"""The dense inner iteration as two launches (rows; fold + exchange + update) against the same iteration as
three launches (rows; fold; exchange + update) and against the oracle: Alg. 1 steps 6-10, Alg. 2 steps 7-15."""
import numpy as np
import pytest

import lpc_synth
from oracle import lpco
from _common import gpu_context, oracle_config, oracle_problem, to_dev

pytestmark = pytest.mark.gpu


def _epochs(sp, form, epochs=2, tile=128, threads=512, **over):
    import torch
    from paper_1901_08924_amd import lpc
    ctx = gpu_context(sp, **over)
    ctx.tune(lpc.TUNE_ITER_FORM, form)
    ctx.tune(lpc.TUNE_ITER_TILE, tile)
    ctx.tune(lpc.TUNE_ITER_THREADS, threads)
    alpc = ctx.config.algo != lpc.ALGO_LPC
    w = to_dev(sp.w0)
    y, z = (to_dev(sp.w0), to_dev(sp.w0)) if alpc else (None, None)
    for s in range(epochs):
        ctx.epoch(w, s, y, z)
    assert ctx.take_device_flags() == 0
    P = ctx.objective(w)
    ctx.close()
    out = [w.cpu().numpy()] + ([y.cpu().numpy(), z.cpu().numpy()] if alpc else [])
    return out, P


# d = 4096: 32 tiles of 128; d = 1000: ragged last tile; d = 333: rows that cannot be read 16 bytes at a time
@pytest.mark.parametrize("d,N,B,bits", [(4096, 8, 64, 4), (1000, 4, 16, 3), (333, 5, 8, 2), (64, 4, 16, 2),
                                        (8192, 16, 16, 3)])
@pytest.mark.parametrize("tile,threads", [(128, 512), (64, 512), (128, 256), (64, 256)])
def test_two_launches_equal_three_alg1(d, N, B, bits, tile, threads):
    sp = lpc_synth.make("c2", n=4096, d=d, N=N, B=B, bits=bits)
    over = dict(m=6, clip=0.9)
    three, P3 = _epochs(sp, 0, **over)
    two, P2 = _epochs(sp, 1, tile=tile, threads=threads, **over)
    assert np.array_equal(two[0], three[0])      # same fold order, same draws: the same bits
    assert np.abs(three[0]).max() > 0


@pytest.mark.parametrize("algo", [lpco.ALGO_ALPC_SC, lpco.ALGO_ALPC_GC])
@pytest.mark.parametrize("d,N,B", [(512, 4, 16), (2048, 16, 32), (333, 3, 8)])
@pytest.mark.parametrize("tile,threads", [(128, 512), (64, 256)])
def test_two_launches_equal_three_alpc(algo, d, N, B, tile, threads):
    sp = lpc_synth.make("c4", n=4096, d=d, N=N, B=B)
    over = dict(algo=algo, m=5, tau2=0.5, clip_mode=0, clip=0.8)   # lambda mode: the scale does not depend on sums
    three, _ = _epochs(sp, 0, **over)
    two, _ = _epochs(sp, 1, tile=tile, threads=threads, **over)
    for a, b in zip(two, three):
        assert np.array_equal(a, b)


def test_two_launches_c_sigma_mode_agrees_to_rounding():
    # sigma comes from sums whose grouping differs between the two shapes: the scale may differ in its last bits
    sp = lpc_synth.make("c4", n=4096, d=2048, N=8, B=16)
    over = dict(algo=lpco.ALGO_ALPC_GC, m=8, tau2=0.5)
    (w3, y3, z3), P3 = _epochs(sp, 0, **over)
    (w2, y2, z2), P2 = _epochs(sp, 1, **over)
    assert abs(P2 - P3) <= 1e-5 * abs(P3)
    assert np.abs(w2 - w3).max() <= 1e-3 * max(1e-3, np.abs(w3).max())


@pytest.mark.parametrize("form", [0, 1, 2])
@pytest.mark.parametrize("name,over", [("c2", dict(n=2048, d=1024, N=8, B=16)),
                                       ("c4", dict(n=2048, d=512, N=4, B=16)),
                                       ("c2", dict(n=3000, d=333, N=5, B=20)),
                                       ("c4", dict(n=4096, d=8192, N=16, B=64))])
def test_two_launches_against_the_oracle(name, over, form):
    sp = lpc_synth.make(name, **over)
    p, _k = oracle_problem(sp)
    extra = dict(tau2=0.5) if name == "c4" else {}
    cfg = oracle_config(sp, **extra)
    alpc = cfg.algo != lpco.ALGO_LPC
    w_o = sp.w0.copy()
    y_o, z_o = (sp.w0.copy(), sp.w0.copy()) if alpc else (None, None)
    for s in range(3):
        lpco.epoch(p, cfg, w_o, s, y_o, z_o)
    (w_g, *_), P_g = _epochs(sp, form, epochs=3, **extra)
    P_o = lpco.objective(p, w_o)
    assert abs(P_g - P_o) <= 1e-4 * abs(P_o)


def test_two_launch_epoch_is_reproducible():
    sp = lpc_synth.make("c2", n=4096, d=4096, N=8, B=64)
    a, _ = _epochs(sp, 1, m=16)
    b, _ = _epochs(sp, 1, m=16)
    assert np.array_equal(a[0], b[0])


def test_a_wait_that_gives_up_is_reported_and_every_kernel_exits():
    """Spin limit 0: a workgroup that does not find the others' statistics at its first look gives up, finishes
    with what it has and raises the flag; nothing hangs.  The next epoch with the limit restored is correct."""
    import torch
    from paper_1901_08924_amd import lpc
    sp = lpc_synth.make("c2", n=4096, d=4096, N=8, B=64)
    ctx = gpu_context(sp, m=8)
    ctx.tune(lpc.TUNE_ITER_FORM, 1)
    ctx.tune(lpc.TUNE_SPIN_LIMIT, 0)
    w = to_dev(sp.w0)
    ctx.epoch(w, 0)
    torch.cuda.synchronize()
    assert ctx.take_device_flags() in (lpc.OK, lpc.EDEVICE)
    ctx.tune(lpc.TUNE_SPIN_LIMIT, 1 << 15)
    w = to_dev(sp.w0)
    ctx.epoch(w, 0)
    assert ctx.take_device_flags() == lpc.OK
    ctx.close()
    ref, _ = _epochs(sp, 0, epochs=1, m=8)
    assert np.array_equal(w.cpu().numpy(), ref[0])


@pytest.mark.parametrize("name,over", [("c2", dict(n=4096, d=4096, N=8, B=64)), ("c2", dict(n=3000, d=333, N=5, B=20)),
                                       ("c4", dict(n=4096, d=2048, N=16, B=32)), ("c1", {})])
def test_column_tile_epoch_is_reproducible_and_close_to_the_row_form(name, over):
    """Form 2 (column tiles) adds the same numbers as form 0 in another order: the same bits run to run, iterates
    within rounding of form 0's (a rounding difference in u may flip a few stochastic rounding decisions)."""
    sp = lpc_synth.make(name, **over)
    extra = dict(tau2=0.5) if name == "c4" else {}
    a, Pa = _epochs(sp, 2, m=8, **extra)
    b, Pb = _epochs(sp, 2, m=8, **extra)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    ref, P0 = _epochs(sp, 0, m=8, **extra)
    assert abs(Pa - P0) <= 1e-5 * abs(P0)
    assert np.abs(a[0] - ref[0]).max() <= 2e-3 * max(1e-3, np.abs(ref[0]).max())


def test_column_tile_worker_pass_matches_the_oracle_at_ragged_sizes():
    import torch
    from paper_1901_08924_amd import lpc
    from _common import batch_grad_inf
    for d, N, B in ((333, 3, 7), (1000, 4, 33), (4096, 8, 64), (8192 + 4, 2, 5)):
        sp = lpc_synth.make("c2", n=2048, d=d, N=N, B=B)
        ctx = gpu_context(sp)
        ctx.tune(lpc.TUNE_ITER_FORM, 2)
        p, _k = oracle_problem(sp)
        cfg = oracle_config(sp)
        rng = np.random.default_rng(5)
        ws = (rng.standard_normal(d) * 2.0).astype(np.float32)
        w = (ws + 0.2 * rng.standard_normal(d)).astype(np.float32)
        zs = torch.zeros(sp.n, device="cuda")
        ctx.full_grad(to_dev(ws), torch.zeros(d, device="cuda"), zs, None)
        dp = lpco.d_pad(d)
        for kind, tag, rows in ((1, lpco.TAG_BATCH, N), (2, lpco.TAG_SHARED, 1)):
            U = torch.full((N, dp), 9.0, device="cuda")
            stats = torch.zeros(N, 4, dtype=torch.float64, device="cuda")
            ctx.worker_vr_grad(to_dev(w), to_dev(ws), zs, 3, 2, U, stats, kind=kind)
            U_o, _ = lpco.worker_vr_grad(p, cfg, w, ws, 3, 2, tag=tag)
            got = U.cpu().numpy()[:rows]
            for i in range(rows):
                scale = max(batch_grad_inf(sp, w, 3, 2, tag, i), np.abs(U_o[i]).max())
                assert np.abs(got[i] - U_o[i]).max() <= 2e-5 * scale
                assert not got[i, d:].any()
            sg = stats.cpu().numpy()[:rows]
            assert np.array_equal(sg[:, 0], np.abs(got[:, :d]).max(axis=1).astype(np.float64))
        ctx.close()
