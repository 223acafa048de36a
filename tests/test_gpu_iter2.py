"""The dense inner iteration as two launches (rows; fold + exchange + update) against the same iteration as
three launches (rows; fold; exchange + update) and against the oracle: Alg. 1 steps 6-10, Alg. 2 steps 7-15."""
import numpy as np
import pytest

import lpc_synth
from oracle import lpco
from _common import gpu_context, oracle_config, oracle_problem, to_dev

pytestmark = pytest.mark.gpu


def _epochs(sp, launches, epochs=2, tile=128, threads=512, **over):
    import torch
    from paper_1901_08924_amd import lpc
    ctx = gpu_context(sp, **over)
    ctx.tune(lpc.TUNE_ITER_LAUNCHES, launches)
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
    three, P3 = _epochs(sp, 3, **over)
    two, P2 = _epochs(sp, 2, tile=tile, threads=threads, **over)
    assert np.array_equal(two[0], three[0])      # same fold order, same draws: the same bits
    assert np.abs(three[0]).max() > 0


@pytest.mark.parametrize("algo", [lpco.ALGO_ALPC_SC, lpco.ALGO_ALPC_GC])
@pytest.mark.parametrize("d,N,B", [(512, 4, 16), (2048, 16, 32), (333, 3, 8)])
@pytest.mark.parametrize("tile,threads", [(128, 512), (64, 256)])
def test_two_launches_equal_three_alpc(algo, d, N, B, tile, threads):
    sp = lpc_synth.make("c4", n=4096, d=d, N=N, B=B)
    over = dict(algo=algo, m=5, tau2=0.5, clip_mode=0, clip=0.8)   # lambda mode: the scale does not depend on sums
    three, _ = _epochs(sp, 3, **over)
    two, _ = _epochs(sp, 2, tile=tile, threads=threads, **over)
    for a, b in zip(two, three):
        assert np.array_equal(a, b)


def test_two_launches_c_sigma_mode_agrees_to_rounding():
    # sigma comes from sums whose grouping differs between the two shapes: the scale may differ in its last bits
    sp = lpc_synth.make("c4", n=4096, d=2048, N=8, B=16)
    over = dict(algo=lpco.ALGO_ALPC_GC, m=8, tau2=0.5)
    (w3, y3, z3), P3 = _epochs(sp, 3, **over)
    (w2, y2, z2), P2 = _epochs(sp, 2, **over)
    assert abs(P2 - P3) <= 1e-5 * abs(P3)
    assert np.abs(w2 - w3).max() <= 1e-3 * max(1e-3, np.abs(w3).max())


@pytest.mark.parametrize("name,over", [("c2", dict(n=2048, d=1024, N=8, B=16)),
                                       ("c4", dict(n=2048, d=512, N=4, B=16))])
def test_two_launches_against_the_oracle(name, over):
    sp = lpc_synth.make(name, **over)
    p, _k = oracle_problem(sp)
    extra = dict(tau2=0.5) if name == "c4" else {}
    cfg = oracle_config(sp, **extra)
    alpc = cfg.algo != lpco.ALGO_LPC
    w_o = sp.w0.copy()
    y_o, z_o = (sp.w0.copy(), sp.w0.copy()) if alpc else (None, None)
    for s in range(3):
        lpco.epoch(p, cfg, w_o, s, y_o, z_o)
    (w_g, *_), P_g = _epochs(sp, 2, epochs=3, **extra)
    P_o = lpco.objective(p, w_o)
    assert abs(P_g - P_o) <= 1e-4 * abs(P_o)


def test_two_launch_epoch_is_reproducible():
    sp = lpc_synth.make("c2", n=4096, d=4096, N=8, B=64)
    a, _ = _epochs(sp, 2, m=16)
    b, _ = _epochs(sp, 2, m=16)
    assert np.array_equal(a[0], b[0])


def test_a_wait_that_gives_up_is_reported_and_every_kernel_exits():
    """Spin limit 0: a workgroup that does not find the others' statistics at its first look gives up, finishes
    with what it has and raises the flag; nothing hangs.  The next epoch with the limit restored is correct."""
    import torch
    from paper_1901_08924_amd import lpc
    sp = lpc_synth.make("c2", n=4096, d=4096, N=8, B=64)
    ctx = gpu_context(sp, m=8)
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
    ref, _ = _epochs(sp, 3, epochs=1, m=8)
    assert np.array_equal(w.cpu().numpy(), ref[0])
