"""The resident form of the dense inner loop (all m iterations of an epoch in one launch whose workgroups hand
each other partial vectors, statistics and iterates on the chip) against the oracle and against the three-launch
form: Alg. 1 steps 5-11, Alg. 2 steps 5-15, Alg. 3."""
import numpy as np
import pytest

import lpc_synth
from oracle import lpco
from _common import gpu_context, oracle_config, oracle_problem, to_dev

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(120)]

RESIDENT = 3


def _epochs(sp, form, epochs=2, **over):
    from paper_1901_08924_amd import lpc
    ctx = gpu_context(sp, **over)
    ctx.tune(lpc.TUNE_ITER_FORM, form)
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


CASES = [
    ("c2", dict(n=2048, d=1024, N=8, B=16), {}),                       # one worker per die, half the compute units hold rows
    ("c2", dict(n=4096, d=4096, N=8, B=64), dict(m=8)),                # the benchmark's shape, short
    ("c2", dict(n=3000, d=332, N=5, B=20), {}),                        # dies without a worker, ragged slices, d_pad > d
    ("c2", dict(n=4096, d=4100, N=11, B=40), dict(m=5, bits=3, clip=0.9)),   # two workers on some dies, 26 slices of 160
    ("c1", {}, {}),                                                    # d = 64: two slices
    ("c2", dict(n=4096, d=2048, N=3, B=100), dict(m=4, bits=8, clip_mode=1, clip=2.5)),  # four rows per compute unit
    ("c4", dict(n=2048, d=512, N=4, B=16), dict(tau2=0.5)),            # Alg. 3, shared batch spread over the dies
    ("c4", dict(n=4096, d=8192, N=16, B=64), dict(tau2=0.5, m=6)),     # the benchmark's shape, short
    ("c4", dict(n=4096, d=2048, N=9, B=7), dict(tau2=0.5, algo=lpco.ALGO_ALPC_SC, m=7)),   # Alg. 2, B < 8
    ("c2", dict(n=4096, d=16384, N=8, B=33), dict(m=3, bits=2)),       # the widest rows, 33 positions per batch
]


@pytest.mark.parametrize("name,over,cfg_over", CASES)
def test_resident_epochs_against_the_oracle(name, over, cfg_over):
    sp = lpc_synth.make(name, **over)
    print("case", name, over, cfg_over, flush=True)
    p, _k = oracle_problem(sp)
    cfg = oracle_config(sp, **cfg_over)
    alpc = cfg.algo != lpco.ALGO_LPC
    w_o = sp.w0.copy()
    y_o, z_o = (sp.w0.copy(), sp.w0.copy()) if alpc else (None, None)
    for s in range(3):
        lpco.epoch(p, cfg, w_o, s, y_o, z_o)
    (w_g, *rest), P_g = _epochs(sp, RESIDENT, epochs=3, **cfg_over)
    P_o = lpco.objective(p, w_o)
    assert np.isfinite(P_g) and abs(P_g - P_o) <= 1e-4 * abs(P_o)
    scale = max(1e-3, float(np.abs(w_o).max()))
    assert np.abs(w_g - w_o).max() <= 2e-2 * scale      # iterates agree up to a few flipped rounding decisions
    if alpc:
        assert np.abs(rest[1] - z_o).max() <= 2e-2 * max(1e-3, float(np.abs(z_o).max()))


@pytest.mark.parametrize("name,over,cfg_over", [CASES[1], CASES[3], CASES[7], CASES[8]])
def test_resident_epochs_are_reproducible_and_close_to_the_launch_per_phase_form(name, over, cfg_over):
    """Every sum has a fixed order: the same bits run to run.  The three-launch form adds the same numbers in another
    order, so the two agree to rounding (a rounding difference in u may flip a few stochastic rounding decisions)."""
    sp = lpc_synth.make(name, **over)
    print("case", name, over, cfg_over, flush=True)
    a, Pa = _epochs(sp, RESIDENT, **cfg_over)
    b, Pb = _epochs(sp, RESIDENT, **cfg_over)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    ref, Pr = _epochs(sp, 0, **cfg_over)
    assert abs(Pa - Pr) <= 1e-5 * abs(Pr)
    assert np.abs(a[0] - ref[0]).max() <= 2e-2 * max(1e-3, float(np.abs(ref[0]).max()))


def test_resident_form_refused_where_it_does_not_apply():
    from paper_1901_08924_amd import lpc
    sp = lpc_synth.make("c2", n=2048, d=333, N=4, B=16)     # rows that cannot be read 16 bytes at a time
    ctx = gpu_context(sp)
    with pytest.raises(lpc.LpcError) as e:
        ctx.tune(lpc.TUNE_ITER_FORM, RESIDENT)
    assert e.value.code == lpc.EUNSUPPORTED
    ctx.close()


def test_a_resident_wait_that_gives_up_is_reported_and_every_workgroup_exits():
    """Spin limit 0: no wait is ever satisfied; every workgroup leaves the loop at its first wait, the flag is raised
    and nothing hangs.  The next epoch with the limit restored is correct."""
    import torch
    from paper_1901_08924_amd import lpc
    sp = lpc_synth.make("c2", n=4096, d=1024, N=8, B=32)
    ctx = gpu_context(sp, m=4)
    ctx.tune(lpc.TUNE_ITER_FORM, RESIDENT)
    ctx.tune(lpc.TUNE_SPIN_LIMIT, 0)
    w = to_dev(sp.w0)
    ctx.epoch(w, 0)
    torch.cuda.synchronize()
    assert ctx.take_device_flags() == lpc.EDEVICE
    ctx.tune(lpc.TUNE_SPIN_LIMIT, 1 << 15)
    w = to_dev(sp.w0)
    ctx.epoch(w, 0)
    assert ctx.take_device_flags() == lpc.OK
    ctx.close()
    again, _ = _epochs(sp, RESIDENT, epochs=1, m=4)
    assert np.array_equal(w.cpu().numpy(), again[0])
