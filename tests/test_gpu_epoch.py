"""GPU parity of whole epochs: Alg. 1 and Alg. 2/3 against the oracle, objective within 1e-4."""
import numpy as np
import pytest

import lpc_synth
from oracle import lpco
from _common import gpu_context, oracle_config, oracle_problem, to_dev

pytestmark = pytest.mark.gpu


def _run_both(sp, epochs, **over):
    ctx = gpu_context(sp, **over)
    p, _k = oracle_problem(sp)
    cfg = oracle_config(sp, **over)
    alpc = cfg.algo != lpco.ALGO_LPC
    w_o = sp.w0.copy()
    y_o, z_o = (sp.w0.copy(), sp.w0.copy()) if alpc else (None, None)
    w_g = to_dev(sp.w0)
    y_g, z_g = (to_dev(sp.w0), to_dev(sp.w0)) if alpc else (None, None)
    hist = []
    for s in range(epochs):
        lpco.epoch(p, cfg, w_o, s, y_o, z_o)
        ctx.epoch(w_g, s, y_g, z_g)
        hist.append((lpco.objective(p, w_o), ctx.objective(w_g), lpco.objective(p, w_g.cpu().numpy())))
    assert ctx.take_device_flags() == 0
    ctx.close()
    return hist, w_o, w_g.cpu().numpy()


def test_c1_ten_epochs_objective_parity():
    sp = lpc_synth.make("c1")      # the full tiny config: n=1024, d=64, N=4, B=16, b=2, c*sigma clip, 10 epochs
    hist, w_o, w_g = _run_both(sp, sp.epochs)
    for P_o, P_g, P_og in hist:
        assert abs(P_g - P_o) <= 1e-4 * abs(P_o)       # spec tolerance
        assert abs(P_g - P_og) <= 1e-5 * abs(P_og)     # the GPU objective of its own iterate
    assert hist[-1][0] < hist[0][0]
    assert np.abs(w_g - w_o).max() <= 1e-3 * max(1.0, np.abs(w_o).max())


@pytest.mark.parametrize("bits,clip_mode,clip", [(32, 0, 1.0), (4, 0, 0.9), (3, 1, 2.0)])
def test_lpc_epochs_small_dense(bits, clip_mode, clip):
    sp = lpc_synth.make("c2", n=2048, d=512, N=4, B=16)
    hist, w_o, w_g = _run_both(sp, 4, bits=bits, clip_mode=clip_mode, clip=clip)
    for P_o, P_g, _ in hist:
        assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    assert hist[-1][0] < hist[0][0]


def test_quantization_off_tracks_the_oracle_closely():
    # without stochastic rounding the two trajectories differ by float rounding only
    sp = lpc_synth.make("c1", n=512, d=40, N=4, B=8)
    hist, w_o, w_g = _run_both(sp, 5, bits=32)
    assert np.abs(w_g - w_o).max() <= 2e-5 * max(1.0, np.abs(w_o).max())


@pytest.mark.parametrize("algo", [lpco.ALGO_ALPC_SC, lpco.ALGO_ALPC_GC])
@pytest.mark.parametrize("bits", [32, 3])
def test_alpc_epochs_ridge(algo, bits):
    sp = lpc_synth.make("c4", n=2048, d=256, N=4, B=16)
    hist, w_o, w_g = _run_both(sp, 4, algo=algo, bits=bits, tau2=0.5)
    for P_o, P_g, _ in hist:
        assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    assert hist[-1][0] < hist[0][0]
    if bits == 32:
        assert np.abs(w_g - w_o).max() <= 5e-5 * max(1.0, np.abs(w_o).max())


def test_epoch_is_reproducible():
    import torch
    sp = lpc_synth.make("c2", n=1024, d=256, N=4, B=16)
    ctx = gpu_context(sp)
    a, b = to_dev(sp.w0), to_dev(sp.w0)
    ctx.epoch(a, 0); ctx.epoch(a, 1)
    ctx.epoch(b, 0); ctx.epoch(b, 1)
    assert torch.equal(a, b)
    ctx.close()


@pytest.mark.parametrize("d,B,over", [
    (50_000, 100, {}),                                  # sparse inner iteration, two rounds of rows per worker
    (50_000, 16, dict(scheme=lpco.SCHEME_B)),           # dense-U worker pass (shared scale), large d
    (2048, 70, {}),                                     # small d: many rows of a batch share columns
    (3000, 32, dict(algo=lpco.ALGO_ALPC_GC, L=0.25, tau2=0.5)),
])
def test_csr_epoch_is_reproducible(d, B, over):
    """CSR data: the snapshot gradient and the workers' differences are summed in a fixed order (no float atomics
    whose arrival order could matter), so two runs give the same bits -- and with them the same stochastic
    rounding decisions and the same iterates."""
    import torch
    sp = lpc_synth.make("c3", n=4096, d=d, nnz_mean=30, N=4, B=B)
    runs = []
    for _ in range(3):
        ctx = gpu_context(sp, m=5, **over)
        alpc = ctx.config.algo != 0
        w = to_dev(sp.w0)
        y, z = (to_dev(sp.w0), to_dev(sp.w0)) if alpc else (None, None)
        for s in range(3):
            ctx.epoch(w, s, y, z)
        mu = torch.zeros(sp.d, device="cuda")
        ctx.full_grad(w, mu, None, None)
        U = torch.zeros(sp.N, lpco.d_pad(sp.d), device="cuda")
        ctx.worker_vr_grad(w, to_dev(sp.w0), None, 7, 3, U, None)
        runs.append((w.clone(), mu, U))
        ctx.close()
    assert runs[0][0].abs().max().item() > 0
    for other in runs[1:]:
        for a, b in zip(runs[0], other):
            assert torch.equal(a, b)


@pytest.mark.parametrize("d,bits", [(2048, 2), (40_000, 2), (40_000, 32)])
def test_lpc_epochs_csr(d, bits):
    # sparse rows: small-d single-launch exchange and the large-d path
    sp = lpc_synth.make("c3", n=4096, d=d, nnz_mean=20, N=4, B=16)
    hist, w_o, w_g = _run_both(sp, 3, bits=bits)
    for P_o, P_g, _ in hist:
        assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    assert hist[-1][0] < hist[0][0]


@pytest.mark.parametrize("scheme", [lpco.SCHEME_B, lpco.SCHEME_C])
@pytest.mark.parametrize("algo", [lpco.ALGO_LPC, lpco.ALGO_ALPC_GC])
def test_shared_scale_schemes_epochs(scheme, algo):
    # Sec. 4.2 (b), (c): parameter-server style exchange with one scale factor for all workers
    name = "c2" if algo == lpco.ALGO_LPC else "c4"
    sp = lpc_synth.make(name, n=2048, d=512, N=4, B=16)
    hist, w_o, w_g = _run_both(sp, 3, algo=algo, scheme=scheme, bits=4, clip_mode=0, clip=1.0, tau2=0.5)
    for P_o, P_g, _ in hist:
        assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    assert hist[-1][0] < hist[0][0]


@pytest.mark.parametrize("bits,clip_mode,clip,n_full", [(2, 0, 1.0, 0), (5, 0, 0.8, 0), (4, 1, 2.0, 0), (3, 0, 1.0, 2048)])
def test_sparse_inner_iteration_matches_the_oracle_coordinate_by_coordinate(bits, clip_mode, clip, n_full):
    """CSR rows that touch few columns take the sparse passes (head partials + marked tail segments).  The
    oracle works on dense vectors; the iterates must agree coordinate by coordinate except where a float
    rounding difference in u (scatter order) flips a stochastic rounding decision: such a flip moves one
    coordinate of w by eta*delta/N, so only a handful of coordinates may differ, and by little."""
    sp = lpc_synth.make("c3", n=4096, d=50_000, nnz_mean=20, N=4, B=16)
    over = dict(bits=bits, clip_mode=clip_mode, clip=clip, m=6, n_full=n_full)
    hist, w_o, w_g = _run_both(sp, 2, **over)
    for P_o, P_g, _ in hist:
        assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    scale = max(np.abs(w_o).max(), 1e-12)
    diff = np.abs(w_g - w_o)
    assert np.count_nonzero(w_o) > 1000                      # the iterate has moved on head and tail columns
    assert np.count_nonzero(w_o[8192:]) > 100
    assert (diff > 1e-5 * scale).mean() <= 2e-3              # a few flipped decisions at most
    assert diff.max() <= 0.05 * scale
    # the same support (the L1 prox zeroes exactly the same coordinates, up to those few)
    assert np.count_nonzero((w_o == 0) != (w_g == 0)) <= 2e-3 * sp.d


@pytest.mark.parametrize("nnz_mean,B", [(80, 16), (160, 70)])
def test_sparse_inner_iteration_with_long_rows_and_the_wide_head(nnz_mean, B):
    """d >= 2^17: the sparse passes treat 16384 leading columns densely.  Rows longer than 64 entries: the worker
    pass stages a row's first 64 pairs and takes the rest from memory (head and tail wavefronts both), B = 70 adds
    a second workgroup per worker, hence a second tail plane.  Same agreement with the dense oracle as above."""
    sp = lpc_synth.make("c3", n=2048, d=140_000, nnz_mean=nnz_mean, N=4, B=B)
    rp = sp.csr[0]
    assert (np.diff(rp) > 64).mean() > 0.1
    hist, w_o, w_g = _run_both(sp, 2, bits=3, m=5)
    for P_o, P_g, _ in hist:
        assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    scale = max(np.abs(w_o).max(), 1e-12)
    diff = np.abs(w_g - w_o)
    assert np.count_nonzero(w_o[:64]) > 32 and np.count_nonzero(w_o[64:16384]) > 1000
    assert np.count_nonzero(w_o[16384:]) > 100
    assert (diff > 1e-5 * scale).mean() <= 2e-3
    assert diff.max() <= 0.05 * scale
    assert np.count_nonzero((w_o == 0) != (w_g == 0)) <= 2e-3 * sp.d


@pytest.mark.parametrize("scheme,bits,clip_mode,clip,d", [
    (lpco.SCHEME_B, 3, 0, 1.0, 50_000), (lpco.SCHEME_C, 4, 0, 0.9, 50_000), (lpco.SCHEME_B, 2, 1, 2.0, 50_000),
    (lpco.SCHEME_C, 3, 0, 1.0, 140_000)])                      # d >= 2^17: 16384 dense head columns
def test_sparse_inner_iteration_with_a_shared_scale_factor(scheme, bits, clip_mode, clip, d):
    """Sec. 4.2 (b), (c) on CSR rows that touch few columns: the sparse worker, statistics and quantizer passes with
    delta = max_i delta_i, then the integer-sum receiver (eq. (5) for scheme (c)).  Coordinate-level agreement
    with the oracle as for scheme (a); the same bits run to run."""
    import torch
    sp = lpc_synth.make("c3", n=4096, d=d, nnz_mean=20, N=4, B=16)
    over = dict(bits=bits, clip_mode=clip_mode, clip=clip, m=6, scheme=scheme)
    hist, w_o, w_g = _run_both(sp, 2, **over)
    for P_o, P_g, _ in hist:
        assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    scale = max(np.abs(w_o).max(), 1e-12)
    diff = np.abs(w_g - w_o)
    assert np.count_nonzero(w_o) > 1000 and np.count_nonzero(w_o[8192:]) > 100
    assert (diff > 1e-5 * scale).mean() <= 2e-3
    assert diff.max() <= 0.05 * scale
    _h, _w, w_again = _run_both(sp, 2, **over)
    assert np.array_equal(w_g, w_again)


@pytest.mark.parametrize("algo,scheme,bits,clip_mode,clip,B", [
    (lpco.ALGO_ALPC_GC, lpco.SCHEME_A, 3, 0, 1.0, 16), (lpco.ALGO_ALPC_SC, lpco.SCHEME_A, 4, 1, 2.0, 16),
    (lpco.ALGO_ALPC_GC, lpco.SCHEME_B, 4, 0, 0.9, 16), (lpco.ALGO_ALPC_GC, lpco.SCHEME_C, 2, 0, 1.0, 16),
    (lpco.ALGO_ALPC_GC, lpco.SCHEME_A, 3, 0, 1.0, 70),         # B = 70: two workgroups (planes) per vector
    (lpco.ALGO_ALPC_GC, lpco.SCHEME_A, 3, 0, 1.0, -70)])       # ... and d >= 2^17: 16384 dense head columns
def test_sparse_inner_iteration_of_alpc_svrg(algo, scheme, bits, clip_mode, clip, B):
    """Alg. 2 / Alg. 3 on CSR rows that touch few columns: the workers' vectors AND the shared batch's
    full-precision difference take the sparse worker and statistics passes; coordinate-level agreement of x~, y and z
    with the oracle (up to a few flipped rounding decisions) and the same bits run to run."""
    d, B = (140_000, -B) if B < 0 else (50_000, B)
    sp = lpc_synth.make("c3", n=4096, d=d, nnz_mean=20, N=4, B=B)
    over = dict(algo=algo, scheme=scheme, bits=bits, clip_mode=clip_mode, clip=clip, m=6, tau2=0.5, L=0.25,
                sigma=1e-3 if algo == lpco.ALGO_ALPC_SC else 0.0)
    runs = []
    for _ in range(2):
        ctx = gpu_context(sp, **over)
        w_g, y_g, z_g = to_dev(sp.w0), to_dev(sp.w0), to_dev(sp.w0)
        for s in range(2):
            ctx.epoch(w_g, s, y_g, z_g)
        assert ctx.take_device_flags() == 0
        P_g = ctx.objective(w_g)
        ctx.close()
        runs.append((w_g.cpu().numpy(), y_g.cpu().numpy(), z_g.cpu().numpy(), P_g))
    p, _k = oracle_problem(sp)
    cfg = oracle_config(sp, **over)
    w_o, y_o, z_o = sp.w0.copy(), sp.w0.copy(), sp.w0.copy()
    for s in range(2):
        lpco.epoch(p, cfg, w_o, s, y_o, z_o)
    P_o = lpco.objective(p, w_o)
    assert abs(runs[0][3] - P_o) <= 1e-4 * abs(P_o)
    for got, want in zip(runs[0][:3], (w_o, y_o, z_o)):
        scale = max(np.abs(want).max(), 1e-12)
        diff = np.abs(got - want)
        assert np.count_nonzero(want) > 1000
        assert (diff > 1e-5 * scale).mean() <= 2e-3
        assert diff.max() <= 0.05 * scale
    for a, b in zip(runs[0][:3], runs[1][:3]):
        assert np.array_equal(a, b)
