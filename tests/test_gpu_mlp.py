"""GPU parity of the MLP instance (matrix-core contractions) against the oracle."""
import ctypes as C

import numpy as np
import pytest

import lpc_synth
from oracle import lpco
from _common import gpu_context, oracle_config, oracle_problem, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,N,K,tA,tB", [(128, 128, 16, 0, 0), (64, 32, 8, 0, 0), (130, 257, 35, 0, 0),
                                          (200, 100, 77, 1, 0), (96, 300, 64, 0, 1), (33, 10, 1024, 1, 1),
                                          (2048, 10, 1024, 0, 0), (3, 5, 6, 0, 0), (512, 384, 256, 1, 0),
                                          (1024, 10, 256, 1, 0), (100, 7, 333, 1, 0), (77, 16, 100, 0, 0),
                                          (300, 3, 2051, 0, 0), (130, 13, 2000, 1, 0)])
def test_matrix_core_contraction(M, N, K, tA, tB):
    import torch
    from paper_1901_08924_amd import lpc
    rng = np.random.default_rng(M + N + K)
    A = rng.standard_normal((K, M) if tA else (M, K)).astype(np.float32)
    B = rng.standard_normal((N, K) if tB else (K, N)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    C0 = rng.standard_normal((M, N)).astype(np.float32)
    ref = (A.T if tA else A).astype(np.float64) @ (B.T if tB else B).astype(np.float64)
    fn = lpc.lib.lpc_debug_gemm      # declared in include/lpc.h, bound in lpc.EXPORTS
    dA, dB, dbias = to_dev(A), to_dev(B), to_dev(bias)
    st = torch.cuda.current_stream().cuda_stream
    for relu, acc in [(0, 0), (1, 0), (0, 1)]:
        dC = to_dev(C0)
        rc = fn(dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), M, N, K, A.shape[1], B.shape[1], N, tA, tB, 0.5,
                dbias.data_ptr(), relu, acc, st)
        assert rc == 0
        want = 0.5 * ref + bias
        if relu:
            want = np.maximum(want, 0)
        if acc:
            want = want + C0
        got = dC.cpu().numpy()
        assert np.abs(got - want).max() <= 2e-5 * max(1.0, np.abs(want).max())


# the last three take the fused last-layer launch (hidden width a multiple of 4, at most 1024; few classes)
MLPS = [((6, 5, 4, 3), 64, 2, 6), ((40, 33, 10), 200, 3, 20), ((300, 129, 70, 10), 640, 4, 32), ((17, 5), 90, 2, 9),
        ((64, 256, 10), 256, 2, 16), ((32, 1024, 12), 128, 2, 8), ((64, 10), 128, 2, 8)]


@pytest.mark.parametrize("dims,n,N,B", MLPS)
def test_mlp_full_gradient(dims, n, N, B):
    import torch
    sp = lpc_synth.make("c5", n=n, dims=dims, N=N, B=B, n_full=n)
    ctx = gpu_context(sp)
    p, _k = oracle_problem(sp)
    w = (sp.w0 + 0.05 * np.random.default_rng(1).standard_normal(sp.d)).astype(np.float32)
    mu = torch.full((sp.d,), 3.0, device="cuda")
    f = torch.zeros(1, dtype=torch.float64, device="cuda")
    ctx.full_grad(to_dev(w), mu, None, f)
    mu_o, _, f_o = lpco.full_grad(p, w)
    assert np.abs(mu.cpu().numpy() - mu_o).max() <= 1e-5 * np.abs(mu_o).max()
    assert abs(f.item() - f_o) <= 1e-5 * abs(f_o)
    assert abs(ctx.objective(to_dev(w)) - lpco.objective(p, w)) <= 1e-5 * abs(lpco.objective(p, w))
    ctx.close()


def test_mlp_full_gradient_partial_snapshot():
    import torch
    sp = lpc_synth.make("c5", n=500, dims=(40, 33, 10), N=3, B=20, n_full=150)     # the first 150 rows only
    ctx = gpu_context(sp)
    p, _k = oracle_problem(sp)
    mu = torch.zeros(sp.d, device="cuda")
    ctx.full_grad(to_dev(sp.w0), mu, None, None)
    mu_o, _, _ = lpco.full_grad(p, sp.w0, n_rows=150)
    assert np.abs(mu.cpu().numpy() - mu_o).max() <= 1e-5 * np.abs(mu_o).max()
    ctx.close()


@pytest.mark.parametrize("n", [10240, 9000])
def test_mlp_full_gradient_over_several_chunks_and_row_blocks(n):
    # the snapshot pass takes 8192 rows at a time; inside a chunk the weight-gradient product of the first
    # layer runs as 2048-row blocks side by side, the bias sums and the 10-column layer as 256-row blocks;
    # n = 9000 leaves a ragged second chunk (three whole 256-row blocks and 40 rows)
    import torch
    sp = lpc_synth.make("c5", n=n, dims=(64, 128, 10), N=3, B=16, n_full=n)
    ctx = gpu_context(sp)
    p, _k = oracle_problem(sp)
    w = (sp.w0 + 0.05 * np.random.default_rng(2).standard_normal(sp.d)).astype(np.float32)
    mu = torch.full((sp.d,), -7.0, device="cuda")
    f = torch.zeros(1, dtype=torch.float64, device="cuda")
    ctx.full_grad(to_dev(w), mu, None, f)
    mu_o, _, f_o = lpco.full_grad(p, w)
    assert np.abs(mu.cpu().numpy() - mu_o).max() <= 1e-5 * np.abs(mu_o).max()
    assert abs(f.item() - f_o) <= 1e-5 * abs(f_o)
    ctx.close()


@pytest.mark.parametrize("dims,n,N,B", MLPS)
def test_mlp_worker_vr_gradient(dims, n, N, B):
    import torch
    sp = lpc_synth.make("c5", n=n, dims=dims, N=N, B=B, n_full=n)
    ctx = gpu_context(sp)
    p, _k = oracle_problem(sp)
    cfg = oracle_config(sp)
    rng = np.random.default_rng(2)
    ws = (sp.w0 + 0.05 * rng.standard_normal(sp.d)).astype(np.float32)
    w = (ws + 0.02 * rng.standard_normal(sp.d)).astype(np.float32)
    dp = lpco.d_pad(sp.d)
    for kind, tag, rows in [(1, lpco.TAG_BATCH, N), (2, lpco.TAG_SHARED, 1)]:
        U = torch.full((N, dp), 9.0, device="cuda")
        stats = torch.zeros(N, 4, dtype=torch.float64, device="cuda")
        ctx.worker_vr_grad(to_dev(w), to_dev(ws), None, 1, 2, U, stats, kind=kind)
        U_o, _ = lpco.worker_vr_grad(p, cfg, w, ws, 1, 2, tag=tag)
        got = U.cpu().numpy()[:rows]
        for i in range(rows):
            idx = lpco.sample_batch(sp.seed, 1, 2, tag, 0xFFFFFF if tag == lpco.TAG_SHARED else i, B, n)
            sub, _ks = lpco.make_problem(sp.loss, sp.y[idx], X=np.ascontiguousarray(sp.X[idx]), d=sp.d, mlp_dims=dims)
            gB = lpco.full_grad(sub, w)[0]               # grad f_B(w): the scale of what is subtracted
            ref_scale = max(np.abs(gB).max(), np.abs(U_o[i]).max())
            assert np.abs(got[i] - U_o[i]).max() <= 2e-5 * ref_scale
            assert not got[i, sp.d:].any()
        assert np.array_equal(stats.cpu().numpy()[:rows, 0], np.abs(got[:, :sp.d]).max(axis=1).astype(np.float64))
    ctx.close()


def test_mlp_epochs():
    sp = lpc_synth.make("c5", n=512, dims=(40, 33, 10), N=4, B=16, n_full=256, m=8)
    import test_gpu_epoch
    hist, w_o, w_g = test_gpu_epoch._run_both(sp, 3)
    for P_o, P_g, _ in hist:
        assert abs(P_g - P_o) <= 1e-4 * abs(P_o)
    assert hist[-1][0] < hist[0][0]
