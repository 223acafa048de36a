"""Pins for the oracle's optimizer loops: Alg. 1, Alg. 2, Alg. 3 (CPU only)."""
import numpy as np
import pytest

import lpc_synth
from oracle import lpco


def _problem_from(sp):
    if sp.csr is not None:
        return lpco.make_problem(sp.loss, sp.y, sp.lambda1, sp.lambda2, csr=(*sp.csr, sp.d))
    return lpco.make_problem(sp.loss, sp.y, sp.lambda1, sp.lambda2, X=sp.X, d=sp.d, mlp_dims=sp.mlp_dims)


def _config_from(sp, **over):
    kw = dict(algo=sp.algo, N=sp.N, B=sp.B, m=sp.m, bits=sp.bits, clip_mode=sp.clip_mode, clip=sp.clip, eta=sp.eta,
              L=sp.L, seed=sp.seed, n_full=sp.n_full)
    kw.update(over)
    return lpco.make_config(**kw)


def _soft(p, thr):
    return np.sign(p) * np.maximum(np.abs(p) - thr, 0.0)


def _slope(loss, z, y):
    return -y / (1 + np.exp(y * z)) if loss == lpco.LOSS_LOGISTIC else z - y


def _fista(X, y, loss, l1, l2, L, iters=20000):
    """Brute-force minimiser of eq. (1) in float64 (accelerated proximal gradient, run to stagnation)."""
    n, d = X.shape
    w = np.zeros(d); v = w.copy(); t = 1.0
    step = 1.0 / L
    for _ in range(iters):
        g = X.T @ _slope(loss, X @ v, y) / n
        w_new = _soft(v - step * g, step * l1) / (1 + step * l2)
        t_new = (1 + np.sqrt(1 + 4 * t * t)) / 2
        v = w_new + (t - 1) / t_new * (w_new - w)
        if np.abs(w_new - w).max() < 1e-15:
            w = w_new
            break
        w, t = w_new, t_new
    return w


def _objective64(X, y, loss, l1, l2, w):
    z = X @ w
    f = np.mean(np.logaddexp(0, -y * z)) if loss == lpco.LOSS_LOGISTIC else 0.5 * np.mean((z - y) ** 2)
    return f + l1 * np.abs(w).sum() + 0.5 * l2 * (w ** 2).sum()


# ---------------------------------------------------------------- Alg. 1

def test_first_inner_iteration_is_an_exact_proximal_gradient_step():
    # x_0 = x~ makes u_0^i = 0, hence u~_0 = 0 for any b: with m = 1 the epoch is
    # x~ <- prox_{eta h}(x~ - eta grad f(x~)), whatever the quantizer settings
    sp = lpc_synth.make("c1", n=128, d=20, N=4, B=8)
    p, _k = _problem_from(sp)
    w0 = (0.1 * np.random.default_rng(0).standard_normal(sp.d)).astype(np.float32)
    X, y = sp.X.astype(np.float64), sp.y.astype(np.float64)
    g = X.T @ _slope(sp.loss, X @ w0.astype(np.float64), y) / sp.n
    expect = _soft(w0 - sp.eta * g, sp.eta * sp.lambda1) / (1 + sp.eta * sp.lambda2)
    for bits in (2, 4, 32):
        w = w0.copy()
        lpco.epoch(p, _config_from(sp, m=1, bits=bits), w, 0)
        assert np.allclose(w, expect, rtol=0, atol=2e-7)


def test_quantization_off_is_minibatch_prox_svrg():
    # with u~_t = (1/N) sum_i u_t^i Alg. 1 is the minibatch prox-SVRG of Theorem 1 (batch N*B per step).
    # Separate float64 implementation, same index streams.
    sp = lpc_synth.make("c1", n=256, d=24, N=4, B=8)
    p, _k = _problem_from(sp)
    cfg = _config_from(sp, bits=32)
    X, y = sp.X.astype(np.float64), sp.y.astype(np.float64)
    w_or = sp.w0.copy()
    w_snap = sp.w0.astype(np.float64)
    for s in range(3):
        lpco.epoch(p, cfg, w_or, s)
        mu = X.T @ _slope(sp.loss, X @ w_snap, y) / sp.n
        x = w_snap.copy()
        for t in range(sp.m):
            idx = np.concatenate([lpco.sample_batch(sp.seed, s, t, lpco.TAG_BATCH, i, sp.B, sp.n)
                                  for i in range(sp.N)])
            coef = _slope(sp.loss, X[idx] @ x, y[idx]) - _slope(sp.loss, X[idx] @ w_snap, y[idx])
            v = (coef[:, None] * X[idx]).mean(axis=0) + mu
            x = _soft(x - sp.eta * v, sp.eta * sp.lambda1) / (1 + sp.eta * sp.lambda2)
        w_snap = x
        assert np.allclose(w_or, w_snap, rtol=0, atol=5e-6 * max(1.0, np.abs(w_snap).max()))


@pytest.mark.parametrize("bits,clip_mode,clip", [(32, 0, 1.0), (4, 0, 1.0), (4, 0, 0.9), (2, 1, 2.0)])
def test_lpc_svrg_reaches_the_minimiser_on_a_tiny_problem(bits, clip_mode, clip):
    sp = lpc_synth.make("c1", n=256, d=16, N=4, B=8)
    p, _k = _problem_from(sp)
    X, y = sp.X.astype(np.float64), sp.y.astype(np.float64)
    l1, l2 = 1e-2, 1e-2
    p.lambda1, p.lambda2 = l1, l2
    w_star = _fista(X, y, sp.loss, l1, l2, sp.L)
    P_star = _objective64(X, y, sp.loss, l1, l2, w_star)
    w = sp.w0.copy()
    cfg = _config_from(sp, bits=bits, clip_mode=clip_mode, clip=clip, eta=1.0 / sp.L)
    P0 = lpco.objective(p, w)
    gaps = []
    for s in range(150):
        lpco.epoch(p, cfg, w, s)
        gaps.append(lpco.objective(p, w) - P_star)
    assert gaps[-1] >= -1e-9
    assert gaps[-1] <= (1e-6 if bits == 32 else 2e-5) * max(1.0, P0)
    assert gaps[-1] < 1e-3 * (P0 - P_star)


def test_epoch_reports_table1_bits():
    sp = lpc_synth.make("c1", n=128, d=20, N=4, B=8)
    p, _k = _problem_from(sp)
    w = sp.w0.copy()
    for bits, scheme, per_iter in [(2, lpco.SCHEME_A, (32 + 2 * 20) * 4 * 3), (3, lpco.SCHEME_C, 4 * (64 + 2 * 3 * 20)),
                                   (3, lpco.SCHEME_B, 4 * (64 + 2 * 3 * 20 + 20 * 2)), (32, 0, 32 * 20 * 4 * 3)]:
        sent = lpco.epoch(p, _config_from(sp, bits=bits, scheme=scheme, clip_mode=0, clip=1.0), w, 0)
        assert sent == sp.m * per_iter


def test_shared_scale_schemes_also_converge():
    sp = lpc_synth.make("c1", n=256, d=16, N=4, B=8)
    p, _k = _problem_from(sp)
    p.lambda1, p.lambda2 = 1e-2, 1e-2
    X, y = sp.X.astype(np.float64), sp.y.astype(np.float64)
    P_star = _objective64(X, y, sp.loss, 1e-2, 1e-2, _fista(X, y, sp.loss, 1e-2, 1e-2, sp.L))
    for scheme in (lpco.SCHEME_B, lpco.SCHEME_C):
        w = sp.w0.copy()
        cfg = _config_from(sp, bits=4, clip_mode=0, clip=1.0, scheme=scheme, eta=1.0 / sp.L)
        for s in range(150):
            lpco.epoch(p, cfg, w, s)
        assert 0 <= lpco.objective(p, w) - P_star + 1e-9 <= 5e-5


def test_epochs_are_reproducible_and_restartable():
    # all randomness is a function of (seed, epoch, iter, worker, index): re-running an epoch from the
    # same state gives the same bits
    sp = lpc_synth.make("c1", n=128, d=20, N=4, B=8)
    p, _k = _problem_from(sp)
    cfg = _config_from(sp)
    a = sp.w0.copy()
    lpco.epoch(p, cfg, a, 0)
    mid = a.copy()
    lpco.epoch(p, cfg, a, 1)
    b = mid.copy()
    lpco.epoch(p, cfg, b, 1)
    assert np.array_equal(a, b)
    c = mid.copy()
    lpco.epoch(p, cfg, c, 2)
    assert not np.array_equal(a, c)


# ---------------------------------------------------------------- Alg. 2 / Alg. 3

def _ridge(n=256, d=12, seed=0, N=4, B=8, l2=0.05):
    sp = lpc_synth.make("c4", n=n, d=d, N=N, B=B, seed=seed)
    sp.lambda2 = l2
    return sp


def test_alpc_parameter_rules():
    sp = _ridge()
    p, _k = _problem_from(sp)
    # Alg. 3 step 3: tau1_s = 2/(s+4), alpha_s = 1/(6 L tau1_s); snapshot is a plain mean (theta = 1)
    for s in range(5):
        t1, t2, a, th = lpco.alpc_params(p, _config_from(sp, algo=lpco.ALGO_ALPC_GC, tau2=0.5), s)
        assert np.isclose(t1, 2 / (s + 4)) and np.isclose(a, 1 / (6 * sp.L * t1), rtol=1e-6) and th == 1.0
        assert t2 == 0.5 and t1 + t2 <= 1 + 1e-7
    # experiments' rule alpha = lrn_rate / tau1
    t1, _, a, _ = lpco.alpc_params(p, _config_from(sp, algo=lpco.ALGO_ALPC_GC, alpha=0.01), 2)
    assert np.isclose(a, 0.01 / t1, rtol=1e-6)
    # Theorem 3: tau1 = sqrt(m sigma / 6L), alpha = 1/(6 tau1 L), tau2 = min(1/2, 5 zeta/3 + 1/2B), theta = 1 + alpha sigma
    cfg = _config_from(sp, algo=lpco.ALGO_ALPC_SC, m=2, bits=8, clip_mode=0, clip=1.0)
    t1, t2, a, th = lpco.alpc_params(p, cfg, 0)
    sigma = sp.lambda2
    assert np.isclose(t1, min(0.5, np.sqrt(2 * sigma / (6 * sp.L))), rtol=1e-6)
    assert np.isclose(a, 1 / (6 * t1 * sp.L), rtol=1e-5) and np.isclose(th, 1 + a * sigma, rtol=1e-6)
    zeta = sp.d / (4 * 127 ** 2) + 1 / (sp.N * sp.B)
    assert np.isclose(t2, min(0.5, 5 * zeta / 3 + 1 / (2 * sp.B)), rtol=1e-6)


def test_alpc_with_one_inner_iteration():
    # m = 1: x_1 = tau1 z_0 + tau2 x~ + (1-tau1-tau2) y_0 = x~ when y_0 = z_0 = x~; u = 0 there, so
    # y_1 = prox_{h/(4L)}(x~ - grad f(x~)/(4L)), z_1 = prox_{alpha h}(x~ - alpha grad f(x~)), x~^1 = y_1
    sp = _ridge()
    p, _k = _problem_from(sp)
    cfg = _config_from(sp, algo=lpco.ALGO_ALPC_SC, m=1, bits=3, clip_mode=0, clip=0.9)
    rng = np.random.default_rng(1)
    w0 = (0.2 * rng.standard_normal(sp.d)).astype(np.float32)
    w, y, z = w0.copy(), w0.copy(), w0.copy()
    _, _, alpha, _ = lpco.alpc_params(p, cfg, 0)
    lpco.epoch(p, cfg, w, 0, y, z)
    X, t = sp.X.astype(np.float64), sp.y.astype(np.float64)
    g = X.T @ (X @ w0.astype(np.float64) - t) / sp.n
    y_ref = (w0 - g / (4 * sp.L)) / (1 + sp.lambda2 / (4 * sp.L))
    z_ref = (w0 - alpha * g) / (1 + alpha * sp.lambda2)
    assert np.allclose(y, y_ref, atol=3e-7) and np.allclose(z, z_ref, atol=3e-7)
    assert np.array_equal(w, y)     # the weighted mean of a single iterate


@pytest.mark.parametrize("algo", [lpco.ALGO_ALPC_SC, lpco.ALGO_ALPC_GC])
def test_alpc_quantization_off_matches_separate_implementation(algo):
    sp = _ridge(n=128, d=10)
    p, _k = _problem_from(sp)
    cfg = _config_from(sp, algo=algo, bits=32, tau2=0.5)
    X, t = sp.X.astype(np.float64), sp.y.astype(np.float64)
    lam2, L = sp.lambda2, sp.L
    w_or, y_or, z_or = sp.w0.copy(), sp.w0.copy(), sp.w0.copy()
    xs = sp.w0.astype(np.float64); y = xs.copy(); z = xs.copy()
    for s in range(3):
        t1, t2, alpha, theta = lpco.alpc_params(p, cfg, s)
        lpco.epoch(p, cfg, w_or, s, y_or, z_or)
        mu = X.T @ (X @ xs - t) / sp.n
        acc, wsum = np.zeros(sp.d), 0.0
        for it in range(sp.m):
            x = t1 * z + t2 * xs + (1 - t1 - t2) * y
            idx = np.concatenate([lpco.sample_batch(sp.seed, s, it, lpco.TAG_BATCH, i, sp.B, sp.n)
                                  for i in range(sp.N)])
            v = ((X[idx] @ (x - xs))[:, None] * X[idx]).mean(axis=0) + mu
            J = lpco.sample_batch(sp.seed, s, it, lpco.TAG_SHARED, 0xFFFFFF, sp.B, sp.n)
            vhat = ((X[J] @ (x - xs))[:, None] * X[J]).mean(axis=0) + mu
            y = (x - v / (4 * L)) / (1 + lam2 / (4 * L))
            z = (z - alpha * vhat) / (1 + alpha * lam2)
            acc += theta ** it * y
            wsum += theta ** it
        xs = acc / wsum
        tol = 2e-5 * max(1.0, np.abs(xs).max())
        assert np.allclose(w_or, xs, atol=tol) and np.allclose(y_or, y, atol=tol) and np.allclose(z_or, z, atol=tol)


@pytest.mark.parametrize("algo", [lpco.ALGO_ALPC_SC, lpco.ALGO_ALPC_GC])
def test_alpc_reaches_the_ridge_closed_form(algo):
    sp = _ridge(n=256, d=12, l2=0.05)
    p, _k = _problem_from(sp)
    X, t = sp.X.astype(np.float64), sp.y.astype(np.float64)
    w_star = np.linalg.solve(X.T @ X / sp.n + sp.lambda2 * np.eye(sp.d), X.T @ t / sp.n)
    P_star = _objective64(X, t, sp.loss, 0.0, sp.lambda2, w_star)
    cfg = _config_from(sp, algo=algo, bits=4, clip_mode=0, clip=1.0, tau2=0.5)
    w, y, z = sp.w0.copy(), sp.w0.copy(), sp.w0.copy()
    P0 = lpco.objective(p, w)
    for s in range(60):
        lpco.epoch(p, cfg, w, s, y, z)
    gap = lpco.objective(p, w) - P_star
    assert -1e-9 <= gap <= 1e-3 * (P0 - P_star)


def test_double_sampling_gradient_is_unbiased():
    # E[v^] = grad f(x): v^ = (1/B) sum_{j in J} [grad f_j(x) - grad f_j(x~)] + grad f(x~)
    sp = _ridge(n=64, d=6)
    p, _k = _problem_from(sp)
    rng = np.random.default_rng(3)
    x = rng.standard_normal(sp.d).astype(np.float32)
    xs = (x + 0.3 * rng.standard_normal(sp.d)).astype(np.float32)
    mu_s = lpco.full_grad(p, xs)[0].astype(np.float64)
    target = lpco.full_grad(p, x)[0].astype(np.float64)
    cfg = _config_from(sp, B=4)
    acc, acc2, T = np.zeros(sp.d), np.zeros(sp.d), 6000
    for it in range(T):
        UJ, _ = lpco.worker_vr_grad(p, cfg, x, xs, 0, it, tag=lpco.TAG_SHARED)
        vhat = UJ[0, :sp.d] + mu_s
        acc += vhat
        acc2 += vhat ** 2
    mean = acc / T
    se = np.sqrt(np.maximum(acc2 / T - mean ** 2, 1e-12) / T)
    assert np.all(np.abs(mean - target) <= 4.5 * se)


# ---------------------------------------------------------------- traces of delta and d_lambda (Sec. 3.2)

def test_traced_epoch_takes_the_same_steps_and_starts_with_a_zero_message():
    sp = lpc_synth.make("c2", n=512, d=96, N=4, B=8)
    p, _k = _problem_from(sp)
    cfg = _config_from(sp, m=6, bits=3, clip_mode=lpco.CLIP_LAMBDA, clip=0.7)
    w_a, w_b = sp.w0.copy(), sp.w0.copy()
    lpco.epoch(p, cfg, w_a, 0)
    dtr, ntr = lpco.epoch_traced(p, cfg, w_b, 0)
    assert np.array_equal(w_a, w_b)
    assert dtr.shape == (6, 4) and ntr.shape == (6, 4)
    # x_0 = x~: every worker's first message is the zero vector, nothing to scale or clip
    assert np.all(dtr[0] == 0.0) and np.all(ntr[0] == 0)
    assert np.all(dtr[1:] > 0.0)
    # lambda < 1 cuts at least the largest coordinate of every later message
    assert np.all(ntr[1:] >= 1)


def test_trace_rows_are_eq3_and_the_clip_count_written_out_by_hand():
    # iteration t = 1 recomputed in float64 numpy: x_1 = prox(x~ - eta*mu) (the first message is zero),
    # u^i = grad f_{B_i}(x_1) - grad f_{B_i}(x~), delta_i = lambda*|u^i|_inf/(2^(b-1)-1), d_lambda = #{u_j outside dom(delta_i, b)}
    sp = lpc_synth.make("c2", n=256, d=48, N=3, B=8)
    p, _k = _problem_from(sp)
    lam, b = 0.6, 4
    cfg = _config_from(sp, m=2, bits=b, clip_mode=lpco.CLIP_LAMBDA, clip=lam)
    w0 = (0.2 * np.random.default_rng(5).standard_normal(sp.d)).astype(np.float32)
    w = w0.copy()
    dtr, ntr = lpco.epoch_traced(p, cfg, w, 7)
    X, y = sp.X.astype(np.float64), sp.y.astype(np.float64)
    snap = w0.astype(np.float64)
    mu = X.T @ _slope(sp.loss, X @ snap, y) / sp.n
    step = float(sp.eta)
    x1 = _soft(snap - step * mu, step * sp.lambda1) / (1 + step * sp.lambda2)
    x1 = x1.astype(np.float32).astype(np.float64)          # the iterate is kept in float
    for i in range(3):
        idx = lpco.sample_batch(sp.seed, 7, 1, lpco.TAG_BATCH, i, 8, sp.n)
        Xb, yb = X[idx], y[idx]
        u = Xb.T @ (_slope(sp.loss, Xb @ x1, yb) - _slope(sp.loss, Xb @ snap, yb)) / 8
        amax = np.abs(u).max()
        assert dtr[1, i] == pytest.approx(lam * amax / (2 ** (b - 1) - 1), rel=2e-5)
        # coordinates within 1e-4 of the threshold could go either way in float: none here, or skip the count
        # outside dom(delta, b) = [-2^(b-1)*delta, (2^(b-1)-1)*delta]: the codebook has one more negative point
        hi, lo = lam * amax, -(2 ** (b - 1)) * lam * amax / (2 ** (b - 1) - 1)
        near = (np.abs(u - hi) < 1e-4 * amax) | (np.abs(u - lo) < 1e-4 * amax)
        if not near.any():
            assert ntr[1, i] == int((u > hi).sum() + (u < lo).sum())


def test_no_clipping_at_lambda_one_and_shared_delta_under_scheme_b():
    sp = lpc_synth.make("c2", n=512, d=64, N=4, B=8)
    p, _k = _problem_from(sp)
    w = sp.w0.copy()
    dtr, ntr = lpco.epoch_traced(p, _config_from(sp, m=5, bits=3, clip_mode=lpco.CLIP_LAMBDA, clip=1.0), w, 0)
    assert np.all(ntr == 0)                                  # Sec. 4.1: lambda = 1 is LP-SVRG, d_lambda = 0
    w = sp.w0.copy()
    dtr_b, _ = lpco.epoch_traced(p, _config_from(sp, m=5, bits=3, clip_mode=lpco.CLIP_LAMBDA, clip=1.0,
                                                 scheme=lpco.SCHEME_B), w, 0)
    assert np.all(dtr_b == dtr_b[:, :1])                     # one scale factor per iteration: max_i delta_i
    assert np.all(dtr_b[1] == dtr[1].max())                  # iteration 1 starts from the same iterate


def test_trace_is_zero_with_quantization_off():
    sp = lpc_synth.make("c1", n=256, d=20, N=2, B=8)
    p, _k = _problem_from(sp)
    w = sp.w0.copy()
    dtr, ntr = lpco.epoch_traced(p, _config_from(sp, m=3, bits=32), w, 0)
    assert np.all(dtr == 0.0) and np.all(ntr == 0)


def test_entropy_coded_sizes_in_the_trace():
    sp = lpc_synth.make("c2", n=512, d=200, N=3, B=8)
    p, _k = _problem_from(sp)
    w = sp.w0.copy()
    cfg = _config_from(sp, m=5, bits=4, clip_mode=lpco.CLIP_LAMBDA, clip=1.0)
    _d, _n, coded = lpco.epoch_traced(p, cfg, w, 0, coded=True)
    # the zero message of t = 0 uses one symbol: a lone symbol costs one bit per coordinate
    assert np.all(coded[0] == sp.d)
    # any prefix code spends at least one bit per coordinate and an optimal one no more than the fixed b bits
    assert np.all(coded[1:] >= sp.d) and np.all(coded[1:] <= 4 * sp.d)
    # the rows are the sizes lpco.huffman_bits gives for the messages an identical epoch produces step by step
    w2 = sp.w0.copy()
    mu, _, _ = lpco.full_grad(p, w2)
    x = w2.copy()
    for t in range(2):
        U, stats = lpco.worker_vr_grad(p, cfg, x, w2, 0, t)
        packed, delta, _c, _r = lpco.quantize_clip(U, sp.d, 4, lpco.CLIP_LAMBDA, 1.0, seed=sp.seed, epoch=0, iter_=t,
                                                   stats=stats)
        for i in range(3):
            size, _lens = lpco.huffman_bits(lpco.code_histogram(packed[i], sp.d, 4))
            assert coded[t, i] == size
        x = lpco.prox_step(x, lpco.dequantize_avg(packed, delta, sp.d, 4), mu, sp.eta, sp.lambda1, sp.lambda2)
    w3 = sp.w0.copy()
    _d, _n, coded32 = lpco.epoch_traced(p, _config_from(sp, m=2, bits=32), w3, 0, coded=True)
    assert np.all(coded32 == 32 * sp.d)
