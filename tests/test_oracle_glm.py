"""Pins for the oracle's gradient oracles, objective and proximal step (CPU only)."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import lpco


def _logistic(seed=0, n=40, d=7, l1=1e-3, l2=1e-2):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d)).astype(np.float32)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    return X, y, lpco.make_problem(lpco.LOSS_LOGISTIC, y, l1, l2, X=X)


def _squared(seed=0, n=40, d=7, l2=1e-2):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d)).astype(np.float32)
    y = rng.standard_normal(n).astype(np.float32)
    return X, y, lpco.make_problem(lpco.LOSS_SQUARED, y, 0.0, l2, X=X)


# ---------------------------------------------------------------- prox (Sec. 3.3)

@pytest.mark.parametrize("l1,l2", [(0.3, 0.0), (0.0, 0.7), (0.2, 0.5), (0.0, 0.0)])
def test_prox_is_the_argmin_of_its_definition(l1, l2):
    # prox_{eta h}(p) = argmin_y h(y) + |y - p|^2/(2 eta), separable: brute force on a fine grid
    eta = 0.37
    pts = np.array([-2.0, -0.6, -0.1, -0.05, 0.0, 0.04, 0.11, 0.5, 1.7], dtype=np.float32)
    w = pts.copy()
    zero = np.zeros_like(w)
    out = lpco.prox_step(w, zero, zero, eta, l1, l2)   # v = 0: prox of the point itself
    grid = np.linspace(-3, 3, 600_001)
    for p, got in zip(pts.astype(np.float64), out):
        obj = l1 * np.abs(grid) + 0.5 * l2 * grid ** 2 + (grid - p) ** 2 / (2 * eta)
        assert abs(grid[np.argmin(obj)] - got) <= 2e-5


def test_prox_step_adds_mu_after_averaging_and_steps_against_v():
    # Alg. 1 steps 9-10: v = u~ + grad f(x~); x <- prox(x - eta v).  With h = 0 this is x - eta (u + mu).
    rng = np.random.default_rng(0)
    w, u, mu = (rng.standard_normal(50).astype(np.float32) for _ in range(3))
    out = lpco.prox_step(w, u, mu, 0.25, 0.0, 0.0)
    assert np.allclose(out, w.astype(np.float64) - 0.25 * (u.astype(np.float64) + mu), rtol=0, atol=1e-6)
    # L1 only: exact zeros inside the threshold
    out = lpco.prox_step(np.array([0.01, -0.01, 1.0], np.float32), np.zeros(3, np.float32), np.zeros(3, np.float32),
                         0.5, 0.1, 0.0)
    assert out[0] == 0 and out[1] == 0 and np.isclose(out[2], 0.95)


# ---------------------------------------------------------------- objective and full gradient

def test_objective_against_library_formulas():
    from sklearn.metrics import log_loss
    X, y, (p, _k) = _logistic(1)
    w = np.random.default_rng(2).standard_normal(7).astype(np.float32)
    prob = 1.0 / (1.0 + np.exp(-(X.astype(np.float64) @ w.astype(np.float64))))
    lib_f = log_loss((y > 0).astype(int), prob, labels=[0, 1])
    reg = 1e-3 * np.abs(w.astype(np.float64)).sum() + 0.5 * 1e-2 * (w.astype(np.float64) ** 2).sum()
    assert np.isclose(lpco.objective(p, w), lib_f + reg, rtol=1e-12)
    X, y, (p, _k) = _squared(1)
    resid = X.astype(np.float64) @ w.astype(np.float64) - y
    assert np.isclose(lpco.objective(p, w), 0.5 * np.mean(resid ** 2) + 0.5 * 1e-2 * (w.astype(np.float64) ** 2).sum(),
                      rtol=1e-12)


@pytest.mark.parametrize("maker", [_logistic, _squared])
def test_full_gradient_by_central_differences(maker):
    # mu = grad f (the smooth part only: h is handled by the prox)
    X, y, (p, keep) = maker(3, n=24, d=6)
    p.lambda1 = 0.0
    p.lambda2 = 0.0
    w = np.random.default_rng(4).standard_normal(6).astype(np.float32)
    mu, z, f = lpco.full_grad(p, w)
    assert np.isclose(f, lpco.objective(p, w), rtol=1e-12)
    assert np.allclose(z, X.astype(np.float64) @ w.astype(np.float64), rtol=0, atol=1e-6)
    h = 2.0 ** -8   # exactly representable steps keep the float32 model vector exact
    for j in range(6):
        wp, wm = w.copy(), w.copy()
        wp[j] += np.float32(h)
        wm[j] -= np.float32(h)
        fd = (lpco.objective(p, wp) - lpco.objective(p, wm)) / (float(wp[j]) - float(wm[j]))
        assert abs(fd - mu[j]) <= 2e-5 * max(1.0, abs(fd))


def test_squared_loss_gradient_is_the_normal_equation_residual():
    X, y, (p, _k) = _squared(5, n=200, d=33)
    w = np.random.default_rng(6).standard_normal(33).astype(np.float32)
    mu, z, _ = lpco.full_grad(p, w)
    X64 = X.astype(np.float64)
    assert np.allclose(mu, X64.T @ (X64 @ w - y) / 200, rtol=0, atol=2e-7 * np.abs(mu).max() + 1e-9)
    # at the least-squares solution the (unregularised) gradient vanishes
    w_ls = np.linalg.lstsq(X64, y.astype(np.float64), rcond=None)[0].astype(np.float32)
    mu_ls, _, _ = lpco.full_grad(p, w_ls)
    assert np.abs(mu_ls).max() <= 1e-6


def test_partial_snapshot_uses_leading_rows_only():
    X, y, (p, _k) = _logistic(7, n=64, d=5)
    w = np.ones(5, np.float32)
    mu_half, _, _ = lpco.full_grad(p, w, n_rows=32)
    p2, _k2 = lpco.make_problem(lpco.LOSS_LOGISTIC, y[:32], X=np.ascontiguousarray(X[:32]))
    mu_ref, _, _ = lpco.full_grad(p2, w)
    assert np.array_equal(mu_half, mu_ref)


def test_csr_and_dense_agree():
    rng = np.random.default_rng(8)
    n, d = 60, 40
    M = sp.random(n, d, density=0.15, format="csr", random_state=3, dtype=np.float32)
    M.sort_indices()
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    w = rng.standard_normal(d).astype(np.float32)
    ws = (w + 0.1 * rng.standard_normal(d)).astype(np.float32)
    pd_, _k1 = lpco.make_problem(lpco.LOSS_LOGISTIC, y, 1e-3, 0.0, X=np.ascontiguousarray(M.toarray()))
    ps_, _k2 = lpco.make_problem(lpco.LOSS_LOGISTIC, y, 1e-3, 0.0, csr=(M.indptr, M.indices, M.data, d))
    a, b = lpco.full_grad(pd_, w), lpco.full_grad(ps_, w)
    assert np.allclose(a[0], b[0], atol=1e-7) and np.allclose(a[1], b[1], atol=1e-6) and np.isclose(a[2], b[2])
    cfg = lpco.make_config(N=3, B=8, seed=5)
    Ud, sd = lpco.worker_vr_grad(pd_, cfg, w, ws, 1, 2)
    Us, ss = lpco.worker_vr_grad(ps_, cfg, w, ws, 1, 2)
    assert np.allclose(Ud, Us, atol=1e-7) and np.allclose(sd, ss, atol=1e-6)
    assert np.isclose(lpco.objective(pd_, w), lpco.objective(ps_, w))


# ---------------------------------------------------------------- variance-reduced difference

@pytest.mark.parametrize("maker,loss", [(_logistic, "log"), (_squared, "sq")])
def test_worker_difference_matches_definition(maker, loss):
    # u^i = (1/B) sum_{a in i_B} [grad f_a(x) - grad f_a(x~)], batch drawn from worker i's stream
    X, y, (p, _k) = maker(9, n=64, d=9)
    rng = np.random.default_rng(10)
    w = rng.standard_normal(9).astype(np.float32)
    ws = (w + 0.3 * rng.standard_normal(9)).astype(np.float32)
    cfg = lpco.make_config(N=4, B=16, seed=21)
    U, stats = lpco.worker_vr_grad(p, cfg, w, ws, epoch=2, iter_=5)
    X64, y64 = X.astype(np.float64), y.astype(np.float64)

    def slope(z):
        return -y64 / (1 + np.exp(y64 * z)) if loss == "log" else z - y64

    full_w, full_s = slope(X64 @ w), slope(X64 @ ws)
    for i in range(4):
        idx = lpco.sample_batch(21, 2, 5, lpco.TAG_BATCH, i, 16, 64)
        ref = ((full_w[idx] - full_s[idx])[:, None] * X64[idx]).mean(axis=0)
        assert np.allclose(U[i, :9], ref, rtol=0, atol=1e-6 * np.abs(ref).max())
        assert not U[i, 9:].any()
        assert stats[i, 0] == np.abs(U[i]).max()
    # shared batch J (double sampling): one row, stream without a worker id
    UJ, _ = lpco.worker_vr_grad(p, cfg, w, ws, 2, 5, tag=lpco.TAG_SHARED)
    idx = lpco.sample_batch(21, 2, 5, lpco.TAG_SHARED, 0xFFFFFF, 16, 64)
    ref = ((full_w[idx] - full_s[idx])[:, None] * X64[idx]).mean(axis=0)
    assert UJ.shape[0] == 1 and np.allclose(UJ[0, :9], ref, atol=1e-6 * np.abs(ref).max())


def test_difference_vanishes_at_the_snapshot():
    # x_0 = x~  =>  u_0^i = 0 exactly (first inner iteration of every epoch of Alg. 1)
    X, y, (p, _k) = _logistic(11)
    w = np.random.default_rng(12).standard_normal(7).astype(np.float32)
    U, stats = lpco.worker_vr_grad(p, lpco.make_config(N=2, B=8), w, w.copy(), 0, 0)
    assert not U.any() and not stats.any()


def test_vr_estimate_is_unbiased():
    # E[u^i] + grad f(x~) = grad f(x)  (Assumption 1 + the SVRG construction)
    X, y, (p, _k) = _logistic(13, n=32, d=5)
    rng = np.random.default_rng(14)
    w = rng.standard_normal(5).astype(np.float32)
    ws = (w + 0.5 * rng.standard_normal(5)).astype(np.float32)
    target = lpco.full_grad(p, w)[0].astype(np.float64) - lpco.full_grad(p, ws)[0]
    cfg = lpco.make_config(N=8, B=4, seed=1)
    acc, acc2, T = np.zeros(5), np.zeros(5), 1500
    for it in range(T):
        U, _ = lpco.worker_vr_grad(p, cfg, w, ws, 0, it)
        acc += U[:, :5].mean(axis=0)
        acc2 += (U[:, :5].astype(np.float64) ** 2).mean(axis=0)
    mean = acc / T
    se = np.sqrt(np.maximum(acc2 / T - mean ** 2, 1e-12) / (8 * T))
    assert np.all(np.abs(mean - target) <= 4.5 * se)


# ---------------------------------------------------------------- MLP (deep model as an instance of eq. (1))

def _mlp(seed=0, n=24, dims=(6, 5, 4, 3)):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[-1], size=n).astype(np.float32)
    parts = []
    for l in range(len(dims) - 1):
        parts += [rng.standard_normal(dims[l] * dims[l + 1]) * 0.5, rng.standard_normal(dims[l + 1]) * 0.1]
    w = np.concatenate(parts).astype(np.float32)
    prob, keep = lpco.make_problem(lpco.LOSS_MLP_SOFTMAX, y, X=X, d=w.size, mlp_dims=dims)
    return X, y, w, dims, (prob, keep)


def _torch_mlp_grad(X, y, w, dims, rows):
    import torch
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    h = torch.tensor(X[rows], dtype=torch.float64)
    off = 0
    for l in range(len(dims) - 1):
        W = wt[off: off + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1]); off += dims[l] * dims[l + 1]
        b = wt[off: off + dims[l + 1]]; off += dims[l + 1]
        h = h @ W + b
        if l + 2 < len(dims):
            h = torch.relu(h)
    loss = torch.nn.functional.cross_entropy(h, torch.tensor(y[rows], dtype=torch.long))
    loss.backward()
    return loss.item(), wt.grad.numpy()


def test_mlp_gradient_against_autograd():
    X, y, w, dims, (p, _k) = _mlp(1)
    mu, _, f = lpco.full_grad(p, w)
    f_ref, g_ref = _torch_mlp_grad(X, y, w, dims, np.arange(X.shape[0]))
    assert np.isclose(f, f_ref, rtol=1e-10)
    assert np.allclose(mu, g_ref, rtol=0, atol=2e-7 * np.abs(g_ref).max())
    assert np.isclose(lpco.objective(p, w), f_ref, rtol=1e-10)
    ws = (w + 0.05 * np.random.default_rng(2).standard_normal(w.size)).astype(np.float32)
    cfg = lpco.make_config(N=2, B=6, seed=3)
    U, _ = lpco.worker_vr_grad(p, cfg, w, ws, 1, 1)
    for i in range(2):
        idx = lpco.sample_batch(3, 1, 1, lpco.TAG_BATCH, i, 6, X.shape[0])
        ref = _torch_mlp_grad(X, y, w, dims, idx)[1] - _torch_mlp_grad(X, y, ws, dims, idx)[1]
        assert np.allclose(U[i, :w.size], ref, rtol=0, atol=1e-6 * max(np.abs(ref).max(), 1e-3))


def test_relu_margin_on_a_hand_built_network():
    """lpco_mlp_relu_margin against a 3-2-2-2 network whose hidden pre-activations are known by construction
    (all numbers exactly representable): a unit that is exactly zero, the minimum taken over both hidden layers
    and over the rows of the batch, negative pre-activations counted by magnitude, the last (softmax) layer's
    tiny logits ignored, and the [in][out] row-major weight layout (a transposed read changes every value)."""
    dims = (3, 2, 2, 2)
    X = np.array([[1.0, 2.0, -1.0], [0.0, 0.0, 0.0]], dtype=np.float32)
    y = np.array([0.0, 1.0], dtype=np.float32)
    W1 = [[1.0, 0.5], [1.0, -1.0], [3.0, 0.25]]          # unit 0 of row 0: 1 + 2 - 3 = 0; unit 1: 0.5 - 2 - 0.25
    W2 = [[2.0, -4.0], [100.0, 100.0]]
    W3 = [[1e-3, 0.0], [0.0, 1e-3]]                      # logits of order 1e-3: not hidden units

    def net(b1, b2):
        return np.concatenate([np.ravel(W1), b1, np.ravel(W2), b2, np.ravel(W3), [0.0, 0.0]]).astype(np.float32)

    p, _k = lpco.make_problem(lpco.LOSS_MLP_SOFTMAX, y, X=X, d=20, mlp_dims=dims)
    # row 0, no biases: layer 1 = (0, -1.75)
    assert lpco.mlp_relu_margin(p, net([0.0, 0.0], [0.25, 0.5]), [0]) == 0.0
    # row 0, b1 = (0.75, 0.5): layer 1 = (0.75, -1.25), h = (0.75, 0); layer 2 = (1.75, -2.5)
    w = net([0.75, 0.5], [0.25, 0.5])
    assert lpco.mlp_relu_margin(p, w, [0]) == 0.75
    # row 1 (x = 0): layer 1 = b1 = (0.75, 0.5); layer 2 = (1.5 + 50 + 0.25, -3 + 50 + 0.5)
    assert lpco.mlp_relu_margin(p, w, [1]) == 0.5
    assert lpco.mlp_relu_margin(p, w, [0, 1]) == 0.5 and lpco.mlp_relu_margin(p, w, [1, 0, 0]) == 0.5
    # the second hidden layer decides when it holds the smallest value: b2 = (-1.5, 0.5) -> row 0: (0, -2.5)
    assert lpco.mlp_relu_margin(p, net([0.75, 0.5], [-1.5, 0.5]), [0]) == 0.0
    assert lpco.mlp_relu_margin(p, net([0.75, 0.5], [-1.625, 0.5]), [0]) == 0.125


# ---------------------------------------------------------------- argument checking

def test_bad_arguments_return_errors():
    X, y, (p, _k) = _logistic(0)
    w = np.zeros(7, np.float32)
    with pytest.raises(lpco.OracleError):
        lpco.worker_vr_grad(p, lpco.make_config(N=2, B=0), w, w, 0, 0)
    with pytest.raises(lpco.OracleError):
        lpco.prox_step(w, w, w, -1.0, 0.0, 0.0)
    p.lambda1 = -1.0
    with pytest.raises(lpco.OracleError):
        lpco.objective(p, w)
