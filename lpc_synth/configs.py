"""Generators for the five benchmark configurations (C1..C5) and scaled-down variants."""
from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

LOSS_LOGISTIC, LOSS_SQUARED, LOSS_MLP_SOFTMAX = 0, 1, 2
ALGO_LPC, ALGO_ALPC_SC, ALGO_ALPC_GC = 0, 1, 2
CLIP_LAMBDA, CLIP_CSIGMA = 0, 1

CONFIG_NAMES = ("c1", "c2", "c3", "c4", "c5")


@dataclass
class SynthProblem:
    name: str
    loss: int
    n: int
    d: int
    y: np.ndarray                      # float32: +-1 labels, real targets, or class ids
    w0: np.ndarray                     # float32 starting point x~^0
    X: Optional[np.ndarray] = None     # dense float32 [n, d] (for the MLP: [n, dims[0]])
    csr: Optional[Tuple[np.ndarray, np.ndarray, np.ndarray]] = None  # (row_ptr i32, col_idx i32, vals f32)
    mlp_dims: Optional[Tuple[int, ...]] = None
    lambda1: float = 0.0
    lambda2: float = 0.0
    # run parameters
    algo: int = ALGO_LPC
    N: int = 1
    B: int = 1
    m: int = 1
    bits: int = 32
    clip_mode: int = CLIP_LAMBDA
    clip: float = 1.0
    eta: float = 0.1
    L: float = 1.0
    epochs: int = 1
    n_full: int = 0                    # rows used by the snapshot gradient (0 = all)
    seed: int = 0
    w_star: Optional[np.ndarray] = None
    notes: dict = field(default_factory=dict)


def _sparse_planted(rng, d, frac, scale=1.0):
    k = max(1, int(np.ceil(frac * d)))
    w = np.zeros(d, dtype=np.float32)
    support = rng.choice(d, size=k, replace=False)
    w[support] = (rng.standard_normal(k) * scale).astype(np.float32)
    return w


def _sign_labels(rng, margin, flip_frac):
    y = np.where(margin >= 0, 1.0, -1.0).astype(np.float32)
    nflip = int(round(flip_frac * y.size))
    if nflip:
        y[rng.choice(y.size, size=nflip, replace=False)] *= -1.0
    return y


def _normalize_rows(X):
    nrm = np.sqrt(np.einsum("ij,ij->i", X, X, dtype=np.float64)).astype(np.float32)
    nrm[nrm == 0] = 1.0
    X /= nrm[:, None]
    return X


def make_c1(seed=0, n=1024, d=64, N=4, B=16, bits=2, epochs=10):
    """Tiny L1-logistic problem: iid N(0,1) design, 10%-sparse planted model, 5% label flips."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d), dtype=np.float32)
    w_star = _sparse_planted(rng, d, 0.10)
    y = _sign_labels(rng, X.astype(np.float64) @ w_star.astype(np.float64), 0.05)
    L = float(np.max(np.einsum("ij,ij->i", X, X, dtype=np.float64)) / 4.0)
    return SynthProblem(name="c1", loss=LOSS_LOGISTIC, n=n, d=d, X=X, y=y, w0=np.zeros(d, np.float32),
                        lambda1=1e-4, lambda2=0.0, N=N, B=B, m=max(1, n // (N * B)), bits=bits,
                        clip_mode=CLIP_CSIGMA, clip=2.0, eta=0.1 / L, L=L, epochs=epochs, seed=seed, w_star=w_star)


def make_c2(seed=0, n=65536, d=4096, N=8, B=64, bits=4, epochs=20, clip=1.0):
    """Dense L1+L2 logistic: rows N(0,I) then l2-normalised, 5%-sparse planted model, 2% flips."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d), dtype=np.float32)
    _normalize_rows(X)
    w_star = _sparse_planted(rng, d, 0.05, scale=float(np.sqrt(d)) / 4.0)
    y = _sign_labels(rng, X @ w_star, 0.02)
    return SynthProblem(name="c2", loss=LOSS_LOGISTIC, n=n, d=d, X=X, y=y, w0=np.zeros(d, np.float32),
                        lambda1=1e-5, lambda2=1e-4, N=N, B=B, m=max(1, n // (N * B)), bits=bits,
                        clip_mode=CLIP_LAMBDA, clip=clip, eta=0.4 / 0.25, L=0.25, epochs=epochs, seed=seed,
                        w_star=w_star)


def make_c3(seed=0, n=1 << 20, d=1 << 20, nnz_mean=50, N=16, B=256, bits=2, epochs=3):
    """Sparse text-like L1 logistic in CSR: Zipf(1.1) column ids, tf-idf-like positive values,
    l2-normalised rows, int32 indices with sorted columns."""
    rng = np.random.default_rng(seed)
    per_row = np.clip(rng.poisson(nnz_mean, size=n), 1, 200).astype(np.int64)
    total = int(per_row.sum())
    # Zipf(1.1) over ranks 0..d-1 by inverse CDF; the column id is the rank
    pmf = 1.0 / np.power(np.arange(1, d + 1, dtype=np.float64), 1.1)
    cdf = np.cumsum(pmf)
    cdf /= cdf[-1]
    cols = np.searchsorted(cdf, rng.random(total), side="left").astype(np.int64)
    np.minimum(cols, d - 1, out=cols)
    rows = np.repeat(np.arange(n, dtype=np.int64), per_row)
    keys = np.unique(rows * d + cols)          # merges duplicates within a row, sorts columns
    rows = (keys // d).astype(np.int64)
    cols = (keys % d).astype(np.int32)
    counts = np.bincount(rows, minlength=n)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    tf = 1.0 + np.log1p(rng.geometric(0.5, size=cols.size).astype(np.float64))
    idf = np.log((d + 1.0) / (1.0 + cols.astype(np.float64)))
    vals = (tf * idf)
    sq = np.add.reduceat(vals * vals, row_ptr[:-1])
    vals = (vals / np.sqrt(sq)[rows]).astype(np.float32)
    w_star = _sparse_planted(rng, d, 0.01)
    margin = np.add.reduceat(vals.astype(np.float64) * w_star[cols].astype(np.float64), row_ptr[:-1])
    y = _sign_labels(rng, margin, 0.0)
    assert row_ptr[-1] < 2 ** 31
    return SynthProblem(name="c3", loss=LOSS_LOGISTIC, n=n, d=d, csr=(row_ptr.astype(np.int32), cols, vals), y=y,
                        w0=np.zeros(d, np.float32), lambda1=1e-6, lambda2=0.0, N=N, B=B,
                        m=max(1, n // (N * B)), bits=bits, clip_mode=CLIP_LAMBDA, clip=1.0, eta=0.4 / 0.25,
                        L=0.25, epochs=epochs, seed=seed, w_star=w_star)


def make_c4(seed=0, n=262144, d=8192, rho=0.5, N=16, B=64, bits=3, epochs=5, clip=2.0, algo=ALGO_ALPC_GC):
    """Ridge least squares with AR(1)-correlated columns for the accelerated variant."""
    from scipy.signal import lfilter
    rng = np.random.default_rng(seed)
    X = np.empty((n, d), dtype=np.float32)
    s = float(np.sqrt(1.0 - rho * rho))
    L = 0.0
    block = max(1, (1 << 25) // d)              # x_0 = eps_0, x_j = rho x_{j-1} + sqrt(1-rho^2) eps_j, row by row
    for r0 in range(0, n, block):
        eps = rng.standard_normal((min(block, n - r0), d), dtype=np.float32)
        eps[:, 0] /= np.float32(s)
        xb = lfilter([s], [1.0, -rho], eps, axis=1).astype(np.float32)
        X[r0:r0 + xb.shape[0]] = xb
        L = max(L, float(np.max(np.einsum("ij,ij->i", xb, xb, dtype=np.float64))))
    w_star = (rng.standard_normal(d) / np.sqrt(d)).astype(np.float32)
    y = (X @ w_star + 0.1 * rng.standard_normal(n).astype(np.float32)).astype(np.float32)
    return SynthProblem(name="c4", loss=LOSS_SQUARED, n=n, d=d, X=X, y=y, w0=np.zeros(d, np.float32),
                        lambda1=0.0, lambda2=1e-3, algo=algo, N=N, B=B, m=max(1, n // (N * B)), bits=bits,
                        clip_mode=CLIP_CSIGMA, clip=clip, eta=0.1 / L, L=L, epochs=epochs, seed=seed,
                        w_star=w_star)


def make_c5(seed=0, n=65536, dims=(3072, 1024, 1024, 10), N=16, B=128, bits=4, epochs=2, n_full=16384, m=32):
    """Gaussian-mixture classification for the 3-layer ReLU MLP; He-normal weights, zero biases."""
    rng = np.random.default_rng(seed)
    C = dims[-1]
    means = (0.5 * rng.standard_normal((C, dims[0]))).astype(np.float32)
    cls = (np.arange(n) % C).astype(np.int64)
    rng.shuffle(cls)
    X = rng.standard_normal((n, dims[0]), dtype=np.float32)
    X += means[cls]
    parts = []
    for l in range(len(dims) - 1):
        fan_in, fan_out = dims[l], dims[l + 1]
        parts.append((rng.standard_normal((fan_in, fan_out)) * np.sqrt(2.0 / fan_in)).astype(np.float32).ravel())
        parts.append(np.zeros(fan_out, np.float32))
    w0 = np.concatenate(parts)
    return SynthProblem(name="c5", loss=LOSS_MLP_SOFTMAX, n=n, d=int(w0.size), X=X, y=cls.astype(np.float32), w0=w0,
                        mlp_dims=tuple(dims), lambda1=0.0, lambda2=0.0, N=N, B=B, m=m, bits=bits,
                        clip_mode=CLIP_LAMBDA, clip=0.85, eta=0.05, L=1.0, epochs=epochs,
                        n_full=min(n_full, n), seed=seed)


_MAKERS = {"c1": make_c1, "c2": make_c2, "c3": make_c3, "c4": make_c4, "c5": make_c5}


def make(name, **overrides):
    """make("c2") is the full-size configuration; pass n=, d=, ... for a scaled-down one."""
    return _MAKERS[name](**overrides)


def gaussian_u(N, d, seed=0, scale=1.0):
    """iid N(0, scale^2) stand-in for the workers' variance-reduced differences (the paper's
    histograms of u are close to Gaussian), padded with zeros to a multiple of 32 columns."""
    rng = np.random.default_rng(seed)
    dp = ((d + 31) // 32) * 32
    U = np.zeros((N, dp), dtype=np.float32)
    U[:, :d] = rng.standard_normal((N, d), dtype=np.float32) * np.float32(scale)
    return U
