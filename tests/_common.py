"""Shared helpers of the tests: build oracle-side and GPU-side handles from one synthetic problem."""
import numpy as np

from oracle import lpco


def oracle_problem(sp):
    if sp.csr is not None:
        return lpco.make_problem(sp.loss, sp.y, sp.lambda1, sp.lambda2, csr=(*sp.csr, sp.d))
    return lpco.make_problem(sp.loss, sp.y, sp.lambda1, sp.lambda2, X=sp.X, d=sp.d, mlp_dims=sp.mlp_dims)


def config_kwargs(sp, **over):
    kw = dict(algo=sp.algo, N=sp.N, B=sp.B, m=sp.m, bits=sp.bits, clip_mode=sp.clip_mode, clip=sp.clip, eta=sp.eta,
              L=sp.L, seed=sp.seed, n_full=sp.n_full)
    kw.update(over)
    return kw


def oracle_config(sp, **over):
    return lpco.make_config(**config_kwargs(sp, **over))


def gpu_context(sp, **over):
    import torch
    from paper_1901_08924_amd import lpc
    dev = torch.device("cuda:0")
    cfg = lpc.make_config(**config_kwargs(sp, **over))
    y = torch.from_numpy(sp.y).to(dev)
    if sp.csr is not None:
        rp, ci, va = (torch.from_numpy(np.ascontiguousarray(a)).to(dev) for a in sp.csr)
        return lpc.Context(sp.loss, y, cfg, csr=(rp, ci, va, sp.d), lambda1=sp.lambda1, lambda2=sp.lambda2)
    X = torch.from_numpy(sp.X).to(dev)
    return lpc.Context(sp.loss, y, cfg, X=X, d=sp.d, mlp_dims=sp.mlp_dims, lambda1=sp.lambda1, lambda2=sp.lambda2)


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def batch_grad_inf(sp, w, epoch, iter_, tag, worker):
    """|grad f_B(w)|_inf for the batch B that `worker` draws at (epoch, iter): the oracle's full gradient over a
    problem made of exactly the sampled rows (duplicates kept).  The scale a variance-reduced difference of
    nearly equal per-sample gradients is compared against."""
    field = 0xFFFFFF if tag == lpco.TAG_SHARED else worker
    idx = lpco.sample_batch(sp.seed, epoch, iter_, tag, field, sp.B, sp.n)
    if sp.csr is not None:
        rp, ci, va = sp.csr
        lens = (rp[idx + 1] - rp[idx]).astype(np.int64)
        sub_rp = np.zeros(idx.size + 1, dtype=np.int32)
        np.cumsum(lens, out=sub_rp[1:])
        take = np.concatenate([np.arange(rp[r], rp[r + 1]) for r in idx]) if lens.sum() else np.zeros(0, np.int64)
        sub, _k = lpco.make_problem(sp.loss, sp.y[idx], csr=(sub_rp, ci[take], va[take], sp.d))
    else:
        sub, _k = lpco.make_problem(sp.loss, sp.y[idx], X=np.ascontiguousarray(sp.X[idx]), d=sp.d,
                                    mlp_dims=sp.mlp_dims)
    return float(np.abs(lpco.full_grad(sub, w)[0]).max())
