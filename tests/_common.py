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
