"""GPU parity: statistics, clipped stochastic quantizer + packing, receiver-side average, prox.

Integer results (codes, packed words, clip counts) must be bit-exact against the oracle given the
same float vector and stream; the average of eq. (4) is bit-exact too because both sides use the
same fixed order of fused multiply-adds."""
import numpy as np
import pytest

import lpc_synth
from oracle import lpco
from _common import gpu_context, to_dev

pytestmark = pytest.mark.gpu


def _ctx(d, N, bits, clip_mode=0, clip=1.0, seed=0):
    # a dummy dense problem carries d; the quantizer calls only use config and d
    sp = lpc_synth.make("c1", n=max(64, N), d=d, N=N, B=1, bits=bits, seed=seed)
    return gpu_context(sp, clip_mode=clip_mode, clip=clip, bits=bits, m=1), sp


def _u(N, d, seed, scale=1.0):
    U = lpc_synth.gaussian_u(N, d, seed=seed, scale=scale)
    U *= np.linspace(0.5, 3.0, N, dtype=np.float32)[:, None]
    return U


CASES = [  # d, N, bits, clip_mode, clip
    (45, 3, 5, 0, 1.0),            # ragged: less than two segments
    (64, 4, 2, 1, 2.0),            # C1 shape
    (4096, 8, 4, 0, 1.0),          # C2 shape, unbiased
    (4096, 8, 4, 0, 0.9),          # the paper's operating point, clipped
    (8192, 16, 3, 1, 2.0),         # C4 shape, odd bit width
    (8192 * 3 + 37, 2, 7, 0, 0.5), # several tiles and a ragged tail
    (100_003, 4, 2, 0, 1.0),
    (20_000, 2, 16, 0, 0.75), (20_000, 2, 9, 0, 1.0), (20_000, 2, 8, 0, 1.0), (20_000, 2, 6, 0, 0.3),
    (5000, 2, 10, 0, 1.0), (5000, 2, 11, 0, 1.0), (5000, 2, 12, 1, 1.0), (5000, 2, 13, 0, 1.0),
    (5000, 2, 14, 0, 0.6), (5000, 2, 15, 0, 1.0),
]


@pytest.mark.parametrize("d,N,bits,clip_mode,clip", CASES)
def test_quantize_pack_bit_exact(d, N, bits, clip_mode, clip):
    import torch
    ctx, _ = _ctx(d, N, bits, clip_mode, clip, seed=7)
    U = _u(N, d, seed=d + bits)
    dU = to_dev(U)
    stats_g = torch.zeros(N, 4, dtype=torch.float64, device="cuda")
    ctx.vector_stats(dU, N, stats_g)
    stats_o = np.stack([lpco.vector_stats(U[i, :d]) for i in range(N)])
    sg = stats_g.cpu().numpy()
    assert np.array_equal(sg[:, 0], stats_o[:, 0]) and np.array_equal(sg[:, 3], stats_o[:, 3])
    assert np.allclose(sg[:, 1:3], stats_o[:, 1:3], rtol=1e-12, atol=1e-9)
    for epoch, it in [(0, 0), (3, 17)]:
        if clip_mode == lpco.CLIP_LAMBDA:
            # delta depends on the order-independent max only: the whole path is reproducible bit for bit
            po, do, co, rc = lpco.quantize_clip(U, d, bits, clip_mode, clip, seed=7, epoch=epoch, iter_=it)
            delta_in = None
        else:
            # sigma depends on the summation order: the oracle's delta is handed to both sides
            do = np.array([lpco.delta_from_stats(stats_o[i], d, bits, clip_mode, clip)[0] for i in range(N)],
                          dtype=np.float32)
            po, do, co, rc = lpco.quantize_clip(U, d, bits, clip_mode, clip, seed=7, epoch=epoch, iter_=it,
                                                delta_in=do)
            delta_in = to_dev(do)
        packed = torch.zeros(N, ctx.W, dtype=torch.int32, device="cuda")
        delta = torch.zeros(N, dtype=torch.float32, device="cuda")
        ncl = torch.zeros(N, dtype=torch.int32, device="cuda")
        ctx.quantize_clip(dU, stats_g, delta_in, epoch, it, packed, delta, ncl)
        assert np.array_equal(delta.cpu().numpy(), do)
        assert np.array_equal(packed.cpu().numpy().view(np.uint32), po)
        assert np.array_equal(ncl.cpu().numpy().view(np.uint32), co)
        # receiver: eq. (4), bit-exact
        avg = torch.zeros(d, dtype=torch.float32, device="cuda")
        ctx.dequantize_avg(to_dev(po.view(np.int32)), to_dev(do), avg)
        assert np.array_equal(avg.cpu().numpy(), lpco.dequantize_avg(po, do, d, bits))
    if clip_mode == lpco.CLIP_CSIGMA:
        # the device-derived delta agrees with the oracle's to the last bit or the one before
        packed = torch.zeros(N, ctx.W, dtype=torch.int32, device="cuda")
        delta = torch.zeros(N, dtype=torch.float32, device="cuda")
        ctx.quantize_clip(dU, stats_g, None, 0, 0, packed, delta, None)
        assert np.allclose(delta.cpu().numpy(), do, rtol=3e-7, atol=0)
    assert ctx.take_device_flags() == 0
    ctx.close()


@pytest.mark.parametrize("d,N,bits,clip", [(4096, 8, 4, 0.9), (8192 * 3 + 37, 3, 4, 1.0), (100_003, 4, 2, 1.0),
                                           (20_000, 2, 8, 0.75), (45, 3, 2, 1.0), (1001, 5, 8, 0.3)])
def test_quantize_pack_without_clip_counts_bit_exact(d, N, bits, clip):
    """The instantiation the epochs use (no clip counts, a draw for every group of four) for the bit widths that pack
    one word per thread: ragged last segments, garbage in the padding, an all-zero vector, and coordinates just
    below zero, whose position on the grid rounds up to the next integer."""
    import torch
    ctx, _ = _ctx(d, N, bits, 0, clip, seed=11)
    U = _u(N, d, seed=3 * d + bits)
    U[0, :] = 0.0                                     # u_0 = 0: every code 0
    tiny = np.float32(-1e-12) * np.abs(U[1]).max()
    U[1, 5:d:97] = tiny                              # s in (-2^-25, 0): s - floor(s) rounds to 1
    U[1, 6:d:97] = -tiny
    dU = to_dev(U)
    dU[:, d:] = -77.0
    stats = torch.zeros(N, 4, dtype=torch.float64, device="cuda")
    ctx.vector_stats(dU, N, stats)
    for epoch, it in [(0, 0), (2, 9)]:
        po, do, _co, _rc = lpco.quantize_clip(U, d, bits, 0, clip, seed=11, epoch=epoch, iter_=it)
        packed = torch.full((N, ctx.W), -1, dtype=torch.int32, device="cuda")
        delta = torch.zeros(N, dtype=torch.float32, device="cuda")
        ctx.quantize_clip(dU, stats, None, epoch, it, packed, delta, None)
        assert np.array_equal(delta.cpu().numpy(), do)
        got = packed.cpu().numpy().view(np.uint32)
        assert np.array_equal(got, po)
        assert not got[0].any()
    assert ctx.take_device_flags() == 0
    ctx.close()


def test_quantizer_degenerate_inputs():
    import torch
    d, N, bits = 1000, 3, 3
    ctx, _ = _ctx(d, N, bits)
    U = np.zeros((N, lpco.d_pad(d)), dtype=np.float32)
    U[1, :d] = np.linspace(-1, 1, d)          # row 0 all zero (u_0 = 0 at t = 0 of every epoch), row 2 one spike
    U[2, 17] = -3.0
    dU = to_dev(U)
    # garbage in the padding must not leak into the message
    dU[:, d:] = 123.0
    stats = torch.zeros(N, 4, dtype=torch.float64, device="cuda")
    ctx.vector_stats(dU, N, stats)
    packed = torch.full((N, ctx.W), -1, dtype=torch.int32, device="cuda")
    delta = torch.full((N,), -1.0, dtype=torch.float32, device="cuda")
    ncl = torch.full((N,), -1, dtype=torch.int32, device="cuda")
    ctx.quantize_clip(dU, stats, None, 1, 2, packed, delta, ncl)
    po, do, co, _ = lpco.quantize_clip(U, d, bits, seed=0, epoch=1, iter_=2)
    assert np.array_equal(packed.cpu().numpy().view(np.uint32), po)
    assert np.array_equal(delta.cpu().numpy(), do) and do[0] == 0 and not po[0].any()
    assert np.array_equal(ncl.cpu().numpy().view(np.uint32), co)
    assert ctx.take_device_flags() == 0
    # non-finite input raises the device flag
    dU[1, 5] = float("nan")
    ctx.vector_stats(dU, N, stats)
    assert stats[1, 3].item() == 1
    assert ctx.take_device_flags() == -5 and ctx.take_device_flags() == 0
    # a vector whose finite entries are all zero but that holds a NaN: scale 0, so the message is all zeros (code
    # 0 at the NaN too), on both sides, through the separate calls and through the one-launch exchange
    U0 = np.zeros((N, lpco.d_pad(d)), dtype=np.float32)
    U0[1, :d] = np.linspace(-1, 1, d)
    U0[0, 7] = np.nan
    po, do, _, _ = lpco.quantize_clip(U0, d, bits, seed=0, epoch=1, iter_=2)
    assert do[0] == 0 and not po[0].any()
    dU0 = to_dev(U0)
    ctx.vector_stats(dU0, N, stats)
    ctx.quantize_clip(dU0, stats, None, 1, 2, packed, delta, ncl)
    assert np.array_equal(packed.cpu().numpy().view(np.uint32), po) and np.array_equal(delta.cpu().numpy(), do)
    assert ctx.take_device_flags() == -5
    avg = torch.zeros(d, device="cuda")
    packed.fill_(-1)
    ctx.exchange(dU0, 1, 2, packed, delta, avg)
    assert np.array_equal(packed.cpu().numpy().view(np.uint32), po) and np.array_equal(delta.cpu().numpy(), do)
    assert ctx.take_device_flags() == -5
    ctx.close()


def test_quantizer_is_reproducible_and_streams_differ():
    import torch
    d, N, bits = 50_000, 4, 4
    ctx, _ = _ctx(d, N, bits, seed=11)
    dU = to_dev(_u(N, d, seed=1))
    stats = torch.zeros(N, 4, dtype=torch.float64, device="cuda")
    ctx.vector_stats(dU, N, stats)
    outs = []
    for epoch, it in [(0, 0), (0, 0), (0, 1), (1, 0)]:
        packed = torch.zeros(N, ctx.W, dtype=torch.int32, device="cuda")
        delta = torch.zeros(N, dtype=torch.float32, device="cuda")
        ctx.quantize_clip(dU, stats, None, epoch, it, packed, delta, None)
        outs.append(packed.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])
    assert not np.array_equal(outs[0], outs[2]) and not np.array_equal(outs[0], outs[3])
    ctx.close()


@pytest.mark.parametrize("d,l1,l2", [(64, 1e-4, 0.0), (4099, 1e-2, 1e-1), (100_000, 0.0, 1e-3)])
def test_prox_step(d, l1, l2):
    import torch
    sp = lpc_synth.make("c1", n=64, d=d, N=1, B=1)
    sp.lambda1, sp.lambda2 = l1, l2
    ctx = gpu_context(sp, m=1)
    rng = np.random.default_rng(d)
    w, u, mu = (rng.standard_normal(d).astype(np.float32) * s for s in (0.05, 1.0, 1.0))
    dw = to_dev(w)
    ctx.prox_step(dw, to_dev(u), to_dev(mu), 0.01)
    ref = lpco.prox_step(w, u, mu, 0.01, l1, l2)
    got = dw.cpu().numpy()
    assert np.allclose(got, ref, rtol=0, atol=2e-7 * max(1.0, np.abs(ref).max()))
    assert np.array_equal(got == 0, ref == 0) or np.mean((got == 0) != (ref == 0)) < 1e-4
    ctx.close()


@pytest.mark.parametrize("d,N,bits,clip", [(64, 4, 2, 1.0), (4096, 8, 4, 0.9), (8192, 16, 3, 1.0), (1000, 5, 7, 0.5),
                                           (4100, 64, 16, 1.0), (16384, 3, 5, 1.0),     # small-d single-launch path
                                           (20_000, 4, 4, 0.9), (4096, 70, 2, 1.0)])    # large-d / many-worker path
def test_exchange_one_call_bit_exact(d, N, bits, clip):
    """lpc_exchange = statistics + eq. (3) + quantize/pack + eq. (4); every output bit-exact (lambda mode)."""
    import torch
    ctx, _ = _ctx(d, N, bits, 0, clip, seed=5)
    U = _u(N, d, seed=3 * d + bits)
    U[N - 1] = 0.0                                   # an all-zero worker
    dU = to_dev(U)
    for epoch, it in [(0, 0), (2, 9)]:
        packed = torch.full((N, ctx.W), -1, dtype=torch.int32, device="cuda")
        delta = torch.full((N,), -1.0, dtype=torch.float32, device="cuda")
        avg = torch.full((d,), -1.0, dtype=torch.float32, device="cuda")
        ctx.exchange(dU, epoch, it, packed, delta, avg)
        po, do, _, _ = lpco.quantize_clip(U, d, bits, 0, clip, seed=5, epoch=epoch, iter_=it)
        assert np.array_equal(delta.cpu().numpy(), do)
        assert np.array_equal(packed.cpu().numpy().view(np.uint32), po)
        assert np.array_equal(avg.cpu().numpy(), lpco.dequantize_avg(po, do, d, bits))
    ctx.close()


@pytest.mark.parametrize("d,N,bits", [(1000, 8, 3), (4096, 16, 4), (30_000, 5, 2), (70, 3, 9)])
def test_shared_scale_receiver_bit_exact(d, N, bits):
    """Schemes (b)/(c): every worker quantized with delta = max_i delta_i; integer code sums; eq. (5)."""
    import torch
    ctx, _ = _ctx(d, N, bits, 0, 1.0, seed=9)
    U = _u(N, d, seed=d + N)
    deltas = [lpco.delta_from_stats(lpco.vector_stats(U[i, :d]), d, bits, lpco.CLIP_LAMBDA, 1.0)[0] for i in range(N)]
    shared = np.full(N, max(deltas), dtype=np.float32)
    po, do, _, _ = lpco.quantize_clip(U, d, bits, seed=9, epoch=1, iter_=4, delta_in=shared)
    packed = torch.zeros(N, ctx.W, dtype=torch.int32, device="cuda")
    delta = torch.zeros(N, device="cuda")
    stats = torch.zeros(N, 4, dtype=torch.float64, device="cuda")
    ctx.vector_stats(to_dev(U), N, stats)
    ctx.quantize_clip(to_dev(U), stats, to_dev(shared), 1, 4, packed, delta, None)
    assert np.array_equal(packed.cpu().numpy().view(np.uint32), po) and np.array_equal(delta.cpu().numpy(), do)
    for requant in (False, True):
        avg = torch.full((d,), -1.0, device="cuda")
        ctx.dequantize_shared(packed, delta, requant, 1, 4, avg)
        ref, _sums = lpco.dequantize_shared(po, float(do[0]), d, bits, requantize=requant, seed=9, epoch=1, iter_=4)
        assert np.array_equal(avg.cpu().numpy(), ref)
    ctx.close()
