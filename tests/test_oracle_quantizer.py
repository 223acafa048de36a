"""Pins for the oracle's quantizer, message format and receiver-side averaging (CPU only).

Each test checks the oracle against something the paper or the mathematics fixes:
Sec. 3.2 (codebook, rules (1)/(2), unbiasedness), Lemma 1 and its proof (exact
variance), Lemma 4 of the supplement (vector bound with clipping), eq. (3), the
"Unbiased quantization" paragraph of Sec. 4.1, Sec. 4.2 (message size, eq. (4),
schemes (b)/(c), Table 1).
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import lpco

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
NDRAW = 1_000_000


def _levels(b):
    return (1 << (b - 1)) - 1


# ---------------------------------------------------------------- rule (1): unbiased, exact variance

@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_unbiased_and_exact_variance_monte_carlo(bits):
    # 1e6 independent draws of Q(x) for several x inside the hull: the mean is x within
    # 3 standard errors (E[Q(x)] = x) and the variance is (x - z)(z + delta - x) <= delta^2/4
    delta = 0.37
    L = _levels(bits)
    rng = np.random.default_rng(bits)
    xs = np.concatenate([rng.uniform(-(L + 1) * delta, L * delta, size=4), [0.25 * delta, -0.5 * delta]])
    for n_x, x in enumerate(xs):
        u = np.full(NDRAW, x, dtype=np.float32)
        codes, _ = lpco.quantize_codes(u, bits, delta, seed=1234 + n_x, epoch=bits, iter_=n_x)
        q = codes.astype(np.float64) * np.float64(np.float32(delta))
        xf = float(np.float32(x))
        z = np.floor(xf / float(np.float32(delta))) * float(np.float32(delta))
        var_exact = (xf - z) * (z + float(np.float32(delta)) - xf)
        assert var_exact <= delta * delta / 4 * (1 + 1e-6)
        assert set(np.unique(codes)) <= {int(round(z / delta)), int(round(z / delta)) + 1}
        se = np.sqrt(max(var_exact, 1e-30) / NDRAW)
        assert abs(q.mean() - xf) <= 3 * se + 1e-6 * delta
        # the variance estimator of a two-point law: relative 1% is > 5 sigma here unless var is tiny
        if var_exact > 1e-3 * delta * delta:
            assert abs(q.var() - var_exact) <= 0.01 * delta * delta / 4 + 5e-3 * var_exact


def test_grid_points_and_end_points_are_fixed_points():
    # a value of dom(delta,b), in particular the smallest and the largest, is returned unchanged
    for bits in (2, 3, 5, 8, 16):
        L = _levels(bits)
        delta = 0.125  # power of two: k*delta is exact
        ks = np.arange(-(L + 1), L + 1, dtype=np.int64)
        if ks.size > 4096:
            ks = np.concatenate([ks[:1024], ks[-1024:], ks[ks.size // 2 - 512: ks.size // 2 + 512]])
        u = (ks * delta).astype(np.float32)
        for it in range(4):
            codes, ncl = lpco.quantize_codes(u, bits, delta, thresh=L * delta, iter_=it)
            assert np.array_equal(codes, ks)
            assert ncl == 0


def test_out_of_hull_projects_to_extreme_codes():
    # rule (2): outside the hull -> smallest / largest codebook value, deterministically
    for bits in (2, 4, 7):
        L = _levels(bits)
        delta = 0.3
        u = np.array([L * 0.3 * 1.01, 1e3, 1e30, -(L + 1) * 0.3 * 1.01, -1e3, -1e30], dtype=np.float32)
        for it in range(8):
            codes, ncl = lpco.quantize_codes(u, bits, delta, thresh=np.float32(L) * np.float32(delta), iter_=it)
            assert list(codes) == [L, L, L, -(L + 1), -(L + 1), -(L + 1)]
            assert ncl == 6


def test_codes_always_adjacent_to_input():
    rng = np.random.default_rng(0)
    u = rng.standard_normal(50_000).astype(np.float32)
    for bits in (2, 3, 4, 6):
        st = lpco.vector_stats(u)
        delta, thresh = lpco.delta_from_stats(st, u.size, bits, lpco.CLIP_LAMBDA, 0.7)
        codes, _ = lpco.quantize_codes(u, bits, delta, thresh)
        L = _levels(bits)
        assert codes.min() >= -(L + 1) and codes.max() <= L
        clipped = np.clip(u.astype(np.float64), -(L + 1) * float(delta), L * float(delta))
        assert np.all(np.abs(codes * float(delta) - clipped) <= float(delta) * (1 + 1e-5))


# ---------------------------------------------------------------- eq. (3) and clipping

def test_delta_rule_lambda_mode():
    rng = np.random.default_rng(1)
    u = (rng.standard_normal(1000) * 3).astype(np.float32)
    st = lpco.vector_stats(u)
    assert st[0] == np.abs(u).max() and st[3] == 0
    assert np.isclose(st[1], u.astype(np.float64).sum()) and np.isclose(st[2], (u.astype(np.float64) ** 2).sum())
    for bits in (2, 3, 4, 8):
        for lam in (1.0, 0.9, 0.5):
            delta, thresh = lpco.delta_from_stats(st, u.size, bits, lpco.CLIP_LAMBDA, lam)
            exact = Fraction(float(np.float32(lam))) * Fraction(float(np.abs(u).max())) / _levels(bits)
            assert abs(Fraction(float(delta)) - exact) <= exact * Fraction(1, 1 << 22)
            assert thresh == np.float32(lam) * np.abs(u).max()


def test_lambda_one_never_clips_and_never_uses_the_extra_negative_code():
    # Sec. 4.1: with lambda = 1 every coordinate is inside the hull
    rng = np.random.default_rng(2)
    for bits in (2, 3, 4, 5):
        U = lpco.d_pad(10_000)
        u = np.zeros((1, U), dtype=np.float32)
        u[0, :10_000] = rng.standard_normal(10_000).astype(np.float32) * 7.3
        packed, delta, ncl, rc = lpco.quantize_clip(u, 10_000, bits, lpco.CLIP_LAMBDA, 1.0, seed=9)
        assert rc == lpco.OK and ncl[0] == 0
        codes = lpco.unpack(packed[0], 10_000, bits)
        L = _levels(bits)
        assert codes.min() >= -L and codes.max() <= L
        # the largest coordinate sits on the last grid point and is reproduced
        j = int(np.argmax(np.abs(u[0])))
        assert abs(codes[j]) == L


def test_clipped_count_is_number_outside_hull():
    # d_lambda of Lemma 2: coordinates exceeding dom(delta, b)
    rng = np.random.default_rng(3)
    d = 20_000
    u = rng.standard_normal(d).astype(np.float32)
    st = lpco.vector_stats(u)
    for bits in (2, 3, 4):
        for lam in (0.9, 0.5, 0.25):
            delta, thresh = lpco.delta_from_stats(st, d, bits, lpco.CLIP_LAMBDA, lam)
            _, ncl = lpco.quantize_codes(u, bits, delta, thresh)
            L = _levels(bits)
            hi = Fraction(float(np.float32(lam))) * Fraction(float(st[0]))
            lo = -Fraction(float(delta)) * (L + 1)
            expect = sum(1 for v in u if Fraction(float(v)) > hi or Fraction(float(v)) < lo)
            # hi is rounded to float once in the oracle; allow coordinates within one ulp of it
            near = sum(1 for v in u if abs(Fraction(float(v)) - hi) <= hi * Fraction(1, 1 << 22))
            assert abs(int(ncl) - expect) <= near


def test_csigma_mode_matches_population_std():
    # build convention (no passage of the paper fixes it): lambda = min(1, c*sigma/|u|_inf)
    rng = np.random.default_rng(4)
    d = 4096
    u = rng.standard_normal(d).astype(np.float32)
    st = lpco.vector_stats(u)
    for c in (1.0, 2.0, 4.0, 100.0):
        delta, thresh = lpco.delta_from_stats(st, d, 4, lpco.CLIP_CSIGMA, c)
        sigma = np.std(u.astype(np.float64))
        lam = min(1.0, c * sigma / np.abs(u).max())
        assert np.isclose(thresh, lam * np.abs(u).max(), rtol=1e-6)
        assert np.isclose(delta, lam * np.abs(u).max() / 7, rtol=1e-6)
    # about 4.6% of a Gaussian vector lies outside 2 sigma
    delta, thresh = lpco.delta_from_stats(st, d, 4, lpco.CLIP_CSIGMA, 2.0)
    _, ncl = lpco.quantize_codes(u, 4, delta, thresh)
    assert 0.03 * d < ncl < 0.06 * d


def test_all_zero_vector_gives_all_zero_message():
    # x_0 = x~ at t = 0 of every epoch of Alg. 1, so u = 0 is a routine input
    d = 100
    U = np.zeros((3, lpco.d_pad(d)), dtype=np.float32)
    packed, delta, ncl, rc = lpco.quantize_clip(U, d, 3)
    assert rc == lpco.OK
    assert not packed.any() and not delta.any() and not ncl.any()
    assert not lpco.dequantize_avg(packed, delta, d, 3).any()


def test_non_finite_input_is_reported():
    d = 64
    U = np.ones((2, d), dtype=np.float32)
    U[1, 5] = np.nan
    _, _, _, rc = lpco.quantize_clip(U, d, 4)
    assert rc == lpco.ENONFINITE
    assert lpco.vector_stats(U[1])[3] == 1


def test_invalid_bit_widths_rejected():
    U = np.ones((1, 32), dtype=np.float32)
    for bits in (0, 1, 17, 31):
        with pytest.raises(lpco.OracleError):
            lpco.quantize_clip(U, 32, bits)


# ---------------------------------------------------------------- Lemma 4 (supplement)

@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("lam", [1.0, 0.9, 0.5])
def test_vector_error_bound_with_clipping(bits, lam):
    # E|Q(w) - w|^2 <= (d - d_lambda) delta^2/4 + d_lambda (1 - lambda)^2 |w|^2
    rng = np.random.default_rng(10 * bits + int(lam * 10))
    d = 2048
    w = rng.standard_normal(d).astype(np.float32)
    st = lpco.vector_stats(w)
    delta, thresh = lpco.delta_from_stats(st, d, bits, lpco.CLIP_LAMBDA, lam)
    errs, ncl = [], 0
    for it in range(200):
        codes, ncl = lpco.quantize_codes(w, bits, delta, thresh, seed=5, iter_=it)
        errs.append(((codes.astype(np.float64) * float(delta) - w.astype(np.float64)) ** 2).sum())
    bound = (d - ncl) * float(delta) ** 2 / 4 + ncl * (1 - lam) ** 2 * float((w.astype(np.float64) ** 2).sum())
    mean, se = np.mean(errs), np.std(errs) / np.sqrt(len(errs))
    assert mean - 3 * se <= bound
    if lam == 1.0:
        # unbiased case: the exact expectation is sum_j (x - z)(z + delta - x)
        x = w.astype(np.float64) / float(delta)
        fr = x - np.floor(x)
        exact = float(delta) ** 2 * (fr * (1 - fr)).sum()
        assert abs(mean - exact) <= 4 * se + 1e-3 * exact


# ---------------------------------------------------------------- ternary special case

def test_two_bits_lambda_one_is_the_ternary_quantizer():
    # b = 2, lambda = 1: one positive level; codes in {-1,0,1}, sign kept,
    # P(code != 0) = |u_j| / |u|_inf  (the ternary gradient quantizer the paper cites)
    p = np.array([1.0, 0.75, 0.5, 0.25, 0.1, 0.0, -0.1, -0.33, -0.9, -1.0])
    reps = 200_000
    u = np.repeat(p, reps).astype(np.float32) * np.float32(2.5)
    st = lpco.vector_stats(u)
    delta, thresh = lpco.delta_from_stats(st, u.size, 2, lpco.CLIP_LAMBDA, 1.0)
    assert delta == np.float32(2.5)
    codes, ncl = lpco.quantize_codes(u, 2, delta, thresh, seed=77)
    assert ncl == 0 and set(np.unique(codes)) <= {-1, 0, 1}
    codes = codes.reshape(len(p), reps)
    for row, pj in zip(codes, p):
        assert np.all(row * np.sign(pj) >= 0)
        freq = np.mean(row != 0)
        assert abs(freq - abs(pj)) <= 4 * np.sqrt(max(abs(pj) * (1 - abs(pj)), 1e-12) / reps) + 1e-7


# ---------------------------------------------------------------- message format

def _bitstream_words(codes, bits):
    """Independent statement of the layout: one little-endian integer bit stream."""
    stream = 0
    for j, k in enumerate(codes):
        stream |= (int(k) & ((1 << bits) - 1)) << (j * bits)
    nwords = ((len(codes) + 31) // 32) * bits
    raw = stream.to_bytes(nwords * 4, "little")
    return np.frombuffer(raw, dtype="<u4")


@pytest.mark.parametrize("bits", list(range(2, 17)))
def test_pack_round_trip_every_code_at_every_lane(bits):
    ncodes = 1 << bits
    reps = min(ncodes, 256)  # every code value meets every lane position when ncodes <= 256
    j = np.arange(32 * reps * (ncodes // reps if ncodes > 256 else 1))
    if ncodes <= 256:
        codes = ((j // 32 + j % 32) % ncodes) - ncodes // 2
    else:
        codes = ((j * 2654435761) % ncodes) - ncodes // 2   # all lanes, a spread of values
        codes[:ncodes] = np.arange(ncodes) - ncodes // 2     # and every value at least once
    codes = codes.astype(np.int32)
    words = lpco.pack(codes, bits)
    assert words.size == lpco.words_per_msg(codes.size, bits) == codes.size // 32 * bits
    assert np.array_equal(lpco.unpack(words, codes.size, bits), codes)
    small = codes[:96 + 7]
    assert np.array_equal(lpco.pack(small, bits), _bitstream_words(small, bits))


def test_message_size_and_table1():
    # Sec. 4.2: 32 + b d bits per message; Table 1 totals (fixture computed by hand)
    with open(os.path.join(GOLDEN, "table1_bits.txt")) as f:
        rows = [list(map(int, l.split())) for l in f if l.strip() and not l.startswith("#")]
    for d, b, N, bits_a, bits_b, bits_c, bits_msg in rows:
        assert lpco.bits_per_message(d, b) == bits_msg
        assert lpco.bits_per_iteration(d, b, N, lpco.SCHEME_A) == bits_a
        assert lpco.bits_per_iteration(d, b, N, lpco.SCHEME_B) == bits_b
        assert lpco.bits_per_iteration(d, b, N, lpco.SCHEME_C) == bits_c
        # communication-reduced factor of schemes (a), (c): 32 / (32/d + b)
        assert np.isclose(32 * d / bits_msg, 32 / (32 / d + b))
        # the packed buffer holds exactly the b*d_pad code bits; delta travels beside it
        assert lpco.words_per_msg(d, b) * 32 == b * lpco.d_pad(d)
    assert lpco.d_pad(1) == 32 and lpco.d_pad(32) == 32 and lpco.d_pad(33) == 64


def test_ragged_tail_is_padded_with_zero_codes():
    d, bits = 45, 5
    U = np.zeros((1, lpco.d_pad(d)), dtype=np.float32)
    U[0, :d] = np.linspace(-1, 1, d, dtype=np.float32)
    packed, delta, _, _ = lpco.quantize_clip(U, d, bits)
    allcodes = lpco.unpack(packed[0], lpco.d_pad(d), bits)
    assert not allcodes[d:].any() and allcodes[:d].any()


# ---------------------------------------------------------------- eq. (4) and schemes (b), (c)

def test_dequantize_avg_matches_exact_rational_average():
    rng = np.random.default_rng(5)
    d, N, bits = 1000, 8, 4
    U = np.zeros((N, lpco.d_pad(d)), dtype=np.float32)
    U[:, :d] = rng.standard_normal((N, d)).astype(np.float32) * rng.uniform(0.1, 10, size=(N, 1)).astype(np.float32)
    packed, delta, _, _ = lpco.quantize_clip(U, d, bits, lpco.CLIP_LAMBDA, 0.9, seed=3)
    avg = lpco.dequantize_avg(packed, delta, d, bits)
    codes = np.stack([lpco.unpack(packed[i], d, bits) for i in range(N)])
    for j in range(0, d, 37):
        exact = sum(Fraction(float(delta[i])) * int(codes[i, j]) for i in range(N)) / N
        scale = sum(abs(Fraction(float(delta[i])) * int(codes[i, j])) for i in range(N)) / N
        assert abs(Fraction(float(avg[j])) - exact) <= scale * Fraction(N, 1 << 23) + Fraction(1, 1 << 140)
    # one worker: the message decodes to delta * code exactly
    one = lpco.dequantize_avg(packed[:1], delta[:1], d, bits)
    assert np.array_equal(one, (delta[0] * codes[0].astype(np.float32)).astype(np.float32))


def test_quantized_average_is_unbiased_when_lambda_is_one():
    # E[u~_t] = (1/N) sum_i u^i for lambda = 1 (Sec. 4.1 + eq. (4))
    rng = np.random.default_rng(6)
    d, N, bits = 64, 4, 3
    U = np.zeros((N, d), dtype=np.float32)
    U[:] = rng.standard_normal((N, d)).astype(np.float32)
    acc = np.zeros(d)
    T = 20_000
    for it in range(T):
        packed, delta, _, _ = lpco.quantize_clip(U, d, bits, seed=8, epoch=1, iter_=it)
        acc += lpco.dequantize_avg(packed, delta, d, bits)
    mean = acc / T
    truth = U.astype(np.float64).mean(axis=0)
    dl = np.abs(U).max(axis=1) / _levels(bits)
    se = np.sqrt((dl ** 2 / 4).sum()) / N / np.sqrt(T)
    assert np.all(np.abs(mean - truth) <= 4.5 * se)


def test_plain_average_when_quantization_is_off():
    rng = np.random.default_rng(7)
    U = rng.standard_normal((8, 96)).astype(np.float32)
    avg = lpco.plain_avg(U, 90)
    assert np.allclose(avg, U[:, :90].astype(np.float64).mean(axis=0), rtol=0, atol=1e-6)


def test_shared_scale_schemes():
    # scheme (b): all workers use delta = max_i delta_i; codes add as integers within
    # ceil(log2 N) extra bits; scheme (c): the average is re-quantized without bias (eq. (5))
    rng = np.random.default_rng(8)
    d, N, bits = 512, 8, 3
    U = (rng.standard_normal((N, d)) * rng.uniform(0.5, 2, size=(N, 1))).astype(np.float32)
    L = _levels(bits)
    deltas = [lpco.delta_from_stats(lpco.vector_stats(U[i]), d, bits, lpco.CLIP_LAMBDA, 1.0)[0] for i in range(N)]
    dmax = max(deltas)
    assert dmax == np.abs(U).max() / np.float32(L)
    shared = np.full(N, dmax, dtype=np.float32)
    packed, dout, _, _ = lpco.quantize_clip(U, d, bits, seed=4, delta_in=shared)
    assert np.all(dout == dmax)
    avg_b, sums = lpco.dequantize_shared(packed, dmax, d, bits)
    codes = np.stack([lpco.unpack(packed[i], d, bits) for i in range(N)])
    assert np.array_equal(sums, codes.sum(axis=0))
    assert np.abs(sums).max() <= N * (L + 1)          # fits b + ceil(log2 N) bits
    assert np.allclose(avg_b, dmax * codes.mean(axis=0), rtol=1e-6, atol=0)
    # (c): values on the grid of delta, adjacent to the scheme-(b) average, unbiased around it
    acc = np.zeros(d)
    T = 4000
    for it in range(T):
        avg_c, _ = lpco.dequantize_shared(packed, dmax, d, bits, requantize=True, seed=4, iter_=it)
        k = avg_c / dmax
        assert np.allclose(k, np.round(k), atol=1e-5) and np.abs(k).max() <= L + 1
        assert np.all(np.abs(avg_c - avg_b) <= dmax * (1 + 1e-5))
        acc += avg_c
    assert np.all(np.abs(acc / T - avg_b) <= 4.5 * dmax / 2 / np.sqrt(T) + 1e-7)
