"""Pins for the oracle's evaluators: gradient mapping (Sec. 3.3), Theorem 2's step-size conditions
(eq. (6), (7)), and the entropy coding of the code stream (Sec. 6.1)."""
import heapq
from fractions import Fraction

import numpy as np
import pytest

import lpc_synth
from oracle import lpco
from _common import oracle_problem


def test_gradient_mapping_reduces_to_the_gradient_without_h():
    # h = 0: prox is the identity, so G_eta(x) = grad f(x) for every eta
    sp = lpc_synth.make("c4", n=128, d=9)
    sp.lambda1 = sp.lambda2 = 0.0
    p, _k = oracle_problem(sp)
    w = np.random.default_rng(0).standard_normal(9).astype(np.float32)
    mu, _, _ = lpco.full_grad(p, w)
    for eta in (0.01, 0.3):
        assert np.isclose(lpco.gradient_mapping(p, w, eta), float((mu.astype(np.float64) ** 2).sum()), rtol=1e-5)


def test_gradient_mapping_vanishes_at_the_minimiser_and_only_there():
    # x* = prox_{eta h}(x* - eta grad f(x*)) characterises the minimiser of eq. (1)
    sp = lpc_synth.make("c4", n=256, d=8)
    sp.lambda2 = 0.1
    p, _k = oracle_problem(sp)
    X, t = sp.X.astype(np.float64), sp.y.astype(np.float64)
    w_star = np.linalg.solve(X.T @ X / sp.n + sp.lambda2 * np.eye(sp.d), X.T @ t / sp.n)
    assert lpco.gradient_mapping(p, w_star.astype(np.float32), 0.05) <= 1e-10
    assert lpco.gradient_mapping(p, (w_star + 0.1).astype(np.float32), 0.05) > 1e-4
    # L1: zero is stationary when |grad f(0)|_inf <= lambda1
    sp1 = lpc_synth.make("c1", n=128, d=10)
    p1, _k1 = oracle_problem(sp1)
    g0 = np.abs(lpco.full_grad(p1, np.zeros(10, np.float32))[0]).max()
    p1.lambda1 = float(g0) * 1.01
    assert lpco.gradient_mapping(p1, np.zeros(10, np.float32), 0.1) == 0.0
    p1.lambda1 = float(g0) * 0.5
    assert lpco.gradient_mapping(p1, np.zeros(10, np.float32), 0.1) > 0.0


def test_theorem2_condition_values():
    # eq. (6): 8 m^2 rho^2 [ d lambda^2 / (4 (2^(b-1)-1)^2) + d_lambda (1-lambda)^2 + 1/(NB) ] + rho, by hand:
    # d=64, b=4 (7 levels), lambda=1, d_lambda=0, N=4, B=16, m=2, rho=0.1:
    #   bracket = 64/(4*49) + 0 + 1/64 = 0.326530612... + 0.015625 = 0.342155612...
    #   8*4*0.01*bracket + 0.1 = 0.32*0.342155612 + 0.1 = 0.209489796
    exact = Fraction(8 * 4, 100) * (Fraction(64, 4 * 49) + Fraction(1, 64)) + Fraction(1, 10)
    assert np.isclose(lpco.theorem2_lhs(64, 4, 1.0, 0, 4, 16, 2, 0.1, lpco.SCHEME_A), float(exact), rtol=1e-12)
    assert np.isclose(float(exact), 0.209489796, atol=1e-9)
    # eq. (7) replaces 1/4 by 3/8 in the first term; clipping adds d_lambda (1-lambda)^2
    exact_c = Fraction(8 * 4, 100) * (Fraction(3 * 64, 8 * 49) + Fraction(1, 64)) + Fraction(1, 10)
    assert np.isclose(lpco.theorem2_lhs(64, 4, 1.0, 0, 4, 16, 2, 0.1, lpco.SCHEME_C), float(exact_c), rtol=1e-12)
    lam = 0.5
    exact_l = Fraction(8 * 4, 100) * (Fraction(64, 4 * 49) * Fraction(1, 4) + 3 * Fraction(1, 4) + Fraction(1, 64)) + Fraction(1, 10)
    assert np.isclose(lpco.theorem2_lhs(64, 4, lam, 3, 4, 16, 2, 0.1, lpco.SCHEME_B), float(exact_l), rtol=1e-12)
    # Corollary 1: with b = O(log sqrt(d)) and eta = O(1/(mL)) the condition can be met: b = log2(sqrt(d)) + 2
    for d in (2 ** 10, 2 ** 16, 2 ** 20):
        b = int(np.log2(np.sqrt(d))) + 2
        m = 64
        assert lpco.theorem2_lhs(d, b, 1.0, 0, 8, 64, m, 0.1 / m, lpco.SCHEME_A) <= 1.0


def _heap_huffman_bits(counts):
    """Textbook Huffman with a heap (independent of the oracle's selection loop)."""
    h = [(int(c), i) for i, c in enumerate(counts) if c > 0]
    if len(h) == 1:
        return h[0][0]
    heapq.heapify(h)
    total, nxt = 0, len(counts)
    while len(h) > 1:
        a = heapq.heappop(h); b = heapq.heappop(h)
        total += a[0] + b[0]           # every merge adds one bit to each leaf below it
        heapq.heappush(h, (a[0] + b[0], nxt)); nxt += 1
    return total


def test_huffman_lengths_known_example_and_bounds():
    # the classic six-symbol example: frequencies 45, 13, 12, 16, 9, 5 -> lengths 1, 3, 3, 3, 4, 4; 224 bits
    bits, lens = lpco.huffman_bits([45, 13, 12, 16, 9, 5])
    assert bits == 224 and sorted(lens) == [1, 3, 3, 3, 4, 4] and lens[0] == 1
    # uniform alphabet of 2^k symbols: exactly k bits each
    bits, lens = lpco.huffman_bits([7] * 16)
    assert bits == 7 * 16 * 4 and set(lens) == {4}
    # a single used symbol costs one bit per coordinate; unused symbols get no code
    bits, lens = lpco.huffman_bits([0, 0, 1000, 0])
    assert bits == 1000 and list(lens) == [0, 0, 1, 0]
    rng = np.random.default_rng(0)
    for _ in range(20):
        counts = rng.integers(0, 1000, size=rng.integers(2, 64))
        if counts.sum() == 0:
            continue
        bits, lens = lpco.huffman_bits(counts)
        assert bits == _heap_huffman_bits(counts)
        used = counts > 0
        if used.sum() > 1:
            assert np.isclose(sum(2.0 ** -l for l in lens[used]), 1.0)       # Kraft equality of a full code tree
            pr = counts[used] / counts.sum()
            H = -(pr * np.log2(pr)).sum()
            assert H * counts.sum() - 1e-6 <= bits < (H + 1) * counts.sum()   # Shannon's bounds


def test_code_histogram_and_entropy_coded_message_size():
    # Gaussian-like u, 7 levels (b=4), lambda = 0.9: most codes are 0 or +-1, so the entropy-coded message
    # is smaller than the fixed b bits per coordinate of Sec. 4.2
    d, bits = 50_000, 4
    U = lpc_synth.gaussian_u(1, d, seed=3)
    packed, delta, _, _ = lpco.quantize_clip(U, d, bits, lpco.CLIP_LAMBDA, 0.9, seed=1)
    counts = lpco.code_histogram(packed[0], d, bits)
    codes = lpco.unpack(packed[0], d, bits)
    assert counts.sum() == d and np.array_equal(counts, np.bincount(codes + 8, minlength=16))
    hb, _ = lpco.huffman_bits(counts)
    assert hb < bits * d and hb >= d


# ---------------------------------------------------------------- the entropy-coded stream itself

def _bitstring(stream, total):
    return "".join(str((int(stream[p >> 5]) >> (p & 31)) & 1) for p in range(total))


def test_stream_of_a_small_message_written_out_by_hand():
    # b = 2: bins 0..3 are the codes -2, -1, 0, 1.  Lengths (3, 2, 1, 3): ordered by (length, bin) the canonical
    # codewords are bin 2 -> "0", bin 1 -> "10", bin 0 -> "110", bin 3 -> "111".
    lens = np.array([3, 2, 1, 3], np.int32)
    codes = np.array([0, 0, -1, 1, 0, -2, -1, 0], np.int32)
    words = lpco.pack(codes, 2)
    stream, total = lpco.huffman_encode(words, len(codes), 2, lens)
    assert _bitstring(stream, total) == "0" + "0" + "10" + "111" + "0" + "110" + "10" + "0"
    assert total == 14 and stream.size == 1
    # the stream's first bit is bit 0 of word 0: "00101110110100" read from the low end
    assert int(stream[0]) == int("00101110110100"[::-1], 2)
    assert np.array_equal(lpco.huffman_decode(stream, total, len(codes), 2, lens), codes)


@pytest.mark.parametrize("bits,d,scale", [(2, 1000, 0.5), (4, 4097, 1.0), (8, 3000, 3.0), (3, 31, 0.1)])
def test_stream_round_trip_and_size(bits, d, scale):
    rng = np.random.default_rng(bits * 100 + d)
    half = 1 << (bits - 1)
    codes = np.clip(np.rint(scale * rng.standard_normal(d)), -half, half - 1).astype(np.int32)
    words = lpco.pack(codes, bits)
    counts = lpco.code_histogram(words, d, bits)
    size, lens = lpco.huffman_bits(counts)
    stream, total = lpco.huffman_encode(words, d, bits, lens)
    assert total == size == int((counts * lens.astype(np.uint64)).sum())
    assert stream.size == (total + 31) // 32
    assert np.array_equal(lpco.huffman_decode(stream, total, d, bits, lens), codes)
    # no codeword is a prefix of another (checked on the bit strings themselves)
    used = np.flatnonzero(lens)
    book = {}
    for k in used:
        one = lpco.pack(np.array([k - half], np.int32), bits)
        s, t = lpco.huffman_encode(one, 1, bits, lens)
        book[int(k)] = _bitstring(s, t)
        assert t == lens[k]
    words_sorted = sorted(book.values())
    for a, b in zip(words_sorted, words_sorted[1:]):
        assert not b.startswith(a)


def test_stream_rejects_lengths_that_are_no_prefix_code_and_unused_symbols():
    codes = np.array([0, 1, -1, 0], np.int32)
    words = lpco.pack(codes, 2)
    with pytest.raises(Exception):
        lpco.huffman_encode(words, 4, 2, np.array([1, 1, 1, 0], np.int32), capacity_words=4)   # Kraft sum 3/2
    with pytest.raises(Exception):
        lpco.huffman_encode(words, 4, 2, np.array([0, 1, 2, 0], np.int32), capacity_words=4)   # code 1 has no codeword
    with pytest.raises(Exception):
        lpco.huffman_encode(words, 4, 2, np.array([0, 2, 1, 2], np.int32), capacity_words=0)   # does not fit
