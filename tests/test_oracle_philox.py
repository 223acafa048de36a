"""Pins for the oracle's counter-based generator and its samplers (CPU only)."""
import os

import numpy as np
import pytest

from oracle import lpco

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(t, 16) for t in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


@pytest.mark.parametrize("ctr,key,out", _kat_rows())
def test_philox_known_answers(ctr, key, out):
    got = lpco.philox4x32_10(ctr, key)
    assert [int(x) for x in got] == out


def test_stream_word_layout():
    # word `index` = lane (index & 3) of the block with counter
    # (index >> 2, tag << 24 | worker, iter, epoch) and key (seed_lo, seed_hi)
    seed = 0x0123456789ABCDEF
    for (epoch, it, tag, worker, index) in [(0, 0, 0, 0, 0), (3, 17, 1, 5, 6), (9, 2, 2, 0xFFFFFF, 1023),
                                           (1, 1, 0, 15, (1 << 34) + 7)]:
        blk = lpco.philox4x32_10([(index >> 2) & 0xFFFFFFFF, (tag << 24) | worker, it, epoch],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        assert lpco.stream_word(seed, epoch, it, tag, worker, index) == int(blk[index & 3])


def test_streams_are_distinct():
    base = [lpco.stream_word(1, 0, 0, 0, 0, j) for j in range(64)]
    for args in [(2, 0, 0, 0, 0), (1, 1, 0, 0, 0), (1, 0, 1, 0, 0), (1, 0, 0, 1, 0), (1, 0, 0, 0, 1)]:
        other = [lpco.stream_word(*args, j) for j in range(64)]
        assert sum(a == b for a, b in zip(base, other)) == 0


def test_uniform_words_bit_balance():
    # each of the 32 bit positions is set about half of the time (binomial, 5 sigma)
    n = 1 << 15
    words = np.array([lpco.stream_word(7, 0, 0, 0, 0, j) for j in range(n)], dtype=np.uint64)
    for b in range(32):
        ones = int(((words >> np.uint64(b)) & np.uint64(1)).sum())
        assert abs(ones - n / 2) < 5 * np.sqrt(n / 4)


def test_sample_batch_uniform_chi_square():
    # Alg. 1 step 6: indices uniform on {0..n-1}; chi-square against the flat law
    from scipy import stats
    n, B = 64, 1 << 16
    idx = lpco.sample_batch(11, 2, 3, lpco.TAG_BATCH, 1, B, n)
    assert idx.min() >= 0 and idx.max() < n
    counts = np.bincount(idx, minlength=n)
    chi2 = ((counts - B / n) ** 2 / (B / n)).sum()
    assert stats.chi2.sf(chi2, n - 1) > 1e-4
    # floor(word * n / 2^32) by an independent big-integer evaluation
    for p in range(32):
        word = lpco.stream_word(11, 2, 3, lpco.TAG_BATCH, 1, p)
        assert idx[p] == (word * n) // (1 << 32)


def test_sample_batch_non_power_of_two_and_with_replacement():
    n, B = 1000, 4096
    idx = lpco.sample_batch(5, 0, 0, lpco.TAG_BATCH, 0, B, n)
    assert idx.min() >= 0 and idx.max() < n
    assert len(np.unique(idx)) < B  # with replacement: B > n forces repeats


def test_worker_batches_differ_and_shared_batch_is_one_stream():
    # Alg. 1 step 6: workers sample independently; Alg. 2 step 11 + Sec. 5: J is the
    # same on every worker (one stream, no worker id in it)
    n, B = 1 << 20, 64
    b0 = lpco.sample_batch(3, 1, 4, lpco.TAG_BATCH, 0, B, n)
    b1 = lpco.sample_batch(3, 1, 4, lpco.TAG_BATCH, 1, B, n)
    J = lpco.sample_batch(3, 1, 4, lpco.TAG_SHARED, 0xFFFFFF, B, n)
    assert (b0 != b1).sum() > B - 3
    assert (J != b0).sum() > B - 3 and (J != b1).sum() > B - 3
    # determinism: the same arguments give the same batch
    assert np.array_equal(b0, lpco.sample_batch(3, 1, 4, lpco.TAG_BATCH, 0, B, n))
    # different iterations are independent draws (Assumption 1)
    assert (b0 != lpco.sample_batch(3, 1, 5, lpco.TAG_BATCH, 0, B, n)).sum() > B - 3
