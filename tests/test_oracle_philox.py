"""Pins for the oracle's random stream (Philox4x32-10 and the uniform / Bernoulli mapping)."""
import os

import numpy as np

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat_rows():
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            w = [int(x, 16) for x in line.split()]
            yield w[0:4], w[4:6], w[6:10]


def test_known_answers():
    rows = list(_kat_rows())
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = oracle.philox4x32_10(ctr, key)
        assert [int(x) for x in got] == want


def test_uniform_is_word_shifted_by_8_times_2_pow_minus_24():
    # atom i uses word i mod 4 of block i div 4; counter words 2,3 carry the stream, the key the seed
    seed, stream = 0x0123456789ABCDEF, 0xFEDCBA9876543210
    u = oracle.uniforms(seed, stream, 37)
    for i in (0, 1, 2, 3, 4, 5, 18, 36):
        blk = i // 4
        words = oracle.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, stream & 0xFFFFFFFF, stream >> 32],
                                     [seed & 0xFFFFFFFF, seed >> 32])
        assert u[i] == np.float32((int(words[i % 4]) >> 8) / 2.0 ** 24)
    assert u.dtype == np.float32
    assert (u >= 0).all() and (u < 1).all()
    assert np.array_equal(u * 2 ** 24, np.floor(u * 2 ** 24))          # exact multiples of 2^-24


def test_uniforms_first_offset_and_streams_differ():
    a = oracle.uniforms(5, 9, 100)
    b = oracle.uniforms(5, 9, 40, first=60)
    assert np.array_equal(a[60:], b)
    assert not np.array_equal(a, oracle.uniforms(5, 10, 100))
    assert not np.array_equal(a, oracle.uniforms(6, 9, 100))
    # high halves of seed and stream matter too
    assert not np.array_equal(a, oracle.uniforms(5 + (1 << 32), 9, 100))
    assert not np.array_equal(a, oracle.uniforms(5, 9 + (1 << 32), 100))


def test_uniforms_are_uniform():
    u = oracle.uniforms(11, 3, 400_000).astype(np.float64)
    n = u.size
    assert abs(u.mean() - 0.5) < 5 * np.sqrt(1 / 12 / n)
    assert abs((u ** 2).mean() - 1 / 3) < 5 * np.sqrt((1 / 5 - 1 / 9) / n)
    hist, _ = np.histogram(u, bins=64, range=(0, 1))
    chi2 = ((hist - n / 64) ** 2 / (n / 64)).sum()
    assert chi2 < 63 + 6 * np.sqrt(2 * 63)
    # neighbouring atoms (words of one block, and of consecutive blocks) are uncorrelated
    for lag in (1, 2, 3, 4):
        c = np.corrcoef(u[:-lag], u[lag:])[0, 1]
        assert abs(c) < 5 / np.sqrt(n)


def test_bernoulli_decision_and_edge_probabilities():
    n = 50_000
    p = np.full(n, 0.3, dtype=np.float32)
    mask = oracle.bernoulli_mask(p, 1, 2)
    u = oracle.uniforms(1, 2, n)
    assert np.array_equal(mask, u < p)
    assert abs(mask.mean() - 0.3) < 5 * np.sqrt(0.21 / n)
    assert oracle.bernoulli_mask(np.ones(n, np.float32), 1, 2).all()       # p = 1 always kept
    assert not oracle.bernoulli_mask(np.zeros(n, np.float32), 1, 2).any()  # p = 0 never kept
