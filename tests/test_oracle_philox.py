"""Pins for the oracle's counter-based uniform draw."""
import math
import os

import numpy as np

from oracle import tsd_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        yield w[:4], w[4:6], tuple(w[6:])


def test_known_answer_vectors():
    n = 0
    for ctr, key, out in _kat():
        assert orc.philox4x32_10(ctr, key) == out
        n += 1
    assert n == 3


def test_bulk_equals_scalar():
    rng = np.random.default_rng(5)
    c = rng.integers(0, 2 ** 32, size=(4, 200), dtype=np.uint64)
    key = (0x1234ABCD, 0x9E3779B9)
    bulk = orc.philox4x32_10_bulk(c[0], c[1], c[2], c[3], key)
    for j in range(200):
        assert int(bulk[j]) == orc.philox4x32_10([int(c[i, j]) for i in range(4)], key)[0]


def test_uniform_lattice():
    # 23-bit mid-point lattice: strictly inside (0, 1) and exact in float32
    assert orc.word_to_uniform(0) == 2.0 ** -24
    assert orc.word_to_uniform(0xFFFFFFFF) == 1.0 - 2.0 ** -24
    for w in (0, 1, 511, 512, 0x80000000, 0xFFFFFFFF, 0x12345678):
        u = orc.word_to_uniform(w)
        assert 0.0 < u < 1.0 and float(np.float32(u)) == u
    # keyed by (seed, series, round, position): changing any of them changes the draw
    base = orc.uniform(7, 3, 2, 1)
    assert len({base, orc.uniform(8, 3, 2, 1), orc.uniform(7, 4, 2, 1), orc.uniform(7, 3, 3, 1),
                orc.uniform(7, 3, 2, 2), orc.uniform(7 + (1 << 32), 3, 2, 1)}) == 6
    # counter layout: (series, round, position, 0), key = (seed low, seed high), word 0
    seed = (0x299F31D0 << 32) | 0xA4093822
    w0 = orc.philox4x32_10((5, 6, 7, 0), (0xA4093822, 0x299F31D0))[0]
    assert orc.uniform(seed, 5, 6, 7) == orc.word_to_uniform(w0)


def test_uniform_statistics():
    # mean 1/2, variance 1/12, and P(log u <= ell) = e^ell (the Bernoulli(alpha) draw of the round)
    n = 400_000
    b = np.arange(n) % 1000
    r = np.arange(n) // 1000
    w = orc.philox4x32_10_bulk(b, r, 1, 0, (2021, 0))
    u = ((w >> np.uint64(9)).astype(np.float64) + 0.5) * 2.0 ** -23
    assert abs(u.mean() - 0.5) < 4 * math.sqrt(1 / 12 / n)
    assert abs(u.var() - 1 / 12) < 1e-3
    for ell in (-0.05, -0.5, -1.0, -3.0):
        p = math.exp(ell)
        frac = np.mean(np.log(u) <= ell)
        assert abs(frac - p) < 4 * math.sqrt(p * (1 - p) / n)
    # successive positions of the same (series, round) are uncorrelated
    w2 = orc.philox4x32_10_bulk(b, r, 2, 0, (2021, 0))
    u2 = ((w2 >> np.uint64(9)).astype(np.float64) + 0.5) * 2.0 ** -23
    assert abs(np.corrcoef(u, u2)[0, 1]) < 4 / math.sqrt(n)


def test_bulk_all_words_equals_scalar():
    # the sampled variants consume all four output words of a block
    rng = np.random.default_rng(5)
    c = rng.integers(0, 2 ** 32, size=(50, 4), dtype=np.uint64)
    key = (0xA4093822, 0x299F31D0)
    w = orc.philox4x32_10_bulk(c[:, 0], c[:, 1], c[:, 2], c[:, 3], key, all_words=True)
    assert w.shape == (50, 4)
    for row, ctr in zip(w, c):
        assert tuple(int(x) for x in row) == orc.philox4x32_10(tuple(int(x) for x in ctr), key)
