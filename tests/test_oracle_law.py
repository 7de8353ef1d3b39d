"""Pins for the throughput law (Eq. 7, Eq. 8) and the marginal-gain criterion for K."""
import math
import os

import numpy as np

from oracle import tsd_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_table_b2_timemoe.txt")


def test_pmf_and_mean():
    for alpha in (0.0, 0.3, 0.9, 1.0):
        for K in (1, 4, 8):
            pmf = orc.block_length_pmf(alpha, K)
            assert math.isclose(pmf.sum(), 1.0, rel_tol=1e-12)
            mean = float(np.dot(np.arange(1, K + 2), pmf))
            assert math.isclose(mean, orc.expected_block_length(alpha, K), rel_tol=1e-12)
            # tail-sum form: E[L] = sum_{j=0..K} alpha^j
            assert math.isclose(mean, sum(alpha ** j for j in range(K + 1)), rel_tol=1e-12)
    assert orc.expected_block_length(0.0, 5) == 1.0 and orc.expected_block_length(1.0, 5) == 6.0


def test_marginal_criterion_is_equivalent_to_comparing_speedups():
    rng = np.random.default_rng(0)
    for _ in range(500):
        a, c, v = rng.uniform(0.05, 0.99), rng.uniform(0.01, 0.8), rng.uniform(0.8, 3.0)
        K = int(rng.integers(1, 9))
        direct = orc.predicted_speedup(a, K + 1, c, v) >= orc.predicted_speedup(a, K, c, v)
        assert orc.next_position_pays(a, K, c, v) == direct
    assert math.isclose(orc.predicted_speedup(0.9, 3, 0.1, 1.0), 3.439 / 1.3, rel_tol=1e-12)


def test_consistent_with_paper_block_size_sweep():
    # Time-MoE rows of the appendix K sweep: the implied round cost E[L]/S must be close to
    # affine in K with intercept v ~ 1 (single-pass verification) and a small positive slope c.
    rows = [tuple(map(float, l.split())) for l in open(GOLD) if not l.startswith("#") and l.strip()]
    K = np.array([r[0] for r in rows])
    cost = np.array([orc.expected_block_length(r[1], int(r[0])) / r[2] for r in rows])
    c, v = np.polyfit(K, cost, 1)
    assert 0.05 < c < 0.25 and 0.8 < v < 1.2
    assert np.abs(np.polyval([c, v], K) - cost).max() < 0.06
    for r in rows:
        assert abs(orc.predicted_speedup(r[1], int(r[0]), c, v) - r[2]) < 0.12


def test_choose_block_size_is_the_argmax_of_eq8():
    # the marginal condition's slack falls strictly with K, so the first K at which it fails maximises S
    rng = np.random.default_rng(3)
    for _ in range(400):
        a, c, v = rng.uniform(0.05, 0.995), rng.uniform(0.005, 0.8), rng.uniform(0.8, 5.0)
        S = [orc.predicted_speedup(a, K, c, v) for K in range(1, 33)]
        assert orc.choose_block_size(a, c, v, 32) == int(np.argmax(S)) + 1
        slack = [a ** (K + 1) * (c * K + v) - c * orc.expected_block_length(a, K) for K in range(1, 33)]
        assert all(x > y - 1e-15 for x, y in zip(slack, slack[1:])) and slack[0] > slack[4]
    assert orc.choose_block_size(0.9, 0.1, 1.0, 3) == 3            # capped
    assert orc.choose_block_size(0.1, 0.9, 1.0, 16) == 1            # nothing pays


def test_hoeffding_halfwidth_bound_and_coverage():
    for n, delta in ((64, 0.05), (256, 0.01), (1024, 0.1)):
        eps = orc.hoeffding_halfwidth(n, delta)
        assert math.isclose(2 * math.exp(-2 * n * eps * eps), delta, rel_tol=1e-12)
    # Monte Carlo: per-history terms in [0, 1] (accepted fraction of a few Bernoulli positions)
    rng = np.random.default_rng(4)
    n, delta, p = 128, 0.05, 0.7
    eps = orc.hoeffding_halfwidth(n, delta)
    terms = rng.binomial(4, p, size=(20000, n)) / 4.0
    miss = np.mean(np.abs(terms.mean(axis=1) - p) >= eps)
    assert miss <= delta                                             # the bound holds (it is loose: miss ~ 0)
    assert eps < 0.13 and orc.hoeffding_halfwidth(4 * n, delta) == eps / 2
