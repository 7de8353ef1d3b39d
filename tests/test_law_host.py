"""The library-side throughput-law helpers (used for reporting) against the oracle's, written
independently, and against the closed forms."""
import math

import numpy as np

from oracle import tsd_oracle as orc
from paper_2511_18191_amd import law


def test_law_helpers_agree_with_oracle():
    rng = np.random.default_rng(1)
    for _ in range(300):
        a, c, v, K = rng.uniform(0.01, 0.999), rng.uniform(0.01, 0.9), rng.uniform(0.7, 4.0), int(rng.integers(1, 12))
        assert math.isclose(law.mean_block_length(a, K), orc.expected_block_length(a, K), rel_tol=1e-12)
        assert math.isclose(law.speedup(a, K, c, v), orc.predicted_speedup(a, K, c, v), rel_tol=1e-12)
        assert law.one_more_position_pays(a, K, c, v) == orc.next_position_pays(a, K, c, v)
    assert law.mean_block_length(1.0, 4) == 5.0 and law.mean_block_length(0.0, 4) == 1.0


def test_best_block_size_is_where_the_marginal_gain_stops():
    for a, c, v in ((0.9, 0.1, 1.0), (0.7, 0.2, 1.0), (0.5, 0.05, 1.2), (0.95, 0.02, 1.0)):
        K = law.best_block_size(a, c, v, k_max=16)
        S = [law.speedup(a, k, c, v) for k in range(1, 17)]
        assert all(S[k] >= S[k - 1] - 1e-15 for k in range(1, K))         # every step up to K paid
        if K < 16:
            assert S[K] < S[K - 1]                                           # the next one does not


def test_planner_arithmetic_agrees_with_oracle():
    rng = np.random.default_rng(2)
    for _ in range(300):
        a, c, v = rng.uniform(0.05, 0.995), rng.uniform(0.005, 0.8), rng.uniform(0.8, 5.0)
        assert law.best_block_size(a, c, v, k_max=16) == orc.choose_block_size(a, c, v, 16)
    for n, d in ((10, 0.05), (256, 0.01)):
        assert math.isclose(law.acceptance_confidence(n, d), orc.hoeffding_halfwidth(n, d), rel_tol=1e-12)
