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


def test_batch_round_simulation_follows_the_capped_geometric_law():
    # the Monte Carlo that predicts a batch's rounds, against what the law fixes: certain acceptance commits K + 1
    # patches a round, certain rejection one; one series with a long horizon commits E[L] of Eq. 7 per round;
    # the number of series still decoding never grows; the horizon cuts the last block
    for K, T in ((4, 8), (6, 15), (1, 5)):
        act, pos = law.simulate_batch_rounds(np.ones(7), K, T, reps=3)
        assert act.shape[1] == -(-T // (K + 1)) and (act == 7).all()
        act, pos = law.simulate_batch_rounds(np.zeros(5), K, T, reps=3)
        assert act.shape[1] == T and (act == 5).all()
        assert (pos[:, -1] == min(K, 1)).all() and (pos[:, 0] == min(K, T)).all()
    for a, K in ((0.5, 3), (0.8, 6), (0.3, 8)):
        T = 4000
        act, _ = law.simulate_batch_rounds([a], K, T, reps=40, seed=3)
        rounds = (act > 0).sum(axis=1)
        L = T / rounds.mean()
        assert abs(L - law.mean_block_length(a, K)) < 0.02 * law.mean_block_length(a, K), (a, K, L)
    rng = np.random.default_rng(5)
    act, pos = law.simulate_batch_rounds(rng.uniform(0.2, 0.95, size=64), 4, 8, reps=50, seed=1)
    assert (np.diff(act, axis=1) <= 0).all() and (act[:, 0] == 64).all() and (act.max(axis=1) == 64).all()
    assert ((pos >= 0) & (pos <= 4)).all() and (pos[act > 0] >= 1).all() and (pos[act == 0] == 0).all()
    # a heterogeneous batch needs more rounds than its average series: the slowest series sets the count
    per_series = np.mean([(law.simulate_batch_rounds([x], 4, 8, reps=200, seed=2)[0] > 0).sum(axis=1).mean() for x in (0.3, 0.9)])
    both = (law.simulate_batch_rounds([0.3, 0.9], 4, 8, reps=200, seed=2)[0] > 0).sum(axis=1).mean()
    assert both > per_series
