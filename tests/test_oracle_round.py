"""Invariants of one speculative round and of the whole forecast loop (oracle only)."""
import itertools
import math

import numpy as np
import pytest
from scipy import stats

import synth
from oracle import tsd_oracle as orc


def _setup(name="cfg1", B=None):
    cfg = synth.get_config(name)
    rng = np.random.default_rng(cfg.weight_seed)
    Wt = orc.as_f64(synth.make_weights(cfg.target, cfg.patch, rng, cfg.dtype))
    Wd = orc.as_f64(synth.make_weights(cfg.draft, cfg.patch, rng, cfg.dtype))
    B = B or cfg.batch
    series = synth.make_series(cfg.series_kind, B, cfg.context + cfg.horizon, cfg.series_seed, cfg.context)
    return cfg, Wt, Wd, series


def _hist(cfg, series, b):
    ctx = series[b, : cfg.context].astype(np.float64)
    m, s = orc.context_stats(ctx)
    return ((ctx - m) / s).reshape(-1, cfg.patch)


def test_single_pass_equals_k_plus_1_passes():
    # invariant 1: one causal pass over [h, x_1..x_K] read at the K+1 boundaries equals K+1
    # separate passes over the growing prefixes
    cfg, Wt, Wd, series = _setup()
    for b in (0, 3):
        h = _hist(cfg, series, b)
        u = lambda i: 0.5
        one = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, cfg.K, 1.0, 1.0, u, single_pass=True)
        sep = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, cfg.K, 1.0, 1.0, u, single_pass=False)
        np.testing.assert_allclose(one["mu_p"], sep["mu_p"], rtol=1e-10, atol=1e-13)
        assert one["n"] == sep["n"]
        # boundary i reads the target's prediction after [h, x_1..x_{i-1}]: check i = 1 and K+1
        np.testing.assert_allclose(sep["mu_p"][0], orc.forward(Wt, cfg.target, h)[-1], rtol=1e-12)
        full = np.vstack([h, one["X"]])
        np.testing.assert_allclose(one["mu_p"][cfg.K], orc.forward(Wt, cfg.target, full)[-1], rtol=1e-12)
        # proposals are the draft's own means, fed back autoregressively
        np.testing.assert_allclose(one["X"][1], orc.forward(Wd, cfg.draft, np.vstack([h, one["X"][:1]]))[-1], rtol=1e-12)


@pytest.mark.parametrize("K", [1, 2, 3])
def test_brute_force_accept_patterns(K):
    # invariant 5: force every accept/reject pattern through the uniforms; first rejection at i
    # commits x_1..x_{i-1}, mu_p^(i); no rejection commits x_1..x_K, mu_p^(K+1)
    cfg, Wt, Wd, series = _setup()
    h = _hist(cfg, series, 1)
    base = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, K, 0.2, 0.2, lambda i: 0.5)
    alphas = np.exp(np.minimum(0.0, [orc.log_ratio(base["X"][i], base["mu_p"][i], base["mu_q"][i], 0.2, 0.2)
                                     for i in range(K)]))
    assert np.all(alphas < 1.0) and np.all(alphas > 0.0)
    for pattern in itertools.product([True, False], repeat=K):
        us = [a * 0.999 if acc else min(a * 1.001 + 1e-9, 1 - 1e-9) for a, acc in zip(alphas, pattern)]
        rec = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, K, 0.2, 0.2, lambda i: us[i - 1])
        first_rej = pattern.index(False) if False in pattern else K
        assert rec["n"] == first_rej
        assert 1 <= rec["commits"].shape[0] == first_rej + 1 <= K + 1          # invariant 2
        np.testing.assert_array_equal(rec["commits"][:first_rej], base["X"][:first_rej])
        np.testing.assert_array_equal(rec["commits"][first_rej], base["mu_p"][first_rej])
        # later positions are never tested
        assert np.all(np.isnan(rec["ell"][first_rej + 1:])) and np.all(np.isnan(rec["logu"][first_rej + 1:]))
    # equality counts as acceptance (u <= alpha)
    rec = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, 1, 0.2, 0.2, lambda i: float(alphas[0]))
    assert rec["n"] == (1 if math.log(float(alphas[0])) <= rec["ell"][0] else 0)


def test_draft_equal_to_target_accepts_everything():
    # invariant 3: Delta = 0 => alpha = 1 => every proposal accepted, output == target-only
    cfg, Wt, _, series = _setup(B=2)
    for b in range(2):
        ctx = series[b, : cfg.context]
        f, st = orc.forecast_spec(Wt, cfg.target, Wt, cfg.target, ctx, cfg.patch, cfg.horizon, cfg.K,
                                  1e-3, 1e-3, seed=1, b=b)
        ref = orc.forecast_target_only(Wt, cfg.target, ctx, cfg.patch, cfg.horizon)
        np.testing.assert_allclose(f, ref, rtol=1e-9, atol=1e-12)
        # every round of a series with r patches left proposes min(K, r) and commits them all plus the bonus
        want, rem = [], cfg.T
        while rem > 0:
            want.append(min(cfg.K, rem) + 1)
            rem -= want[-1]
        assert st["lengths"] == want and st["rounds"] == math.ceil(cfg.T / (cfg.K + 1))
        assert st["accepted"] == sum(L - 1 for L in want) and st["tested"] == st["accepted"]


def test_sigma_to_zero_recovers_target_only():
    cfg, Wt, Wd, series = _setup(B=2)
    for b in range(2):
        ctx = series[b, : cfg.context]
        f, st = orc.forecast_spec(Wt, cfg.target, Wd, cfg.draft, ctx, cfg.patch, cfg.horizon, cfg.K,
                                  1e-6, 1e-6, seed=1, b=b)
        ref = orc.forecast_target_only(Wt, cfg.target, ctx, cfg.patch, cfg.horizon)
        # every commit is the target's own mean (BLAS blocking differs between a row computed
        # alone and inside a longer pass, hence rounding-level slack)
        np.testing.assert_allclose(f, ref, rtol=1e-10, atol=1e-13)
        assert st["accepted"] == 0 and st["lengths"] == [1] * cfg.T and st["tested"] == cfg.T


def test_forecast_bookkeeping_and_truncation():
    cfg, Wt, Wd, series = _setup(B=3)
    for H in (96, 90, 17):                                # T = 6, 6, 2 at P = 16
        T = -(-H // cfg.patch)
        trace = []
        f, st = orc.forecast_spec(Wt, cfg.target, Wd, cfg.draft, series[2, : cfg.context], cfg.patch, H,
                                  cfg.K, 0.05, 0.05, seed=5, b=2, trace=trace)
        assert f.shape == (H,) and st["committed"] == T
        assert all(1 <= L <= cfg.K + 1 for L in st["lengths"])
        assert sum(st["lengths"][:-1]) < T <= sum(st["lengths"])
        assert st["accepted"] == sum(L - 1 for L in st["lengths"])
        assert st["tested"] == sum(r["n"] + (r["n"] < r["X"].shape[0]) for r in trace)
        # no round proposes more than the patches the series still needs
        left = T
        for r in trace:
            assert r["X"].shape[0] == min(cfg.K, left)
            left -= min(r["n"] + 1, left)
        # each round's history is the context plus everything committed before it
        m, s = orc.context_stats(series[2, : cfg.context].astype(np.float64))
        y = np.vstack([r["commits"] for r in trace])[:T].reshape(-1) * s + m
        np.testing.assert_allclose(f, y[:H], rtol=1e-12)
    # a shifted context shifts the forecast (statistics are frozen on the context)
    ctx = series[0, : cfg.context].astype(np.float64)
    f0, _ = orc.forecast_spec(Wt, cfg.target, Wd, cfg.draft, ctx, cfg.patch, 32, cfg.K, 1.0, 1.0, seed=5, b=0)
    f1, _ = orc.forecast_spec(Wt, cfg.target, Wd, cfg.draft, ctx + 7.0, cfg.patch, 32, cfg.K, 1.0, 1.0, seed=5, b=0)
    np.testing.assert_allclose(f1, f0 + 7.0, rtol=1e-9)


def test_block_length_law_under_injected_rate():
    # invariant 4: with an injected i.i.d. acceptance rate the committed-patches-per-round
    # histogram is capped geometric and its mean is Eq. 7
    m = synth.ModelCfg(1, 16, 1, 32)
    W = orc.as_f64(synth.make_weights(m, 4, np.random.default_rng(0)))
    h = np.random.default_rng(1).standard_normal((3, 4))
    for alpha, K, n in ((0.9, 3, 3000), (0.75, 6, 3000)):
        Ls = np.array([orc.spec_round(W, m, W, m, h, K, 1.0, 1.0, (lambda i, r=r: orc.uniform(11, 0, r, i)),
                                      alpha_override=alpha)["n"] + 1 for r in range(n)])
        pmf = orc.block_length_pmf(alpha, K)
        counts = np.bincount(Ls, minlength=K + 2)[1:]
        chi2 = ((counts - n * pmf) ** 2 / (n * pmf)).sum()
        assert chi2 < stats.chi2.ppf(0.999, K)
        EL = orc.expected_block_length(alpha, K)
        assert abs(Ls.mean() - EL) < 4 * Ls.std() / math.sqrt(n)
    assert math.isclose(orc.expected_block_length(0.9, 3), 3.439, rel_tol=1e-12)
    assert math.isclose(orc.expected_block_length(0.75, 6), (1 - 0.75 ** 7) / 0.25, rel_tol=1e-12)


def test_not_proposing_past_the_horizon_changes_no_forecast():
    # a round of a series with r < K patches left proposes r positions; running the full K and
    # truncating the commits at T (the other possible reading) gives the same patches: positions
    # past the horizon can only produce commits that are dropped
    cfg, Wt, Wd, series = _setup(B=2)
    P, K = cfg.patch, cfg.K
    for H, sigma in ((96, 0.3), (90, 1.0), (40, 2.0)):
        T = -(-H // P)
        ctx = series[1, : cfg.context].astype(np.float64)
        m, s = orc.context_stats(ctx)
        hist = ((ctx - m) / s).reshape(-1, P)
        Y = np.empty((0, P))
        r = 0
        while Y.shape[0] < T:                                   # the full-K reading, written out
            rec = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, np.vstack([hist, Y]), K, sigma, sigma,
                                 lambda i, r=r: orc.uniform(9, 1, r, i))
            Y = np.vstack([Y, rec["commits"]])[:T]
            r += 1
        want = (Y.reshape(-1) * s + m)[:H]
        got, st = orc.forecast_spec(Wt, cfg.target, Wd, cfg.draft, ctx, P, H, K, sigma, sigma, seed=9, b=1)
        np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
        assert st["rounds"] == r
