"""Pins of the threshold acceptance rule and of the batch-synchronised loop (oracle only).

Table "TiRex configuration", acceptance row: the inequality ||.||_d^2 <= sigma^2, batch kept in step.
"""
import math

import numpy as np
import pytest

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


def _sigma_between(cfg, Wt, Wd, series, b, K):
    """A sigma that splits the round's proposals of series b: some inside the ball, some outside."""
    rec = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, _hist(cfg, series, b), K, 1.0, 1.0, lambda i: 0.5)
    d = np.sqrt(np.mean((rec["X"] - rec["mu_p"][:K]) ** 2, axis=1))  # per-position scaled distance
    return rec, d


def test_threshold_on_a_hand_built_boundary():
    # d = 4, x - mu_p = (2, 0, 0, 0): ||.||_d^2 = 4 / 4 = 1, so sigma = 1 is exactly on the boundary
    # (inside: the rule is "<="), sigma just below 1 is outside, per-dimension scales (2, 1, 1, 1)
    # give a scaled Mahalanobis distance of 1/4 (inside) and (0.5, 1, 1, 1) give 4 (outside)
    x, mu = np.array([2.0, 0, 0, 0]), np.zeros(4)
    assert orc.within_threshold(x, mu, 1.0)
    assert not orc.within_threshold(x, mu, 0.999)
    assert orc.within_threshold(x, mu, 1.001)
    assert orc.within_threshold(x, mu, np.array([2.0, 1, 1, 1]))
    assert not orc.within_threshold(x, mu, np.array([0.5, 1, 1, 1]))
    # the unscaled norm (a dropped 1/d) would reject at sigma = 1.5: 4 > 2.25, the scaled one accepts
    assert orc.within_threshold(x, mu, 1.5)


def test_threshold_rule_is_the_ratio_rule_at_a_constant_draw():
    # with mean proposals and equal scales Eq. 6 reads ell = -||x - mu_p||_d^2 / (2 sigma^2), and
    # u <= exp(ell) at the constant u = exp(-1/2) is ||x - mu_p||_d^2 <= sigma^2: the already pinned
    # ratio rule, driven with that draw, must give the same counts and commits as the threshold rule
    cfg, Wt, Wd, series = _setup()
    K = cfg.K
    u_half = math.exp(-0.5)
    seen = set()
    for b in range(4):
        _, d = _sigma_between(cfg, Wt, Wd, series, b, K)
        for sigma in list(0.5 * (np.sort(d)[:-1] + np.sort(d)[1:])) + [d.min() * 0.5, d.max() * 2.0]:
            sigma = float(sigma)
            h = _hist(cfg, series, b)
            thr = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, K, sigma, sigma, lambda i: 0.123, rule="threshold")
            rat = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, K, sigma, sigma, lambda i: u_half, rule="ratio")
            assert thr["n"] == rat["n"]
            np.testing.assert_array_equal(thr["commits"], rat["commits"])
            # the log form carried in the record is the same decision
            t = thr["n"] + (thr["n"] < K)
            np.testing.assert_allclose(thr["ell"][:t], rat["ell"][:t], rtol=1e-12)
            assert np.all(thr["logu"][:t] == -0.5) and np.all(np.isnan(thr["logu"][t:]))
            # and the count is the number of leading positions inside the ball, recomputed here
            inside = d <= sigma
            assert thr["n"] == (int(np.argmin(inside)) if not inside.all() else K)
            seen.add(thr["n"])
    assert len(seen) >= 3  # the sigmas really did split the proposals in several places


def test_threshold_rule_ignores_the_draw_and_the_draft_scale():
    cfg, Wt, Wd, series = _setup()
    h = _hist(cfg, series, 2)
    _, d = _sigma_between(cfg, Wt, Wd, series, 2, cfg.K)
    sigma = float(np.median(d))
    a = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, cfg.K, sigma, sigma, lambda i: 1e-6, rule="threshold")
    b = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, cfg.K, sigma, 7.0 * sigma, lambda i: 1 - 1e-6, rule="threshold")
    assert a["n"] == b["n"]
    np.testing.assert_array_equal(a["commits"], b["commits"])


def test_threshold_draft_equal_to_target_and_vanishing_sigma():
    cfg, Wt, Wd, series = _setup(B=2)
    ctx = series[0, : cfg.context]
    ref = orc.forecast_target_only(Wt, cfg.target, ctx, cfg.patch, cfg.horizon)
    f, st = orc.forecast_spec(Wt, cfg.target, Wt, cfg.target, ctx, cfg.patch, cfg.horizon, cfg.K, 1e-6, 1e-6,
                              seed=1, b=0, rule="threshold")
    np.testing.assert_allclose(f, ref, rtol=1e-9, atol=1e-12)
    assert st["accepted"] == st["tested"]
    # a different draft with sigma -> 0: nothing passes, every round commits one target patch
    f, st = orc.forecast_spec(Wt, cfg.target, Wd, cfg.draft, ctx, cfg.patch, cfg.horizon, cfg.K, 1e-9, 1e-9,
                              seed=1, b=0, rule="threshold")
    np.testing.assert_allclose(f, ref, rtol=1e-9, atol=1e-12)
    assert st["accepted"] == 0 and st["rounds"] == -(-cfg.horizon // cfg.patch)


@pytest.mark.parametrize("rule", ["ratio", "threshold"])
def test_sync_of_one_series_is_the_plain_loop(rule):
    cfg, Wt, Wd, series = _setup(B=3)
    for b in (0,):  # the synchronised loop numbers its series from 0: series 0 alone draws the same uniforms
        ctx = series[b, : cfg.context]
        f1, s1 = orc.forecast_spec(Wt, cfg.target, Wd, cfg.draft, ctx, cfg.patch, cfg.horizon, cfg.K, 0.05, 0.05,
                                   seed=5, b=b, rule=rule)
        f2, s2 = orc.forecast_spec_sync(Wt, cfg.target, Wd, cfg.draft, ctx[None, :], cfg.patch, cfg.horizon, cfg.K,
                                        0.05, 0.05, seed=5, rule=rule)
        np.testing.assert_array_equal(f1, f2[0])
        for k in ("rounds", "tested", "accepted", "committed", "lengths"):
            assert s1[k] == s2[0][k]


def test_sync_on_identical_series_under_the_threshold_rule():
    # the threshold rule draws nothing, so copies of one series decide alike in every round: the
    # minimum changes nothing and each copy's forecast is the unsynchronised one
    cfg, Wt, Wd, series = _setup(B=2)
    ctx = series[1, : cfg.context]
    _, d = _sigma_between(cfg, Wt, Wd, series, 1, cfg.K)
    sigma = float(np.median(d))
    f1, s1 = orc.forecast_spec(Wt, cfg.target, Wd, cfg.draft, ctx, cfg.patch, cfg.horizon, cfg.K, sigma, sigma,
                               seed=5, b=0, rule="threshold")
    f3, s3 = orc.forecast_spec_sync(Wt, cfg.target, Wd, cfg.draft, np.stack([ctx] * 3), cfg.patch, cfg.horizon,
                                    cfg.K, sigma, sigma, seed=5, rule="threshold")
    for b in range(3):
        np.testing.assert_array_equal(f3[b], f1)
        assert s3[b]["lengths"] == s1["lengths"] and s3[b]["accepted"] == s1["accepted"]
    assert 0 < s1["accepted"] < s1["tested"]  # the case has both outcomes


@pytest.mark.parametrize("rule", ["ratio", "threshold"])
def test_sync_keeps_the_minimum_of_the_series_own_counts(rule):
    cfg, Wt, Wd, series = _setup(B=4)
    B, K, P = 4, cfg.K, cfg.patch
    T = -(-cfg.horizon // P)
    sigma = float(np.median(_sigma_between(cfg, Wt, Wd, series, 0, K)[1]))  # mixed outcomes under both rules
    trace = []
    f, st = orc.forecast_spec_sync(Wt, cfg.target, Wd, cfg.draft, series[:B, : cfg.context], P, cfg.horizon, K,
                                   sigma, sigma, seed=9, rule=rule, trace=trace)
    Y = [np.empty((0, P)) for _ in range(B)]
    some_cut = False
    for r, recs in enumerate(trace):
        K_r = min(K, T - Y[0].shape[0])
        own = []
        for b in range(B):
            # each series' own record is what the plain round gives on the history committed so far
            solo = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, np.vstack([_hist(cfg, series, b), Y[b]]), K_r, sigma,
                                  sigma, lambda i, b=b: orc.uniform(9, b, r, i), rule=rule)
            assert solo["n"] == recs[b]["n"]
            np.testing.assert_array_equal(solo["X"], recs[b]["X"])
            own.append(solo["n"])
        n_min = min(own)
        some_cut |= max(own) > n_min
        for b in range(B):
            assert recs[b]["n_sync"] == n_min
            blk = np.vstack([recs[b]["X"][:n_min], recs[b]["mu_p"][n_min][None]])
            Y[b] = np.vstack([Y[b], blk])[:T]
        assert len({y.shape[0] for y in Y}) == 1          # the batch stays in step
    assert some_cut                                        # synchronisation did cost some series proposals
    for b in range(B):
        m, s = orc.context_stats(series[b, : cfg.context].astype(np.float64))
        np.testing.assert_allclose(f[b], (Y[b].reshape(-1) * s + m)[: cfg.horizon], rtol=0, atol=0)
        assert st[b]["committed"] == T and sum(st[b]["lengths"]) >= T
        assert st[b]["accepted"] >= sum(L - 1 for L in st[b]["lengths"][:-1])  # own counts are never below the kept ones


def test_sync_never_finishes_in_fewer_rounds_than_the_slowest_series_alone():
    cfg, Wt, Wd, series = _setup(B=4)
    sigma = float(np.median(_sigma_between(cfg, Wt, Wd, series, 0, cfg.K)[1]))
    f, st = orc.forecast_spec_sync(Wt, cfg.target, Wd, cfg.draft, series[:4, : cfg.context], cfg.patch, cfg.horizon,
                                   cfg.K, sigma, sigma, seed=9, rule="threshold")
    alone = [orc.forecast_spec(Wt, cfg.target, Wd, cfg.draft, series[b, : cfg.context], cfg.patch, cfg.horizon, cfg.K,
                               sigma, sigma, seed=9, b=b, rule="threshold")[1]["rounds"] for b in range(4)]
    assert st[0]["rounds"] >= max(alone)
