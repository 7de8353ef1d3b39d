"""Pins for the sampled variants of the round (Sec. "Fallback Correction and Sampled Variants",
"Bonus Patch on Full Acceptance", Proposition "Equal-covariance acceptance"): the counter-based
normal draws, sampled proposals x_i = mu_q + sigma_q eps, fallback noise t = mu_p + r eps."""
import math

import numpy as np
import pytest
from scipy import integrate, stats

import synth
from oracle import tsd_oracle as orc


# ---- the normal draws ----------------------------------------------------------------------------
def test_normal_scalar_equals_bulk_and_blocks_are_keyed():
    z = orc.normal(11, 5, 3, 2, orc.STREAM_PROPOSAL, 96)
    zb = orc.normal_bulk(11, np.array([4, 5]), 3, 2, orc.STREAM_PROPOSAL, 96)
    np.testing.assert_array_equal(zb[1], z)
    assert z.shape == (96,)
    # a shorter patch is a prefix (element e depends on e only through its block and slot)
    np.testing.assert_array_equal(orc.normal(11, 5, 3, 2, orc.STREAM_PROPOSAL, 10), z[:10])
    # every key component matters
    for other in (orc.normal(12, 5, 3, 2, 1, 96), orc.normal(11, 6, 3, 2, 1, 96), orc.normal(11, 5, 4, 2, 1, 96),
                  orc.normal(11, 5, 3, 1, 1, 96), orc.normal(11, 5, 3, 2, orc.STREAM_FALLBACK, 96)):
        assert np.abs(other - z).min() > 0


def test_normal_is_standard_normal():
    # Kolmogorov-Smirnov against the normal cdf, moments, and the two Box-Muller slots separately
    z = orc.normal_bulk(2021, np.arange(4000), 0, 1, orc.STREAM_PROPOSAL, 96)       # 384000 draws
    flat = z.reshape(-1)
    assert stats.kstest(flat, "norm").pvalue > 1e-3
    n = flat.size
    assert abs(flat.mean()) < 4 / math.sqrt(n)
    assert abs(flat.var() - 1) < 4 * math.sqrt(2 / n)
    assert abs(stats.skew(flat)) < 4 * math.sqrt(6 / n)
    assert abs(stats.kurtosis(flat)) < 4 * math.sqrt(24 / n)
    for slot in range(4):
        assert stats.kstest(z[:, slot::4].reshape(-1), "norm").pvalue > 1e-3
    # tails exist on the 23-bit lattice: the largest radius is sqrt(-2 ln 2^-24) = 5.77
    assert 4.0 < np.abs(flat).max() <= math.sqrt(-2 * math.log(2.0 ** -24)) + 1e-12


def test_normal_draws_are_uncorrelated_across_slots_streams_positions():
    b = np.arange(20000)
    a = orc.normal_bulk(5, b, 0, 1, orc.STREAM_PROPOSAL, 8)
    f = orc.normal_bulk(5, b, 0, 1, orc.STREAM_FALLBACK, 8)
    p2 = orc.normal_bulk(5, b, 0, 2, orc.STREAM_PROPOSAL, 8)
    r1 = orc.normal_bulk(5, b, 1, 1, orc.STREAM_PROPOSAL, 8)
    lim = 4.5 / math.sqrt(b.size)
    c = np.corrcoef(a.T)                                   # elements of one patch (cos/sin partners included)
    assert np.abs(c - np.eye(8)).max() < lim
    for other in (f, p2, r1):
        assert abs(np.corrcoef(a[:, 0], other[:, 0])[0, 1]) < lim
        assert abs(np.corrcoef(a[:, 1], other[:, 1])[0, 1]) < lim
    # and from the acceptance uniform of the same (series, round, position)
    u = np.array([orc.uniform(5, int(x), 0, 1) for x in b[:4000]])
    assert abs(np.corrcoef(a[:4000, 0], u)[0, 1]) < 4.5 / math.sqrt(4000)


# ---- acceptance under sampled proposals ------------------------------------------------------------
def _mc_acceptance(d, delta_vec, sigma, temper, n, seed):
    """Mean of 1[log u <= min(0, temper * ell)] over x = mu_q + sigma eps with the oracle's own draws."""
    mu_q = np.linspace(-0.3, 0.4, d)
    mu_p = mu_q + delta_vec
    eps = orc.normal_bulk(seed, np.arange(n), 0, 1, orc.STREAM_PROPOSAL, d)
    acc = 0
    for k in range(n):
        x = mu_q + sigma * eps[k]
        ell = temper * orc.log_ratio(x, mu_p, mu_q, sigma, sigma)
        acc += math.log(orc.uniform(seed, k, 0, 1)) <= min(0.0, ell)
    return acc / n


@pytest.mark.parametrize("d,scale", [(8, 0.9), (32, 0.35)])
def test_unscaled_stochastic_rule_has_overlap_2phi(d, scale):
    # Proposition "Equal-covariance acceptance": with sampled proposals and the unscaled ratio
    # (ell multiplied back by d) the mean acceptance is the overlap 2 Phi(-Delta / 2),
    # Delta = ||mu_p - mu_q||_2 / sigma
    sigma = 0.5
    delta_vec = scale * sigma * np.cos(np.arange(d)) / math.sqrt(d) * 2.0
    Delta = np.linalg.norm(delta_vec) / sigma
    n = 40000
    got = _mc_acceptance(d, delta_vec, sigma, float(d), n, seed=77)
    want = 2 * stats.norm.cdf(-Delta / 2)
    assert 0.2 < want < 0.9
    assert abs(got - want) < 4 * math.sqrt(want * (1 - want) / n)


def test_tempered_stochastic_rule_matches_quadrature():
    # Under x ~ q the log density ratio is -(Delta z + Delta^2 / 2) with z ~ N(0, 1), so the
    # tempered rule accepts with probability E min(1, exp(-(Delta z + Delta^2/2) / d)): a
    # one-dimensional integral evaluated here by quadrature, independently of the oracle
    d, sigma = 16, 0.4
    delta_vec = 3.0 * sigma * np.sin(1 + np.arange(d)) / math.sqrt(d) * 2.0
    Delta = np.linalg.norm(delta_vec) / sigma
    f = lambda z: min(1.0, math.exp(-(Delta * z + Delta * Delta / 2) / d)) * stats.norm.pdf(z)
    want = integrate.quad(f, -12, 12, points=[-Delta / 2])[0]
    n = 40000
    got = _mc_acceptance(d, delta_vec, sigma, 1.0, n, seed=78)
    assert 0.5 < want < 0.99
    assert abs(got - want) < 4 * math.sqrt(want * (1 - want) / n)
    # and tempering raises acceptance above the unscaled overlap at the same Delta
    assert want > 2 * stats.norm.cdf(-Delta / 2)


# ---- the round with noise ------------------------------------------------------------------------
def _setup(name="cfg1"):
    cfg = synth.get_config(name)
    rng = np.random.default_rng(cfg.weight_seed)
    Wt = orc.as_f64(synth.make_weights(cfg.target, cfg.patch, rng, cfg.dtype))
    Wd = orc.as_f64(synth.make_weights(cfg.draft, cfg.patch, rng, cfg.dtype))
    series = synth.make_series(cfg.series_kind, 4, cfg.context + cfg.horizon, cfg.series_seed, cfg.context)
    ctx = series[1, : cfg.context].astype(np.float64)
    m, s = orc.context_stats(ctx)
    return cfg, Wt, Wd, ((ctx - m) / s).reshape(-1, cfg.patch), series


def test_sampled_proposals_condition_the_draft_and_the_target():
    cfg, Wt, Wd, h, _ = _setup()
    K, sq = 3, 0.3
    eps = lambda stream, i: orc.normal(9, 1, 0, i, stream, cfg.patch)
    rec = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, K, 0.3, sq, lambda i: 0.5, eps_fn=eps, sample_proposals=True)
    for i in range(K):
        np.testing.assert_allclose(rec["X"][i] - rec["mu_q"][i], sq * eps(orc.STREAM_PROPOSAL, i + 1), rtol=0, atol=1e-15)
    # step 2 of the draft and boundary 2 of the target saw the DRAW x_1, not the mean
    np.testing.assert_allclose(rec["mu_q"][1], orc.forward(Wd, cfg.draft, np.vstack([h, rec["X"][:1]]))[-1], rtol=1e-12)
    np.testing.assert_allclose(rec["mu_p"][1], orc.forward(Wt, cfg.target, np.vstack([h, rec["X"][:1]]))[-1], rtol=1e-10)
    mean_path = orc.forward(Wd, cfg.draft, np.vstack([h, rec["mu_q"][:1]]))[-1]
    assert np.abs(mean_path - rec["mu_q"][1]).max() > 1e-6
    # the statistic is the general Eq. 5 at the draw
    for i in range(rec["n"] + (rec["n"] < K)):
        assert rec["ell"][i] == orc.log_ratio(rec["X"][i], rec["mu_p"][i], rec["mu_q"][i], 0.3, sq)
    # single pass == K+1 passes also under sampling
    sep = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, K, 0.3, sq, lambda i: 0.5, eps_fn=eps, sample_proposals=True,
                         single_pass=False)
    np.testing.assert_allclose(rec["mu_p"], sep["mu_p"], rtol=1e-10, atol=1e-13)


def test_sampling_with_vanishing_noise_is_mean_propagation():
    cfg, Wt, Wd, h, _ = _setup()
    eps = lambda stream, i: orc.normal(9, 1, 0, i, stream, cfg.patch)
    base = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, 3, 0.3, 0.3, lambda i: 0.5)
    # proposal noise scale -> 0 with the acceptance temperatures held: pass the noise through eps_fn
    tiny = lambda stream, i: 1e-9 * eps(stream, i)
    rec = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, 3, 0.3, 0.3, lambda i: 0.5, eps_fn=tiny, sample_proposals=True,
                         fallback_r=0.3)
    np.testing.assert_allclose(rec["X"], base["X"], atol=1e-7)
    np.testing.assert_allclose(rec["commits"], base["commits"], atol=1e-7)
    assert rec["n"] == base["n"]
    # defaults ignore eps_fn altogether
    same = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, 3, 0.3, 0.3, lambda i: 0.5, eps_fn=eps)
    np.testing.assert_array_equal(same["commits"], base["commits"])


@pytest.mark.parametrize("force", ["reject_first", "accept_all"])
def test_fallback_noise_lands_on_the_corrected_or_bonus_patch_only(force):
    cfg, Wt, Wd, h, _ = _setup()
    K, r = 3, 0.2
    eps = lambda stream, i: orc.normal(4, 1, 0, i, stream, cfg.patch)
    u = (lambda i: 1 - 1e-7) if force == "reject_first" else (lambda i: 1e-7)
    sig = 1e-3 if force == "reject_first" else 50.0
    rec = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, K, sig, sig, u, eps_fn=eps, fallback_r=r)
    n = rec["n"]
    assert n == (0 if force == "reject_first" else K)
    np.testing.assert_array_equal(rec["commits"][:n], rec["X"][:n])                       # accepted proposals untouched
    np.testing.assert_array_equal(rec["X"], rec["mu_q"])                                    # mean proposals
    np.testing.assert_allclose(rec["commits"][n] - rec["mu_p"][n], r * eps(orc.STREAM_FALLBACK, n + 1), atol=1e-15)


def test_fallback_noise_energy_is_r_squared():
    # Lemma "fallback noise only hurts": E ||t - mu_p||_d^2 = r^2 (the clean fallback has 0)
    P, r = 32, 0.35
    z = orc.normal_bulk(8, np.arange(20000), 3, 2, orc.STREAM_FALLBACK, P)
    e = ((r * z) ** 2).mean(axis=1)
    assert abs(e.mean() - r * r) < 4 * r * r * math.sqrt(2 / (P * 20000))


def test_forecast_with_noise_uses_per_round_draws_and_keeps_length_law():
    cfg, Wt, Wd, h, series = _setup()
    trace = []
    y, st = orc.forecast_spec(Wt, cfg.target, Wd, cfg.draft, series[1, : cfg.context], cfg.patch, cfg.horizon, cfg.K, 0.5, 0.5,
                              seed=3, b=1, trace=trace, sample_proposals=True, fallback_r=0.25)
    assert y.shape == (cfg.horizon,) and np.isfinite(y).all()
    assert st["committed"] == cfg.T and all(1 <= L <= cfg.K + 1 for L in st["lengths"])
    for r, rec in enumerate(trace):
        np.testing.assert_allclose(rec["X"][0] - rec["mu_q"][0], 0.5 * orc.normal(3, 1, r, 1, orc.STREAM_PROPOSAL, cfg.patch), atol=1e-14)
        n = rec["n"]
        np.testing.assert_allclose(rec["commits"][n] - rec["mu_p"][n], 0.25 * orc.normal(3, 1, r, n + 1, orc.STREAM_FALLBACK, cfg.patch),
                                   atol=1e-14)
    # without noise the forecast differs (the knobs do something) and the default call is unchanged
    y0, _ = orc.forecast_spec(Wt, cfg.target, Wd, cfg.draft, series[1, : cfg.context], cfg.patch, cfg.horizon, cfg.K, 0.5, 0.5, seed=3, b=1)
    assert np.abs(y - y0).max() > 1e-3


def test_round_with_diagonal_scales():
    # per-dimension scales enter the statistic (Mahalanobis energies, log-det) and the proposal draw
    cfg, Wt, Wd, h, _ = _setup()
    P, K = cfg.patch, 3
    sp, sq = np.linspace(0.3, 0.9, P), np.linspace(0.8, 0.2, P)
    eps = lambda stream, i: orc.normal(6, 1, 0, i, stream, P)
    rec = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, K, sp, sq, lambda i: 1e-9, eps_fn=eps, sample_proposals=True)
    assert rec["n"] == K                                    # u tiny: everything accepted, all K statistics recorded
    for i in range(K):
        np.testing.assert_allclose(rec["X"][i] - rec["mu_q"][i], sq * eps(orc.STREAM_PROPOSAL, i + 1), atol=1e-15)
        assert rec["ell"][i] == orc.log_ratio_diag(rec["X"][i], rec["mu_p"][i], rec["mu_q"][i], sp, sq)
    # constant vectors reproduce the isotropic round exactly
    iso = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, K, 0.4, 0.4, lambda i: 0.5)
    vec = orc.spec_round(Wt, cfg.target, Wd, cfg.draft, h, K, np.full(P, 0.4), np.full(P, 0.4), lambda i: 0.5)
    np.testing.assert_allclose(vec["ell"][: iso["n"] + 1], iso["ell"][: iso["n"] + 1], rtol=1e-12, atol=1e-15)
    assert vec["n"] == iso["n"]
