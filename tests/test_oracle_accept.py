"""Pins for the acceptance statistic (Eq. 5), its mean-propagating form (Eq. 6) and the
deterministic fidelity identity (Eq. 9)."""
import math

import numpy as np
from scipy import stats

from oracle import tsd_oracle as orc


def test_energy_is_per_dimension():
    assert orc.energy(np.full(96, 2.0)) == 4.0          # ||u||^2 / d
    assert orc.energy(np.array([3.0, 4.0])) == 12.5


def test_eq5_equals_scaled_log_density_ratio():
    # ell = (1/d) log[p(x)/q(x)] for the isotropic Gaussians of Eq. 4, via scipy's log-pdf
    rng = np.random.default_rng(0)
    for d, sp, sq in ((16, 1.0, 1.0), (96, 0.3, 0.3), (32, 0.7, 0.2), (5, 0.2, 1.3)):
        x, mp, mq = rng.standard_normal((3, d))
        lp = stats.multivariate_normal(mean=mp, cov=sp ** 2 * np.eye(d)).logpdf(x)
        lq = stats.multivariate_normal(mean=mq, cov=sq ** 2 * np.eye(d)).logpdf(x)
        assert math.isclose(orc.log_ratio(x, mp, mq, sp, sq), (lp - lq) / d, rel_tol=1e-10, abs_tol=1e-12)


def test_eq6_distance_gate_hand_values():
    d = 96
    mq = np.linspace(-1, 1, d)
    # Delta^2 = ||mu_q - mu_p||_d^2 = c^2 when the two means differ by c in every coordinate
    for c, sigma in ((0.5, 1.0), (0.3, 0.25), (1.0, 2.0)):
        ell = orc.log_ratio(mq, mq - c, mq, sigma, sigma)
        assert math.isclose(ell, -c * c / (2 * sigma * sigma), rel_tol=1e-12)
    # Delta^2 = 2 sigma^2  =>  alpha = 1/e (the maximiser in the proof of the fidelity bound)
    sigma = 0.4
    c = math.sqrt(2) * sigma
    assert math.isclose(math.exp(orc.log_ratio(mq, mq + c, mq, sigma, sigma)), math.exp(-1), rel_tol=1e-12)
    # Delta = 0  =>  ell = 0  =>  always accepted
    assert orc.log_ratio(mq, mq, mq, 0.3, 0.3) == 0.0


def test_log_determinant_term():
    # x = mu_q = mu_p leaves exactly (1/2) log(sigma_q^2 / sigma_p^2) = log(sigma_q / sigma_p)
    x = np.ones(8)
    assert math.isclose(orc.log_ratio(x, x, x, 2.0, 0.5), math.log(0.5 / 2.0), rel_tol=1e-12)
    assert math.isclose(orc.log_ratio(x, x, x, 0.5, 2.0), math.log(2.0 / 0.5), rel_tol=1e-12)
    # omitting it with sigma_q << sigma_p inflates ell by log(sigma_p / sigma_q) > 0 and drives
    # alpha to ~1 whatever the gap (remark "The normalization term is load-bearing")
    sp, sq = 1.0, 0.05
    mp = x + 0.02
    with_term = orc.log_ratio(x, mp, x, sp, sq)
    omitted = with_term + math.log(sp / sq)
    assert math.exp(with_term) < 0.06 and math.exp(omitted) > 0.999


def test_without_tempering_acceptance_collapses():
    # Component ablation: dropping the 1/d scaling multiplies ell by d; at d = 96 and a gap that
    # the tempered rule accepts ~70% of the time, the untempered probability is ~0.
    d, sigma = 96, 0.25
    mq = np.zeros(d)
    c = sigma * math.sqrt(2 * 0.35)
    ell = orc.log_ratio(mq, mq + c, mq, sigma, sigma)
    assert 0.68 < math.exp(ell) < 0.72
    assert math.exp(d * ell) < 1e-14


def test_fidelity_identity_monte_carlo():
    # E||Y - mu_p||_d^2 = Delta^2 exp(-Delta^2 / 2 sigma^2) <= 2 sigma^2 / e, with Y = mu_q when
    # log u <= ell and mu_p otherwise; u from the keyed Philox stream.
    d, sigma, n = 16, 0.5, 200_000
    w = orc.philox4x32_10_bulk(np.arange(n), 0, 1, 0, (99, 0))
    logu = np.log(((w >> np.uint64(9)).astype(np.float64) + 0.5) * 2.0 ** -23)
    for delta2 in (0.1, 2 * sigma ** 2, 2.0):
        mp = np.zeros(d)
        mq = mp + math.sqrt(delta2)
        ell = orc.log_ratio(mq, mp, mq, sigma, sigma)
        acc = logu <= min(0.0, ell)
        err = np.where(acc, orc.energy(mq - mp), 0.0)
        expect = delta2 * math.exp(-delta2 / (2 * sigma ** 2))
        assert expect <= 2 * sigma ** 2 / math.e + 1e-15
        assert abs(err.mean() - expect) < 4 * delta2 * math.sqrt(0.25 / n)
    assert math.isclose(2 * sigma ** 2 * math.exp(-1), 2 * sigma ** 2 / math.e)


def test_diagonal_covariance_statistic():
    # Remark "General covariances": (1/d) log[p(x)/q(x)] for diagonal Gaussians, via scipy's log-pdf
    rng = np.random.default_rng(3)
    for d in (4, 32, 96):
        x, mp, mq = rng.standard_normal((3, d))
        sp, sq = rng.uniform(0.2, 1.5, d), rng.uniform(0.2, 1.5, d)
        lp = stats.multivariate_normal(mean=mp, cov=np.diag(sp ** 2)).logpdf(x)
        lq = stats.multivariate_normal(mean=mq, cov=np.diag(sq ** 2)).logpdf(x)
        assert math.isclose(orc.log_ratio_diag(x, mp, mq, sp, sq), (lp - lq) / d, rel_tol=1e-10, abs_tol=1e-12)
        # the isotropic case recovers Eq. 5, with scalars or constant vectors
        assert math.isclose(orc.log_ratio_diag(x, mp, mq, 0.7, 0.4), orc.log_ratio(x, mp, mq, 0.7, 0.4), rel_tol=1e-12)
        assert math.isclose(orc.log_ratio_diag(x, mp, mq, np.full(d, 0.7), np.full(d, 0.4)), orc.log_ratio(x, mp, mq, 0.7, 0.4),
                            rel_tol=1e-12)
    # a dimension the target is sure about (small s_p) dominates the energy: hand value
    x, mp, mq = np.zeros(2), np.array([1.0, 1.0]), np.zeros(2)
    sp, sq = np.array([0.5, 2.0]), np.array([1.0, 1.0])
    want = (-0.5 * (1 / 0.25 + 1 / 4.0) + 0.0 + 0.5 * (0.0 - math.log(0.25) - math.log(4.0))) / 2
    assert math.isclose(orc.log_ratio_diag(x, mp, mq, sp, sq), want, rel_tol=1e-12)


def test_diagonal_log_determinant_is_load_bearing():
    # a confident draft (s_q << s_p in every dimension) proposing its own mean: without the
    # normalisation term the statistic is positive (always accept) however far the means are apart
    d = 16
    mq, mp = np.zeros(d), np.full(d, 0.3)
    sp, sq = np.linspace(0.8, 1.2, d), np.linspace(0.05, 0.1, d)
    with_term = orc.log_ratio_diag(mq, mp, mq, sp, sq)
    logdet = (np.sum(np.log(sq ** 2)) - np.sum(np.log(sp ** 2))) / (2 * d)
    assert with_term < -2.0 and with_term - logdet > -0.1
