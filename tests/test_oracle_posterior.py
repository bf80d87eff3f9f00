"""Pins for the oracle's KDE and Bayesian acceptance posterior (Section 4.4; CPU only).

The paper gives the Bayes formula and says the densities come from KDE (citing
Silverman 1986) without naming kernel or bandwidth; the reading built here is a
Gaussian kernel with Silverman's reference-rule bandwidth.  Expected values come from
scipy's gaussian_kde, hand arithmetic and properties -- never from the oracle."""
import math

import numpy as np
import pytest
from scipy.integrate import quad
from scipy.stats import gaussian_kde


def test_hand_computed_two_plus_two(oracle):
    # L_A = {0.2, 0.4}, L_R = {0.6, 0.9}, query d = 0.5, Silverman: h = (4/(3n))^(1/5) * std(n-1)
    LA, LR, d = [0.2, 0.4], [0.6, 0.9], 0.5
    LA32, LR32 = np.float32(LA).astype(np.float64), np.float32(LR).astype(np.float64)

    def dens(s):
        n = len(s)
        mean = sum(s) / n
        sd = math.sqrt(sum((x - mean) ** 2 for x in s) / (n - 1))
        h = (4.0 / (3.0 * n)) ** 0.2 * sd
        return sum(math.exp(-0.5 * ((d - x) / h) ** 2) for x in s) / (n * h * math.sqrt(2 * math.pi))

    pa, pr = dens(list(LA32)), dens(list(LR32))
    prior_a = prior_r = 0.5
    expect = pa * prior_a / (pa * prior_a + pr * prior_r)
    assert oracle.posterior(d, LA, LR) == pytest.approx(expect, rel=1e-12)
    assert math.exp(oracle.kde_logpdf(d, LA)) == pytest.approx(pa, rel=1e-12)


@pytest.mark.parametrize("rule,name", [(0, "silverman"), (1, "scott")])
def test_kde_matches_scipy(oracle, rule, name):
    rng = np.random.default_rng(0)
    for n in (2, 5, 64, 1000):
        s = np.float32(np.clip(rng.normal(0.3, 0.1, n), 1e-3, 1 - 1e-3))
        kde = gaussian_kde(s.astype(np.float64), bw_method=name)
        for d in (0.0, 0.05, 0.3, 0.55, 1.0):
            assert math.exp(oracle.kde_logpdf(d, s, rule)) == pytest.approx(
                float(kde.evaluate([d])[0]), rel=1e-10, abs=1e-300)


def test_kde_integrates_to_one(oracle):
    rng = np.random.default_rng(1)
    s = np.float32(rng.uniform(0.1, 0.9, 17))
    total, _ = quad(lambda x: math.exp(oracle.kde_logpdf(x, s)), -2.0, 3.0, limit=400,
                    points=list(np.sort(s.astype(np.float64))))
    assert total == pytest.approx(1.0, abs=1e-7)


def test_posterior_matches_bayes_rule_with_scipy_densities_and_size_priors(oracle):
    rng = np.random.default_rng(2)
    LA = np.float32(np.clip(rng.normal(0.25, 0.07, 90), 1e-3, 1 - 1e-3))
    LR = np.float32(np.clip(rng.normal(0.55, 0.12, 30), 1e-3, 1 - 1e-3))   # unequal priors 3:1
    ka = gaussian_kde(LA.astype(np.float64), bw_method="silverman")
    kr = gaussian_kde(LR.astype(np.float64), bw_method="silverman")
    for d in np.linspace(0.0, 1.0, 21):
        a = float(ka.evaluate([d])[0]) * 90 / 120
        r = float(kr.evaluate([d])[0]) * 30 / 120
        assert oracle.posterior(d, LA, LR) == pytest.approx(a / (a + r), rel=1e-9, abs=1e-300)


def test_swapping_lists_complements_the_posterior(oracle):
    rng = np.random.default_rng(3)
    LA, LR = np.float32(rng.uniform(0.05, 0.5, 40)), np.float32(rng.uniform(0.3, 0.95, 25))
    for d in (0.1, 0.33, 0.4, 0.8):
        assert oracle.posterior(d, LA, LR) + oracle.posterior(d, LR, LA) == pytest.approx(1.0, abs=1e-14)


def test_identical_lists_give_one_half(oracle):
    s = np.float32([0.1, 0.2, 0.35, 0.7])
    for d in (0.0, 0.3, 0.9):
        assert oracle.posterior(d, s, s) == pytest.approx(0.5, abs=1e-15)


def test_posterior_decreases_with_distance_when_accepted_mass_sits_left(oracle):
    # the qualitative claim of the acceptance-probability figure: smaller distance, higher probability
    rng = np.random.default_rng(4)
    LA = np.float32(np.clip(rng.normal(0.2, 0.05, 64), 1e-3, 1 - 1e-3))
    LR = np.float32(np.clip(rng.normal(0.4, 0.05, 64), 1e-3, 1 - 1e-3))
    ds = np.linspace(0.1, 0.5, 81)
    P = [oracle.posterior(d, LA, LR) for d in ds]
    assert all(a >= b - 1e-12 for a, b in zip(P, P[1:]))
    assert P[0] > 0.99 and P[-1] < 0.01
    mid = float(ds[np.argmin(np.abs(np.array(P) - 0.5))])
    assert 0.25 < mid < 0.35


def test_far_queries_stay_finite(oracle):
    # both densities underflow in linear space; the log-domain Bayes ratio is still defined
    LA, LR = np.float32([0.10, 0.11, 0.12]), np.float32([0.13, 0.14, 0.15])
    for d in (0.0, 0.9, 1.0):
        P = oracle.posterior(d, LA, LR)
        assert 0.0 <= P <= 1.0 and not math.isnan(P)
    assert oracle.posterior(1.0, LA, LR) < 1e-6      # closer to the rejected cluster
    assert oracle.posterior(0.0, LA, LR) > 1 - 1e-6


def test_degenerate_histories_switch_the_test_off(oracle):
    ok = np.float32([0.2, 0.3, 0.4])
    assert oracle.posterior(0.3, [], ok) == 0.0
    assert oracle.posterior(0.3, ok, []) == 0.0
    assert oracle.posterior(0.3, np.float32([0.2]), ok) == 0.0
    assert oracle.posterior(0.3, np.float32([0.2, 0.2, 0.2]), ok) == 0.0      # zero variance
    assert oracle.posterior(0.3, ok, ok, min_n=4) == 0.0
    assert oracle.posterior(0.3, ok, ok, min_n=3) == pytest.approx(0.5)
