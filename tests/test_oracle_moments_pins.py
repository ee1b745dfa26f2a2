"""Pins of the moment-tracking oracle (Sec. 3.2.2): library sample variance, the decomposition of nu_adam and
nu_micro into mu^2 and sigma^2, unbiasedness by Monte-Carlo, closed forms of the EMA.  No GPU needed."""
import numpy as np
import pytest

from oracle import moments as om


def _per_example(n, B, seed, mu_scale=0.3, sigma_scale=1.0):
    rng = np.random.default_rng(seed)
    mu = rng.standard_normal(n) * mu_scale
    sigma = np.abs(rng.standard_normal(n)) * sigma_scale + 0.1
    g = mu[None, :] + sigma[None, :] * rng.standard_normal((B, n))
    return mu, sigma, g


def test_one_step_without_memory_is_the_sample_variance_and_its_complement():
    """beta2 = 0: sigma^2-hat is numpy's unbiased sample variance over the examples, mu^2-hat = mean^2 - var/B."""
    n, B = 500, 7
    _, _, g = _per_example(n, B, 0)
    a, q, s = om.moment_track_step(np.zeros(n), np.zeros(n), g.sum(0), (g * g).sum(0), 0.0, 1.0 / B, 1.0 / B, B, 1)
    var = np.var(g, axis=0, ddof=1)
    np.testing.assert_allclose(s.sum_sigma2, var.sum(), rtol=1e-12)
    np.testing.assert_allclose(s.sum_mu2, (g.mean(0) ** 2 - var / B).sum(), rtol=1e-10)
    np.testing.assert_allclose(a, g.mean(0) ** 2, rtol=1e-13)
    np.testing.assert_allclose(q, (g * g).mean(0), rtol=1e-13)


def test_the_estimators_decompose_both_second_moments():
    """nu_adam-hat = mu^2-hat + sigma^2-hat / B and nu_micro-hat = mu^2-hat + sigma^2-hat, summed over parameters."""
    n, B, beta2 = 300, 5, 0.95
    a, q = np.zeros(n), np.zeros(n)
    for t in range(1, 6):
        _, _, g = _per_example(n, B, 10 + t)
        a, q, s = om.moment_track_step(a, q, g.sum(0), (g * g).sum(0), beta2, 1.0 / B, 1.0 / B, B, t)
        corr = 1.0 / (1.0 - beta2 ** t)
        np.testing.assert_allclose(s.sum_mu2 + s.sum_sigma2 / B, (a * corr).sum(), rtol=1e-12)
        np.testing.assert_allclose(s.sum_mu2 + s.sum_sigma2, (q * corr).sum(), rtol=1e-12)


def test_unbiasedness_by_monte_carlo():
    """E[mu^2-hat] = mu^2 and E[sigma^2-hat] = sigma^2 (stated with Eq. (musq_sigsq_est)): over 400k independent
    parameters the means must agree within 5 standard errors; exchanging the two formulas, dropping the 1/B or the
    1/(1 - 1/B) would miss by far more."""
    n, B = 400_000, 4
    mu, sigma, g = _per_example(n, B, 3)
    _, _, s = om.moment_track_step(np.zeros(n), np.zeros(n), g.sum(0), (g * g).sum(0), 0.0, 1.0 / B, 1.0 / B, B, 1)
    # Var[sigma^2-hat] = 2 sigma^4 / (B-1); Var[mean^2] ~ 4 mu^2 sigma^2 / B + 2 sigma^4 / B^2
    se_sig = np.sqrt((2 * sigma ** 4 / (B - 1)).sum()) / n
    se_mu = np.sqrt((4 * mu ** 2 * sigma ** 2 / B + 2 * sigma ** 4 / B ** 2 + 2 * sigma ** 4 / (B * B * (B - 1))).sum()) / n
    assert abs(s.sum_sigma2 / n - (sigma ** 2).mean()) < 5 * se_sig
    assert abs(s.sum_mu2 / n - (mu ** 2).mean()) < 5 * se_mu
    # the planted mistakes are far outside the band
    biased_mu2 = (g.mean(0) ** 2).mean()                         # nu_adam itself: off by sigma^2 / B
    assert abs(biased_mu2 - (mu ** 2).mean()) > 50 * se_mu


def test_mean_loss_cotangents_give_the_same_estimates():
    """Cotangents of the mean loss are 1/B of those of the summed loss: grad_scale 1 and sq_scale B undo it."""
    n, B = 200, 6
    _, _, g = _per_example(n, B, 4)
    r1 = om.moment_track_step(np.zeros(n), np.zeros(n), g.sum(0), (g * g).sum(0), 0.9, 1.0 / B, 1.0 / B, B, 1)
    gm = g / B
    r2 = om.moment_track_step(np.zeros(n), np.zeros(n), gm.sum(0), (gm * gm).sum(0), 0.9, 1.0, float(B), B, 1)
    np.testing.assert_allclose(r1[2].sum_mu2, r2[2].sum_mu2, rtol=1e-12)
    np.testing.assert_allclose(r1[2].sum_sigma2, r2[2].sum_sigma2, rtol=1e-12)


def test_constant_inputs_are_recovered_at_every_step_and_the_raw_ema_follows_its_closed_form():
    n, B, beta2 = 50, 8, 0.95
    _, _, g = _per_example(n, B, 5)
    S_id, S_sq = g.sum(0), (g * g).sum(0)
    a, q = np.zeros(n), np.zeros(n)
    first = None
    for t in range(1, 8):
        a, q, s = om.moment_track_step(a, q, S_id, S_sq, beta2, 1.0 / B, 1.0 / B, B, t)
        np.testing.assert_allclose(a, (1 - beta2 ** t) * g.mean(0) ** 2, rtol=1e-12)      # geometric series
        first = first or s
        np.testing.assert_allclose(s.sum_mu2, first.sum_mu2, rtol=1e-11)
        np.testing.assert_allclose(s.sum_sigma2, first.sum_sigma2, rtol=1e-11)
    # without the correction the estimates are scaled by 1 - beta2^t
    _, _, raw = om.moment_track_step(np.zeros(n), np.zeros(n), S_id, S_sq, beta2, 1.0 / B, 1.0 / B, B, 1, debias=False)
    np.testing.assert_allclose(raw.sum_sigma2, (1 - beta2) * first.sum_sigma2, rtol=1e-12)


def test_ratios_and_argument_checks():
    s = om.MomentSums(2.0, 8.0, 0.0, 4)
    assert om.ratio_to_sigma_eff(s, 4, "adam") == pytest.approx(1.0)
    assert om.ratio_to_sigma_eff(s, 4, "microadam") == pytest.approx(0.25)
    with pytest.raises(ValueError):
        om.moment_track_step(np.zeros(3), np.zeros(3), np.zeros(3), np.zeros(3), 0.9, 1.0, 1.0, 1, 1)
