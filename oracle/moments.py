"""fp64 oracle of the on-line measurement of mu^2 and sigma^2 (Sec. 3.2.2, "Expectation and variance of gradients").

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

Two EMAs with the optimizer's beta2 track nu_adam = (mean gradient)^2 and nu_micro = mean of squared per-example
gradients; the unbiased estimators of Eq. (musq_sigsq_est) are formed from the EMAs and averaged over all
parameters (caption of the figure that plots them).  Readings where the text is silent:

* the EMAs are bias-corrected by 1/(1 - beta2^t) before the estimators are formed (``debias``); the factor is
  common to both EMAs, so the ratio mu^2-hat / sigma^2-hat does not depend on it;
* "averaged over all parameters" is read as the mean of mu^2-hat and the mean of sigma^2-hat, each taken
  separately (the sums are returned; the caller divides by the parameter count and forms ratios);
* sigma_eff^2 is sigma^2 / B for Adam and sigma^2 for MicroAdam (Sec. 3.2.2).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class MomentSums:
    sum_mu2: float       # sum over parameters of mu^2-hat
    sum_sigma2: float    # sum over parameters of sigma^2-hat
    sum_abs: float       # sum over parameters of |nu_adam-hat| + |nu_micro-hat| / B, the size of the terms that cancel
    n: int


def moment_track_step(ema_adam, ema_micro, S_id, S_sq, beta2: float, grad_scale: float, sq_scale: float, B: int,
                      step: int, debias: bool = True):
    """One tracking step; returns (new ema_adam, new ema_micro, MomentSums)."""
    if B < 2:
        raise ValueError("the unbiased estimators need B >= 2")
    a = np.asarray(ema_adam, dtype=np.float64)
    q = np.asarray(ema_micro, dtype=np.float64)
    mu_t = np.float64(grad_scale) * np.asarray(S_id, dtype=np.float64)
    nu_adam = mu_t * mu_t                                        # Eq. (nu_defs), right
    nu_micro = np.float64(sq_scale) * np.asarray(S_sq, dtype=np.float64)   # Eq. (nu_defs), left
    a_t = beta2 * a + (1.0 - beta2) * nu_adam
    q_t = beta2 * q + (1.0 - beta2) * nu_micro
    corr = 1.0 / (1.0 - beta2 ** step) if debias else 1.0
    a_hat, q_hat = a_t * corr, q_t * corr
    c = 1.0 / (1.0 - 1.0 / B)
    mu2 = c * (a_hat - q_hat / B)                                # Eq. (musq_sigsq_est), first line
    sigma2 = c * (q_hat - a_hat)                                 # Eq. (musq_sigsq_est), second line
    sums = MomentSums(float(mu2.sum()), float(sigma2.sum()), float((np.abs(a_hat) + np.abs(q_hat) / B).sum() * c),
                      int(mu2.size))
    return a_t, q_t, sums


def ratio_to_sigma_eff(sums: MomentSums, B: int, algorithm: str) -> float:
    """mean(mu^2-hat) / mean(sigma_eff^2-hat): sigma_eff^2 = sigma^2/B for 'adam', sigma^2 for 'microadam'."""
    if algorithm == "adam":
        return sums.sum_mu2 / (sums.sum_sigma2 / B)
    if algorithm == "microadam":
        return sums.sum_mu2 / sums.sum_sigma2
    raise ValueError(f"unknown algorithm {algorithm}")
