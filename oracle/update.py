"""fp64 elementwise oracle of the optimizer updates that consume the statistics.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

``adam_family_step`` follows Algorithm 1 (App. E) step by step in its order and
notation, with these readings where the printed listing is garbled or silent:

* The MicroAdamVar / MicroAdamMSQ lines of Algorithm 1 carry a factor B/(1-B)
  (negative for B > 1) and the MSQ line as printed has no 1/B on nu_micro; the
  estimators actually meant are those of Eq. (musq_sigsq_est), Sec. 3.2:
  sigma^2-hat = (nu_micro - nu_adam) / (1 - 1/B),
  mu^2-hat    = (nu_adam - nu_micro / B) / (1 - 1/B).
  Their unbiasedness (stated with the equation) is what pins this reading.
* epsilon: the main text (Sec. 3.2.3) puts it outside the root, Algorithm 1
  inside.  Both are exposed: u = m-hat / (sqrt(v-hat + eps_root) + eps).
* The max(0, .) filter is applied to the bias-corrected v-hat only when forming
  u (the stored EMA stays unclamped, Sec. 3.2.3), for MSQ as printed and also
  for Var, where it is a no-op in exact arithmetic.
* One EMA of the combined nu (Algorithm 1) rather than two EMAs combined later
  (App. D): identical by linearity.
* Weight decay (App. D) is decoupled and not multiplied by the learning rate:
  theta <- theta - lr * u - wd * theta.
* grad_scale / sq_scale turn the sums S_id, S_sq into the mean gradient mu_t and
  nu_micro (1/B and 1/B when the cotangents are those of the summed loss).

* Gradient clipping (Sec. 3.2.3 and App. C use it with threshold 1e-2 to stabilise MicroAdam, MicroAdamVar and
  MicroAdamMSQ; its form is not spelled out): read as clipping by the global norm of the mean gradient,
  kappa = min(1, c / ||mu_t||) with the norm over all parameters, applied to every per-example gradient alike -- so
  the mean gradient scales by kappa and the per-example second moment by kappa^2 (``clip_factor``,
  ``adam_family_step_clipped``).

``microsignsgd_step`` is Sec. 3.1: EMA o avg o sign; ``sign_family_step`` covers the three orderings of
avg, EMA and sign that Sec. 3.1 compares (SignEMA, SignSGD, MicroSignSGD).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

ADAM, MICROADAM, MICROADAM_VAR, MICROADAM_MSQ = 0, 1, 2, 3


@dataclass
class AdamParams:
    lr: float = 2.0 / 1024.0      # App. D, base learning rate
    beta1: float = 0.9            # App. D
    beta2: float = 0.95           # App. D
    eps: float = 1e-8
    eps_root: float = 0.0
    weight_decay: float = 0.0
    grad_scale: float = 1.0
    sq_scale: float = 1.0
    step: int = 1                 # t in Algorithm 1, first step is 1
    B: int = 1


def nu_of_variant(variant: int, mu_t: np.ndarray, nu_micro: np.ndarray, B: int) -> np.ndarray:
    """The preconditioner input nu_t of Algorithm 1 for each variant."""
    nu_adam = mu_t * mu_t                                   # Eq. (nu_defs), right
    if variant == ADAM:
        return nu_adam
    if variant == MICROADAM:
        return nu_micro                                     # Eq. (nu_defs), left
    if B < 2:
        raise ValueError("the unbiased estimators need B >= 2")
    c = 1.0 / (1.0 - 1.0 / B)
    if variant == MICROADAM_VAR:
        return c * (nu_micro - nu_adam)                     # sigma^2-hat, Eq. (musq_sigsq_est)
    if variant == MICROADAM_MSQ:
        return c * (nu_adam - nu_micro / B)                 # mu^2-hat, Eq. (musq_sigsq_est)
    raise ValueError(f"unknown variant {variant}")


def adam_family_step(theta, m, v, S_id, S_sq, variant: int, p: AdamParams):
    """One step of Algorithm 1; returns new (theta, m, v) as fp64 arrays."""
    theta = np.asarray(theta, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    mu_t = np.float64(p.grad_scale) * np.asarray(S_id, dtype=np.float64)
    if variant == ADAM:
        nu_micro = None
    else:
        nu_micro = np.float64(p.sq_scale) * np.asarray(S_sq, dtype=np.float64)
    m_t = p.beta1 * m + (1.0 - p.beta1) * mu_t
    nu_t = nu_of_variant(variant, mu_t, nu_micro, p.B)
    v_t = p.beta2 * v + (1.0 - p.beta2) * nu_t
    m_hat = m_t / (1.0 - p.beta1 ** p.step)
    v_hat = v_t / (1.0 - p.beta2 ** p.step)
    if variant in (MICROADAM_VAR, MICROADAM_MSQ):
        v_hat = np.maximum(0.0, v_hat)
    u_t = m_hat / (np.sqrt(v_hat + p.eps_root) + p.eps)
    theta_t = theta - p.lr * u_t - p.weight_decay * theta
    return theta_t, m_t, v_t


def clip_factor(sum_sq_of_S_id: float, grad_scale: float, max_norm: float) -> float:
    """kappa = min(1, max_norm / ||mu_t||), ||mu_t|| = |grad_scale| * sqrt(sum over all parameters of S_id^2)."""
    norm = abs(grad_scale) * float(np.sqrt(sum_sq_of_S_id))
    return 1.0 if norm <= max_norm else max_norm / norm


def adam_family_step_clipped(theta, m, v, S_id, S_sq, variant: int, p: AdamParams, sum_sq_of_S_id: float, max_norm: float):
    """Algorithm 1 on per-example gradients all multiplied by the global clipping factor."""
    kappa = clip_factor(sum_sq_of_S_id, p.grad_scale, max_norm)
    q = AdamParams(**{**p.__dict__, "grad_scale": p.grad_scale * kappa, "sq_scale": p.sq_scale * kappa * kappa})
    return adam_family_step(theta, m, v, S_id, S_sq, variant, q)


def microsignsgd_step(theta, m, S_sign, lr: float, beta: float, weight_decay: float, B: int,
                      debias: bool, step: int):
    """MicroSignSGD = EMA o avg o sign (Sec. 3.1); returns new (theta, m)."""
    theta = np.asarray(theta, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    avg_sign = np.asarray(S_sign, dtype=np.float64) / float(B)
    m_t = beta * m + (1.0 - beta) * avg_sign
    d = m_t / (1.0 - beta ** step) if debias else m_t
    theta_t = theta - lr * d - weight_decay * theta
    return theta_t, m_t


MICROSIGNSGD, SIGNSGD, SIGNEMA = 0, 1, 2


def sign_family_step(theta, m, S, variant: int, lr: float, beta: float, weight_decay: float, B: int,
                     debias: bool, step: int):
    """One step of the three placements of sign in SignSGD (Sec. 3.1); returns new (theta, m).

      MicroSignSGD = EMA o avg o sign : S is the sum of per-example signs;   m <- EMA(S/B),        step along m
      SignSGD      = EMA o sign o avg : S is the sum of gradients;           m <- EMA(sign(S/B)),  step along m
      SignEMA      = sign o EMA o avg : S is the sum of gradients;           m <- EMA(S/B),        step along sign(m)
    Weight decay is decoupled and not multiplied by the learning rate (App. D).  ``debias`` divides the EMA by
    1 - beta^t before it is used (for SignEMA this cannot change the sign and is ignored).
    """
    theta = np.asarray(theta, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    avg = np.asarray(S, dtype=np.float64) / float(B)
    if variant == SIGNSGD:
        avg = np.sign(avg)
    elif variant not in (MICROSIGNSGD, SIGNEMA):
        raise ValueError(f"unknown variant {variant}")
    m_t = beta * m + (1.0 - beta) * avg
    if variant == SIGNEMA:
        d = np.sign(m_t)
    else:
        d = m_t / (1.0 - beta ** step) if debias else m_t
    theta_t = theta - lr * d - weight_decay * theta
    return theta_t, m_t
