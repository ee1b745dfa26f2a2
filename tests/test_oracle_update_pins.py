"""Pins of the fp64 optimizer-update oracle: library optimizers, closed forms and
the unbiasedness statements that go with Eq. (musq_sigsq_est).  No GPU needed."""
import numpy as np
import pytest
import torch

from oracle import update as ou


def _rand(n, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(n) * scale


def test_adam_variant_is_library_adam():
    """Variant 'Original' of Algorithm 1 = torch.optim.Adam fed the mean gradient (eps outside the root)."""
    n, steps = 257, 5
    theta0 = _rand(n, 0, 0.02)
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-8)
    theta, m, v = theta0.copy(), np.zeros(n), np.zeros(n)
    B = 8
    for t in range(1, steps + 1):
        S_id = _rand(n, 10 + t) * B                       # a sum over B examples
        p.grad = torch.tensor(S_id / B, dtype=torch.float64)
        opt.step()
        prm = ou.AdamParams(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, grad_scale=1.0 / B, step=t, B=B)
        theta, m, v = ou.adam_family_step(theta, m, v, S_id, None, ou.ADAM, prm)
        np.testing.assert_allclose(theta, p.detach().numpy(), rtol=1e-12, atol=1e-15)


def test_decoupled_weight_decay_matches_adamw():
    """theta - lr*u - wd*theta equals torch AdamW when wd = lr * wd_torch (constant lr)."""
    n, lr, wdt = 64, 1e-2, 0.1
    theta0 = _rand(n, 1)
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=lr, betas=(0.9, 0.95), eps=1e-8, weight_decay=wdt)
    theta, m, v = theta0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, 4):
        g = _rand(n, 20 + t)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        prm = ou.AdamParams(lr=lr, eps=1e-8, weight_decay=lr * wdt, step=t, B=1)
        theta, m, v = ou.adam_family_step(theta, m, v, g, None, ou.ADAM, prm)
    np.testing.assert_allclose(theta, p.detach().numpy(), rtol=1e-12)


def test_B1_microadam_is_adam():
    """With one example nu_micro = nu_adam (Eq. nu_defs), so MicroAdam = Adam."""
    n = 100
    g = _rand(n, 2)
    th, m, v = _rand(n, 3), _rand(n, 4) * 0.1, np.abs(_rand(n, 5)) * 0.01
    prm = ou.AdamParams(step=3, B=1)
    a = ou.adam_family_step(th, m, v, g, None, ou.ADAM, prm)
    b = ou.adam_family_step(th, m, v, g, g * g, ou.MICROADAM, prm)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


def test_estimators_are_sample_variance_and_its_complement():
    """sigma^2-hat is the textbook unbiased sample variance (numpy ddof=1); mu^2-hat = mean^2 - var/B."""
    B, n = 6, 500
    g = np.random.default_rng(6).standard_normal((B, n)) * 0.7 + 0.3
    mu_t, nu_micro = g.mean(0), (g * g).mean(0)
    var = ou.nu_of_variant(ou.MICROADAM_VAR, mu_t, nu_micro, B)
    msq = ou.nu_of_variant(ou.MICROADAM_MSQ, mu_t, nu_micro, B)
    np.testing.assert_allclose(var, g.var(axis=0, ddof=1), rtol=1e-12)
    np.testing.assert_allclose(msq, mu_t ** 2 - g.var(axis=0, ddof=1) / B, rtol=1e-10, atol=1e-14)
    assert np.all(var >= 0)
    assert np.any(msq < 0)          # the mean-square estimator can be negative (Sec. 3.2.3)
    assert np.all(ou.nu_of_variant(ou.MICROADAM, mu_t, nu_micro, B) > 0)


def test_estimators_unbiased_monte_carlo():
    """E[mu^2-hat] = mu^2 and E[sigma^2-hat] = sigma^2 for iid gradients (Eq. musq_sigsq_est)."""
    mu, sigma, B, trials = 0.4, 1.3, 4, 400_000
    g = np.random.default_rng(7).standard_normal((B, trials)) * sigma + mu
    mu_t, nu_micro = g.mean(0), (g * g).mean(0)
    var = ou.nu_of_variant(ou.MICROADAM_VAR, mu_t, nu_micro, B).mean()
    msq = ou.nu_of_variant(ou.MICROADAM_MSQ, mu_t, nu_micro, B).mean()
    assert abs(var - sigma ** 2) < 0.01
    assert abs(msq - mu ** 2) < 0.01
    # and the raw moments of Eq. (basic_nu_averages)
    assert abs((mu_t ** 2).mean() - (mu ** 2 + sigma ** 2 / B)) < 0.01
    assert abs(nu_micro.mean() - (mu ** 2 + sigma ** 2)) < 0.01


@pytest.mark.parametrize("variant", [ou.MICROADAM_VAR, ou.MICROADAM_MSQ])
def test_one_ema_equals_two_emas(variant):
    """EMA of the combined nu (Algorithm 1) = combination of the EMAs of nu_adam and nu_micro (App. D)."""
    B, n, beta2 = 8, 50, 0.95
    v = np.zeros(n)
    ea, em = np.zeros(n), np.zeros(n)
    th, m = np.zeros(n), np.zeros(n)
    for t in range(1, 6):
        g = np.random.default_rng(30 + t).standard_normal((B, n))
        S_id, S_sq = g.sum(0), (g * g).sum(0)
        prm = ou.AdamParams(beta2=beta2, grad_scale=1 / B, sq_scale=1 / B, step=t, B=B)
        th, m, v = ou.adam_family_step(th, m, v, S_id, S_sq, variant, prm)
        ea = beta2 * ea + (1 - beta2) * (S_id / B) ** 2
        em = beta2 * em + (1 - beta2) * (S_sq / B)
    c = 1 / (1 - 1 / B)
    two = c * (em - ea) if variant == ou.MICROADAM_VAR else c * (ea - em / B)
    np.testing.assert_allclose(v, two, rtol=1e-11, atol=1e-14)


def test_constant_gradient_closed_form():
    """Constant g: m-hat = g and v-hat = g^2 at every step, so theta_t = theta_0 - t*lr*g/(|g|+eps)."""
    n, lr, eps = 10, 1e-2, 1e-8
    g = np.linspace(-2, 2, n) + 0.05
    th, m, v = np.zeros(n), np.zeros(n), np.zeros(n)
    for t in range(1, 8):
        prm = ou.AdamParams(lr=lr, eps=eps, step=t, B=1)
        th, m, v = ou.adam_family_step(th, m, v, g, g * g, ou.MICROADAM, prm)
        np.testing.assert_allclose(th, -t * lr * g / (np.abs(g) + eps), rtol=1e-12)
    np.testing.assert_allclose(m, g * (1 - 0.9 ** 7), rtol=1e-12)
    np.testing.assert_allclose(v, g * g * (1 - 0.95 ** 7), rtol=1e-12)


def test_msq_relu_and_eps_root():
    """A negative mu^2-hat is clamped only when forming u; v keeps the unclamped value."""
    B = 4
    S_id = np.array([0.0, 4.0])          # mean 0 and 1
    S_sq = np.array([4.0, 4.0])          # nu_micro = 1 in both
    prm = ou.AdamParams(lr=1.0, eps=1e-6, grad_scale=1 / B, sq_scale=1 / B, step=1, B=B)
    th, m, v = ou.adam_family_step(np.zeros(2), np.zeros(2), np.zeros(2), S_id, S_sq, ou.MICROADAM_MSQ, prm)
    c = 1 / (1 - 1 / B)
    np.testing.assert_allclose(v, (1 - 0.95) * c * np.array([0 - 0.25, 1 - 0.25]), rtol=1e-12)
    assert v[0] < 0
    assert th[0] == 0.0                                  # m-hat = 0 there
    np.testing.assert_allclose(th[1], -1.0 / (np.sqrt(c * 0.75) + 1e-6), rtol=1e-12)
    # eps inside the root (Algorithm 1's placement)
    prm2 = ou.AdamParams(lr=1.0, eps=0.0, eps_root=1e-2, grad_scale=1 / B, sq_scale=1 / B, step=1, B=B)
    th2, _, _ = ou.adam_family_step(np.zeros(2), np.zeros(2), np.zeros(2), S_id, S_sq, ou.MICROADAM_MSQ, prm2)
    np.testing.assert_allclose(th2[1], -1.0 / np.sqrt(c * 0.75 + 1e-2), rtol=1e-12)
    with pytest.raises(ValueError):
        ou.adam_family_step(np.zeros(2), np.zeros(2), np.zeros(2), S_id, S_sq, ou.MICROADAM_VAR, ou.AdamParams(B=1))


def test_microsignsgd_pins():
    """B=1: EMA o avg o sign = EMA o sign (SignSGD with momentum); |m| <= 1; all-agree limit m_t = 1 - beta^t."""
    n, beta, lr = 40, 0.9, 1e-3
    g = _rand(n, 8)
    th, m = _rand(n, 9), np.zeros(n)
    th_ref, m_ref = th.copy(), m.copy()
    for t in range(1, 5):
        th, m = ou.microsignsgd_step(th, m, np.sign(g), lr, beta, 0.0, 1, False, t)
        m_ref = beta * m_ref + (1 - beta) * np.sign(g)
        th_ref = th_ref - lr * m_ref
    np.testing.assert_allclose(th, th_ref, rtol=1e-13)
    B = 16
    th, m = np.zeros(3), np.zeros(3)
    for t in range(1, 30):
        th, m = ou.microsignsgd_step(th, m, np.array([B, -B, 0.0]), lr, beta, 0.0, B, False, t)
        assert np.all(np.abs(m) <= 1.0)
        np.testing.assert_allclose(m, np.array([1, -1, 0]) * (1 - beta ** t), rtol=1e-12, atol=0)
    # debias makes the all-agree direction exactly +-1; weight decay is not multiplied by lr
    th2, m2 = ou.microsignsgd_step(np.ones(3), np.zeros(3), np.array([B, -B, 0.0]), lr, beta, 0.5, B, True, 1)
    np.testing.assert_allclose(th2, 1.0 - lr * np.array([1, -1, 0]) - 0.5, rtol=1e-13)


def test_sign_family_pins():
    """The three placements of sign (Sec. 3.1): MicroSignSGD variant = the dedicated routine; with B = 1 MicroSignSGD
    and SignSGD coincide; SignEMA equals torch.sign of a hand-rolled EMA; constant-gradient closed forms."""
    n, beta, lr, wd = 30, 0.9, 1e-3, 1e-2
    rng = np.random.default_rng(12)
    th0 = rng.standard_normal(n)
    # (a) variant 0 is the MicroSignSGD routine
    S = rng.integers(-8, 9, n).astype(np.float64) * 2
    a = ou.sign_family_step(th0, np.zeros(n), S, ou.MICROSIGNSGD, lr, beta, wd, 16, True, 3)
    b = ou.microsignsgd_step(th0, np.zeros(n), S, lr, beta, wd, 16, True, 3)
    np.testing.assert_array_equal(a[0], b[0]); np.testing.assert_array_equal(a[1], b[1])
    # (b) one example per batch: the sign of the average is the average of the signs
    g = rng.standard_normal(n)
    th_a, m_a, th_b, m_b = th0.copy(), np.zeros(n), th0.copy(), np.zeros(n)
    for t in range(1, 6):
        th_a, m_a = ou.sign_family_step(th_a, m_a, np.sign(g), ou.MICROSIGNSGD, lr, beta, 0.0, 1, False, t)
        th_b, m_b = ou.sign_family_step(th_b, m_b, g, ou.SIGNSGD, lr, beta, 0.0, 1, False, t)
    np.testing.assert_allclose(th_a, th_b, rtol=1e-14)
    # (c) SignEMA against a hand-rolled recursion and the library sign; every step has size lr exactly
    th, m, ema = th0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, 6):
        S = rng.standard_normal(n) * 16
        prev = th.copy()
        th, m = ou.sign_family_step(th, m, S, ou.SIGNEMA, lr, beta, 0.0, 16, False, t)
        ema = beta * ema + (1 - beta) * S / 16
        np.testing.assert_allclose(m, ema, rtol=1e-13)
        np.testing.assert_allclose(np.abs(th - prev), lr, rtol=1e-9)
        np.testing.assert_allclose(th, prev - lr * np.sign(ema), rtol=1e-12, atol=1e-15)
    # (d) constant gradient: SignSGD's EMA tends to sign(g) as 1 - beta^t; weight decay is not scaled by lr
    th, m = np.ones(3), np.zeros(3)
    S = np.array([3.0, -0.5, 0.0])
    for t in range(1, 20):
        th, m = ou.sign_family_step(th, m, S, ou.SIGNSGD, lr, beta, 0.0, 4, False, t)
        np.testing.assert_allclose(m, np.array([1, -1, 0]) * (1 - beta ** t), rtol=1e-12)
    th2, _ = ou.sign_family_step(np.ones(3), np.zeros(3), S, ou.SIGNEMA, lr, beta, 0.5, 4, False, 1)
    np.testing.assert_allclose(th2, 1.0 - lr * np.array([1, -1, 0]) - 0.5, rtol=1e-13)
    # (e) the ordering matters once B > 1: a batch whose mean and whose majority disagree
    per_example = np.array([[5.0], [-1.0], [-1.0]])            # mean +1, two of three negative
    _, m_micro = ou.sign_family_step(np.zeros(1), np.zeros(1), np.sign(per_example).sum(0), ou.MICROSIGNSGD, lr, beta, 0.0, 3, False, 1)
    _, m_sgd = ou.sign_family_step(np.zeros(1), np.zeros(1), per_example.sum(0), ou.SIGNSGD, lr, beta, 0.0, 3, False, 1)
    assert m_micro[0] < 0 < m_sgd[0]


def test_clipping_is_the_library_global_norm_clip_and_acts_on_every_example():
    """kappa scales the mean gradient exactly like torch's clip_grad_norm_ (up to its 1e-6 guard), leaves gradients
    under the threshold alone, and the clipped MicroAdam step equals the plain step on per-example gradients that
    were all multiplied by kappa."""
    rng = np.random.default_rng(7)
    n, B = 300, 6
    g = rng.standard_normal((B, n)) * 0.3
    S_id, S_sq = g.sum(0), (g * g).sum(0)
    mean = S_id / B
    for max_norm in (0.5, 100.0):
        kappa = ou.clip_factor(float((S_id ** 2).sum()), 1.0 / B, max_norm)
        p = torch.nn.Parameter(torch.zeros(n, dtype=torch.float64))
        p.grad = torch.tensor(mean.copy())
        torch.nn.utils.clip_grad_norm_([p], max_norm)
        np.testing.assert_allclose(kappa * mean, p.grad.numpy(), rtol=2e-6)
        if max_norm > 10:
            assert kappa == 1.0
        else:
            assert kappa < 1.0 and abs(np.linalg.norm(kappa * mean) - max_norm) < 1e-12
        prm = ou.AdamParams(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, grad_scale=1.0 / B, sq_scale=1.0 / B, step=2, B=B)
        th, m, v = rng.standard_normal(n), rng.standard_normal(n) * 0.1, np.abs(rng.standard_normal(n)) * 0.01
        for variant in (ou.ADAM, ou.MICROADAM, ou.MICROADAM_VAR, ou.MICROADAM_MSQ):
            a = ou.adam_family_step_clipped(th, m, v, S_id, S_sq, variant, prm, float((S_id ** 2).sum()), max_norm)
            gk = kappa * g
            b = ou.adam_family_step(th, m, v, gk.sum(0), (gk * gk).sum(0), variant, prm)
            for x, y in zip(a, b):
                np.testing.assert_allclose(x, y, rtol=1e-12, atol=1e-15)
