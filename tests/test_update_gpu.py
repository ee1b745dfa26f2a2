"""GPU parity of the optimizer-update kernels against the fp64 elementwise oracle, over consecutive steps."""
import numpy as np
import pytest
import torch

import paper_2510_00236_amd as pex
import synth_inputs as si
from oracle import update as ou

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

VARIANTS = [("adam", ou.ADAM), ("microadam", ou.MICROADAM), ("microadam_var", ou.MICROADAM_VAR),
            ("microadam_msq", ou.MICROADAM_MSQ)]


def _stats(n, B, seed, mean=0.05):
    """Synthetic S_id, S_sq of B per-example gradients g_b ~ N(mean, 1) * 1e-2 (fp32, as pex_stat would emit)."""
    g = torch.Generator().manual_seed(seed)
    gb = (torch.randn(B, n, generator=g) + mean) * 1e-2
    return gb.sum(0).contiguous(), (gb * gb).sum(0).contiguous()


@pytest.mark.parametrize("name,code", VARIANTS)
@pytest.mark.parametrize("n", [1 << 20, 1000003, 7])
def test_adam_family_matches_oracle(name, code, n):
    B, steps = 32, 3
    theta0, m0, v0 = si.optimizer_state(n, seed=1)
    th, m, v = theta0.to(DEV), m0.to(DEV), v0.to(DEV)
    rth, rm, rv = theta0.double().numpy(), m0.double().numpy(), v0.double().numpy()
    eps = 1e-6 if name == "microadam_msq" else 1e-8
    lr = 2.0 / 1024
    for t in range(1, steps + 1):
        # mean/sigma = 1 keeps most mu^2-hat and sigma^2-hat estimates away from zero
        S_id, S_sq = _stats(n, B, 100 + t, mean=1.0)
        kw = dict(lr=lr, beta1=0.9, beta2=0.95, eps=eps, eps_root=0.0, weight_decay=1e-4,
                  grad_scale=1.0 / B, sq_scale=1.0 / B, step=t, B=B)
        prev_got, prev_ref = th.cpu().double().numpy(), rth
        pex.pex_adam_update(th, m, v, S_id.to(DEV), None if name == "adam" else S_sq.to(DEV), name, pex.AdamParams(**kw))
        rth, rm, rv = ou.adam_family_step(rth, rm, rv, S_id.numpy(), S_sq.numpy(), code, ou.AdamParams(**kw))
        torch.cuda.synchronize()
        gm, gv, gth = m.cpu().double().numpy(), v.cpu().double().numpy(), th.cpu().double().numpy()
        assert np.isfinite(gth).all() and np.isfinite(gv).all()
        # fp32 arithmetic on fp32 inputs: a few ulp of the largest term on m; v of the Var/MSQ variants is a
        # difference of two O(nu_micro) terms, so its error is measured against that scale.
        np.testing.assert_allclose(gm, rm, rtol=2e-6, atol=4e-7 * np.abs(rm).max())
        nu_scale = float((S_sq.double().numpy() / B).max())
        np.testing.assert_allclose(gv, rv, rtol=4e-6, atol=4e-7 * nu_scale)
        # The increment of theta is lr*m-hat/(sqrt(v-hat)+eps): its sensitivity to v-hat is unbounded as
        # v-hat -> 0 (and it has a kink where the max(0, .) filter acts), so increments are compared where
        # v-hat is at least 1e-3 of the second-moment scale; elsewhere they must be finite, bounded by
        # lr*|m-hat|/eps and carry the sign of -m-hat.
        inc_got, inc_ref = gth - prev_got, rth - prev_ref
        v_hat = rv / (1.0 - 0.95 ** t)
        m_hat = rm / (1.0 - 0.9 ** t)
        well = v_hat > 1e-3 * nu_scale
        assert well.mean() > 0.9 or n < 100
        if well.any():
            assert np.abs(inc_got - inc_ref)[well].max() <= 1e-3 * np.abs(inc_ref[well]).max(), name
            np.testing.assert_allclose(inc_got[well], inc_ref[well], rtol=2e-3, atol=1e-9)
        ill = ~well
        if ill.any():
            assert (np.abs(inc_got[ill]) <= lr * np.abs(m_hat[ill]) / eps * 1.001 + 1e-3 * np.abs(prev_got[ill]) + 1e-9).all()


def test_msq_negative_estimates_are_clamped():
    """mu^2-hat < 0 where the mean is ~0: v stays negative in memory, the step stays finite (Sec. 3.2.3)."""
    n, B = 4096, 8
    S_id = torch.zeros(n)
    S_sq = torch.full((n,), 8.0e-4)
    th, m, v = (torch.ones(n, device=DEV), torch.zeros(n, device=DEV), torch.zeros(n, device=DEV))
    p = pex.AdamParams(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-6, eps_root=0.0, weight_decay=0.0,
                       grad_scale=1.0 / B, sq_scale=1.0 / B, step=1, B=B)
    pex.pex_adam_update(th, m, v, S_id.to(DEV), S_sq.to(DEV), "microadam_msq", p)
    torch.cuda.synchronize()
    assert (v < 0).all() and torch.isfinite(th).all() and torch.equal(th, torch.ones(n, device=DEV))


@pytest.mark.parametrize("n", [1 << 20, 1000003, 5])
@pytest.mark.parametrize("debias", [False, True])
def test_microsignsgd_matches_oracle(n, debias):
    B, beta, lr, wd = 64, 0.9, 3.47e-3, 1e-4
    theta0, m0, _ = si.optimizer_state(n, seed=2)
    th, m = theta0.to(DEV), m0.to(DEV)
    rth, rm = theta0.double().numpy(), m0.double().numpy()
    g = torch.Generator().manual_seed(5)
    for t in range(1, 4):
        S_sign = torch.randint(-B // 2, B // 2 + 1, (n,), generator=g).float() * 2   # same parity as B
        pex.pex_signsgd_update(th, m, S_sign.to(DEV), lr, beta, wd, B, debias=debias, step=t)
        rth, rm = ou.microsignsgd_step(rth, rm, S_sign.numpy(), lr, beta, wd, B, debias, t)
    torch.cuda.synchronize()
    np.testing.assert_allclose(m.cpu().double().numpy(), rm, rtol=2e-6, atol=4e-7)
    assert (m.abs() <= 1).all()
    d_ref, d_got = rth - theta0.double().numpy(), th.cpu().double().numpy() - theta0.double().numpy()
    assert np.abs(d_got - d_ref).max() <= 2e-5 * np.abs(d_ref).max() + 1e-9


@pytest.mark.parametrize("variant", ["microsignsgd", "signsgd", "signema"])
@pytest.mark.parametrize("n", [1 << 20, 1000003])
def test_sign_family_matches_oracle(variant, n):
    B, beta, lr, wd = 64, 0.9, 1.1e-3, 1e-4
    code = {"microsignsgd": ou.MICROSIGNSGD, "signsgd": ou.SIGNSGD, "signema": ou.SIGNEMA}[variant]
    theta0, m0, _ = si.optimizer_state(n, seed=4)
    th, m = theta0.to(DEV), m0.to(DEV)
    rth, rm = theta0.double().numpy(), m0.double().numpy()
    g = torch.Generator().manual_seed(6)
    for t in range(1, 4):
        if variant == "microsignsgd":
            S = torch.randint(-B // 2, B // 2 + 1, (n,), generator=g).float() * 2
        else:
            S = torch.randn(n, generator=g) * B
            S[::97] = 0.0                                  # sgn(0) = 0
        pex.pex_sign_update(th, m, S.to(DEV), variant, lr, beta, wd, B, debias=True, step=t)
        rth, rm = ou.sign_family_step(rth, rm, S.numpy(), code, lr, beta, wd, B, True, t)
    torch.cuda.synchronize()
    np.testing.assert_allclose(m.cpu().double().numpy(), rm, rtol=3e-6, atol=4e-7)
    d_ref, d_got = rth - theta0.double().numpy(), th.cpu().double().numpy() - theta0.double().numpy()
    if variant == "signema":
        # sign(m) is decided in fp32 on the GPU and in fp64 by the oracle: they may differ only where m is within
        # rounding of zero (not the exact zeros planted above, where both give 0); everywhere else the steps agree
        # to fp32 rounding of theta
        near_zero = (np.abs(rm) < 1e-6) & (rm != 0.0)
        assert near_zero.mean() < 1e-3
        assert np.abs(d_got - d_ref)[~near_zero].max() <= 1e-6
    else:
        assert np.abs(d_got - d_ref).max() <= 2e-5 * np.abs(d_ref).max() + 1e-9


def test_end_to_end_stat_then_update():
    """Config-2 layer: statistics from pex_stat feed the MicroAdam update; compared with the oracle chain."""
    import oracle
    w = si.WORKLOADS["c2_mlp_in"]
    X, G = si.make(w, seed=1)
    Xd, Gd = X.to(DEV), G.to(DEV)
    S_id, S_sq = pex.pex_stat(Xd, Gd, "identity"), pex.pex_stat(Xd, Gd, "square")
    n = w.din * w.dout
    theta0, m0, v0 = si.optimizer_state(n, seed=3)
    th, m, v = theta0.to(DEV), m0.to(DEV), v0.to(DEV)
    kw = dict(lr=2.0 / 1024, beta1=0.9, beta2=0.95, eps=1e-8, eps_root=0.0, weight_decay=0.0,
              grad_scale=1.0 / w.B, sq_scale=1.0 / w.B, step=1, B=w.B)
    pex.pex_adam_update(th, m, v, S_id.view(-1), S_sq.view(-1), "microadam", pex.AdamParams(**kw))
    torch.cuda.synchronize()
    st = oracle.stat(si.widen(X), si.widen(G))
    rth, rm, rv = ou.adam_family_step(theta0.double().numpy(), m0.double().numpy(), v0.double().numpy(),
                                      st.S_id.ravel(), st.S_sq.ravel(), ou.MICROADAM, ou.AdamParams(**kw))
    np.testing.assert_allclose(v.cpu().double().numpy(), rv, rtol=1e-4)
    d_ref, d_got = rth - theta0.double().numpy(), th.cpu().double().numpy() - theta0.double().numpy()
    assert np.abs(d_got - d_ref).max() <= 1e-3 * np.abs(d_ref).max()


@pytest.mark.parametrize("n", [1 << 20, 1000003, 3])
@pytest.mark.parametrize("debias", [True, False])
def test_moment_tracking_matches_oracle(n, debias):
    """EMAs of nu_adam and nu_micro and the summed mu^2 / sigma^2 estimators (Sec. 3.2.2) over several steps."""
    from oracle import moments as om
    B, beta2 = 8, 0.95
    rng = np.random.default_rng(n)
    mu = rng.standard_normal(n) * 0.05
    a = torch.zeros(n, device=DEV)
    q = torch.zeros(n, device=DEV)
    a_ref, q_ref = np.zeros(n), np.zeros(n)
    for t in range(1, 5):
        g = (mu[None, :] + rng.standard_normal((B, n))).astype(np.float32)
        S_id = torch.from_numpy(g.sum(0)).to(DEV)
        S_sq = torch.from_numpy((g * g).sum(0)).to(DEV)
        prm = pex.MomentParams(beta2=beta2, grad_scale=1.0 / B, sq_scale=1.0 / B, B=B, debias=int(debias), step=t)
        sums = pex.pex_moment_track(a, q, S_id, S_sq, prm).cpu().numpy()
        a_ref, q_ref, ref = om.moment_track_step(a_ref, q_ref, S_id.cpu().double().numpy(), S_sq.cpu().double().numpy(),
                                                 float(np.float32(beta2)), float(np.float32(1.0 / B)), float(np.float32(1.0 / B)), B, t, debias)
        np.testing.assert_allclose(a.cpu().double().numpy(), a_ref, rtol=2e-6, atol=1e-30)
        np.testing.assert_allclose(q.cpu().double().numpy(), q_ref, rtol=2e-6, atol=1e-30)
        # the sums cancel (mu^2 << sigma^2 here): the bar is relative to the size of the terms, fp32 EMAs give ~1e-7 of it
        assert abs(sums[0] - ref.sum_mu2) <= 2e-6 * ref.sum_abs, (sums, ref)
        assert abs(sums[1] - ref.sum_sigma2) <= 2e-6 * ref.sum_abs, (sums, ref)
    # run-to-run determinism of the reduction
    a2, q2 = a.clone(), q.clone()
    s1 = pex.pex_moment_track(a, q, S_id, S_sq, prm).clone()
    s2 = pex.pex_moment_track(a2, q2, S_id, S_sq, prm)
    assert torch.equal(s1, s2) and torch.equal(a, a2)


def test_moment_tracking_recovers_planted_moments():
    """Per-example gradients with known mu and sigma: after one step without memory the averaged estimators land on
    mu^2 and sigma^2 within the Monte-Carlo error, through the whole GPU path (statistics, then tracking)."""
    B, T, din, dout = 16, 4, 256, 512
    X, G = si.custom(B, T, din, dout, dtype="bf16", seed=5)
    Xd, Gd = X.to(DEV), G.to(DEV)
    out = pex.pex_stat_multi(Xd, Gd, ("identity", "square"))
    n = din * dout
    a, q = torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    prm = pex.MomentParams(beta2=0.0, grad_scale=1.0 / B, sq_scale=1.0 / B, B=B, debias=1, step=1)
    sums = pex.pex_moment_track(a, q, out["identity"].view(-1), out["square"].view(-1), prm).cpu().numpy() / n
    # entries of X_b^T G_b are sums of T products of independent unit normals: mean 0, variance T
    assert abs(sums[1] - T) < 0.02 * T
    assert abs(sums[0]) < 0.1 * T / B            # nu_adam itself would sit at T / B


@pytest.mark.parametrize("n", [1 << 20, 1000003, 5])
def test_sum_of_squares_and_clipped_updates_match_oracle(n):
    """Global-norm clipping without a host round trip: the norm accumulates on the GPU over two 'layers', the update
    reads it there.  Thresholds on both sides of the actual norm."""
    rng = np.random.default_rng(n)
    B = 8
    S_id_t, S_sq_t = _stats(n, B, seed=n % 1000)
    parts = [S_id_t.numpy(), rng.standard_normal(n // 2 + 3).astype(np.float32) * 0.05]
    acc = pex.pex_sum_squares(torch.from_numpy(parts[0]).to(DEV))
    acc = pex.pex_sum_squares(torch.from_numpy(parts[1]).to(DEV), acc=acc, accumulate=True)
    ref_sumsq = float((parts[0].astype(np.float64) ** 2).sum() + (parts[1].astype(np.float64) ** 2).sum())
    assert abs(float(acc.cpu()[0]) - ref_sumsq) <= 1e-12 * ref_sumsq
    again = pex.pex_sum_squares(torch.from_numpy(parts[0]).to(DEV))
    again = pex.pex_sum_squares(torch.from_numpy(parts[1]).to(DEV), acc=again, accumulate=True)
    assert torch.equal(acc, again)                       # fixed summation order
    S_id, S_sq = parts[0], S_sq_t.numpy()
    norm = np.sqrt(ref_sumsq) / B
    for max_norm in (0.25 * norm, 4.0 * norm):
        for name, code in VARIANTS:
            theta0 = rng.standard_normal(n).astype(np.float32) * 0.02
            m0 = rng.standard_normal(n).astype(np.float32) * 0.01
            v0 = (rng.standard_normal(n).astype(np.float32) ** 2) * 0.01
            th, m, v = (torch.from_numpy(x.copy()).to(DEV) for x in (theta0, m0, v0))
            prm = pex.AdamParams(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, eps_root=0.0, weight_decay=0.0,
                                 grad_scale=1.0 / B, sq_scale=1.0 / B, step=3, B=B)
            pex.pex_adam_update_clipped(th, m, v, torch.from_numpy(S_id).to(DEV), torch.from_numpy(S_sq).to(DEV), name, prm,
                                        acc, float(max_norm))
            op = ou.AdamParams(lr=float(np.float32(1e-2)), beta1=float(np.float32(0.9)), beta2=float(np.float32(0.95)),
                               eps=float(np.float32(1e-8)), grad_scale=float(np.float32(1.0 / B)),
                               sq_scale=float(np.float32(1.0 / B)), step=3, B=B)
            rt, rm, rv = ou.adam_family_step_clipped(theta0, m0, v0, S_id, S_sq, code, op, ref_sumsq, float(np.float32(max_norm)))
            np.testing.assert_allclose(m.cpu().double().numpy(), rm, rtol=3e-6, atol=1e-9)
            np.testing.assert_allclose(v.cpu().double().numpy(), rv, rtol=3e-6, atol=1e-10)
            ok = np.abs(rv) / (1 - 0.95 ** 3) >= 1e-3 * np.abs(rv).max() / (1 - 0.95 ** 3)
            d_gpu, d_ref = th.cpu().double().numpy() - theta0, rt - theta0
            np.testing.assert_allclose(d_gpu[ok], d_ref[ok], rtol=2e-4, atol=2e-8)      # theta is fp32: one ulp of 0.1 is 7e-9
    # under the threshold the clipped call is the plain call, bit for bit
    th1, m1, v1 = (torch.from_numpy(x.copy()).to(DEV) for x in (theta0, m0, v0))
    th2, m2, v2 = (torch.from_numpy(x.copy()).to(DEV) for x in (theta0, m0, v0))
    Sd, Sq = torch.from_numpy(S_id).to(DEV), torch.from_numpy(S_sq).to(DEV)
    pex.pex_adam_update_clipped(th1, m1, v1, Sd, Sq, "microadam", prm, acc, float(4.0 * norm))
    pex.pex_adam_update(th2, m2, v2, Sd, Sq, "microadam", prm)
    assert torch.equal(th1, th2) and torch.equal(m1, m2) and torch.equal(v1, v2)


def test_updates_at_the_full_parameter_count_of_the_1b_layer():
    """One MicroAdam and one MicroSignSGD step over the 16,777,216 parameters of the 2048 x 8192 layer (the size
    bench.py times): every parameter against the fp64 oracle."""
    n, B = 2048 * 8192, 16
    theta0, m0, v0 = si.optimizer_state(n, seed=3)
    g = torch.Generator().manual_seed(77)
    S_id = torch.randn(n, generator=g) * (B ** 0.5) * 1e-2 + B * 1e-2
    S_sq = (S_id * S_id) / B + torch.rand(n, generator=g) * B * 1e-4            # >= S_id^2 / B, as Cauchy-Schwarz demands
    S_sg = torch.randint(-B // 2, B // 2 + 1, (n,), generator=g).float() * 2    # same parity as B
    kw = dict(lr=2.0 / 1024, beta1=0.9, beta2=0.95, eps=1e-8, eps_root=0.0, weight_decay=1e-4,
              grad_scale=1.0 / B, sq_scale=1.0 / B, step=1, B=B)
    th, m, v = theta0.to(DEV), m0.to(DEV), v0.to(DEV)
    pex.pex_adam_update(th, m, v, S_id.to(DEV), S_sq.to(DEV), "microadam", pex.AdamParams(**kw))
    th2, m2 = theta0.to(DEV), m0.to(DEV)
    pex.pex_signsgd_update(th2, m2, S_sg.to(DEV), 1e-3, 0.9, 1e-4, B)
    torch.cuda.synchronize()
    t0 = theta0.double().numpy()
    rth, rm, rv = ou.adam_family_step(t0, m0.double().numpy(), v0.double().numpy(), S_id.numpy(), S_sq.numpy(),
                                      ou.MICROADAM, ou.AdamParams(**kw))
    np.testing.assert_allclose(m.cpu().double().numpy(), rm, rtol=2e-6, atol=4e-7 * np.abs(rm).max())
    np.testing.assert_allclose(v.cpu().double().numpy(), rv, rtol=4e-6, atol=4e-7 * np.abs(rv).max())
    inc_got, inc_ref = th.cpu().double().numpy() - t0, rth - t0
    assert np.abs(inc_got - inc_ref).max() <= 1e-3 * np.abs(inc_ref).max()
    rth2, rm2 = ou.microsignsgd_step(t0, m0.double().numpy(), S_sg.numpy(), 1e-3, 0.9, 1e-4, B, False, 1)
    np.testing.assert_allclose(m2.cpu().double().numpy(), rm2, rtol=2e-6, atol=1e-9)
    inc2_got, inc2_ref = th2.cpu().double().numpy() - t0, rth2 - t0
    assert np.abs(inc2_got - inc2_ref).max() <= 1e-3 * np.abs(inc2_ref).max() + 1e-9
