"""Pins of the norm / weighted-sum oracle against the already pinned matrix oracle, the Gram ("ghost") route that
never forms a per-example gradient, closed forms and brute force."""
import numpy as np

import oracle
from oracle import norms as on


def _rand(B, T, din, dout, seed):
    r = np.random.default_rng(seed)
    return r.standard_normal((B, T, din)).astype(np.float32), r.standard_normal((B, T, dout)).astype(np.float32)


def test_example_norms_three_ways():
    X, G = _rand(4, 11, 9, 7, 0)
    N = on.example_norms(X, G)
    # the C oracle's own per-example norms (a different loop nest)
    np.testing.assert_allclose(N, oracle.stat(X, G).normsq, rtol=1e-12)
    # ghost route: <X_b X_b^T, G_b G_b^T> through the T x T Gram matrices, no M_b
    Xd, Gd = X.astype(np.float64), G.astype(np.float64)
    ghost = np.array([((Xd[b] @ Xd[b].T) * (Gd[b] @ Gd[b].T)).sum() for b in range(4)])
    np.testing.assert_allclose(N, ghost, rtol=1e-12)
    # the sum over examples is the total of the square statistic
    np.testing.assert_allclose(N.sum(), oracle.stat(X, G).S_sq.sum(), rtol=1e-12)


def test_token_norms():
    X, G = _rand(3, 8, 6, 5, 1)
    Nt = on.token_norms(X, G)
    assert Nt.shape == (3, 8)
    # the total is the total of the per-token square statistic (Sec. 2.3)
    np.testing.assert_allclose(Nt.sum(), oracle.token_sq(X, G).sum(), rtol=1e-12)
    # T = 1: gradients are rank one, so the per-token norm is the per-example norm
    X1, G1 = _rand(5, 1, 6, 5, 2)
    np.testing.assert_allclose(on.token_norms(X1, G1)[:, 0], on.example_norms(X1, G1), rtol=1e-12)
    # Cauchy-Schwarz on the sum of T rank-one terms: ||sum_t x g^T||^2 <= T * sum_t ||x||^2 ||g||^2
    assert (on.example_norms(X, G) <= 8 * Nt.sum(axis=1) * (1 + 1e-12)).all()
    # library check
    np.testing.assert_allclose(Nt, (X.astype(np.float64) ** 2).sum(-1) * (G.astype(np.float64) ** 2).sum(-1), rtol=1e-12)


def test_weighted_sum_and_clipping():
    X, G = _rand(5, 7, 6, 4, 3)
    st = oracle.stat(X, G)
    np.testing.assert_allclose(on.weighted_sum(X, G, np.ones(5)), st.S_id, rtol=1e-12, atol=1e-12)
    # a unit weight vector picks one per-example gradient
    ii, jj = np.meshgrid(np.arange(6), np.arange(4), indexing="ij")
    M = oracle.per_example_at(X, G, ii.ravel(), jj.ravel()).reshape(5, 6, 4)
    for k in range(5):
        e = np.zeros(5); e[k] = 1.0
        np.testing.assert_allclose(on.weighted_sum(X, G, e), M[k], rtol=1e-12, atol=1e-12)
    # linear in the weights
    w1, w2 = np.random.default_rng(4).standard_normal((2, 5))
    np.testing.assert_allclose(on.weighted_sum(X, G, 2 * w1 - w2), 2 * on.weighted_sum(X, G, w1) - on.weighted_sum(X, G, w2), rtol=1e-10, atol=1e-12)
    # clipping: every clipped gradient has norm <= c, examples already inside the ball are untouched
    N = on.example_norms(X, G)
    c = float(np.sqrt(np.median(N)))
    w = on.clip_weights(N, c)
    assert ((w * np.sqrt(N)) <= c * (1 + 1e-12)).all() and (w[np.sqrt(N) <= c] == 1.0).all() and (w < 1).any()
    np.testing.assert_allclose(on.weighted_sum(X, G, w), sum(w[b] * M[b] for b in range(5)), rtol=1e-12, atol=1e-12)


def test_all_ones_closed_form_and_integer_brute_force():
    # all ones: M_b = T everywhere, N_b = din*dout*T^2; N_bl = din*dout
    X, G = np.ones((3, 5, 4), dtype=np.float32), np.ones((3, 5, 6), dtype=np.float32)
    assert np.array_equal(on.example_norms(X, G), np.full(3, 4 * 6 * 25.0))
    assert np.array_equal(on.token_norms(X, G), np.full((3, 5), 24.0))
    r = np.random.default_rng(5)
    X = r.integers(-2, 3, size=(2, 3, 3)).astype(np.float32)
    G = r.integers(-2, 3, size=(2, 3, 2)).astype(np.float32)
    for b in range(2):
        tot = 0
        for i in range(3):
            for j in range(2):
                m = sum(int(X[b, t, i]) * int(G[b, t, j]) for t in range(3))
                tot += m * m
        assert on.example_norms(X, G)[b] == tot


def test_power_statistic():
    X, G = _rand(5, 7, 6, 4, 8)
    st = oracle.stat(X, G)
    # alpha = 2 is the square statistic; B = 1, alpha = 1 is |S_id|
    np.testing.assert_allclose(on.power_stat(X, G, 2.0), st.S_sq, rtol=1e-12)
    np.testing.assert_allclose(on.power_stat(X[:1], G[:1], 1.0), np.abs(oracle.stat(X[:1], G[:1]).S_id), rtol=1e-12)
    # T = 1: gradients are rank one and the power factorises (Sec. 2.3): (|X|^a)^T (|G|^a)
    X1, G1 = _rand(6, 1, 5, 3, 9)
    a = 1.5
    fact = (np.abs(X1.astype(np.float64)) ** a).reshape(6, 5).T @ (np.abs(G1.astype(np.float64)) ** a).reshape(6, 3)
    np.testing.assert_allclose(on.power_stat(X1, G1, a), fact, rtol=1e-12)
    # scaling one example's cotangents by c multiplies its contribution by |c|^alpha (c a power of two: exact in fp32)
    G2 = G.copy(); G2[2] *= -4.0
    ii, jj = np.meshgrid(np.arange(6), np.arange(4), indexing="ij")
    M2 = np.abs(oracle.per_example_at(X, G, ii.ravel(), jj.ravel()).reshape(5, 6, 4)[2])
    np.testing.assert_allclose(on.power_stat(X, G2, a) - on.power_stat(X, G, a), (4.0 ** a - 1.0) * M2 ** a, rtol=1e-9, atol=1e-12)


def test_clip_weights_over_layers_is_per_example_norm_clipping_of_the_whole_model():
    """Two dense layers: clipping every example's whole gradient (both layers together) to norm c with the library
    routine, then summing over examples, equals the weighted sums with the weights of clip_weights_over_layers."""
    import torch
    B = 6
    X1, G1 = _rand(B, 7, 6, 4, 11)
    X2, G2 = _rand(B, 7, 5, 3, 12)
    X2 = X2 * np.linspace(0.2, 3.0, B, dtype=np.float32)[:, None, None]          # spread the norms around the threshold
    N = np.stack([on.example_norms(X1, G1), on.example_norms(X2, G2)])
    c = float(np.sqrt(np.median(N.sum(axis=0))))
    w = on.clip_weights_over_layers(N, c)
    assert (w < 1).any() and (w == 1).any()
    want1, want2 = np.zeros((6, 4)), np.zeros((5, 3))
    for b in range(B):
        p1 = torch.nn.Parameter(torch.zeros(6, 4, dtype=torch.float64))
        p2 = torch.nn.Parameter(torch.zeros(5, 3, dtype=torch.float64))
        p1.grad = torch.from_numpy(X1[b].astype(np.float64).T @ G1[b].astype(np.float64))
        p2.grad = torch.from_numpy(X2[b].astype(np.float64).T @ G2[b].astype(np.float64))
        torch.nn.utils.clip_grad_norm_([p1, p2], c)
        want1 += p1.grad.numpy()
        want2 += p2.grad.numpy()
    # the library routine divides by (norm + 1e-6): agreement to that guard
    np.testing.assert_allclose(on.weighted_sum(X1, G1, w), want1, rtol=1e-5, atol=1e-9)
    np.testing.assert_allclose(on.weighted_sum(X2, G2, w), want2, rtol=1e-5, atol=1e-9)
    # one layer: the single-layer rule; a zero gradient is left alone
    np.testing.assert_allclose(on.clip_weights_over_layers(N[:1], c), on.clip_weights(N[0], c), rtol=1e-15)
    assert np.array_equal(on.clip_weights_over_layers(np.zeros((3, 2)), 1.0), np.ones(2))
