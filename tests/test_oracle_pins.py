"""Pins of the fp64 CPU oracle against things other than itself.

Every check here fixes the oracle to the paper's worked example, a closed form,
an algebraic identity stated in the paper, a library routine on a special case,
or exact integer brute force -- chosen so that a dropped term, a wrong sign or
index, or a transposed operand fails at least one of them.  No GPU needed.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si


def _inputs(B, T, din, dout, dtype="bf16", seed=0, **kw):
    X, G = si.custom(B, T, din, dout, dtype=dtype, seed=seed, **kw)
    return si.widen(X), si.widen(G)


def _einsum_M(X, G):
    """Per-example gradients through a library contraction (Sec. 2.3: BLD,BLF->BDF)."""
    return np.einsum("bti,btj->bij", X.astype(np.float64), G.astype(np.float64))


# ----------------------------------------------------------------------------- worked example

def test_worked_example_all_ones(golden_dir):
    """App. A, first listing: B=10, d=4, all ones => avg_sq_grads = ones(4,4)."""
    vals = {}
    with open(os.path.join(golden_dir, "all_ones_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = float(v)
    B, d = int(vals["B"]), int(vals["d"])
    X = np.ones((B, 1, d), dtype=np.float32)
    G = np.ones((B, 1, d), dtype=np.float32)
    st = oracle.stat(X, G)
    assert np.array_equal(st.S_id, np.full((d, d), vals["S_id"]))
    assert np.array_equal(st.S_sq, np.full((d, d), vals["S_sq"]))
    assert np.array_equal(st.S_sign, np.full((d, d), vals["S_sign"]))
    assert np.array_equal(oracle.token_sq(X, G), np.full((d, d), vals["S_tok"]))
    assert np.array_equal(st.S_sq / B, np.full((d, d), vals["avg_sq_grads"]))


# ----------------------------------------------------------------------------- S_id

@pytest.mark.parametrize("shape", [(3, 5, 7, 11), (4, 16, 64, 64), (2, 33, 40, 24)])
def test_identity_is_the_batch_gradient(shape):
    """phi = identity gives the ordinary weight gradient X_flat^T G_flat (K = B*T)."""
    B, T, din, dout = shape
    X, G = _inputs(*shape, dtype="f32", seed=1)
    ref = X.reshape(B * T, din).astype(np.float64).T @ G.reshape(B * T, dout).astype(np.float64)
    st = oracle.stat(X, G)
    assert st.S_id.shape == (din, dout)
    np.testing.assert_allclose(st.S_id, ref, rtol=1e-12, atol=1e-12 * np.abs(ref).max())


# ----------------------------------------------------------------------------- library contraction

@pytest.mark.parametrize("shape", [(3, 5, 7, 11), (5, 8, 16, 9), (1, 4, 3, 2)])
def test_all_statistics_against_einsum(shape):
    """Small shapes: materialise M with a library einsum, apply phi with numpy."""
    X, G = _inputs(*shape, dtype="bf16", seed=2)
    M = _einsum_M(X, G)
    st = oracle.stat(X, G)
    scale = np.abs(M).max()
    np.testing.assert_allclose(st.S_id, M.sum(0), rtol=0, atol=1e-12 * scale)
    np.testing.assert_allclose(st.S_sq, (M * M).sum(0), rtol=1e-12)
    assert np.array_equal(st.S_sign, np.sign(M).sum(0))
    np.testing.assert_allclose(st.maxabs, np.abs(M).max(axis=(1, 2)), rtol=1e-13)
    np.testing.assert_allclose(st.normsq, (M * M).sum(axis=(1, 2)), rtol=1e-12)


def test_long_double_brute_force_config1():
    """Config-1 shape, a different loop order and extended precision."""
    X, G = si.make("c1_tiny", seed=0)
    X, G = si.widen(X), si.widen(G)
    B, T, din, dout = 4, 16, 64, 64
    Xl, Gl = X.astype(np.longdouble), G.astype(np.longdouble)
    S_id = np.zeros((din, dout), dtype=np.longdouble)
    S_sq = np.zeros((din, dout), dtype=np.longdouble)
    S_sg = np.zeros((din, dout), dtype=np.longdouble)
    for b in range(B):
        M = np.zeros((din, dout), dtype=np.longdouble)
        for t in reversed(range(T)):                   # reversed t, outer-product order
            M += np.outer(Xl[b, t], Gl[b, t])
        S_id += M
        S_sq += M * M
        S_sg += np.sign(M)
    st = oracle.stat(X, G)
    np.testing.assert_allclose(st.S_id, S_id.astype(np.float64), rtol=0, atol=1e-13 * 50)
    np.testing.assert_allclose(st.S_sq, S_sq.astype(np.float64), rtol=1e-13)
    assert np.array_equal(st.S_sign, S_sg.astype(np.float64))


# ----------------------------------------------------------------------------- T = 1 factorisation

def test_T1_square_factorises():
    """Sec. 2.3, MLP dense layer: sum_b (h_b l_b^T)^2 = (H o H)^T (L o L)."""
    X, G = _inputs(9, 1, 12, 7, dtype="bf16", seed=3)
    H, L = X[:, 0].astype(np.float64), G[:, 0].astype(np.float64)
    st = oracle.stat(X, G)
    np.testing.assert_allclose(st.S_sq, (H * H).T @ (L * L), rtol=1e-13)
    np.testing.assert_allclose(oracle.token_sq(X, G), st.S_sq, rtol=1e-13)


def test_T1_sign_factorises():
    """Sec. 2.3: sign is factorable, so for rank-one gradients S_sign = sign(H)^T sign(L)."""
    X, G = _inputs(9, 1, 12, 7, dtype="bf16", seed=4)
    X[0, 0, 3] = 0.0                                   # a zero row: sgn(0) = 0 must be counted as 0
    H, L = X[:, 0].astype(np.float64), G[:, 0].astype(np.float64)
    st = oracle.stat(X, G)
    assert np.array_equal(st.S_sign, np.sign(H).T @ np.sign(L))


# ----------------------------------------------------------------------------- B = 1

def test_B1_reductions():
    X, G = _inputs(1, 6, 10, 13, dtype="bf16", seed=5)
    st = oracle.stat(X, G)
    np.testing.assert_allclose(st.S_sq, st.S_id ** 2, rtol=1e-13)
    assert np.array_equal(st.S_sign, np.sign(st.S_id))


# ----------------------------------------------------------------------------- ghost norm

def test_ghost_norm_gram_route():
    """||M_b||_F^2 = <X_b X_b^T, G_b G_b^T>: a route that never forms M_b (Sec. 2.3 remark)."""
    B, T, din, dout = 4, 9, 14, 6
    X, G = _inputs(B, T, din, dout, dtype="bf16", seed=6)
    st = oracle.stat(X, G)
    Xd, Gd = X.astype(np.float64), G.astype(np.float64)
    N = np.array([np.sum((Xd[b] @ Xd[b].T) * (Gd[b] @ Gd[b].T)) for b in range(B)])
    np.testing.assert_allclose(st.normsq, N, rtol=1e-12)
    np.testing.assert_allclose(st.S_sq.sum(), N.sum(), rtol=1e-12)


# ----------------------------------------------------------------------------- inequalities / structure

def test_cauchy_schwarz_and_parity():
    """nu_micro >= nu_adam elementwise (variance estimate >= 0, Sec. 3.2); |S_sign| <= B, same parity as B."""
    B = 7
    X, G = _inputs(B, 5, 20, 17, dtype="f32", seed=7)
    st = oracle.stat(X, G)
    assert np.all(st.S_sq / B >= (st.S_id / B) ** 2 - 1e-12 * st.S_sq.max())
    assert np.all(st.S_sq > 0)
    assert np.all(np.abs(st.S_sign) <= B)
    M = _einsum_M(X, G)
    nz = np.all(M != 0, axis=0)
    assert np.all((st.S_sign[nz].astype(np.int64) - B) % 2 == 0)


def test_scaling_and_flip_laws():
    """G_b -> c_b G_b scales example b's square by c_b^2; negative c_b flips its sign, positive leaves it."""
    B, T, din, dout = 5, 4, 8, 6
    X, G = _inputs(B, T, din, dout, dtype="f32", seed=8)
    c = np.array([2.0, -0.5, 1.0, -4.0, 0.25], dtype=np.float32)   # powers of two: exact rescale
    Gs = G * c[:, None, None]
    M = _einsum_M(X, G)
    st = oracle.stat(X, Gs)
    np.testing.assert_allclose(st.S_sq, ((c[:, None, None].astype(np.float64) ** 2) * M * M).sum(0), rtol=1e-12)
    assert np.array_equal(st.S_sign, (np.sign(c)[:, None, None] * np.sign(M)).sum(0))
    np.testing.assert_allclose(st.S_id, (c[:, None, None] * M).sum(0), rtol=0, atol=1e-12 * np.abs(M).max() * 4)


def test_permutation_invariance():
    """Independent of within-batch indexing (Sec. 3.1) and of token order inside an example."""
    B, T, din, dout = 6, 7, 9, 5
    X, G = _inputs(B, T, din, dout, dtype="bf16", seed=9)
    rng = np.random.default_rng(0)
    pb = rng.permutation(B)
    st0 = oracle.stat(X, G)
    st1 = oracle.stat(X[pb], G[pb])
    np.testing.assert_allclose(st1.S_sq, st0.S_sq, rtol=1e-12)
    assert np.array_equal(st1.S_sign, st0.S_sign)
    X2, G2 = X.copy(), G.copy()
    for b in range(B):
        pt = rng.permutation(T)
        X2[b], G2[b] = X[b][pt], G[b][pt]
    st2 = oracle.stat(X2, G2)
    np.testing.assert_allclose(st2.S_sq, st0.S_sq, rtol=1e-12)
    np.testing.assert_allclose(st2.S_id, st0.S_id, rtol=0, atol=1e-12 * np.abs(st0.S_id).max())
    # permuting tokens of X only must change the result (guards against a t-independent bug)
    X3 = X.copy()
    X3[0] = X[0][::-1]
    assert not np.allclose(oracle.stat(X3, G).S_sq, st0.S_sq)


def test_second_moment_statistics():
    """iid zero-mean inputs: E[M_b[i,j]^2] = T sx^2 sg^2, so mean(S_sq) ~ B T sx^2 sg^2 (Eq. basic_nu_averages with mu = 0)."""
    B, T, din, dout = 8, 32, 48, 40
    X, G = _inputs(B, T, din, dout, dtype="f32", seed=10, g_std=0.5)
    st = oracle.stat(X, G)
    expect = B * T * 1.0 * 0.25
    assert abs(st.S_sq.mean() / expect - 1.0) < 0.05
    assert abs(oracle.token_sq(X, G).mean() / expect - 1.0) < 0.05
    assert abs(st.S_sign.mean()) < 0.2                      # symmetric inputs: signs cancel on average


# ----------------------------------------------------------------------------- exact integer brute force

def test_integer_brute_force_pure_python():
    """Tiny integer inputs, exact Python-int arithmetic, four nested loops."""
    B, T, din, dout = 3, 4, 5, 6
    X, G = si.integer_valued(B, T, din, dout, dtype="bf16", seed=11)
    Xn, Gn = si.widen(X), si.widen(G)
    Xi, Gi = Xn.astype(int).tolist(), Gn.astype(int).tolist()
    S_id = [[0] * dout for _ in range(din)]
    S_sq = [[0] * dout for _ in range(din)]
    S_sg = [[0] * dout for _ in range(din)]
    S_tk = [[0] * dout for _ in range(din)]
    for b, i, j in itertools.product(range(B), range(din), range(dout)):
        m = 0
        for t in range(T):
            m += Xi[b][t][i] * Gi[b][t][j]
            S_tk[i][j] += Xi[b][t][i] ** 2 * Gi[b][t][j] ** 2
        S_id[i][j] += m
        S_sq[i][j] += m * m
        S_sg[i][j] += (m > 0) - (m < 0)
    st = oracle.stat(Xn, Gn)
    assert np.array_equal(st.S_id, np.array(S_id, dtype=np.float64))
    assert np.array_equal(st.S_sq, np.array(S_sq, dtype=np.float64))
    assert np.array_equal(st.S_sign, np.array(S_sg, dtype=np.float64))
    assert np.array_equal(oracle.token_sq(Xn, Gn), np.array(S_tk, dtype=np.float64))


# ----------------------------------------------------------------------------- per-token square

def test_token_sq_pins():
    B, T, din, dout = 4, 6, 10, 7
    X, G = _inputs(B, T, din, dout, dtype="bf16", seed=12)
    S = oracle.token_sq(X, G)
    Xd, Gd = X.astype(np.float64), G.astype(np.float64)
    # (i) identity statistic of the squared inputs (squares of bf16 values are exact in fp32)
    st = oracle.stat((Xd * Xd).astype(np.float32), (Gd * Gd).astype(np.float32))
    np.testing.assert_allclose(S, st.S_id, rtol=1e-13)
    # (ii) rank-one sum over tokens
    ref = np.zeros((din, dout))
    for b in range(B):
        for t in range(T):
            ref += np.outer(Xd[b, t] ** 2, Gd[b, t] ** 2)
    np.testing.assert_allclose(S, ref, rtol=1e-13)
    # (iii) total = sum of per-token norm products (per-token norms remark, Sec. 2.3)
    np.testing.assert_allclose(S.sum(), ((Xd ** 2).sum(-1) * (Gd ** 2).sum(-1)).sum(), rtol=1e-12)
    # it is not the per-example square when T > 1
    assert not np.allclose(S, oracle.stat(X, G).S_sq)


# ----------------------------------------------------------------------------- sampled-entry routes

def test_sampled_routes_match_full():
    B, T, din, dout = 5, 9, 21, 17
    X, G = _inputs(B, T, din, dout, dtype="bf16", seed=13)
    M = _einsum_M(X, G)
    rng = np.random.default_rng(1)
    ii, jj = rng.integers(0, din, 50), rng.integers(0, dout, 50)
    Ms = oracle.per_example_at(X, G, ii, jj)
    np.testing.assert_allclose(Ms, M[:, ii, jj], rtol=0, atol=1e-12 * np.abs(M).max())
    full = oracle.stat(X, G)
    part = oracle.stat_at(X, G, ii, jj)
    np.testing.assert_allclose(part.S_sq, full.S_sq[ii, jj], rtol=1e-12)
    assert np.array_equal(part.S_sign, full.S_sign[ii, jj])
    assert np.all(part.maxabs <= full.maxabs + 1e-12)
    np.testing.assert_allclose(oracle.token_sq_at(X, G, ii, jj), oracle.token_sq(X, G)[ii, jj], rtol=1e-12)


def test_ambiguity_mask():
    """amb counts examples whose |M_b[i,j]| is below 1e-6 * max|M_b|; an exact zero is ambiguous too."""
    # B=2, T=2, din=2, dout=2; example 0 has M[0,0] = 2^-24 (tiny), M[1,1] = 1; example 1 is all ones.
    X = np.zeros((2, 2, 2), dtype=np.float32)
    G = np.zeros((2, 2, 2), dtype=np.float32)
    X[0, 0] = [2.0 ** -24, 0.0]
    G[0, 0] = [1.0, 0.0]
    X[0, 1] = [0.0, 1.0]
    G[0, 1] = [0.0, 1.0]
    X[1] = 1.0
    G[1] = 0.5
    st = oracle.stat(X, G)
    assert st.maxabs.tolist() == [1.0, 1.0]
    assert st.amb.tolist() == [[1, 1], [1, 0]]             # example 0: tiny, 0, 0 are inside the band
    assert st.S_sign.tolist() == [[2.0, 1.0], [1.0, 2.0]]


def test_bad_arguments_raise():
    X, G = _inputs(2, 3, 4, 5)
    with pytest.raises(ValueError):
        oracle.stat(X, G[:, :2])
    with pytest.raises(ValueError):
        oracle.stat(X[:0], G[:0])
    with pytest.raises(RuntimeError):
        oracle.per_example_at(X, G, np.array([4]), np.array([0]))
