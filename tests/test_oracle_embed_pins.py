"""Pins of the embedding-table oracle: the dense-layer oracle on one-hot inputs (an independent C loop nest),
closed forms for T = 1 and B = 1, brute force, symmetries.  No GPU needed."""
import numpy as np
import pytest

import oracle
import synth_inputs as si
from oracle import embed as oe


def _case(B, T, V, d, seed, pad=0.0):
    ids = si.token_ids(B, T, V, seed=seed, pad_fraction=pad).numpy()
    G = si.widen(si.custom(B, T, 8, d, dtype="bf16", seed=seed)[1])
    return ids, G


def test_equals_the_dense_layer_oracle_on_one_hot_inputs():
    """An embedding is a dense layer on one-hot rows (Sec. 2.3): all three statistics must agree with the dense oracle."""
    B, T, V, d = 5, 40, 23, 24
    ids, G = _case(B, T, V, d, 1, pad=0.1)
    X = np.zeros((B, T, V), dtype=np.float32)
    for b in range(B):
        for t in range(T):
            if ids[b, t] >= 0:
                X[b, t, ids[b, t]] = 1.0
    ref = oracle.stat(X, G)
    got = oe.embed_stat(ids, G, V)
    np.testing.assert_allclose(got.S_id, ref.S_id, rtol=1e-13, atol=1e-300)
    np.testing.assert_allclose(got.S_sq, ref.S_sq, rtol=1e-13, atol=1e-300)
    np.testing.assert_array_equal(got.S_sign, ref.S_sign)


def test_identity_is_the_ordinary_embedding_gradient():
    """S_id is what a library scatter-add over all B*T positions gives (numpy add.at)."""
    B, T, V, d = 4, 30, 50, 16
    ids, G = _case(B, T, V, d, 2)
    ref = np.zeros((V, d))
    np.add.at(ref, ids.reshape(-1), G.reshape(-1, d).astype(np.float64))
    np.testing.assert_allclose(oe.embed_stat(ids, G, V).S_id, ref, rtol=1e-13, atol=1e-300)


def test_one_token_per_example_factorises():
    """T = 1: M_b has one non-zero row, so S_sq[v] = sum over the examples holding v of G_b^2, S_sign likewise."""
    B, V, d = 60, 11, 8
    ids, G = _case(B, 1, V, d, 3)
    got = oe.embed_stat(ids, G, V)
    for v in range(V):
        rows = G[ids[:, 0] == v, 0, :].astype(np.float64)
        np.testing.assert_allclose(got.S_sq[v], (rows ** 2).sum(0), rtol=1e-13, atol=1e-300)
        np.testing.assert_array_equal(got.S_sign[v], np.sign(rows).sum(0))


def test_one_example_gives_square_and_sign_of_the_gradient():
    ids, G = _case(1, 64, 17, 8, 4)
    got = oe.embed_stat(ids, G, 17)
    np.testing.assert_allclose(got.S_sq, got.S_id ** 2, rtol=1e-13)
    np.testing.assert_array_equal(got.S_sign, np.sign(got.S_id))


def test_repeated_tokens_are_summed_before_phi_not_after():
    """Two positions of one example holding the same token with opposite cotangents cancel: the square statistic is 0
    there, while squaring per position (the per-token quantity) would not be."""
    ids = np.array([[3, 3, 1]])
    G = np.array([[[1.0, -2.0], [-1.0, 2.0], [0.5, 0.25]]])
    got = oe.embed_stat(ids, G, 5)
    assert np.all(got.S_sq[3] == 0) and np.all(got.S_sign[3] == 0)
    np.testing.assert_array_equal(got.S_sq[1], [0.25, 0.0625])
    # the same two positions in different examples do not cancel
    got2 = oe.embed_stat(np.array([[3], [3]]), np.array([[[1.0, -2.0]], [[-1.0, 2.0]]]), 5)
    np.testing.assert_array_equal(got2.S_sq[3], [2.0, 8.0])
    np.testing.assert_array_equal(got2.S_sign[3], [0.0, 0.0])
    np.testing.assert_array_equal(got2.S_id[3], [0.0, 0.0])


def test_symmetries_and_padding():
    B, T, V, d = 6, 25, 19, 8
    ids, G = _case(B, T, V, d, 5, pad=0.2)
    ref = oe.embed_stat(ids, G, V)
    perm_b = np.random.default_rng(0).permutation(B)
    perm_t = np.random.default_rng(1).permutation(T)
    a = oe.embed_stat(ids[perm_b][:, perm_t], G[perm_b][:, perm_t], V)
    np.testing.assert_allclose(a.S_sq, ref.S_sq, rtol=1e-12, atol=1e-300)
    np.testing.assert_array_equal(a.S_sign, ref.S_sign)
    # relabelling the vocabulary permutes the rows
    relabel = np.random.default_rng(2).permutation(V)
    ids2 = np.where(ids >= 0, relabel[np.clip(ids, 0, V - 1)], -1)
    c = oe.embed_stat(ids2, G, V)
    np.testing.assert_allclose(c.S_sq[relabel], ref.S_sq, rtol=1e-13, atol=1e-300)
    # padded positions contribute nothing: dropping them from G changes nothing
    G0 = G.copy()
    G0[ids < 0] = 123.0
    np.testing.assert_array_equal(oe.embed_stat(ids, G0, V).S_id, ref.S_id)
    # rows of absent tokens are zero, and ids >= V are ignored like padding
    absent = np.setdiff1d(np.arange(V), ids[ids >= 0])
    assert np.all(ref.S_sq[absent] == 0)
    np.testing.assert_array_equal(oe.embed_stat(np.where(ids < 0, V + 5, ids), G, V).S_sq, ref.S_sq)


def test_bounds_and_parity_of_the_sign_counts():
    B, T, V, d = 7, 12, 9, 8
    ids, G = _case(B, T, V, d, 6)
    got = oe.embed_stat(ids, G, V)
    present = np.stack([(ids == v).any(axis=1) for v in range(V)]).sum(axis=1)     # examples that contain token v
    assert np.all(np.abs(got.S_sign) <= present[:, None])
    assert np.all(got.S_sq * present[:, None] >= got.S_id ** 2 * (1 - 1e-12))      # Cauchy-Schwarz over the examples present
