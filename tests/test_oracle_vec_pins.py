"""Pins of the vector-parameter oracle (offsets and elementwise scales, App. B "Affine operations") against things
other than itself: the already pinned matrix oracle, library reductions, closed forms and brute force."""
import numpy as np

import oracle
from oracle import vec as ov


def _rand(B, T, d, seed):
    r = np.random.default_rng(seed)
    return r.standard_normal((B, T, d)).astype(np.float32), r.standard_normal((B, T, d)).astype(np.float32)


def test_offset_is_the_matrix_statistic_with_a_column_of_ones():
    """An offset is a weight row fed by a constant 1 (the paper's cast of affine maps as contractions): the matrix
    oracle on X = ones[B,T,1] must give the same three statistics."""
    A, _ = _rand(5, 13, 24, 0)
    st = oracle.stat(np.ones((5, 13, 1), dtype=np.float32), A)
    vs = ov.vec_stat(A)
    np.testing.assert_allclose(vs.s_id, st.S_id[0], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(vs.s_sq, st.S_sq[0], rtol=1e-12, atol=1e-12)
    assert np.array_equal(vs.s_sign, st.S_sign[0])
    assert np.array_equal(vs.amb, st.amb[0])


def test_scale_is_the_diagonal_of_the_matrix_statistic():
    """v_b[j] = sum_t A[b,t,j] C[b,t,j] is the diagonal of C_b^T A_b."""
    A, C = _rand(4, 9, 12, 1)
    st = oracle.stat(C, A)
    vs = ov.vec_stat(A, C)
    np.testing.assert_allclose(vs.s_id, np.diag(st.S_id), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(vs.s_sq, np.diag(st.S_sq), rtol=1e-12, atol=1e-12)
    assert np.array_equal(vs.s_sign, np.diag(st.S_sign))


def test_against_library_reductions():
    A, C = _rand(6, 20, 17, 2)
    v = np.einsum("btj,btj->bj", A.astype(np.float64), C.astype(np.float64))
    vs = ov.vec_stat(A, C)
    np.testing.assert_allclose(vs.v, v, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(vs.s_id, v.sum(0), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(vs.s_sq, (v * v).sum(0), rtol=1e-12)
    assert np.array_equal(vs.s_sign, np.sign(v).sum(0))
    # identity = the ordinary bias gradient of the flattened batch
    np.testing.assert_allclose(ov.vec_stat(A).s_id, A.astype(np.float64).reshape(-1, 17).sum(0), rtol=1e-12, atol=1e-12)


def test_closed_forms_and_special_cases():
    # all ones: every example's offset gradient is T, so mean square = T^2, sign count = B
    vs = ov.vec_stat(np.ones((10, 7, 4), dtype=np.float32))
    assert np.array_equal(vs.s_id, np.full(4, 70.0)) and np.array_equal(vs.s_sq, np.full(4, 490.0))
    assert np.array_equal(vs.s_sign, np.full(4, 10.0)) and not vs.amb.any()
    # T = 1: the square statistic factorises into sum_b A^2 C^2 (Sec. 2.3, rank-one case)
    A, C = _rand(8, 1, 5, 3)
    np.testing.assert_allclose(ov.vec_stat(A, C).s_sq, ((A.astype(np.float64) ** 2) * (C.astype(np.float64) ** 2)).sum((0, 1)), rtol=1e-12)
    # B = 1: square of the sum, sign of the sum
    A, C = _rand(1, 11, 6, 4)
    vs = ov.vec_stat(A, C)
    np.testing.assert_allclose(vs.s_sq, vs.s_id ** 2, rtol=1e-12)
    assert np.array_equal(vs.s_sign, np.sign(vs.s_id))
    # Cauchy-Schwarz: nu_micro >= nu_adam
    A, C = _rand(9, 5, 7, 5)
    vs = ov.vec_stat(A, C)
    assert (vs.s_sq * 9 >= vs.s_id ** 2 - 1e-9).all()


def test_laws_and_the_ambiguity_mask():
    A, C = _rand(5, 6, 8, 6)
    base = ov.vec_stat(A, C)
    perm = np.array([2, 0, 4, 1, 3])
    p = ov.vec_stat(A[perm], C[perm])
    np.testing.assert_allclose(p.s_sq, base.s_sq, rtol=1e-12)
    assert np.array_equal(p.s_sign, base.s_sign)
    A2 = A.copy()
    A2[3] *= -1                        # flipping one example's cotangents flips its contribution
    f = ov.vec_stat(A2, C)
    np.testing.assert_allclose(f.s_id, base.s_id - 2 * base.v[3], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(f.s_sq, base.s_sq, rtol=1e-12)
    assert np.array_equal(f.s_sign, base.s_sign - 2 * np.sign(base.v[3]))
    # an exactly cancelling column is a zero (sgn 0 = 0) and counts as ambiguous for that example
    Z = np.zeros((2, 2, 3), dtype=np.float32)
    Z[0, :, 0] = [1.0, -1.0]
    Z[0, :, 1] = [2.0, 1.0]
    Z[1, :, :] = 1.0
    z = ov.vec_stat(Z)
    assert np.array_equal(z.s_sign, [1.0, 2.0, 1.0]) and np.array_equal(z.amb, [1, 0, 1])


def test_exact_integer_brute_force():
    r = np.random.default_rng(7)
    A = r.integers(-3, 4, size=(4, 5, 6)).astype(np.float32)
    C = r.integers(-3, 4, size=(4, 5, 6)).astype(np.float32)
    vs = ov.vec_stat(A, C)
    for j in range(6):
        vb = [sum(int(A[b, t, j]) * int(C[b, t, j]) for t in range(5)) for b in range(4)]
        assert vs.s_id[j] == sum(vb) and vs.s_sq[j] == sum(x * x for x in vb)
        assert vs.s_sign[j] == sum((x > 0) - (x < 0) for x in vb)
