"""fp64 CPU oracle for per-example statistics of vector parameters (offsets, elementwise scales).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``): nothing in the product package imports this.

An offset added on both the batch and the length axis is a tensor contraction of the cotangents with a vector of
ones (App. B, "Affine operations"): its per-example gradient is the reduction over the length axis,
``v_b[j] = sum_t A[b,t,j]``; an elementwise scale applied to an activation ``C`` has
``v_b[j] = sum_t A[b,t,j] * C[b,t,j]``.  The statistic is then, exactly as for weight matrices (Sec. 2.3),
``s = sum_b phi(v_b)`` for phi in {identity, square, sign}.  Plain loops over the examples in fp64, no blocking.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SIGN_BAND = 1e-6   # an entry with |v_b[j]| below SIGN_BAND * max_j |v_b| is sign-ambiguous for example b


@dataclass
class VecStat:
    """Statistics of one vector parameter; arrays are [d] fp64 unless noted."""
    s_id: np.ndarray     # sum_b v_b
    s_sq: np.ndarray     # sum_b v_b**2
    s_sign: np.ndarray   # sum_b sgn(v_b), integer valued, sgn(0) = 0
    amb: np.ndarray      # int32: how many examples are sign-ambiguous at j
    v: np.ndarray        # [B, d] the per-example gradients themselves (small: B * d)


def vec_stat(A, C=None) -> VecStat:
    """``A`` [B,T,d] cotangents, ``C`` [B,T,d] activations or None (offset: a vector of ones)."""
    A = np.asarray(A)
    if A.ndim != 3 or 0 in A.shape:
        raise ValueError(f"expected a non-empty [B,T,d] array, got {A.shape}")
    if C is not None:
        C = np.asarray(C)
        if C.shape != A.shape:
            raise ValueError(f"A{A.shape} and C{C.shape} differ")
    B, T, d = A.shape
    v = np.empty((B, d), dtype=np.float64)
    for b in range(B):
        a = A[b].astype(np.float64)
        if C is not None:
            a = a * C[b].astype(np.float64)
        acc = np.zeros(d, dtype=np.float64)
        for t in range(T):            # the reduction over the length axis, one token at a time
            acc += a[t]
        v[b] = acc
    s_id = np.zeros(d)
    s_sq = np.zeros(d)
    s_sign = np.zeros(d)
    amb = np.zeros(d, dtype=np.int32)
    for b in range(B):
        s_id += v[b]
        s_sq += v[b] * v[b]
        s_sign += (v[b] > 0).astype(np.float64) - (v[b] < 0).astype(np.float64)
        amb += (np.abs(v[b]) < SIGN_BAND * np.abs(v[b]).max()).astype(np.int32)
    return VecStat(s_id, s_sq, s_sign, amb, v)
