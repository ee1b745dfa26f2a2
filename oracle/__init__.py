"""fp64 CPU oracle for the per-example gradient statistics and the optimizer updates.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may.  It shares no code with the HIP library.

``stat`` / ``token_sq`` and their ``*_at`` variants call the plain C loops in
``pex_oracle.c`` (the "memory intensive" definition of Sec. 2.1 applied to the
sequence dense layer of Sec. 2.3).  ``update.py`` holds the elementwise fp64
optimizer steps of Algorithm 1 and Sec. 3.1.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pex_oracle.c")
_LIB = os.path.join(_HERE, "libpex_oracle.so")

SIGN_BAND = 1e-6  # same constant as PEX_ORACLE_SIGN_BAND in pex_oracle.c


def build(force: bool = False) -> str:
    """Compile pex_oracle.c with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.pex_oracle_stat.argtypes = [p, p, i64, i64, i64, i64, p, p, p, p, p, p]
        lib.pex_oracle_stat.restype = ctypes.c_int
        lib.pex_oracle_per_example_at.argtypes = [p, p, i64, i64, i64, i64, i64, p, p, p]
        lib.pex_oracle_per_example_at.restype = ctypes.c_int
        lib.pex_oracle_token_sq.argtypes = [p, p, i64, i64, i64, i64, p]
        lib.pex_oracle_token_sq.restype = ctypes.c_int
        lib.pex_oracle_token_sq_at.argtypes = [p, p, i64, i64, i64, i64, i64, p, p, p]
        lib.pex_oracle_token_sq_at.restype = ctypes.c_int
        lib.pex_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the C loops will use (OpenMP default for this process)."""
    return int(_load().pex_oracle_num_threads())


def _f32(a, shape_len):
    a = np.ascontiguousarray(np.asarray(a), dtype=np.float32)
    if a.ndim != shape_len:
        raise ValueError(f"expected a {shape_len}-d array, got shape {a.shape}")
    return a


def _check(X, G):
    X, G = _f32(X, 3), _f32(G, 3)
    if X.shape[:2] != G.shape[:2]:
        raise ValueError(f"X{X.shape} and G{G.shape} disagree on (B,T)")
    if 0 in X.shape or 0 in G.shape:
        raise ValueError("empty inputs have no statistic")
    return X, G


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


@dataclass
class Stat:
    """All statistics of one (X, G) pair.  Arrays are [din, dout] fp64 unless noted."""
    S_id: np.ndarray      # sum_b M_b
    S_sq: np.ndarray      # sum_b M_b**2
    S_sign: np.ndarray    # sum_b sgn(M_b), integer valued
    amb: np.ndarray       # int32: how many examples are sign-ambiguous at (i, j)
    maxabs: np.ndarray    # [B] max_ij |M_b|
    normsq: np.ndarray    # [B] ||M_b||_F^2


def stat(X, G) -> Stat:
    """Materialise each per-example gradient M_b = X_b^T G_b and reduce (Sec. 2.3)."""
    X, G = _check(X, G)
    B, T, din = X.shape
    dout = G.shape[2]
    out = Stat(np.empty((din, dout)), np.empty((din, dout)), np.empty((din, dout)),
               np.empty((din, dout), dtype=np.int32), np.empty(B), np.empty(B))
    rc = _load().pex_oracle_stat(_ptr(X), _ptr(G), B, T, din, dout, _ptr(out.S_id), _ptr(out.S_sq),
                                 _ptr(out.S_sign), _ptr(out.amb), _ptr(out.maxabs), _ptr(out.normsq))
    if rc != 0:
        raise RuntimeError(f"pex_oracle_stat failed with code {rc}")
    return out


def per_example_at(X, G, ii, jj) -> np.ndarray:
    """M[b, k] = (X_b^T G_b)[ii[k], jj[k]] for sampled output positions; fp64 [B, n]."""
    X, G = _check(X, G)
    B, T, din = X.shape
    dout = G.shape[2]
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    if ii.shape != jj.shape or ii.ndim != 1:
        raise ValueError("ii and jj must be 1-d and of equal length")
    M = np.empty((B, ii.size))
    rc = _load().pex_oracle_per_example_at(_ptr(X), _ptr(G), B, T, din, dout, ii.size, _ptr(ii),
                                           _ptr(jj), _ptr(M))
    if rc != 0:
        raise RuntimeError(f"pex_oracle_per_example_at failed with code {rc}")
    return M


def stat_at(X, G, ii, jj) -> Stat:
    """The statistics at sampled positions, from per-example values M[b, k].

    ``maxabs`` is the max over the *sampled* entries only, a lower bound of the
    true per-example max, so the ambiguity band it gives is narrower (stricter)
    than the one the full oracle would give.
    """
    M = per_example_at(X, G, ii, jj)
    mx = np.abs(M).max(axis=1)
    amb = (np.abs(M) < SIGN_BAND * mx[:, None]).sum(axis=0).astype(np.int32)
    sgn = (M > 0).astype(np.float64) - (M < 0).astype(np.float64)
    return Stat(M.sum(axis=0), (M * M).sum(axis=0), sgn.sum(axis=0), amb, mx, (M * M).sum(axis=1))


def token_sq(X, G) -> np.ndarray:
    """S_tok = sum_{b,t} (x_bt o x_bt)(g_bt o g_bt)^T (Sec. 2.3, per-token second moments)."""
    X, G = _check(X, G)
    B, T, din = X.shape
    dout = G.shape[2]
    S = np.empty((din, dout))
    rc = _load().pex_oracle_token_sq(_ptr(X), _ptr(G), B, T, din, dout, _ptr(S))
    if rc != 0:
        raise RuntimeError(f"pex_oracle_token_sq failed with code {rc}")
    return S


def token_sq_at(X, G, ii, jj) -> np.ndarray:
    """S_tok at sampled positions; fp64 [n]."""
    X, G = _check(X, G)
    B, T, din = X.shape
    dout = G.shape[2]
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    out = np.empty(ii.size)
    rc = _load().pex_oracle_token_sq_at(_ptr(X), _ptr(G), B, T, din, dout, ii.size, _ptr(ii),
                                        _ptr(jj), _ptr(out))
    if rc != 0:
        raise RuntimeError(f"pex_oracle_token_sq_at failed with code {rc}")
    return out
