"""fp64 CPU oracle for per-example and per-token gradient norms and for per-example weighted sums (clipping).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``): nothing in the product package imports this.

* ``example_norms``: N_b = ||X_b^T G_b||_F^2, the squared norm of the per-example gradient of a dense sequence
  layer (the quantity of the "ghost clipping" remark of Sec. 2.3), by materialising M_b.
* ``token_norms``: N_bl = ||x_bl||^2 ||g_bl||^2, the per-sample per-token norm of Sec. 2.3 (the squared norm of the
  rank-one term x_bl g_bl^T).
* ``weighted_sum``: sum_b w_b X_b^T G_b, what a clipping nonlinearity phi(g_b) = min(1, c/||g_b||) g_b of Sec. 2.1
  needs once the norms are known.
Plain per-example loops; the library matmul is the step that forms M_b.
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    a = np.asarray(a, dtype=np.float64)
    if a.ndim != 3 or 0 in a.shape:
        raise ValueError(f"expected a non-empty [B,T,d] array, got {a.shape}")
    return a


def example_norms(X, G) -> np.ndarray:
    X, G = _f64(X), _f64(G)
    out = np.empty(X.shape[0])
    for b in range(X.shape[0]):
        M = X[b].T @ G[b]
        out[b] = (M * M).sum()
    return out


def token_norms(X, G) -> np.ndarray:
    X, G = _f64(X), _f64(G)
    B, T, _ = X.shape
    out = np.empty((B, T))
    for b in range(B):
        for t in range(T):
            out[b, t] = (X[b, t] * X[b, t]).sum() * (G[b, t] * G[b, t]).sum()
    return out


def weighted_sum(X, G, w) -> np.ndarray:
    X, G = _f64(X), _f64(G)
    w = np.asarray(w, dtype=np.float64)
    if w.shape != (X.shape[0],):
        raise ValueError("one weight per example")
    S = np.zeros((X.shape[2], G.shape[2]))
    for b in range(X.shape[0]):
        S += w[b] * (X[b].T @ G[b])
    return S


def power_stat(X, G, alpha: float) -> np.ndarray:
    """sum_b |X_b^T G_b|^alpha elementwise: the power nonlinearity phi(s) = s^alpha of Sec. 2.3 on a sequence layer."""
    X, G = _f64(X), _f64(G)
    S = np.zeros((X.shape[2], G.shape[2]))
    for b in range(X.shape[0]):
        S += np.abs(X[b].T @ G[b]) ** alpha
    return S


def clip_weights_over_layers(layer_norms_sq, c) -> np.ndarray:
    """Per-example clipping (the clip nonlinearity of Sec. 2.1) in a model of several layers: the gradient of example
    b is the concatenation of its per-layer gradients, so ||g_b||^2 is the sum over the layers of the per-layer
    squared norms (``layer_norms_sq`` is [layers, B]), and w_b = min(1, c / ||g_b||).  An example whose gradient
    is exactly zero keeps w_b = 1."""
    n = np.asarray(layer_norms_sq, dtype=np.float64)
    if n.ndim != 2:
        raise ValueError("expected [layers, B] squared norms")
    total = np.zeros(n.shape[1])
    for l in range(n.shape[0]):
        total = total + n[l]
    w = np.ones(n.shape[1])
    for b in range(n.shape[1]):
        norm = np.sqrt(total[b])
        if norm > c:
            w[b] = c / norm
    return w


def clip_weights(norms_sq, c) -> np.ndarray:
    """w_b = min(1, c / ||g_b||): the factor of the clipping nonlinearity for squared norms ``norms_sq``."""
    n = np.sqrt(np.asarray(norms_sq, dtype=np.float64))
    return np.minimum(1.0, c / np.maximum(n, 1e-300))
