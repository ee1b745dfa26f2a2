"""fp64 oracle of per-example gradient statistics of an embedding table.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

An embedding lookup h[b,t,:] = E[ids[b,t],:] is a dense layer applied to one-hot inputs, so the per-example gradient
of the table is M_b = onehot(ids_b)^T G_b (Sec. 2.3 with X one-hot): row v of M_b is the sum of the cotangents of the
positions of example b that hold token v, and rows of tokens that example b does not contain are zero.  The
statistics are S = sum_b phi(M_b) for phi = identity, square, sign (sgn(0) = 0), exactly as for a dense layer.
Positions whose id lies outside [0, V) (padding) contribute nothing.

Written as the definition: every M_b is materialised as a dense [V, d] array.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SIGN_BAND = 1e-6   # an entry with |M_b| below this fraction of max|M_b| is sign-ambiguous (same rule as the dense oracle)


@dataclass
class EmbedStat:
    S_id: np.ndarray      # [V, d]
    S_sq: np.ndarray
    S_sign: np.ndarray
    amb: np.ndarray       # [V, d] int32: examples that hold token v and whose entry is inside the ambiguity band


def embed_stat(ids, G, V: int) -> EmbedStat:
    ids = np.asarray(ids)
    G = np.asarray(G, dtype=np.float64)
    if ids.ndim != 2 or G.ndim != 3 or G.shape[:2] != ids.shape:
        raise ValueError("ids must be [B,T] and G [B,T,d]")
    B, T = ids.shape
    d = G.shape[2]
    out = EmbedStat(np.zeros((V, d)), np.zeros((V, d)), np.zeros((V, d)), np.zeros((V, d), dtype=np.int32))
    for b in range(B):
        M = np.zeros((V, d))
        present = np.zeros(V, dtype=bool)
        for t in range(T):
            v = int(ids[b, t])
            if 0 <= v < V:
                M[v] += G[b, t]
                present[v] = True
        mx = np.abs(M).max()
        out.S_id += M
        out.S_sq += M * M
        out.S_sign += (M > 0).astype(np.float64) - (M < 0).astype(np.float64)
        out.amb += ((np.abs(M) < SIGN_BAND * mx) & present[:, None]).astype(np.int32)
    return out
