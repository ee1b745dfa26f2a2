"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds none of the method's arithmetic: it only draws activations X,
cotangents G and optimizer state with the shapes and value structure of the
workloads (transformer dense layers; the 2048 x 8192 shape is the MLP layer of
the 1.2B model of App. D).  Both the HIP path and the CPU oracle are handed the
very same rounded payloads; neither imports the other.

Streams: X from seed*2, G from seed*2+1, per-token scale / mask from seed*2+2,
optimizer state from seed*2+3, token ids from seed*2+4.  All draws use a CPU ``torch.Generator`` so they
are identical on every machine.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    T: int
    din: int
    dout: int
    dtype: str            # "f32" or "bf16": storage type of X and G
    g_std: float = 1.0    # standard deviation of G before per-token scaling
    g_token: str = "none"  # "none" | "lognormal" (exp(N(0,1)) per token) | "sparse" (80% of tokens x 1e-3)


WORKLOADS = {
    "c1_tiny":        Workload("c1_tiny", 4, 16, 64, 64, "f32"),
    "c2_mlp_in":      Workload("c2_mlp_in", 32, 256, 512, 2048, "bf16", g_std=1e-2),
    "c3_gpt2_qkv":    Workload("c3_gpt2_qkv", 64, 1024, 768, 2304, "bf16", g_token="lognormal"),
    "c3_gpt2_proj":   Workload("c3_gpt2_proj", 64, 1024, 768, 768, "bf16", g_token="lognormal"),
    "c3_gpt2_fc":     Workload("c3_gpt2_fc", 64, 1024, 768, 3072, "bf16", g_token="lognormal"),
    "c3_gpt2_fcproj": Workload("c3_gpt2_fcproj", 64, 1024, 3072, 768, "bf16", g_token="lognormal"),
    "c4_1b_up":       Workload("c4_1b_up", 16, 2048, 2048, 8192, "bf16"),
    "c4_1b_down":     Workload("c4_1b_down", 16, 2048, 8192, 2048, "bf16"),
    "c5_long":        Workload("c5_long", 4, 8192, 4096, 4096, "bf16", g_token="sparse"),
}


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def _store(x: torch.Tensor, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return x.to(torch.bfloat16)       # round to nearest even
    if dtype == "f32":
        return x
    raise ValueError(f"unknown dtype {dtype}")


def token_scale(w: Workload, seed: int) -> torch.Tensor | None:
    """Per-token multiplier of G, shape [B, T, 1] fp32, or None."""
    if w.g_token == "none":
        return None
    g = _gen(seed * 2 + 2)
    if w.g_token == "lognormal":
        return torch.exp(torch.randn(w.B, w.T, 1, generator=g))
    if w.g_token == "sparse":
        u = torch.rand(w.B, w.T, 1, generator=g)
        return torch.where(u < 0.8, torch.full_like(u, 1e-3), torch.ones_like(u))
    raise ValueError(f"unknown token structure {w.g_token}")


def make(w: Workload | str, seed: int = 0):
    """Return (X[B,T,din], G[B,T,dout]) as CPU tensors in the workload's storage dtype."""
    if isinstance(w, str):
        w = WORKLOADS[w]
    gx, gg = _gen(seed * 2), _gen(seed * 2 + 1)
    scale = token_scale(w, seed)
    st = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    X = torch.empty(w.B, w.T, w.din, dtype=st)
    G = torch.empty(w.B, w.T, w.dout, dtype=st)
    for b in range(w.B):                      # per example, to bound the fp32 temporaries
        X[b] = _store(torch.randn(w.T, w.din, generator=gx), w.dtype)
        g = torch.randn(w.T, w.dout, generator=gg) * w.g_std
        if scale is not None:
            g = g * scale[b]
        G[b] = _store(g, w.dtype)
    return X, G


def custom(B: int, T: int, din: int, dout: int, dtype: str = "bf16", seed: int = 0,
           g_std: float = 1.0, g_token: str = "none"):
    """Gaussian inputs of an arbitrary shape (ragged tails, edge cases)."""
    return make(Workload("custom", B, T, din, dout, dtype, g_std, g_token), seed)


def integer_valued(B: int, T: int, din: int, dout: int, dtype: str = "bf16", seed: int = 0,
                   lo: int = -3, hi: int = 3):
    """Small-integer inputs: every product and partial sum is exact in bf16/fp32/fp64."""
    gx, gg = _gen(seed * 2), _gen(seed * 2 + 1)
    X = torch.randint(lo, hi + 1, (B, T, din), generator=gx).to(torch.float32)
    G = torch.randint(lo, hi + 1, (B, T, dout), generator=gg).to(torch.float32)
    return _store(X, dtype), _store(G, dtype)


def token_ids(B: int, T: int, V: int, seed: int = 0, exponent: float = 1.0, pad_fraction: float = 0.0):
    """Token ids [B, T] int64 with a Zipf-like rank-frequency law p(v) ~ 1/(v + 2.7)^exponent (id = frequency rank,
    the shape of natural-language token counts); a fraction of the positions can be set to the padding id -1."""
    g = _gen(seed * 2 + 4)
    p = 1.0 / (torch.arange(V, dtype=torch.float64) + 2.7) ** exponent
    ids = torch.multinomial(p / p.sum(), B * T, replacement=True, generator=g).reshape(B, T)
    if pad_fraction > 0:
        ids = torch.where(torch.rand(B, T, generator=g) < pad_fraction, torch.full_like(ids, -1), ids)
    return ids


def optimizer_state(n: int, seed: int = 0):
    """theta ~ N(0, 0.02), m = v = 0, all fp32 of length n."""
    g = _gen(seed * 2 + 3)
    theta = torch.randn(n, generator=g) * 0.02
    return theta, torch.zeros(n), torch.zeros(n)


def widen(x: torch.Tensor):
    """Exact fp32 numpy view of a bf16/fp32 payload (what the CPU oracle reads)."""
    return x.to(torch.float32).contiguous().numpy()
