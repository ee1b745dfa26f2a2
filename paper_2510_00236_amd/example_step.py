"""One MicroAdam step with global-norm clipping over every parameter kind of a transformer block, through libpex only.

    python -m paper_2510_00236_amd.example_step            # GPT-2-small shapes, synthetic activations and cotangents

What a training loop hands over per step: for every dense layer its input activations X[B,T,din] and the cotangents
G[B,T,dout] of its outputs (the backward pass already has both), for an offset the cotangents of the sum it was
added to, for an elementwise scale those cotangents and the activation it multiplied, for the embedding the token ids
and the cotangents of the looked-up vectors.  Per parameter tensor the library returns S_id = sum_b g_b and
S_sq = sum_b g_b^2 without ever storing a per-example gradient; the optimizer kernels consume them in place.
Order of a step (everything stays on the GPU, nothing synchronises with the host):
  1. statistics of every tensor (one contraction per dense layer gives both S_id and S_sq);
  2. the squared global norm of the summed gradient, accumulated over the tensors;
  3. the update of every tensor, which forms the clipping factor from that norm on the device;
  4. optionally the running mu^2 / sigma^2 measurement of Sec. 3.2.2.
"""
from __future__ import annotations

import argparse
import time

import torch

import paper_2510_00236_amd as pex


class Tensor:
    """Optimizer state and statistics buffers of one parameter tensor."""

    def __init__(self, name, shape, dev):
        self.name, self.shape = name, tuple(shape)
        n = 1
        for s in shape:
            n *= s
        self.n = n
        self.theta = torch.randn(n, device=dev) * 0.02
        self.m = torch.zeros(n, device=dev)
        self.v = torch.zeros(n, device=dev)
        self.S_id = torch.empty(n, device=dev)
        self.S_sq = torch.empty(n, device=dev)
        self.ema_a = torch.zeros(n, device=dev)
        self.ema_q = torch.zeros(n, device=dev)


def block_inputs(B, T, d, V, dev, seed=0):
    """Synthetic activations / cotangents with the shapes of one GPT-2-style block plus the token embedding."""
    g = torch.Generator(device=dev).manual_seed(seed)
    rnd = lambda *s: torch.randn(*s, device=dev, generator=g).to(torch.bfloat16)
    ids = torch.randint(0, V, (B, T), device=dev, generator=g)
    return {
        "ids": ids,
        "dense": {                       # name: (X, G)
            "attn.qkv": (rnd(B, T, d), rnd(B, T, 3 * d)),
            "attn.proj": (rnd(B, T, d), rnd(B, T, d)),
            "mlp.fc": (rnd(B, T, d), rnd(B, T, 4 * d)),
            "mlp.proj": (rnd(B, T, 4 * d), rnd(B, T, d)),
        },
        "scale": {"ln1.scale": (rnd(B, T, d), rnd(B, T, d))},    # (cotangents, normalised activations)
        "embed_cot": rnd(B, T, d),
    }


def microadam_step(tensors, inputs, V, step, B, lr=2e-3, max_norm=1e-2, workspace=None, track=True):
    dense, scale = inputs["dense"], inputs["scale"]
    ws = workspace
    # 1. statistics
    for name, (X, G) in dense.items():
        w, b = tensors[name], tensors[name + ".bias"]
        din, dout = X.shape[2], G.shape[2]
        pex.pex_stat_multi(X, G, ("identity", "square"),
                           out={"identity": w.S_id.view(din, dout), "square": w.S_sq.view(din, dout)}, workspace=ws)
        pex.pex_vec_stat(G, None, ("identity", "square"), out={"identity": b.S_id, "square": b.S_sq}, workspace=ws)
    for name, (A, C) in scale.items():
        t = tensors[name]
        pex.pex_vec_stat(A, C, ("identity", "square"), out={"identity": t.S_id, "square": t.S_sq}, workspace=ws)
    e = tensors["embed"]
    d = inputs["embed_cot"].shape[2]
    pex.pex_embed_stat(inputs["ids"], inputs["embed_cot"], V, ("identity", "square"),
                       out={"identity": e.S_id.view(V, d), "square": e.S_sq.view(V, d)}, workspace=ws)
    # 2. global norm of the summed gradient
    acc = tensors["_norm"]
    first = True
    for t in tensors.values():
        if isinstance(t, Tensor):
            pex.pex_sum_squares(t.S_id, acc=acc, accumulate=not first, workspace=ws)
            first = False
    # 3. clipped update, 4. moment tracking
    prm = pex.AdamParams(lr=lr, beta1=0.9, beta2=0.95, eps=1e-8, eps_root=0.0, weight_decay=0.0,
                         grad_scale=1.0 / B, sq_scale=1.0 / B, step=step, B=B)
    mp = pex.MomentParams(beta2=0.95, grad_scale=1.0 / B, sq_scale=1.0 / B, B=B, debias=1, step=step)
    sums = tensors["_moments"]
    for k, t in enumerate(x for x in tensors.values() if isinstance(x, Tensor)):
        if track:
            pex.pex_moment_track(t.ema_a, t.ema_q, t.S_id, t.S_sq, mp, sums=sums[k], workspace=ws)
        pex.pex_adam_update_clipped(t.theta, t.m, t.v, t.S_id, t.S_sq, "microadam", prm, acc, max_norm)


def build(B, T, d, V, dev):
    inputs = block_inputs(B, T, d, V, dev)
    tensors = {}
    for name, (X, G) in inputs["dense"].items():
        tensors[name] = Tensor(name, (X.shape[2], G.shape[2]), dev)
        tensors[name + ".bias"] = Tensor(name + ".bias", (G.shape[2],), dev)
    for name, (A, _) in inputs["scale"].items():
        tensors[name] = Tensor(name, (A.shape[2],), dev)
    tensors["embed"] = Tensor("embed", (V, d), dev)
    n_t = sum(isinstance(t, Tensor) for t in tensors.values())
    tensors["_norm"] = torch.zeros(1, dtype=torch.float64, device=dev)
    tensors["_moments"] = torch.zeros(n_t, 2, dtype=torch.float64, device=dev)
    need = [16]
    for X, G in inputs["dense"].values():
        need.append(pex.pex_stat_multi_workspace_bytes(B, T, X.shape[2], G.shape[2], pex.PEX_BF16, 3))
        need.append(pex.pex_vec_stat_workspace_bytes(B, T, G.shape[2], pex.PEX_BF16))
    need.append(pex.pex_vec_stat_workspace_bytes(B, T, d, pex.PEX_BF16))
    need.append(pex.pex_embed_stat_workspace_bytes(B, T, V, d))
    biggest = max(t.n for t in tensors.values() if isinstance(t, Tensor))
    need += [pex.pex_sum_squares_workspace_bytes(biggest), pex.pex_moment_track_workspace_bytes(biggest)]
    ws = torch.empty(max(need), dtype=torch.uint8, device=dev)
    return inputs, tensors, ws


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--B", type=int, default=64)
    ap.add_argument("--T", type=int, default=1024)
    ap.add_argument("--d", type=int, default=768)
    ap.add_argument("--V", type=int, default=50257)
    ap.add_argument("--steps", type=int, default=5)
    a = ap.parse_args()
    dev = torch.device("cuda:0")
    inputs, tensors, ws = build(a.B, a.T, a.d, a.V, dev)
    microadam_step(tensors, inputs, a.V, 1, a.B, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(2, a.steps + 2):
        microadam_step(tensors, inputs, a.V, s, a.B, workspace=ws)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / a.steps * 1e3
    n_params = sum(t.n for t in tensors.values() if isinstance(t, Tensor))
    mom = tensors["_moments"].sum(0).cpu()
    norm = float(tensors["_norm"].cpu()[0]) ** 0.5 / a.B
    print(f"block d={a.d} B={a.B} T={a.T} V={a.V}: {n_params / 1e6:.1f} M parameters, {ms:.3f} ms per MicroAdam step "
          f"(statistics of every tensor, clipped update, moment tracking)")
    print(f"  gradient norm {norm:.4g}, mean mu^2-hat {float(mom[0]) / n_params:.4g}, mean sigma^2-hat {float(mom[1]) / n_params:.4g}")


if __name__ == "__main__":
    main()
