"""GPU parity of pex_vec_stat (per-example statistics of offsets and elementwise scales) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2510_00236_amd as pex
import synth_inputs as si
from oracle import vec as ov

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(B, T, d, dtype, seed, scale=True):
    X, G = si.custom(B, T, d, d, dtype=dtype, seed=seed)      # two independent [B,T,d] Gaussian tensors
    return (G, X) if scale else (G, None)


def _check(A, C, dtype, tag):
    Ad = A.to(DEV)
    Cd = C.to(DEV) if C is not None else None
    got = pex.pex_vec_stat(Ad, Cd)
    torch.cuda.synchronize()
    ref = ov.vec_stat(si.widen(A), si.widen(C) if C is not None else None)
    # products of bf16 (or fp32) values summed in fp32 over T then B: relative to the largest entry
    bar = 2e-5
    for name, r in (("identity", ref.s_id), ("square", ref.s_sq)):
        g = got[name].cpu().double().numpy()
        err = np.abs(g - r).max() / max(np.abs(r).max(), 1e-300)
        assert err <= bar, f"{tag} {name}: {err:.3e}"
    if A.shape[0] >= 3:
        g = got["square"].cpu().double().numpy()
        assert (np.abs(g - ref.s_sq) <= 1e-4 * ref.s_sq + 1e-30).all(), f"{tag} square elementwise"
    d = np.abs(got["sign"].cpu().double().numpy() - ref.s_sign)
    assert (d <= 2 * ref.amb).all(), f"{tag} sign: counts differ outside the ambiguity band"


@pytest.mark.parametrize("B,T,d,dtype", [
    (5, 77, 520, "bf16"), (3, 100, 136, "bf16"), (2, 37, 33, "bf16"), (2, 37, 33, "f32"), (3, 50, 129, "f32"),
    (1, 64, 96, "bf16"), (40, 1, 128, "bf16"), (1, 1, 1, "f32"), (7, 300, 1024, "bf16"), (4, 16, 64, "f32"),
])
def test_offsets_and_scales_on_ragged_shapes(B, T, d, dtype):
    for scale in (False, True):
        A, C = _inputs(B, T, d, dtype, seed=B * 100 + T, scale=scale)
        _check(A, C, dtype, f"B{B} T{T} d{d} {dtype} scale={scale}")


def test_integer_inputs_are_bit_exact():
    r = torch.Generator().manual_seed(5)
    A = torch.randint(-3, 4, (6, 45, 264), generator=r).to(torch.bfloat16)
    C = torch.randint(-3, 4, (6, 45, 264), generator=r).to(torch.bfloat16)
    got = pex.pex_vec_stat(A.to(DEV), C.to(DEV))
    torch.cuda.synchronize()
    ref = ov.vec_stat(si.widen(A), si.widen(C))
    assert np.array_equal(got["identity"].cpu().double().numpy(), ref.s_id)
    assert np.array_equal(got["square"].cpu().double().numpy(), ref.s_sq)
    assert np.array_equal(got["sign"].cpu().double().numpy(), ref.s_sign)


def test_full_size_bias_of_the_1b_layer_and_subsets():
    """The offset of the 2048 -> 8192 layer at B=16, T=2048 (the oracle finishes in seconds at this size)."""
    w = si.WORKLOADS["c4_1b_up"]
    _, G = si.make(w, seed=0)
    _check(G, None, "bf16", "c4 bias")
    Gd = G.to(DEV)
    full = pex.pex_vec_stat(Gd)
    only = pex.pex_vec_stat(Gd, want=("square",))
    torch.cuda.synchronize()
    assert set(only) == {"square"} and torch.equal(only["square"], full["square"])
    again = pex.pex_vec_stat(Gd)
    assert all(torch.equal(full[k], again[k]) for k in full)     # run-to-run determinism


def test_offset_equals_the_matrix_statistic_with_a_column_of_ones():
    """Cross-check of the two GPU paths: an offset is a weight row fed by a constant 1."""
    X, G = si.custom(6, 64, 32, 256, dtype="bf16", seed=3)
    ones = torch.ones_like(X)
    Gd = G.to(DEV)
    vs = pex.pex_vec_stat(Gd)
    sq = pex.pex_stat(ones.to(DEV), Gd, "square")
    sg = pex.pex_stat(ones.to(DEV), Gd, "sign")
    torch.cuda.synchronize()
    assert torch.allclose(vs["square"], sq[0], rtol=1e-5, atol=0)
    assert (vs["sign"] - sg[0]).abs().max() <= 0
