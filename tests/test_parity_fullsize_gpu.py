"""GPU parity at the full workload sizes, in the launch configuration bench.py times: the oracle evaluates the
per-example gradients entry by entry at sampled output positions (tile corners, tile seams, the ragged last
tile, and random positions), and every statistic is compared there."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00236_amd as pex
import synth_inputs as si
from parity_util import assert_real_stat, assert_sign_stat, TOKEN_SQ_BF16_BAR

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _sample_positions(din, dout, n_random, seed):
    rng = np.random.default_rng(seed)
    ii = list(rng.integers(0, din, n_random))
    jj = list(rng.integers(0, dout, n_random))
    # seams of the 64/128/192/256-wide tiles the kernels use, first and last rows/columns
    edges_i = sorted({0, 1, 31, 32, 63, 64, 127, 128, 255, 256, din // 2 - 1, din // 2, din - 257, din - 256, din - 2, din - 1} & set(range(din)))
    edges_j = sorted({0, 1, 31, 32, 63, 64, 127, 128, 191, 192, 255, 256, dout // 2 - 1, dout // 2, dout - 129, dout - 128, dout - 2, dout - 1} & set(range(dout)))
    for a in edges_i:
        for b in edges_j:
            ii.append(a)
            jj.append(b)
    return np.array(ii, dtype=np.int64), np.array(jj, dtype=np.int64)


@pytest.mark.parametrize("name", ["c3_gpt2_qkv", "c3_gpt2_proj", "c3_gpt2_fc", "c3_gpt2_fcproj", "c4_1b_up", "c4_1b_down", "c5_long"])
def test_full_size_sampled(name):
    w = si.WORKLOADS[name]
    X, G = si.make(w, seed=0)
    Xd, Gd = X.to(DEV), G.to(DEV)
    got = {phi: pex.pex_stat(Xd, Gd, phi) for phi in ("identity", "square", "sign")}
    got["token_sq"] = pex.pex_token_sq(Xd, Gd)
    torch.cuda.synchronize()
    for k, v in got.items():
        assert torch.isfinite(v).all(), f"{name} {k}: non-finite"
    ii, jj = _sample_positions(w.din, w.dout, 3000, seed=1)
    Xn, Gn = si.widen(X), si.widen(G)
    st = oracle.stat_at(Xn, Gn, ii, jj)
    tok = oracle.token_sq_at(Xn, Gn, ii, jj)
    del Xn, Gn
    pick = lambda t: t[torch.as_tensor(ii, device=DEV), torch.as_tensor(jj, device=DEV)].cpu().numpy().astype(np.float64)
    assert_real_stat(pick(got["identity"]), st.S_id, "bf16", f"{name} identity", elementwise=False)
    assert_real_stat(pick(got["square"]), st.S_sq, "bf16", f"{name} square", elementwise=True)
    n_diff = assert_sign_stat(pick(got["sign"]), st.S_sign, st.amb, f"{name} sign")
    assert_real_stat(pick(got["token_sq"]), tok, "bf16", f"{name} token_sq", elementwise=True, bar=TOKEN_SQ_BF16_BAR, eng=None)
    # properties that hold at any size, over the whole output
    S_sq, S_id, S_sg = got["square"], got["identity"], got["sign"]
    assert (S_sq >= 0).all()
    assert (S_sq * w.B >= S_id * S_id * (1 - 1e-4) - 1e-6 * S_sq.max()).all()      # Cauchy-Schwarz: nu_micro >= nu_adam
    assert (S_sg.abs() <= w.B).all() and torch.equal(S_sg, S_sg.round())
    assert ((S_sg.long() - w.B) % 2 == 0).float().mean() > 0.999                    # parity of B wherever no M_b is exactly 0
    print(f"{name}: sign mismatches inside the ambiguity band: {n_diff}")


@pytest.mark.parametrize("name", ["c4_1b_up", "c5_long"])
def test_full_size_shared_contraction_weighted_and_power(name):
    """The entry points that share the contraction kernels (several statistics from one pass, clipping-weighted
    sums, |.|^alpha) at the sizes bench.py times, against per-example values the oracle computes at sampled positions."""
    w = si.WORKLOADS[name]
    X, G = si.make(w, seed=2)
    Xd, Gd = X.to(DEV), G.to(DEV)
    multi = pex.pex_stat_multi(Xd, Gd, ("identity", "square", "sign"))
    pair = pex.pex_stat_multi(Xd, Gd, ("identity", "square"))
    wts = torch.linspace(0.25, 1.0, w.B)
    S_w = pex.pex_weighted_sum(Xd, Gd, wts.to(DEV))
    S_p = pex.pex_stat_power(Xd, Gd, 1.0)
    N = pex.pex_example_norms(Xd, Gd)
    torch.cuda.synchronize()
    ii, jj = _sample_positions(w.din, w.dout, 2000, seed=3)
    M = oracle.per_example_at(si.widen(X), si.widen(G), ii, jj)             # [B, n] fp64
    pick = lambda t: t[torch.as_tensor(ii, device=DEV), torch.as_tensor(jj, device=DEV)].cpu().numpy().astype(np.float64)
    mx = np.abs(M).max(axis=1)
    amb = (np.abs(M) < oracle.SIGN_BAND * mx[:, None]).sum(axis=0)
    for got, what in ((multi, "three at once"), (pair, "identity and square")):
        assert_real_stat(pick(got["identity"]), M.sum(axis=0), "bf16", f"{name} {what}: identity", elementwise=False)
        assert_real_stat(pick(got["square"]), (M * M).sum(axis=0), "bf16", f"{name} {what}: square", elementwise=True)
    assert_sign_stat(pick(multi["sign"]), np.sign(M).sum(axis=0), amb, f"{name} three at once: sign")
    assert_real_stat(pick(S_w), (wts.double().numpy()[:, None] * M).sum(axis=0), "bf16", f"{name} weighted", elementwise=False)
    assert_real_stat(pick(S_p), np.abs(M).sum(axis=0), "bf16", f"{name} |.|^1", elementwise=True)
    # the norms cover every entry; the total of the square statistic is the same number by another kernel
    tot = float(multi["square"].double().sum())
    assert abs(float(N.double().sum()) - tot) <= 1e-5 * tot


def test_full_size_fp32_inputs_sampled():
    """fp32 inputs at a transformer-layer size (B=8, T=1024, 1024 x 4096) on the fp32 MFMA kernel, 1e-4 bar."""
    B, T, din, dout = 8, 1024, 1024, 4096
    X, G = si.custom(B, T, din, dout, dtype="f32", seed=4)
    Xd, Gd = X.to(DEV), G.to(DEV)
    got = {phi: pex.pex_stat(Xd, Gd, phi) for phi in ("identity", "square", "sign")}
    got["token_sq"] = pex.pex_token_sq(Xd, Gd)
    torch.cuda.synchronize()
    ii, jj = _sample_positions(din, dout, 2000, seed=5)
    Xn, Gn = si.widen(X), si.widen(G)
    st = oracle.stat_at(Xn, Gn, ii, jj)
    tok = oracle.token_sq_at(Xn, Gn, ii, jj)
    pick = lambda t: t[torch.as_tensor(ii, device=DEV), torch.as_tensor(jj, device=DEV)].cpu().numpy().astype(np.float64)
    assert_real_stat(pick(got["identity"]), st.S_id, "f32", "fp32 identity", elementwise=False)
    assert_real_stat(pick(got["square"]), st.S_sq, "f32", "fp32 square", elementwise=True)
    assert_sign_stat(pick(got["sign"]), st.S_sign, st.amb, "fp32 sign")
    assert_real_stat(pick(got["token_sq"]), tok, "f32", "fp32 token_sq", elementwise=True)


def test_full_size_every_entry_c4_1b_up():
    """One layer at full size with nothing sampled: all 16.8 M entries of identity, square and sign from one pass of
    the fp64 oracle over B=16, T=2048, 2048 x 8192, and all entries of the per-token square from a second."""
    w = si.WORKLOADS["c4_1b_up"]
    X, G = si.make(w, seed=0)
    Xd, Gd = X.to(DEV), G.to(DEV)
    got = {phi: pex.pex_stat(Xd, Gd, phi) for phi in ("identity", "square", "sign")}
    got["token_sq"] = pex.pex_token_sq(Xd, Gd)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy().astype(np.float64) for k, v in got.items()}
    del Xd, Gd
    Xn, Gn = si.widen(X), si.widen(G)
    st = oracle.stat(Xn, Gn)
    assert_real_stat(got["identity"], st.S_id, "bf16", "c4_1b_up identity, every entry", elementwise=False)
    assert_real_stat(got["square"], st.S_sq, "bf16", "c4_1b_up square, every entry", elementwise=True)
    n_diff = assert_sign_stat(got["sign"], st.S_sign, st.amb, "c4_1b_up sign, every entry")
    print(f"c4_1b_up, every entry: {n_diff} sign counts differ inside the ambiguity band, {int((st.amb > 0).sum())} entries in it")
    del st
    tok = oracle.token_sq(Xn, Gn)
    assert_real_stat(got["token_sq"], tok, "bf16", "c4_1b_up token_sq, every entry", elementwise=True, bar=8e-3, eng=None)
