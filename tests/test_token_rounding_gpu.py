"""The rounding of the per-token square on bf16 layers, pinned against the oracle.

Each squared operand is formed exactly (a product of two bf16 values has 16 significant bits) and rounded to bf16
to nearest even before the bf16 contraction.  Feeding the fp64 oracle those rounded squares turns the per-token
square into a plain contraction it can follow to fp32-accumulation accuracy, so the library is held to the 2e-5 bar
there -- a bar that an implementation which truncates the squares (error about 5e-3, all of one sign) cannot meet.
Against the exact per-token square the bar is 8e-3 elementwise: (1 + 2^-8)^2 - 1 is the worst case of two operands
each rounded to nearest with 8 significant bits."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00236_amd as pex
import synth_inputs as si
from parity_util import ENGINEERING_BAR, assert_real_stat, elementwise_rel_err, max_norm_err

RNE_ELEMENTWISE_BAR = 8e-3
DEV = "cuda:0"


def _squares_rne(t):
    """bf16(t^2), round to nearest even (torch's conversion), from the exact fp32 square."""
    return (t.float() * t.float()).to(torch.bfloat16)


def _squares_truncated(t):
    """bf16 squares with the low 16 bits of the fp32 square dropped: the mistake the test must catch."""
    sq = (t.float() * t.float()).contiguous()
    return (sq.view(torch.int32) & -65536).view(torch.float32).to(torch.bfloat16)


def test_a_truncating_square_would_fail_both_bars():
    """On the CPU, through the oracle only: truncated squares miss the rounded-squares result by far more than the
    2e-5 bar the library is held to (so that bar tells the two apart), and rounding itself stays inside 8e-3."""
    X, G = si.custom(5, 77, 136, 72, dtype="bf16", seed=21)
    pin = oracle.stat(si.widen(_squares_rne(X)), si.widen(_squares_rne(G))).S_id
    trunc = oracle.stat(si.widen(_squares_truncated(X)), si.widen(_squares_truncated(G))).S_id
    exact = oracle.token_sq(si.widen(X), si.widen(G))
    assert max_norm_err(trunc, pin) > 100 * ENGINEERING_BAR
    assert (trunc < pin).all()                                   # truncation errs in one direction
    assert elementwise_rel_err(pin, exact) <= RNE_ELEMENTWISE_BAR
    assert elementwise_rel_err(trunc, exact) > 3 * elementwise_rel_err(pin, exact)


@pytest.mark.gpu
@pytest.mark.parametrize("route", [0, 2])
@pytest.mark.parametrize("B,T,din,dout", [(5, 77, 520, 264), (3, 100, 200, 136), (9, 64, 256, 256)])
def test_token_square_rounds_to_nearest_on_both_routes(pex_option, route, B, T, din, dout):
    """route 0: operands squared inside the contraction; route 2: through bf16 copies of the squares."""
    pex_option("token_presquare", route)
    X, G = si.custom(B, T, din, dout, dtype="bf16", seed=B * 100 + T)
    S = pex.pex_token_sq(X.to(DEV), G.to(DEV))
    torch.cuda.synchronize()
    got = S.cpu().numpy().astype(np.float64)
    pin = oracle.stat(si.widen(_squares_rne(X)), si.widen(_squares_rne(G))).S_id
    assert_real_stat(got, pin, "bf16", f"token_sq route {route} vs rounded squares", elementwise=True, bar=1e-4)
    exact = oracle.token_sq(si.widen(X), si.widen(G))
    assert_real_stat(got, exact, "bf16", f"token_sq route {route} vs exact", elementwise=True, bar=RNE_ELEMENTWISE_BAR, eng=None)
    # the planted mistake, for the record: truncated squares through the oracle do not pass the bar `got` passed
    trunc = oracle.stat(si.widen(_squares_truncated(X)), si.widen(_squares_truncated(G))).S_id
    assert max_norm_err(trunc, pin) > ENGINEERING_BAR


@pytest.mark.gpu
@pytest.mark.parametrize("name", ["c4_1b_up", "c5_long"])
def test_token_square_rounding_at_full_size_sampled(name):
    """The launch configuration bench.py times (cost-model route), at sampled output positions."""
    w = si.WORKLOADS[name]
    X, G = si.make(w, seed=0)
    S = pex.pex_token_sq(X.to(DEV), G.to(DEV))
    torch.cuda.synchronize()
    rng = np.random.default_rng(7)
    ii, jj = rng.integers(0, w.din, 1500), rng.integers(0, w.dout, 1500)
    got = S[torch.as_tensor(ii, device=DEV), torch.as_tensor(jj, device=DEV)].cpu().numpy().astype(np.float64)
    X2, G2 = si.widen(_squares_rne(X)), si.widen(_squares_rne(G))
    pin = oracle.stat_at(X2, G2, ii, jj).S_id
    del X2, G2
    assert_real_stat(got, pin, "bf16", f"{name} token_sq vs rounded squares", elementwise=True, bar=1e-4)
    exact = oracle.token_sq_at(si.widen(X), si.widen(G), ii, jj)
    assert_real_stat(got, exact, "bf16", f"{name} token_sq vs exact", elementwise=True, bar=RNE_ELEMENTWISE_BAR, eng=None)
