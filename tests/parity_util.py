"""Comparison helpers of the GPU parity tests: the tolerances and metrics, written out once."""
import numpy as np

# Bars named by the workload definition: max relative error 1e-4 (fp32 inputs) / 2e-2 (bf16 inputs, fp32
# accumulation).  The engineering bar is what fp32 accumulation of exact products should give
# (unit roundoff 6e-8 times a modest growth factor); it catches dropped slabs or mis-scaled partial sums
# that the wide bf16 bar would let through.
BAR = {"f32": 1e-4, "bf16": 2e-2}
ENGINEERING_BAR = 2e-5
TOKEN_SQ_BF16_BAR = 8e-3   # two operands each rounded to nearest with 8 significant bits after squaring: (1 + 2^-8)^2 - 1


def max_norm_err(S, S0):
    """max_ij |S - S0| / max_ij |S0|."""
    return float(np.abs(S - S0).max() / np.abs(S0).max())


def elementwise_rel_err(S, S0):
    """max_ij |S - S0| / |S0| over entries with S0 != 0."""
    nz = S0 != 0
    return float((np.abs(S - S0)[nz] / np.abs(S0)[nz]).max()) if nz.any() else 0.0


def assert_real_stat(S, S0, dtype, what, elementwise, bar=None, eng=ENGINEERING_BAR):
    bar = BAR[dtype] if bar is None else bar
    e = max_norm_err(S, S0)
    assert np.isfinite(S).all(), f"{what}: non-finite output"
    assert e <= bar, f"{what}: max-norm error {e:.3e} > {bar:.1e}"
    if eng is not None:
        assert e <= eng, f"{what}: max-norm error {e:.3e} above the fp32-accumulation bar {eng:.1e}"
    if elementwise:
        r = elementwise_rel_err(S, S0)
        assert r <= bar, f"{what}: elementwise relative error {r:.3e} > {bar:.1e}"
    return e


def assert_sign_stat(S, S0, amb, what):
    """Exact integer equality outside the ambiguity mask; at an entry where `a` examples lie inside the
    1e-6 * max|M_b| band the count may differ by at most 2a (a flip is +-2, a zero is +-1)."""
    assert np.array_equal(S, np.round(S)), f"{what}: non-integer sign count"
    d = np.abs(S - S0)
    bad = d > 2 * amb
    assert not bad.any(), (f"{what}: {int(bad.sum())} sign counts differ outside the ambiguity band "
                           f"(first at {np.argwhere(bad)[0].tolist()}, got {S[bad][0]}, want {S0[bad][0]})")
    return int((d > 0).sum())
