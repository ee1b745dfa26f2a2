"""pex_stat_noalloc (the entry point for callers that cannot allocate) through the C ABI against pex_stat: the same
kernels on the same plan, so the outputs must agree bit for bit -- and both against the fp64 oracle.  Two calls in a
row share the library's static scratch, the second on a smaller input, so stale partial sums of the first call would
show.  Collected last on purpose: a failure here must not hide the other GPU tests."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2510_00236_amd as pex
import synth_inputs as si
from parity_util import assert_real_stat, assert_sign_stat

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
PHI = ("identity", "square", "sign")


def _noalloc(Xd, Gd, phi, S):
    """Straight through the C symbol: raw pointers, no workspace argument."""
    B, T, din = Xd.shape
    dout = Gd.shape[2]
    dt = pex.PEX_BF16 if Xd.dtype == torch.bfloat16 else pex.PEX_F32
    rc = pex.lib().pex_stat_noalloc(Xd.data_ptr(), Gd.data_ptr(), B, T, din, dout, dt, pex.PHI[phi], S.data_ptr(),
                                    ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == pex.PEX_OK, pex.status_string(rc)


# first call, then a smaller one whose partial sums cover only the front of the scratch the first call filled
CASES = [
    ("bf16", (24, 96, 512, 384), (8, 40, 136, 72)),      # MFMA kernel, batch split over workgroups both times
    ("f32", (12, 50, 260, 132), (4, 19, 45, 51)),        # fp32 MFMA kernel, then the SIMT kernel
]


@pytest.mark.parametrize("dtype,first,second", CASES)
def test_noalloc_matches_pex_stat_on_two_calls_in_a_row(dtype, first, second):
    code = pex.PEX_BF16 if dtype == "bf16" else pex.PEX_F32
    inputs = []
    for k, (B, T, din, dout) in enumerate((first, second)):
        X, G = si.custom(B, T, din, dout, dtype=dtype, seed=91 + k)
        inputs.append((X, G, X.to(DEV), G.to(DEV)))
        for phi in PHI:
            need = pex.pex_stat_workspace_bytes(B, T, din, dout, code, phi)
            assert 0 < need <= pex.NOALLOC_SCRATCH_BYTES, (phi, need)   # the scratch really is in use
    # all six launches back to back on one stream, outputs preallocated: nothing between them clears the scratch
    outs = [{phi: torch.full((Xd.shape[2], Gd.shape[2]), float("nan"), device=DEV) for phi in PHI} for _, _, Xd, Gd in inputs]
    for (_, _, Xd, Gd), out in zip(inputs, outs):
        for phi in PHI:
            _noalloc(Xd, Gd, phi, out[phi])
    torch.cuda.synchronize()
    for (X, G, Xd, Gd), out in zip(inputs, outs):
        st = oracle.stat(si.widen(X), si.widen(G))
        tag = f"noalloc {tuple(X.shape)}x{G.shape[2]} {dtype}"
        for phi in PHI:
            want = pex.pex_stat(Xd, Gd, phi)
            torch.cuda.synchronize()
            assert torch.equal(out[phi], want), f"{tag} {phi}: differs from pex_stat"
        got = {phi: out[phi].cpu().numpy().astype(np.float64) for phi in PHI}
        assert_real_stat(got["identity"], st.S_id, dtype, f"{tag} identity", elementwise=False)
        assert_real_stat(got["square"], st.S_sq, dtype, f"{tag} square", elementwise=True)
        assert_sign_stat(got["sign"], st.S_sign, st.amb, f"{tag} sign")


def test_noalloc_without_scratch_need_and_over_the_limit():
    """A layer with enough tiles needs no scratch at all; one that needs more than the static buffer is refused."""
    X, G = si.custom(2, 64, 2048, 2048, dtype="bf16", seed=5)     # 64 tiles of 256 x 256, B = 2
    Xd, Gd = X.to(DEV), G.to(DEV)
    S = torch.empty(2048, 2048, device=DEV)
    _noalloc(Xd, Gd, "identity", S)
    want = pex.pex_stat(Xd, Gd, "identity")
    torch.cuda.synchronize()
    assert torch.equal(S, want)
    B, T, din, dout = 64, 1024, 768, 768          # nine tiles: many groups of examples, partial sums of 60 MB and more
    assert pex.pex_stat_workspace_bytes(B, T, din, dout, pex.PEX_BF16, "identity") > pex.NOALLOC_SCRATCH_BYTES
    Xb = torch.zeros(B, T, din, dtype=torch.bfloat16, device=DEV)
    Gb = torch.zeros(B, T, dout, dtype=torch.bfloat16, device=DEV)
    Sb = torch.full((din, dout), 7.0, device=DEV)
    with pytest.raises(pex.PexError) as ei:
        pex.pex_stat_noalloc(Xb, Gb, "identity", Sb)
    assert ei.value.code == 8
    torch.cuda.synchronize()
    assert bool((Sb == 7.0).all())                                  # nothing was launched
