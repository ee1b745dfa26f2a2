"""The worked example (one MicroAdam step over every parameter kind of a transformer block) against the oracles, on a
small block: dense weights, offsets, an elementwise scale, the embedding table, clipping and moment tracking."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from oracle import embed as oe, moments as om, update as ou, vec as ov
from paper_2510_00236_amd import example_step as ex

pytestmark = pytest.mark.gpu


def test_block_step_matches_the_oracles():
    B, T, d, V = 6, 48, 64, 97
    dev = torch.device("cuda:0")
    inputs, tensors, ws = ex.build(B, T, d, V, dev)
    theta0 = {k: t.theta.cpu().double().numpy().copy() for k, t in tensors.items() if isinstance(t, ex.Tensor)}
    ex.microadam_step(tensors, inputs, V, 1, B, lr=1e-2, max_norm=5.0, workspace=ws)
    torch.cuda.synchronize()
    wide = lambda t: t.float().cpu().numpy()
    ref = {}
    for name, (X, G) in inputs["dense"].items():
        st = oracle.stat(wide(X), wide(G))
        ref[name] = (st.S_id.reshape(-1), st.S_sq.reshape(-1))
        vs = ov.vec_stat(wide(G))
        ref[name + ".bias"] = (vs.s_id, vs.s_sq)
    for name, (A, C) in inputs["scale"].items():
        vs = ov.vec_stat(wide(A), wide(C))
        ref[name] = (vs.s_id, vs.s_sq)
    es = oe.embed_stat(inputs["ids"].cpu().numpy(), wide(inputs["embed_cot"]), V)
    ref["embed"] = (es.S_id.reshape(-1), es.S_sq.reshape(-1))
    sumsq = sum(float((r[0] ** 2).sum()) for r in ref.values())
    assert abs(float(tensors["_norm"].cpu()[0]) - sumsq) <= 1e-5 * sumsq
    prm = ou.AdamParams(lr=float(np.float32(1e-2)), beta1=float(np.float32(0.9)), beta2=float(np.float32(0.95)),
                        eps=float(np.float32(1e-8)), grad_scale=float(np.float32(1.0 / B)), sq_scale=float(np.float32(1.0 / B)),
                        step=1, B=B)
    k = 0
    for name, t in tensors.items():
        if not isinstance(t, ex.Tensor):
            continue
        S_id, S_sq = ref[name]
        got_id = t.S_id.cpu().double().numpy()
        assert np.abs(got_id - S_id).max() <= 2e-5 * max(np.abs(S_id).max(), 1e-30), name
        assert np.abs(t.S_sq.cpu().double().numpy() - S_sq).max() <= 2e-5 * max(np.abs(S_sq).max(), 1e-30), name
        rt, rm, rv = ou.adam_family_step_clipped(theta0[name], np.zeros(t.n), np.zeros(t.n), S_id, S_sq, ou.MICROADAM, prm, sumsq, 5.0)
        np.testing.assert_allclose(t.m.cpu().double().numpy(), rm, rtol=1e-4, atol=1e-6 * np.abs(rm).max())
        np.testing.assert_allclose(t.v.cpu().double().numpy(), rv, rtol=1e-4, atol=1e-6 * np.abs(rv).max())
        well = rv >= 1e-3 * rv.max()
        np.testing.assert_allclose((t.theta.cpu().double().numpy() - theta0[name])[well], (rt - theta0[name])[well], rtol=2e-3, atol=2e-8)
        _, _, ms = om.moment_track_step(np.zeros(t.n), np.zeros(t.n), S_id, S_sq, float(np.float32(0.95)), float(np.float32(1.0 / B)),
                                        float(np.float32(1.0 / B)), B, 1)
        got = tensors["_moments"][k].cpu().numpy()
        assert abs(got[0] - ms.sum_mu2) <= 1e-4 * ms.sum_abs and abs(got[1] - ms.sum_sigma2) <= 1e-4 * ms.sum_abs, name
        k += 1
