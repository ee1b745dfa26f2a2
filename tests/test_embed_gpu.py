"""GPU parity of the embedding-table statistics against the fp64 oracle (a dense layer on one-hot inputs)."""
import numpy as np
import pytest
import torch

import paper_2510_00236_amd as pex
import synth_inputs as si
from oracle import embed as oe
from parity_util import assert_real_stat, assert_sign_stat

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = [
    # B, T, V, d, dtype, ids dtype, Zipf exponent, padding
    (5, 40, 23, 24, "bf16", torch.int64, 1.0, 0.1),
    (3, 700, 11, 64, "bf16", torch.int32, 1.5, 0.0),      # every row has far more than 64 positions: whole-workgroup path
    (4, 300, 300, 20, "bf16", torch.int64, 1.0, 0.05),    # rows not a multiple of 16 bytes: element-wise loads; two sort passes
    (6, 50, 70000, 16, "f32", torch.int32, 0.5, 0.0),     # three sort passes, almost every row empty
    (2, 1500, 5, 520, "f32", torch.int64, 1.0, 0.3),      # several column blocks, heavy rows
    (7, 129, 257, 1032, "bf16", torch.int32, 1.2, 0.0),   # ragged last column block, mix of light and heavy rows
    (1, 1, 1, 1, "f32", torch.int64, 1.0, 0.0),
    (9, 1030, 2, 8, "bf16", torch.int64, 0.0, 0.0),       # more than one sort tile per example, two tokens only
    (3, 50000, 1000, 8, "bf16", torch.int32, 1.0, 0.02),  # more positions than 64 tiles of 2048: larger sort tiles
]


def _inputs(B, T, V, d, dtype, idt, exponent, pad, seed):
    ids = si.token_ids(B, T, V, seed=seed, exponent=exponent, pad_fraction=pad).to(idt)
    G = si.custom(B, T, 8, d, dtype=dtype, seed=seed)[1]
    return ids, G


@pytest.mark.parametrize("B,T,V,d,dtype,idt,exponent,pad", CASES)
def test_embedding_statistics_match_the_oracle(B, T, V, d, dtype, idt, exponent, pad):
    ids, G = _inputs(B, T, V, d, dtype, idt, exponent, pad, seed=B + T)
    got = pex.pex_embed_stat(ids.to(DEV), G.to(DEV), V, ("identity", "square", "sign"))
    torch.cuda.synchronize()
    ref = oe.embed_stat(ids.numpy(), si.widen(G), V)
    f = lambda t: t.cpu().numpy().astype(np.float64)
    assert_real_stat(f(got["identity"]), ref.S_id, dtype, "identity", elementwise=False)
    assert_real_stat(f(got["square"]), ref.S_sq, dtype, "square", elementwise=True)
    assert_sign_stat(f(got["sign"]), ref.S_sign, ref.amb, "sign")
    # each statistic on its own is the same bits as in the joint pass, and a second run repeats them
    for name in ("identity", "square", "sign"):
        alone = pex.pex_embed_stat(ids.to(DEV), G.to(DEV), V, (name,))[name]
        assert torch.equal(alone, got[name]), name
    again = pex.pex_embed_stat(ids.to(DEV), G.to(DEV), V, ("identity", "square", "sign"))
    assert all(torch.equal(again[k], got[k]) for k in got)


def test_integer_cotangents_are_bit_exact():
    B, T, V, d = 6, 500, 40, 72
    ids = si.token_ids(B, T, V, seed=3, exponent=1.3, pad_fraction=0.1)
    G = si.integer_valued(B, T, 8, d, dtype="bf16", seed=3)[1]
    got = pex.pex_embed_stat(ids.to(DEV), G.to(DEV), V, 7)
    ref = oe.embed_stat(ids.numpy(), si.widen(G), V)
    for k, r in (("identity", ref.S_id), ("square", ref.S_sq), ("sign", ref.S_sign)):
        assert np.array_equal(got[k].cpu().numpy().astype(np.float64), r), k


def test_agrees_with_the_dense_kernels_on_one_hot_inputs():
    """The same statistic through the contraction kernels, with X the one-hot encoding of the ids."""
    B, T, V, d = 4, 96, 64, 128
    ids = si.token_ids(B, T, V, seed=5)
    G = si.integer_valued(B, T, 8, d, dtype="bf16", seed=5)[1]
    X = torch.nn.functional.one_hot(ids, V).to(torch.bfloat16)
    emb = pex.pex_embed_stat(ids.to(DEV), G.to(DEV), V, 7)
    dense = pex.pex_stat_multi(X.to(DEV), G.to(DEV), 7)
    for k in emb:
        assert torch.equal(emb[k], dense[k]), k


def test_output_buffers_workspace_and_stream():
    B, T, V, d = 3, 64, 50, 32
    ids, G = _inputs(B, T, V, d, "bf16", torch.int64, 1.0, 0.0, seed=8)
    idd, Gd = ids.to(DEV), G.to(DEV)
    ref = pex.pex_embed_stat(idd, Gd, V, ("square",))["square"]
    out = {"square": torch.full((V, d), 7.0, device=DEV)}
    ws = torch.empty(pex.pex_embed_stat_workspace_bytes(B, T, V, d), dtype=torch.uint8, device=DEV)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        pex.pex_embed_stat(idd, Gd, V, ("square",), out=out, workspace=ws, stream=st)
    st.synchronize()
    assert torch.equal(out["square"], ref)
    with pytest.raises(ValueError, match="workspace holds 64 bytes"):        # the binding's own check
        pex.pex_embed_stat(idd, Gd, V, ("square",), workspace=ws[:64])
    rc = pex.lib().pex_embed_stat(idd.data_ptr(), 8, Gd.data_ptr(), B, T, V, d, pex.PEX_BF16, 2, None, out["square"].data_ptr(),
                                  None, ws.data_ptr(), 64, None)                  # and the library's, through the C symbol
    assert rc == 6
    with pytest.raises(TypeError):
        pex.pex_embed_stat(idd.to(torch.int16), Gd, V, ("square",))


def test_full_size_gpt2_token_embedding_on_sampled_rows():
    """B=64, T=1024, V=50257, d=768 (the token embedding of the 151M-parameter model of App. D).  The oracle is run on
    a sample of the vocabulary rows: all other ids are turned into padding and the sampled rows renumbered, which leaves
    the sampled rows' statistics unchanged because rows do not interact."""
    B, T, V, d = 64, 1024, 50257, 768
    ids = si.token_ids(B, T, V, seed=0)
    G = si.make(si.Workload("emb", B, T, 8, d, "bf16", g_token="lognormal"), seed=0)[1]
    got = pex.pex_embed_stat(ids.to(DEV), G.to(DEV), V, 7)
    torch.cuda.synchronize()
    counts = torch.bincount(ids.reshape(-1), minlength=V)
    rng = np.random.default_rng(0)
    present = torch.nonzero(counts).reshape(-1).numpy()
    absent = torch.nonzero(counts == 0).reshape(-1).numpy()
    rows = np.unique(np.concatenate([np.arange(12), rng.choice(present, 150, replace=False), rng.choice(absent, 30, replace=False), [V - 1]]))
    remap = np.full(V, -1, dtype=np.int64)
    remap[rows] = np.arange(rows.size)
    ref = oe.embed_stat(remap[ids.numpy()], si.widen(G), rows.size)
    pick = lambda t: t[torch.as_tensor(rows, device=DEV)].cpu().numpy().astype(np.float64)
    assert_real_stat(pick(got["identity"]), ref.S_id, "bf16", "identity", elementwise=False)
    assert_real_stat(pick(got["square"]), ref.S_sq, "bf16", "square", elementwise=True)
    assert_sign_stat(pick(got["sign"]), ref.S_sign, ref.amb, "sign")
    # over the whole table: rows of absent tokens are zero, the column totals are those of all cotangents
    ab = torch.as_tensor(absent, device=DEV)
    assert all(float(got[k][ab].abs().max()) == 0.0 for k in got)
    tot = G.to(DEV).float().reshape(-1, d).double().sum(0)
    err = (got["identity"].double().sum(0) - tot).abs().max() / tot.abs().max()
    assert float(err) < 1e-4
    n_ex = torch.stack([(ids == int(v)).any(dim=1).sum() for v in rows[:12]]).to(DEV)
    assert (got["sign"][torch.as_tensor(rows[:12], device=DEV)].abs().max(dim=1).values <= n_ex).all()
