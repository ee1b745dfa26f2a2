"""GPU parity: libpex through its C ABI against the fp64 CPU oracle, element by element, on the same
seeded inputs -- sizes the oracle finishes in seconds, spanning several tiles and ragged tails."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_00236_amd as pex
import synth_inputs as si
from parity_util import assert_real_stat, assert_sign_stat, TOKEN_SQ_BF16_BAR

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _run_all(X, G):
    Xd, Gd = X.to(DEV), G.to(DEV)
    out = {phi: pex.pex_stat(Xd, Gd, phi) for phi in ("identity", "square", "sign")}
    out["token_sq"] = pex.pex_token_sq(Xd, Gd)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy().astype(np.float64) for k, v in out.items()}


def _compare(X, G, dtype, tag, elementwise=True):
    got = _run_all(X, G)
    Xn, Gn = si.widen(X), si.widen(G)
    st = oracle.stat(Xn, Gn)
    tok = oracle.token_sq(Xn, Gn)
    assert_real_stat(got["identity"], st.S_id, dtype, f"{tag} identity", elementwise=False)
    assert_real_stat(got["square"], st.S_sq, dtype, f"{tag} square", elementwise=elementwise)
    assert_sign_stat(got["sign"], st.S_sign, st.amb, f"{tag} sign")
    if dtype == "bf16":
        assert_real_stat(got["token_sq"], tok, dtype, f"{tag} token_sq", elementwise=True, bar=TOKEN_SQ_BF16_BAR, eng=None)
    else:
        assert_real_stat(got["token_sq"], tok, dtype, f"{tag} token_sq", elementwise=True)
    return got, st


def test_config1_tiny_fp32():
    X, G = si.make("c1_tiny", seed=0)
    _compare(X, G, "f32", "c1")


def test_config2_mlp_in_bf16():
    X, G = si.make("c2_mlp_in", seed=0)
    _compare(X, G, "bf16", "c2")


# (B, T, din, dout, dtype): ragged tails in every dimension, on both kernels
SHAPES = [
    (3, 100, 200, 136, "bf16"),    # multiples of 8: MFMA path with zero-filled tile edges, T not a slab multiple
    (5, 77, 520, 264, "bf16"),     # several tiles per dimension plus ragged edges
    (2, 37, 70, 33, "bf16"),       # rows not 16-byte multiples: SIMT path on bf16
    (2, 37, 70, 33, "f32"),
    (3, 50, 129, 65, "f32"),
    (7, 33, 256, 128, "bf16"),     # exactly one tile, odd T
    (1, 64, 96, 160, "bf16"),      # B = 1
    (40, 1, 128, 96, "bf16"),      # T = 1 (rank-one gradients)
    (2, 16, 32, 32, "bf16"),       # smallest shape the MFMA path takes
    (1, 1, 1, 1, "f32"),           # degenerate
    (1, 1, 8, 8, "bf16"),
    (2100, 1, 64, 96, "bf16"),     # more examples than packed sign counts can hold: fp32 counts
    (40, 24, 512, 520, "bf16"),    # 256-wide tiles with a ragged last tile column
    (3, 50, 132, 68, "f32"),       # fp32 MFMA path: ragged 128-wide tiles, T not a multiple of the 16-token slab
    (5, 77, 520, 264, "f32"),      # fp32 MFMA path: several tiles, batch split over workgroups
    (2, 16, 32, 32, "f32"),        # smallest shape the fp32 MFMA path takes
    (40, 1, 128, 96, "f32"),       # T = 1 on the fp32 MFMA path
    (7, 33, 256, 128, "f32"),
]


@pytest.mark.parametrize("B,T,din,dout,dtype", SHAPES)
def test_ragged_and_edge_shapes(B, T, din, dout, dtype):
    X, G = si.custom(B, T, din, dout, dtype=dtype, seed=B * 1000 + T)
    # with B = 1 an entry of S_sq is a single squared cancelling sum: only the max-norm metric is meaningful
    _compare(X, G, dtype, f"B{B} T{T} {din}x{dout} {dtype}", elementwise=(B >= 3))


@pytest.mark.parametrize("B,T,din,dout,dtype", [(5, 48, 264, 136, "bf16"), (3, 19, 45, 51, "bf16"), (4, 16, 64, 64, "f32"),
                                                (6, 40, 264, 136, "f32")])
def test_integer_inputs_are_bit_exact(B, T, din, dout, dtype):
    """Small-integer inputs: every product and partial sum is exact, so every statistic must match bit for bit."""
    X, G = si.integer_valued(B, T, din, dout, dtype=dtype, seed=3)
    got = _run_all(X, G)
    Xn, Gn = si.widen(X), si.widen(G)
    st = oracle.stat(Xn, Gn)
    assert np.array_equal(got["identity"], st.S_id)
    assert np.array_equal(got["square"], st.S_sq)
    assert np.array_equal(got["sign"], st.S_sign)          # includes exact zeros: sgn(0) = 0
    assert (st.S_sign != np.sign(st.S_id) * B).any()
    assert np.array_equal(got["token_sq"], oracle.token_sq(Xn, Gn))


def test_sign_count_at_the_packing_limit():
    """2048 examples that all agree: the count 2048 must come out exactly (and -2048 with the cotangents negated)."""
    X = torch.ones(2048, 1, 64, dtype=torch.bfloat16)
    G = torch.ones(2048, 1, 96, dtype=torch.bfloat16)
    G[:, :, 48:] = -1
    S = pex.pex_stat(X.to(DEV), G.to(DEV), "sign").cpu()
    assert torch.equal(S[:, :48], torch.full((64, 48), 2048.0)) and torch.equal(S[:, 48:], torch.full((64, 48), -2048.0))


def test_zero_example_gives_zero_sign():
    """An example whose activations are all zero contributes sgn(0) = 0 everywhere."""
    X, G = si.custom(3, 40, 64, 64, dtype="bf16", seed=5)
    X[1] = 0
    got = _run_all(X, G)
    st = oracle.stat(si.widen(X), si.widen(G))
    assert_sign_stat(got["sign"], st.S_sign, st.amb, "zero example")   # max|M_b| = 0: the band is empty, the zeros are exact
    assert np.abs(got["sign"]).max() <= 2


def test_run_to_run_determinism():
    X, G = si.custom(16, 96, 512, 384, dtype="bf16", seed=7)
    Xd, Gd = X.to(DEV), G.to(DEV)
    for phi in ("identity", "square", "sign"):
        a = pex.pex_stat(Xd, Gd, phi).clone()
        b = pex.pex_stat(Xd, Gd, phi)
        torch.cuda.synchronize()
        assert torch.equal(a, b), phi
    a = pex.pex_token_sq(Xd, Gd).clone()
    assert torch.equal(a, pex.pex_token_sq(Xd, Gd))


def test_batch_permutation_and_output_overwrite():
    """S does not depend on the order of examples (Sec. 3.1) and is overwritten, not accumulated into."""
    X, G = si.custom(6, 64, 256, 128, dtype="bf16", seed=8)
    perm = torch.tensor([3, 0, 5, 1, 4, 2])
    Xd, Gd = X.to(DEV), G.to(DEV)
    S = torch.full((256, 128), 1e30, device=DEV)
    pex.pex_stat(Xd, Gd, "sign", S=S)
    S2 = pex.pex_stat(Xd[perm].contiguous(), Gd[perm].contiguous(), "sign")
    torch.cuda.synchronize()
    assert torch.equal(S, S2)
    assert S.abs().max() <= 6


def test_non_default_stream():
    X, G = si.custom(4, 64, 128, 128, dtype="bf16", seed=9)
    Xd, Gd = X.to(DEV), G.to(DEV)
    ref = pex.pex_stat(Xd, Gd, "square")
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        out = pex.pex_stat(Xd, Gd, "square", stream=s)
    s.synchronize()
    assert torch.equal(ref, out)


def test_workspace_errors_on_gpu():
    X, G = si.custom(64, 32, 256, 128, dtype="bf16", seed=10)      # one tile, many examples: the batch is split
    Xd, Gd = X.to(DEV), G.to(DEV)
    need = pex.pex_stat_workspace_bytes(64, 32, 256, 128, pex.PEX_BF16, "square")
    assert need > 0
    small = torch.empty(need - 16, dtype=torch.uint8, device=DEV)
    with pytest.raises(ValueError, match="workspace holds"):          # the binding's own check
        pex.pex_stat(Xd, Gd, "square", workspace=small)
    S = torch.full((256, 128), 7.0, device=DEV)
    rc = pex.lib().pex_stat(Xd.data_ptr(), Gd.data_ptr(), 64, 32, 256, 128, pex.PEX_BF16, pex.PEX_PHI_SQUARE, S.data_ptr(),
                            small.data_ptr(), need - 16, None)          # and the library's, through the C symbol
    torch.cuda.synchronize()
    assert rc == 6 and bool((S == 7.0).all())


MULTI_SHAPES = [
    (5, 77, 520, 264, "bf16"),     # several tiles, ragged edges, batch split over workgroups (workspace)
    (3, 100, 200, 136, "bf16"),
    (7, 33, 256, 128, "bf16"),     # exactly one tile
    (2100, 1, 64, 96, "bf16"),     # fp32 sign counts inside a pair
    (127, 3, 64, 96, "bf16"),      # the most examples the byte-wide sign counters of the three-in-one launch hold
    (128, 3, 64, 96, "bf16"),      # one more: identity and square share a contraction, sign runs alone
    (3, 50, 129, 65, "f32"),       # SIMT kernel: one statistic at a time
]


@pytest.mark.parametrize("B,T,din,dout,dtype", MULTI_SHAPES)
def test_multi_statistics_match_the_oracle_and_the_single_calls(B, T, din, dout, dtype):
    """Every subset of {identity, square, sign} through pex_stat_multi: same bars as the single calls; square is
    bit-identical to pex_stat (same tile, same order), sign counts agree wherever no example is ambiguous."""
    X, G = si.custom(B, T, din, dout, dtype=dtype, seed=B + T)
    Xd, Gd = X.to(DEV), G.to(DEV)
    st = oracle.stat(si.widen(X), si.widen(G))
    single = {phi: pex.pex_stat(Xd, Gd, phi) for phi in ("identity", "square", "sign")}
    for want in (("identity", "square"), ("identity", "sign"), ("square", "sign"), ("identity", "square", "sign"),
                 ("square",), ("identity",), ("sign",)):
        poison = {w: torch.full((din, dout), 3e33, device=DEV) for w in want}     # outputs are overwritten
        got = pex.pex_stat_multi(Xd, Gd, want, out=poison)
        torch.cuda.synchronize()
        assert set(got) == set(want)
        tag = f"multi{want} B{B} T{T} {din}x{dout} {dtype}"
        if "identity" in got:
            assert_real_stat(got["identity"].cpu().double().numpy(), st.S_id, dtype, tag + " identity", elementwise=False)
        if "square" in got:
            assert_real_stat(got["square"].cpu().double().numpy(), st.S_sq, dtype, tag + " square", elementwise=(B >= 3))
            assert torch.equal(got["square"], single["square"]), tag
        if "sign" in got:
            assert_sign_stat(got["sign"].cpu().double().numpy(), st.S_sign, st.amb, tag + " sign")
            clear = torch.from_numpy(st.amb == 0).to(DEV)
            assert torch.equal(got["sign"][clear], single["sign"][clear]), tag


def test_byte_sign_counters_at_their_limit():
    """127 examples that all agree (and all disagree): the three-in-one launch must return +-127 exactly."""
    X = torch.ones(127, 2, 64, dtype=torch.bfloat16)
    G = torch.ones(127, 2, 96, dtype=torch.bfloat16)
    G[:, :, 48:] = -1
    got = pex.pex_stat_multi(X.to(DEV), G.to(DEV), ("identity", "square", "sign"))
    torch.cuda.synchronize()
    S = got["sign"].cpu()
    assert torch.equal(S[:, :48], torch.full((64, 48), 127.0)) and torch.equal(S[:, 48:], torch.full((64, 48), -127.0))
    assert torch.equal(got["identity"].cpu(), 2.0 * S) and torch.equal(got["square"].cpu(), torch.full((64, 96), 4.0 * 127))


def test_multi_on_integer_inputs_is_bit_exact():
    X, G = si.integer_valued(6, 40, 264, 136, dtype="bf16", seed=11)
    st = oracle.stat(si.widen(X), si.widen(G))
    got = pex.pex_stat_multi(X.to(DEV), G.to(DEV), ("identity", "square", "sign"))
    torch.cuda.synchronize()
    assert np.array_equal(got["identity"].cpu().double().numpy(), st.S_id)
    assert np.array_equal(got["square"].cpu().double().numpy(), st.S_sq)
    assert np.array_equal(got["sign"].cpu().double().numpy(), st.S_sign)


def test_token_square_through_presquared_copies_is_the_same_bits(pex_option):
    """The per-token square has two routes on bf16 layers (operands squared inside the contraction, or bf16 copies
    of the squares made first); both round the squares the same way and must agree bit for bit."""
    X, G = si.custom(5, 77, 520, 264, dtype="bf16", seed=21)
    Xd, Gd = X.to(DEV), G.to(DEV)
    pex_option("token_presquare", 0)
    fused = pex.pex_token_sq(Xd, Gd).clone()
    ws_fused = pex.pex_token_sq_workspace_bytes(5, 77, 520, 264, pex.PEX_BF16)
    pex_option("token_presquare", 2)
    copy_bytes = 2 * 5 * 77 * (520 + 264)
    assert 0 <= pex.pex_token_sq_workspace_bytes(5, 77, 520, 264, pex.PEX_BF16) - ws_fused - copy_bytes < 256
    copies = pex.pex_token_sq(Xd, Gd)
    torch.cuda.synchronize()
    assert torch.equal(fused, copies)
    tok = oracle.token_sq(si.widen(X), si.widen(G))
    assert_real_stat(copies.cpu().double().numpy(), tok, "bf16", "token_sq copies", elementwise=True, bar=TOKEN_SQ_BF16_BAR, eng=None)


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for k in range(n):
        B = int(rng.integers(1, 41))
        T = int(rng.integers(1, 301))
        if k % 3 == 2:      # any widths: the SIMT kernel (or fp32 inputs)
            din, dout = int(rng.integers(1, 400)), int(rng.integers(1, 400))
            dtype = "f32" if k % 2 else "bf16"
        else:               # multiples of 8 from 32 up: the MFMA kernel, tile edges anywhere
            din, dout = 8 * int(rng.integers(4, 90)), 8 * int(rng.integers(4, 90))
            dtype = "bf16"
        out.append((B, T, din, dout, dtype))
    return out


@pytest.mark.parametrize("B,T,din,dout,dtype", _random_shapes(24, seed=2510))
def test_seeded_sweep_of_shapes(B, T, din, dout, dtype):
    """Shapes drawn once from a fixed seed: tile edges, slab tails and batch splits fall where nobody chose them.
    Every statistic through its own call, then identity, square and sign again from one shared contraction."""
    X, G = si.custom(B, T, din, dout, dtype=dtype, seed=B + 41 * T + din)
    got, st = _compare(X, G, dtype, f"B{B} T{T} {din}x{dout} {dtype}", elementwise=(B >= 3))
    multi = pex.pex_stat_multi(X.to(DEV), G.to(DEV), ("identity", "square", "sign"))
    f = lambda t: t.cpu().numpy().astype(np.float64)
    assert_real_stat(f(multi["identity"]), st.S_id, dtype, "shared identity", elementwise=False)
    assert_real_stat(f(multi["square"]), st.S_sq, dtype, "shared square", elementwise=(B >= 3))
    assert_sign_stat(f(multi["sign"]), st.S_sign, st.amb, "shared sign")


def test_mfma_probe_runs_and_counts_its_flop():
    """The measurement aid: deterministic output, FLOP count = workgroups x 8 waves x iters x 64 MFMAs x 2*16*16*32."""
    ops = torch.randn(pex.lib().pex_mfma_probe_operand_bytes() // 2, device=DEV).to(torch.bfloat16)
    flop, s1 = pex.pex_mfma_probe(ops, 4, 10)
    assert flop == 4 * 8 * 10 * 64 * 2 * 16 * 16 * 32
    _, s2 = pex.pex_mfma_probe(ops, 4, 10)
    torch.cuda.synchronize()
    assert s1.shape == (4 * 512,) and torch.isfinite(s1).all() and torch.equal(s1, s2)
    with pytest.raises(ValueError):
        pex.pex_mfma_probe(ops[:100], 4, 10)
    with pytest.raises(pex.PexError):
        pex.pex_mfma_probe(ops, 0, 10)


@pytest.mark.parametrize("B,T,din,dout,dtype", [(1, 100_000, 64, 96, "bf16"), (2, 40_000, 64, 64, "f32"), (3, 33_333, 40, 72, "bf16")])
def test_long_sequences(B, T, din, dout, dtype):
    """Contractions over tens of thousands of tokens per example: thousands of slabs through the LDS ring, fp32
    accumulation error still far inside the bars, the batch split (plain contractions split the flattened rows)."""
    X, G = si.custom(B, T, din, dout, dtype=dtype, seed=T)
    _compare(X, G, dtype, f"B{B} T{T} {din}x{dout} {dtype}", elementwise=(B >= 3))


@pytest.mark.parametrize("B,T,din,dout,dtype", [(5, 77, 521, 265, "bf16"), (3, 50, 131, 67, "f32"), (7, 33, 255, 129, "bf16")])
def test_simt_kernel_on_layers_of_several_tiles(B, T, din, dout, dtype):
    """Rows that are not multiples of 16 bytes go to the SIMT kernel whatever their size: several 64 x 64 tiles with
    ragged edges and the batch split over workgroups, one element off the shapes the MFMA kernels are tested on."""
    X, G = si.custom(B, T, din, dout, dtype=dtype, seed=B * 1000 + T)
    _compare(X, G, dtype, f"SIMT B{B} T{T} {din}x{dout} {dtype}", elementwise=(B >= 3))


# Plain contractions with at least 1024 rows per workgroup run on the four-wave kernel (one wave per SIMD, 128 x 128
# per wave): ragged tile edges, a last slab of 1, 23 and 31 rows, an odd and an even number of slabs, one tile and
# several, with the planner's split of the rows over workgroups and (small shapes) with the split switched off.
@pytest.mark.parametrize("B,T,din,dout,max_split", [(1, 1024, 256, 256, 1), (1, 1025, 256, 256, 1), (3, 701, 328, 200, 1),
                                                    (5, 411, 264, 520, 1), (1, 2079, 1032, 40, 2), (3, 7171, 520, 776, None),
                                                    (2, 20000, 512, 512, None)])
def test_four_wave_kernel_shapes(pex_option, B, T, din, dout, max_split):
    if max_split is not None:
        pex_option("max_split", max_split)
    nsplit = max(1, pex.pex_stat_workspace_bytes(B, T, din, dout, pex.PEX_BF16, "identity") // (din * dout * 4))
    assert B * T // nsplit >= 1024, "shape chosen so that the four-wave kernel takes it"
    X, G = si.custom(B, T, din, dout, dtype="bf16", seed=B + T)
    S = pex.pex_stat(X.to(DEV), G.to(DEV), "identity")
    torch.cuda.synchronize()
    st = oracle.stat(si.widen(X), si.widen(G))
    assert_real_stat(S.cpu().numpy().astype(np.float64), st.S_id, "bf16", f"four-wave identity {B}x{T}x{din}x{dout}", elementwise=False)


# phi = square, weighted sums and |.|^alpha have two block shapes on bf16 layers; option wide_blocks = 2 puts as many
# columns as fit on the 256 x 192 one and the rest on the 256 x 128 one, in two launches side by side.
@pytest.mark.parametrize("B,T,din,dout", [(5, 77, 520, 264), (3, 100, 200, 192), (7, 33, 256, 456), (4, 64, 512, 1024),
                                          (6, 40, 264, 392), (40, 24, 512, 200), (2, 50, 96, 1160)])
def test_wide_blocks_side_by_side_with_narrow_ones(pex_option, B, T, din, dout):
    X, G = si.custom(B, T, din, dout, dtype="bf16", seed=B * 10 + T)
    Xd, Gd = X.to(DEV), G.to(DEV)
    wts = torch.linspace(0.5, 1.5, B)
    pex_option("wide_blocks", 0)
    narrow = (pex.pex_stat(Xd, Gd, "square").clone(), pex.pex_weighted_sum(Xd, Gd, wts.to(DEV)).clone(), pex.pex_stat_power(Xd, Gd, 1.0).clone())
    pex_option("wide_blocks", 2)
    need = pex.pex_stat_workspace_bytes(B, T, din, dout, pex.PEX_BF16, "square")
    assert need % (din * 8 * 4) == 0 and need <= 32 * din * dout * 4      # groups of whole rows of the two column ranges
    wide = (pex.pex_stat(Xd, Gd, "square"), pex.pex_weighted_sum(Xd, Gd, wts.to(DEV)), pex.pex_stat_power(Xd, Gd, 1.0))
    torch.cuda.synchronize()
    st = oracle.stat(si.widen(X), si.widen(G))
    f = lambda t: t.cpu().numpy().astype(np.float64)
    assert_real_stat(f(wide[0]), st.S_sq, "bf16", "square on wide blocks", elementwise=(B >= 3))
    M = np.einsum("bti,btj->bij", si.widen(X).astype(np.float64), si.widen(G).astype(np.float64))
    assert_real_stat(f(wide[1]), (wts.double().numpy()[:, None, None] * M).sum(0), "bf16", "weighted sum on wide blocks", elementwise=False)
    assert_real_stat(f(wide[2]), np.abs(M).sum(0), "bf16", "|.|^1 on wide blocks", elementwise=(B >= 3))
    # either block shape folds the same per-example tiles; only the grouping of the sum over b may differ
    for a, b in zip(wide, narrow):
        assert float((a - b).abs().max()) <= 2e-6 * float(b.abs().max())


# The same three statistics have a third route on bf16 layers (option memory_fold): 256 x 256 blocks with one register
# tile, phi(M_b) stored (first example of a group) or added (the others) to the output in memory at the end of every
# example.  Forced here on ragged shapes: one group and several, tiles cut by both edges of the layer, a single example
# (stores only), rows whose pitch is not a multiple of the tile.
@pytest.mark.parametrize("B,T,din,dout,max_split", [(5, 77, 520, 264, 1), (3, 100, 200, 192, 1), (7, 33, 256, 456, 3), (4, 64, 512, 1024, 32),
                                                    (1, 70, 264, 392, 1), (12, 24, 512, 200, 4), (2, 50, 96, 1160, 1)])
def test_examples_folded_in_memory(pex_option, B, T, din, dout, max_split):
    X, G = si.custom(B, T, din, dout, dtype="bf16", seed=B * 10 + T + 1)
    Xd, Gd = X.to(DEV), G.to(DEV)
    wts = torch.linspace(0.5, 1.5, B)
    pex_option("max_split", max_split)
    pex_option("memory_fold", 0)
    in_registers = (pex.pex_stat(Xd, Gd, "square").clone(), pex.pex_weighted_sum(Xd, Gd, wts.to(DEV)).clone(),
                    pex.pex_stat_power(Xd, Gd, 1.0).clone())
    pex_option("memory_fold", 2)
    need = pex.pex_stat_workspace_bytes(B, T, din, dout, pex.PEX_BF16, "square")
    assert need % (din * dout * 4) == 0 and need <= max_split * din * dout * 4 and (max_split > 1 or need == 0)
    # the outputs start from garbage: the first example of a group must store, not add
    S = [torch.full((din, dout), float("nan"), device=DEV) for _ in range(3)]
    pex.pex_stat(Xd, Gd, "square", S=S[0])
    pex.pex_weighted_sum(Xd, Gd, wts.to(DEV), S=S[1])
    pex.pex_stat_power(Xd, Gd, 1.0, S=S[2])
    again = pex.pex_stat(Xd, Gd, "square").clone()
    torch.cuda.synchronize()
    st = oracle.stat(si.widen(X), si.widen(G))
    f = lambda t: t.cpu().numpy().astype(np.float64)
    assert_real_stat(f(S[0]), st.S_sq, "bf16", "square folded in memory", elementwise=(B >= 3))
    M = np.einsum("bti,btj->bij", si.widen(X).astype(np.float64), si.widen(G).astype(np.float64))
    assert_real_stat(f(S[1]), (wts.double().numpy()[:, None, None] * M).sum(0), "bf16", "weighted sum folded in memory", elementwise=False)
    assert_real_stat(f(S[2]), np.abs(M).sum(0), "bf16", "|.|^1 folded in memory", elementwise=(B >= 3))
    assert torch.equal(again, S[0])                      # one owner per entry, examples in order: the same bits every time
    for a, b in zip(S, in_registers):
        assert float((a - b).abs().max()) <= 2e-6 * float(b.abs().max())


@pytest.mark.parametrize("B,expect_bytes", [(254, True), (256, False)])
def test_sign_partials_at_the_byte_limit(pex_option, B, expect_bytes):
    """Two groups of 127 examples exchange their sign counts as bytes (+-127 is the largest a byte holds), two groups of
    128 as fp32; all examples agree in sign, so every partial count sits at the limit."""
    pex_option("max_split", 2)
    T, din, dout = 64, 256, 248
    need = pex.pex_stat_workspace_bytes(B, T, din, dout, pex.PEX_BF16, "sign")
    assert need == (2 * 256 * 256 if expect_bytes else 2 * din * dout * 4)
    X = torch.ones(B, T, din, dtype=torch.bfloat16)
    G = torch.ones(B, T, dout, dtype=torch.bfloat16)
    G[:, :, 48:] = -1
    G[:, :, 95] = 0                                           # a column of exact zeros: sgn(0) = 0 through the bytes too
    S = pex.pex_stat(X.to(DEV), G.to(DEV), "sign").cpu()
    assert torch.equal(S[:, :48], torch.full((din, 48), float(B)))
    assert torch.equal(S[:, 48:95], torch.full((din, 47), -float(B)))
    assert torch.equal(S[:, 95], torch.zeros(din))
    assert torch.equal(S[:, 96:], torch.full((din, dout - 96), -float(B)))
