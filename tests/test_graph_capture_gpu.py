"""The entry points only enqueue kernels on the caller's stream (no allocation, no host synchronisation, no memset
nodes) when outputs and workspace are supplied, so a whole optimizer step can be captured into a HIP graph and
replayed.  Every replay is compared with the eager result, with eager work and synchronisations in between."""
import pytest
import torch

import paper_2510_00236_amd as pex
import synth_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_a_whole_step_replays_from_a_graph():
    B, T, din, dout, V = 6, 80, 328, 200, 500
    n = din * dout
    X, G = si.custom(B, T, din, dout, dtype="bf16", seed=3)
    Xd, Gd = X.to(DEV), G.to(DEV)
    ids = si.token_ids(B, T, V, seed=3).to(DEV)
    theta0, _, _ = si.optimizer_state(n, seed=3)
    prm = pex.AdamParams(lr=2e-3, beta1=0.9, beta2=0.95, eps=1e-8, eps_root=0.0, weight_decay=0.0,
                         grad_scale=1.0 / B, sq_scale=1.0 / B, step=1, B=B)
    mp = pex.MomentParams(beta2=0.95, grad_scale=1.0 / B, sq_scale=1.0 / B, B=B, debias=1, step=1)

    def buffers():
        d = dict(S_id=torch.empty(din, dout, device=DEV), S_sq=torch.empty(din, dout, device=DEV),
                 S_sg=torch.empty(din, dout, device=DEV), S_tk=torch.empty(din, dout, device=DEV),
                 theta=theta0.to(DEV), m=torch.zeros(n, device=DEV), v=torch.zeros(n, device=DEV),
                 ema_a=torch.zeros(n, device=DEV), ema_q=torch.zeros(n, device=DEV),
                 sums=torch.zeros(2, dtype=torch.float64, device=DEV), norms=torch.empty(B, device=DEV),
                 E_sq=torch.empty(V, din, device=DEV))
        ws = max(pex.pex_stat_multi_workspace_bytes(B, T, din, dout, pex.PEX_BF16, 7),
                 pex.pex_token_sq_workspace_bytes(B, T, din, dout, pex.PEX_BF16),
                 pex.pex_example_norms_workspace_bytes(B, T, din, dout, pex.PEX_BF16),
                 pex.pex_moment_track_workspace_bytes(n), pex.pex_embed_stat_workspace_bytes(B, T, V, din), 16)
        d["ws"] = torch.empty(ws, dtype=torch.uint8, device=DEV)
        return d

    def step(b):
        pex.pex_stat_multi(Xd, Gd, 7, out={"identity": b["S_id"], "square": b["S_sq"], "sign": b["S_sg"]}, workspace=b["ws"])
        pex.pex_token_sq(Xd, Gd, S=b["S_tk"], workspace=b["ws"])
        pex.pex_example_norms(Xd, Gd, N=b["norms"], workspace=b["ws"])
        pex.pex_embed_stat(ids, Xd, V, ("square",), out={"square": b["E_sq"]}, workspace=b["ws"])
        pex.pex_moment_track(b["ema_a"], b["ema_q"], b["S_id"].view(-1), b["S_sq"].view(-1), mp, sums=b["sums"], workspace=b["ws"])
        pex.pex_adam_update(b["theta"], b["m"], b["v"], b["S_id"].view(-1), b["S_sq"].view(-1), "microadam", prm)

    eager = buffers()
    for _ in range(3):
        step(eager)
    torch.cuda.synchronize()

    graphed = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):            # warm-up on the capture stream, then restore the state it touched
        step(graphed)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    fresh = buffers()
    for k in ("theta", "m", "v", "ema_a", "ema_q"):
        graphed[k].copy_(fresh[k])
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(graphed)
    for k in ("theta", "m", "v", "ema_a", "ema_q"):      # capture does not run anything, but be explicit
        graphed[k].copy_(fresh[k])
    torch.cuda.synchronize()
    reference = buffers()
    for replay in range(3):
        g.replay()
        torch.cuda.synchronize()
        step(reference)                       # the program's own eager work between the replays
        torch.cuda.synchronize()
        for k in ("S_id", "S_sq", "S_sg", "S_tk", "norms", "E_sq", "sums", "theta", "m", "v", "ema_a", "ema_q"):
            assert torch.equal(graphed[k], reference[k]), f"replay {replay}: {k} differs from the eager run"
    for k in ("theta", "m", "v", "S_sq", "E_sq"):
        assert torch.equal(graphed[k], eager[k]), k


def test_four_wave_contraction_is_deterministic_and_replays_from_a_graph(pex_option):
    """The plain contraction on its four-wave kernel (rows unsplit, so every workgroup runs the long loop): two eager
    runs agree bit for bit (no atomics, fixed order), and so do three replays of a captured launch, with eager work
    between them."""
    pex_option("max_split", 1)
    B, T, din, dout = 3, 701, 328, 520
    X, G = si.custom(B, T, din, dout, dtype="bf16", seed=11)
    Xd, Gd = X.to(DEV), G.to(DEV)
    ws = torch.empty(max(pex.pex_stat_workspace_bytes(B, T, din, dout, pex.PEX_BF16, "identity"), 16), dtype=torch.uint8, device=DEV)
    first = pex.pex_stat(Xd, Gd, "identity", workspace=ws).clone()
    second = pex.pex_stat(Xd, Gd, "identity", workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(first, second)

    S = torch.empty(din, dout, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pex.pex_stat(Xd, Gd, "identity", S=S, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pex.pex_stat(Xd, Gd, "identity", S=S, workspace=ws)
    for _ in range(3):
        S.fill_(-1.0)
        pex.pex_stat(Xd, Gd, "square", workspace=ws)      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(S, first)


def test_a_per_example_clipped_gradient_sum_replays_from_a_graph():
    """Norms of two layers -> clipping weights -> clipped gradient sums, all through the library, captured once and
    replayed three times with eager work in between: every replay equals the eager run bit for bit.  The statistic
    without a workspace argument (static scratch) is part of the captured work too."""
    B, T = 10, 64
    X1, G1 = si.custom(B, T, 264, 136, dtype="bf16", seed=41)
    X2, G2 = si.custom(B, T, 136, 520, dtype="bf16", seed=42)
    scale = torch.linspace(0.2, 3.0, B)[:, None, None]           # gradient norms from about 500 to 8000
    X1, X2 = (X1.float() * scale).to(torch.bfloat16), (X2.float() * scale).to(torch.bfloat16)
    d = [t.to(DEV) for t in (X1, G1, X2, G2)]
    shapes = [(264, 136), (136, 520)]

    def buffers():
        b = dict(N=torch.empty(2, B, device=DEV), w=torch.empty(B, device=DEV),
                 S=[torch.empty(*s, device=DEV) for s in shapes], Q=torch.empty(264, 136, device=DEV))
        nb = [max(pex.pex_example_norms_workspace_bytes(B, T, s[0], s[1], pex.PEX_BF16),
                  pex.pex_weighted_sum_workspace_bytes(B, T, s[0], s[1], pex.PEX_BF16), 16) for s in shapes]
        b["ws"] = [torch.empty(n, dtype=torch.uint8, device=DEV) for n in nb]
        return b

    def step(b):
        for l in range(2):
            pex.pex_example_norms(d[2 * l], d[2 * l + 1], N=b["N"][l], workspace=b["ws"][l])
        pex.pex_clip_weights(b["N"], 2600.0, w=b["w"])
        for l in range(2):
            pex.pex_weighted_sum(d[2 * l], d[2 * l + 1], b["w"], S=b["S"][l], workspace=b["ws"][l])
        pex.pex_stat_noalloc(d[0], d[1], "square", b["Q"])

    eager = buffers()
    step(eager)
    torch.cuda.synchronize()
    assert float(eager["w"].min()) < 1.0 and float(eager["w"].max()) == 1.0     # the threshold cuts some examples, not all

    graphed = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):            # first calls outside capture (the scratch address is looked up here)
        step(graphed)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(graphed)
    torch.cuda.synchronize()
    other = buffers()
    for replay in range(3):
        for t in (graphed["N"], graphed["w"], graphed["Q"], *graphed["S"]):
            t.fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        step(other)                           # the program's own eager work between the replays
        torch.cuda.synchronize()
        for k in ("N", "w", "Q"):
            assert torch.equal(graphed[k], eager[k]), f"replay {replay}: {k}"
        for l in range(2):
            assert torch.equal(graphed["S"][l], eager["S"][l]), f"replay {replay}: S[{l}]"
