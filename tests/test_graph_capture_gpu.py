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
