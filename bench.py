#!/usr/bin/env python3
"""Benchmark of the per-example gradient statistic hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input for the 1B-scale layer pair
(B=16, T=2048, 2048x8192 and 8192x2048, bf16): for each of the two layers
    S_id  = pex_stat(identity),  S_sq = pex_stat(square)  ->  pex_adam_update(MicroAdam)
    S_sgn = pex_stat(sign)                                 ->  pex_signsgd_update
    S_tok = pex_token_sq
Inputs are resident in HBM before the timed region.  `value` is the contraction work of the step
(2*B*T*din*dout FLOP per statistic) divided by the wall time of the step, in TFLOP/s.

Prints ONE JSON line.  `roofline` is measured live with HIP events around launches of the dominant kernel on
the stream it runs on.  The kernel that takes the largest share of the step (41 % in the kernel trace under
profiles/) is the plain 256 x 256-tile contraction: pex_stat(identity) launches it once per layer and
pex_token_sq launches it once more on the pre-squared operands; the events bracket the pex_stat(identity)
launches.  `square_roofline` reports phi = square (27 % of the step: its two contraction launches and the small
reduction between them) the same way, `sign_roofline` phi = sign (22 %).  `traffic` is not measured by this run: it
is the bytes beyond L2 per launch from the committed counter summary under profiles/ (FETCH_SIZE and WRITE_SIZE
runs of this very command, scaled by a copy of known size).  `configs` times every other workload shape per launch,
after the timed region.
`cpu_baseline` times the fp64 oracle on a bounded sample of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "per-example-stat TFLOP/s (Σ_b φ(X_bᵀG_b)) and % of MI355X MFMA peak"
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0

LAYER_SETS = {
    "c4_1b": ["c4_1b_up", "c4_1b_down"],
    "c5_long": ["c5_long"],
    "c3_gpt2": ["c3_gpt2_qkv", "c3_gpt2_proj", "c3_gpt2_fc", "c3_gpt2_fcproj"],
    "c2_mlp_in": ["c2_mlp_in"],
}


def measured_traffic(workload: str, which: str):
    """Bytes beyond L2 per launch of a contraction kernel (`which` = identity | square), from the committed
    rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size); None if no summary
    covers this workload."""
    path = os.path.join(ROOT, "profiles", f"stat_bf16_{workload}_pmc.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith(f"traffic_bytes_per_launch_{which}:"):
                    return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4_1b", choices=sorted(LAYER_SETS))
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-shared-step", action="store_true",
                    help="skip the informational step with shared contractions (profiling runs: the trace then "
                         "holds the headline step only)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="before the timed region, copy 1 GiB device to device once: a kernel of known traffic "
                         "against which the FETCH_SIZE / WRITE_SIZE counters of a profiling run are scaled")
    ap.add_argument("--no-probe", action="store_true",
                    help="skip the MFMA-only ceiling measurement (profiling runs: the trace then holds the step's kernels only)")
    ap.add_argument("--probe-only", choices=["gaussian", "zero"], default=None,
                    help="profiling aid: run nothing but the MFMA-only probe (operands drawn from N(0,1), or all zero) and "
                         "print its own small JSON line; with rocprofv3 --pmc SQ_BUSY_CU_CYCLES the cycles per compute unit "
                         "divided by the kernel's duration give the clock the chip sustains on those operands")
    ap.add_argument("--spin-up-seconds", type=float, default=0.3,
                    help="untimed work before the warm-up steps that brings the chip from idle to its running clocks")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the per-launch timing of the other workload shapes (profiling runs)")
    ap.add_argument("--extras", action="store_true",
                    help="after the timed region also time, per launch, the entry points outside the headline step "
                         "(vector parameters, norms, weighted sums, power, embedding table, moment tracking) on the "
                         "first layer's shapes; reported under \"extras\", not part of `value`")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (per-example statistics shard over the batch axis, "
              "one all-reduce of S per statistic; no multi-GPU path is built). Use --gpus 1.", file=sys.stderr)
        return 2

    import torch

    import paper_2510_00236_amd as pex
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libpex has no CPU path", file=sys.stderr)
        return 2
    pex.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.probe_only is not None:
        n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
        nel = pex.lib().pex_mfma_probe_operand_bytes() // 2
        ops = (torch.randn(nel, device=dev) if args.probe_only == "gaussian" else torch.zeros(nel, device=dev)).to(torch.bfloat16)
        iters = 1500
        _, sink = pex.pex_mfma_probe(ops, n_cu, iters)
        w0 = time.perf_counter()
        while time.perf_counter() - w0 < args.spin_up_seconds:
            pex.pex_mfma_probe(ops, n_cu, iters, sink=sink)
            torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.steps):
            flop, _ = pex.pex_mfma_probe(ops, n_cu, iters, sink=sink)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / args.steps
        print(json.dumps({"probe": "mfma_probe_kernel", "operands": args.probe_only, "launches": args.steps, "launch_ms": round(ms, 4),
                          "TFLOP/s": round(flop / (ms * 1e-3) / 1e12, 1), "frac_of_bf16_peak": round(flop / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                          "compute_units": n_cu}))
        return 0

    layers = []
    for name in LAYER_SETS[args.workload]:
        w = si.WORKLOADS[name]
        X, G = si.make(w, seed=args.seed)
        n = w.din * w.dout
        theta, m, v = si.optimizer_state(n, seed=args.seed)
        L = dict(w=w, X=X.to(dev), G=G.to(dev), n=n,
                 theta=theta.to(dev), m=m.to(dev), v=v.to(dev),
                 theta_s=theta.to(dev), m_s=torch.zeros(n, device=dev),
                 S_id=torch.empty(w.din, w.dout, device=dev), S_sq=torch.empty(w.din, w.dout, device=dev),
                 S_sg=torch.empty(w.din, w.dout, device=dev), S_tk=torch.empty(w.din, w.dout, device=dev))
        ws = max(pex.pex_stat_workspace_bytes(w.B, w.T, w.din, w.dout, pex.PEX_BF16, p) for p in ("identity", "square", "sign"))
        ws = max(ws, pex.pex_token_sq_workspace_bytes(w.B, w.T, w.din, w.dout, pex.PEX_BF16))
        L["ws"] = torch.empty(max(ws, 16), dtype=torch.uint8, device=dev)
        L["keep_cpu"] = (X, G) if name == LAYER_SETS[args.workload][0] else None
        layers.append(L)
    torch.cuda.synchronize()

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    id_events = []          # (start, stop) around every launch of the plain contraction by pex_stat(identity)
    sq_events = []          # ... of the phi = square contraction
    upd_events = []
    sgn_events = []         # ... of the MicroSignSGD update
    sc_events = []          # ... of the phi = sign contraction
    tk_events = []          # ... of the per-token square (both squaring passes and the contraction)

    def step(t: int, record: bool):
        for L in layers:
            w = L["w"]
            if record:
                i0, i1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                i0.record()
            pex.pex_stat(L["X"], L["G"], "identity", S=L["S_id"], workspace=L["ws"])
            if record:
                i1.record()
                id_events.append((i0, i1, w))
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            pex.pex_stat(L["X"], L["G"], "square", S=L["S_sq"], workspace=L["ws"])
            if record:
                e1.record()
                sq_events.append((e0, e1, w))
            p = pex.AdamParams(lr=2.0 / 1024, beta1=0.9, beta2=0.95, eps=1e-8, eps_root=0.0, weight_decay=0.0,
                               grad_scale=1.0 / w.B, sq_scale=1.0 / w.B, step=t, B=w.B)
            if record:
                u0, u1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                u0.record()
            pex.pex_adam_update(L["theta"], L["m"], L["v"], L["S_id"].view(-1), L["S_sq"].view(-1), "microadam", p)
            if record:
                u1.record()
                upd_events.append((u0, u1, w))
            if record:
                s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                s0.record()
            pex.pex_stat(L["X"], L["G"], "sign", S=L["S_sg"], workspace=L["ws"])
            if record:
                s1.record()
                sc_events.append((s0, s1, w))
                g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                g0.record()
            pex.pex_signsgd_update(L["theta_s"], L["m_s"], L["S_sg"].view(-1), 3.47e-3, 0.9, 0.0, w.B, False, t)
            if record:
                g1.record()
                sgn_events.append((g0, g1, w))
            if record:
                k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                k0.record()
            pex.pex_token_sq(L["X"], L["G"], S=L["S_tk"], workspace=L["ws"])
            if record:
                k1.record()
                tk_events.append((k0, k1, w))

    # The chip has idled while the host drew the inputs (many seconds) and needs some tens of milliseconds of work to
    # come back to its running clocks: spin it up on the step itself before the W warm-up steps, outside every count.
    spin_up_steps = 0
    s0 = time.perf_counter()
    while time.perf_counter() - s0 < args.spin_up_seconds:
        step(1, False)
        torch.cuda.synchronize()
        spin_up_steps += 1
    for t in range(1, args.warmup + 1):
        step(t, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.warmup + 1, args.warmup + args.steps + 1):
        step(t, True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # ---- for information, outside the timed region: the same outputs with identity, square and sign taken from
    # one contraction (pex_stat_multi).  Not part of `value`: the metric counts one contraction per statistic.
    def multi_step(t: int):
        for L in layers:
            w = L["w"]
            pex.pex_stat_multi(L["X"], L["G"], ("identity", "square", "sign"),
                               out={"identity": L["S_id"], "square": L["S_sq"], "sign": L["S_sg"]}, workspace=L["ws_multi"])
            p = pex.AdamParams(lr=2.0 / 1024, beta1=0.9, beta2=0.95, eps=1e-8, eps_root=0.0, weight_decay=0.0,
                               grad_scale=1.0 / w.B, sq_scale=1.0 / w.B, step=t, B=w.B)
            pex.pex_adam_update(L["theta"], L["m"], L["v"], L["S_id"].view(-1), L["S_sq"].view(-1), "microadam", p)
            pex.pex_signsgd_update(L["theta_s"], L["m_s"], L["S_sg"].view(-1), 3.47e-3, 0.9, 0.0, w.B, False, t)
            pex.pex_token_sq(L["X"], L["G"], S=L["S_tk"], workspace=L["ws"])

    for L in layers:
        w = L["w"]
        nb = pex.pex_stat_multi_workspace_bytes(w.B, w.T, w.din, w.dout, pex.PEX_BF16, ("identity", "square", "sign"))
        L["ws_multi"] = torch.empty(max(nb, 16), dtype=torch.uint8, device=dev)
    t_last = args.warmup + args.steps
    multi_ms = None
    if not args.no_shared_step:
        multi_step(t_last + 1)
        torch.cuda.synchronize()
        m0 = time.perf_counter()
        for t in range(t_last + 2, t_last + 2 + args.steps):
            multi_step(t)
        torch.cuda.synchronize()
        multi_ms = (time.perf_counter() - m0) / args.steps * 1e3

    # ---- what the MFMA pipes sustain with nothing else going on (same register shape, Gaussian operands like X):
    # the contraction kernels are reported against this measured ceiling beside the datasheet peak
    n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
    ceiling, probe_ms = None, None
    if not args.no_probe:
        probe_ops = torch.randn(pex.lib().pex_mfma_probe_operand_bytes() // 2, device=dev).to(torch.bfloat16)
        probe_iters = 1500
        _, probe_sink = pex.pex_mfma_probe(probe_ops, n_cu, probe_iters)
        for _ in range(3):
            pex.pex_mfma_probe(probe_ops, n_cu, probe_iters, sink=probe_sink)
        torch.cuda.synchronize()
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        probe_reps = 10
        p0.record()
        for _ in range(probe_reps):
            probe_flop, _ = pex.pex_mfma_probe(probe_ops, n_cu, probe_iters, sink=probe_sink)
        p1.record()
        torch.cuda.synchronize()
        probe_ms = p0.elapsed_time(p1) / probe_reps
        ceiling = probe_flop / (probe_ms * 1e-3) / 1e12

    # ---- for information: the other entry points, one at a time, on the first layer's shapes
    extras = None
    if args.extras:
        L = layers[0]
        w = L["w"]
        X, G = L["X"], L["G"]
        flop = 2.0 * w.B * w.T * w.din * w.dout
        n = w.din * w.dout
        V = 32000                                  # vocabulary of the 1.2B model's tokenizer class; embedding width = din
        ids = si.token_ids(w.B, w.T, V, seed=args.seed).to(dev)
        Ge = X                                     # cotangents of the looked-up vectors: [B, T, din] bf16
        wts = torch.linspace(0.25, 1.0, w.B, device=dev)
        ema_a, ema_q = torch.zeros(n, device=dev), torch.zeros(n, device=dev)
        mp = pex.MomentParams(beta2=0.95, grad_scale=1.0 / w.B, sq_scale=1.0 / w.B, B=w.B, debias=1, step=1)
        emb_out = {k: torch.empty(V, w.din, device=dev) for k in ("identity", "square")}
        el = 2                                     # bytes per bf16 element

        def timed(fn, reps=5):
            for _ in range(10):         # fresh buffers: the first launches on new memory run slower
                fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        def entry(ms, flops=None, nbytes=None):
            e = {"ms": round(ms, 4)}
            if flops is not None:
                e["TFLOP/s"] = round(flops / (ms * 1e-3) / 1e12, 1)
            if nbytes is not None:
                e["GB/s"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
            return e

        extras = {"shapes": {"B": w.B, "T": w.T, "din": w.din, "dout": w.dout, "V": V}}
        extras["pex_stat_multi(identity,square)"] = entry(timed(lambda: pex.pex_stat_multi(X, G, ("identity", "square"))), flops=flop)
        extras["pex_stat_multi(identity,square,sign)"] = entry(timed(lambda: pex.pex_stat_multi(X, G, ("identity", "square", "sign"))), flops=flop)
        extras["pex_example_norms"] = entry(timed(lambda: pex.pex_example_norms(X, G)), flops=flop)
        extras["pex_weighted_sum"] = entry(timed(lambda: pex.pex_weighted_sum(X, G, wts)), flops=flop)
        extras["pex_stat_power(alpha=1.5)"] = entry(timed(lambda: pex.pex_stat_power(X, G, 1.5)), flops=flop)
        extras["pex_token_norms"] = entry(timed(lambda: pex.pex_token_norms(X, G)), nbytes=w.B * w.T * (w.din + w.dout) * el)
        extras["pex_vec_stat(offset of dout)"] = entry(timed(lambda: pex.pex_vec_stat(G, None, ("identity", "square", "sign"))),
                                                       nbytes=w.B * w.T * w.dout * el)
        extras["pex_embed_stat(identity,square)"] = entry(
            timed(lambda: pex.pex_embed_stat(ids, Ge, V, ("identity", "square"), out=emb_out)),
            nbytes=w.B * w.T * w.din * el + 2 * V * w.din * 4 + w.B * w.T * 8)
        extras["pex_moment_track"] = entry(timed(lambda: pex.pex_moment_track(ema_a, ema_q, L["S_id"].view(-1), L["S_sq"].view(-1), mp)),
                                           nbytes=24.0 * n)
        extras["pex_sign_update(signema)"] = entry(
            timed(lambda: pex.pex_sign_update(L["theta_s"], L["m_s"], L["S_id"].view(-1), "signema", 3.47e-3, 0.9, 0.0, w.B)),
            nbytes=20.0 * n)
        del ids, emb_out, ema_a, ema_q

    # ---- the other workload shapes, per launch, after the timed region.  Not part of `value`: the headline stays on
    # the 1B-scale layer pair.  Every statistic is timed alone with events on the launch stream, a quarter of a second of
    # warm-up launches and `reps` timed ones; layers whose inputs fit the 256 MB memory-side cache alternate between two sets of
    # input buffers so that cache residency does not flatter them.
    configs = None
    if not args.no_configs:
        configs = {}
        others = [n for k, names in LAYER_SETS.items() if k != args.workload for n in names]
        for name in sorted(others):
            w = si.WORKLOADS[name]
            in_bytes = w.B * w.T * (w.din + w.dout) * 2
            nsets = 2 if in_bytes < (256 << 20) else 1
            sets = []
            for k in range(nsets):
                Xc, Gc = si.make(w, seed=args.seed + 17 * k)
                sets.append((Xc.to(dev), Gc.to(dev)))
            S = torch.empty(w.din, w.dout, device=dev)
            nb = max(pex.pex_stat_workspace_bytes(w.B, w.T, w.din, w.dout, pex.PEX_BF16, p) for p in ("identity", "square", "sign"))
            nb = max(nb, pex.pex_token_sq_workspace_bytes(w.B, w.T, w.din, w.dout, pex.PEX_BF16), 16)
            wsc = torch.empty(nb, dtype=torch.uint8, device=dev)
            flop = 2.0 * w.B * w.T * w.din * w.dout
            reps = 20 if flop < 5e11 else 10

            def per_launch(fn):
                # The chip idles while the host draws the inputs and takes some tens of milliseconds of work to come
                # back to its running clocks: warm up for a quarter of a second, not for a fixed number of launches.
                w0, k = time.perf_counter(), 0
                while k < 10 or time.perf_counter() - w0 < 0.25:
                    fn(*sets[k % nsets])
                    k += 1
                    if k % 10 == 0:
                        torch.cuda.synchronize()
                torch.cuda.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for k in range(reps):
                    fn(*sets[k % nsets])
                b.record()
                torch.cuda.synchronize()
                return a.elapsed_time(b) / reps

            c = {"B": w.B, "T": w.T, "din": w.din, "dout": w.dout, "flop_per_statistic": flop,
                 "input_buffer_sets": nsets, "launches_timed": reps}
            for phi in ("identity", "square", "sign"):
                ms = per_launch(lambda Xc, Gc, phi=phi: pex.pex_stat(Xc, Gc, phi, S=S, workspace=wsc))
                c[phi] = {"us": round(ms * 1e3, 1), "TFLOP/s": round(flop / (ms * 1e-3) / 1e12, 1),
                          "frac_of_bf16_peak": round(flop / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
            ms = per_launch(lambda Xc, Gc: pex.pex_token_sq(Xc, Gc, S=S, workspace=wsc))
            c["token_sq"] = {"us": round(ms * 1e3, 1), "TFLOP/s": round(flop / (ms * 1e-3) / 1e12, 1),
                             "frac_of_bf16_peak": round(flop / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
            if name == "c2_mlp_in":      # this workload names the MicroAdam update over its 512 x 2048 parameters
                n = w.din * w.dout
                th, mm, vv = (t.to(dev) for t in si.optimizer_state(n, seed=args.seed))
                Sa, Sq = torch.randn(n, device=dev), torch.rand(n, device=dev) + 1.0
                pp = pex.AdamParams(lr=2.0 / 1024, beta1=0.9, beta2=0.95, eps=1e-8, eps_root=0.0, weight_decay=0.0,
                                    grad_scale=1.0 / w.B, sq_scale=1.0 / w.B, step=1, B=w.B)
                ms = per_launch(lambda Xc, Gc: pex.pex_adam_update(th, mm, vv, Sa, Sq, "microadam", pp))
                c["microadam_update"] = {"us": round(ms * 1e3, 1), "GB/s": round(32.0 * n / (ms * 1e-3) / 1e9, 1),
                                         "frac_of_hbm_peak": round(32.0 * n / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
            configs[name] = c
            del sets, S, wsc
        torch.cuda.empty_cache()

    flop_per_stat = [2.0 * L["w"].B * L["w"].T * L["w"].din * L["w"].dout for L in layers]
    flop_per_step = 4.0 * sum(flop_per_stat)          # identity, square, sign, per-token square
    ms_per_step = elapsed / args.steps * 1e3
    value = flop_per_step / (elapsed / args.steps) / 1e12

    # ---- rooflines of the contraction kernels, per launch
    def contraction_roofline(events, kernel, which):
        ms = [a.elapsed_time(b) for a, b, _ in events]
        flop = [2.0 * w.B * w.T * w.din * w.dout for _, _, w in events]
        avg_ms = sum(ms) / len(ms)
        achieved = (sum(flop) / len(flop)) / (avg_ms * 1e-3) / 1e12
        return {"bound": "mfma", "kernel": kernel, "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "frac_of_measured_mfma_ceiling": None if ceiling is None else round(achieved / ceiling, 4), "avg_launch_ms": round(avg_ms, 4),
                "launches": len(ms), "traffic": measured_traffic(args.workload, which)}

    roofline = contraction_roofline(id_events, "stat_bf16_quad_kernel (256x256 tile, four waves of 128x128; pex_stat phi=identity; also "
                                               "the contraction inside pex_token_sq)", "identity")
    square_roofline = contraction_roofline(sq_events, "pex_stat phi=square as a whole: stat_bf16_kernel<256x192 tile, square> on the columns that fill one "
                                                      "round of 256 workgroups, stat_bf16_kernel<256x128 tile, square> on the rest in two groups of "
                                                      "examples, reduce_partials_cols_kernel", "square")
    sign_roofline = contraction_roofline(sc_events, "stat_bf16_kernel<256x256 tile, sign with packed counts> (pex_stat phi=sign)", "sign")
    token_roofline = contraction_roofline(tk_events, "pex_token_sq as a whole: square_bf16_kernel on X and on G, then stat_bf16_quad_kernel "
                                                     "on the copies; FLOP of the contraction only", "token")
    upd_ms = [a.elapsed_time(b) for a, b, _ in upd_events]
    upd_bytes = [32.0 * w.din * w.dout for _, _, w in upd_events]
    upd_gbs = (sum(upd_bytes) / len(upd_bytes)) / (sum(upd_ms) / len(upd_ms) * 1e-3) / 1e9
    update_roofline = {"bound": "hbm", "kernel": "adam_update_kernel<microadam>", "achieved": round(upd_gbs, 1),
                       "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(upd_gbs / PEAK_HBM_GBS, 4),
                       "avg_launch_ms": round(sum(upd_ms) / len(upd_ms), 4)}

    sgn_ms = [a.elapsed_time(b) for a, b, _ in sgn_events]
    sgn_gbs = (sum(20.0 * w.din * w.dout for _, _, w in sgn_events) / len(sgn_events)) / (sum(sgn_ms) / len(sgn_ms) * 1e-3) / 1e9
    sign_update_roofline = {"bound": "hbm", "kernel": "signsgd_update_kernel<microsignsgd>", "achieved": round(sgn_gbs, 1),
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(sgn_gbs / PEAK_HBM_GBS, 4),
                            "avg_launch_ms": round(sum(sgn_ms) / len(sgn_ms), 4)}

    # ---- CPU baseline: the fp64 oracle as it stands, on a bounded sample of the first layer
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        X, G = layers[0]["keep_cpu"]
        w = layers[0]["w"]
        per_example = 2.0 * w.T * w.din * w.dout
        # pilot on a thin slice to learn this host's rate, then size the sample for ~cpu_seconds of work
        pr = min(w.din, 128)
        Xp, Gp = si.widen(X[:1, :, :pr]), si.widen(G[:1])
        c0 = time.perf_counter()
        oracle.stat(Xp, Gp)
        rate = 2.0 * w.T * pr * w.dout / (time.perf_counter() - c0)
        budget = args.cpu_seconds * rate
        nb = max(1, min(w.B, int(budget / per_example)))
        rows = w.din
        if nb == 1 and per_example > 2 * budget:
            rows = max(64, int(w.din * budget / per_example) // 64 * 64)
        Xs, Gs = si.widen(X[:nb, :, :rows]), si.widen(G[:nb])
        c0 = time.perf_counter()
        oracle.stat(Xs, Gs)
        cs = time.perf_counter() - c0
        cpu = {"value": round(2.0 * nb * w.T * rows * w.dout / cs / 1e12, 6), "unit": "TFLOP/s",
               "cores": oracle.num_threads(), "kind": "oracle", "seconds": round(cs, 2),
               "sample": f"{w.name}: first {nb} of {w.B} examples, {rows} of {w.din} rows of S, all three phi in "
                         f"one fp64 pass (identity, square, sign)"}

    out = {
        "metric": METRIC, "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "spin_up_steps": spin_up_steps, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "pct_of_bf16_mfma_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "config": {"workload": args.workload, "layers": [L["w"].name for L in layers],
                   "B": layers[0]["w"].B, "T": layers[0]["w"].T,
                   "shapes": [[L["w"].din, L["w"].dout] for L in layers],
                   "step": "per layer: pex_stat identity+square -> MicroAdam update; pex_stat sign -> MicroSignSGD update; pex_token_sq",
                   "flop_per_step": flop_per_step, "seed": args.seed},
        "roofline": roofline, "square_roofline": square_roofline, "sign_roofline": sign_roofline,
        "token_roofline": token_roofline, "update_roofline": update_roofline,
        "sign_update_roofline": sign_update_roofline,
        "mfma_only_ceiling": None if ceiling is None else {
            "achieved": round(ceiling, 1), "unit": "TFLOP/s", "frac_of_peak": round(ceiling / PEAK_BF16_TFLOPS, 4),
            "kernel": "mfma_probe_kernel: nothing but v_mfma_f32_16x16x32_bf16, 8 waves on each of "
                      f"{n_cu} compute units, Gaussian operands", "launch_ms": round(probe_ms, 4)},
        "cpu_baseline": cpu,
        "shared_contraction_step": None if multi_ms is None else {"ms_per_step": round(multi_ms, 4),
                                    "note": "same outputs with identity, square and sign from one contraction per layer "
                                            "(pex_stat_multi); informational, not used in value"},
    }
    if configs is not None:
        out["configs"] = configs
    if extras is not None:
        out["extras"] = extras
    print(json.dumps(out, ensure_ascii=False))
    return 0


if __name__ == "__main__":
    sys.exit(main())
