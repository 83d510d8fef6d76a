#!/usr/bin/env python3
"""Benchmark of the M2RNN scan hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3]

One "step" is one pass of the whole hot path over one batch of synthetic
input: m2rnn_fwd (writing checkpoints) followed by m2rnn_bwd, both through the
C ABI, inputs resident in HBM before the timed region.  Prints ONE JSON line:
tokens/s (tokens = B*T per step), the roofline object of the dominant kernel
(the backward scan) and the float64 oracle timed on the host cores.

The roofline is the vector-ALU one (tanh and gating bind this path, not the
matrix cores or HBM): algorithmic lane-operations per element-step, with a
transcendental counted as two issue slots (measured half rate on gfx950),
against 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-op/s.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Algorithmic vector-ALU work per state element per time step, (plain fp32 ops, transcendental
# ops).  Forward: k.v FMA, 1 + e, gate FMAs, readout, convert = 7, plus exp2 and rcp of the
# tanh.  Backward given H_{t-1}: recompute 3, dq 1, G 1, df 2, dS 3, carry 1, dk + dv 2,
# converts 1 = 14, plus exp2 and rcp.  The chunk recompute of the backward is not counted.
ALU_OPS = {"fwd": (7, 2), "bwd": (14, 2)}
TRANS_SLOTS = 2                       # issue slots of v_exp_f32 / v_rcp_f32 relative to v_fma_f32
PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9  # lane-ops per second, packed fp32 not used

# HBM bytes per launch of the dominant kernel (the backward scan kernel; the forward one for
# forward-only workloads), from two rocprofv3 --pmc runs of this script (FETCH_SIZE, then
# WRITE_SIZE, in KiB; each scaled by what the same counter reads for the --calib-copy-mib
# copy).  These are figures of the profiled runs whose summaries are named here, not of the
# run that prints them: (fetch KiB, fetch scale, write KiB, write scale, summary file).
MEASURED_TRAFFIC = {
    "C3": (420591, 2.000, 437767, 1.000, "profiles/c3_fwd_bwd_pmc_counters.txt"),
    "C4": (738301, 2.000, 1358613, 1.000, "profiles/c4_fwd_bwd_pmc_counters.txt"),
    "C5": (426252, 2.000, 2097664, 1.000, "profiles/c5_fwd_pmc_counters.txt"),
    "P1": (776987, 2.000, 1551132, 1.000, "profiles/p1_fwd_bwd_pmc_counters.txt"),
    "R1": (424524, 2.000, 504935, 1.000, "profiles/r1_fwd_bwd_pmc_counters.txt"),
}

MFMA_PEAK = 2.5e15   # dense fp16 / bf16 flop/s
HBM_PEAK = 8.0e12    # bytes/s


def algorithmic_bytes(wl, chunk, kind):
    """HBM bytes the method itself must move per call: the per-step vectors of every
    (b, n) unit-step (q, k, v, f in, y out; for the backward also dy in and dq, dk, dv, df
    out) plus one fp32 checkpoint per chunk and unit (written by the forward, read by the
    backward).  W, H0, H_T, dW, dH0 are per launch and negligible."""
    io = 2 if wl.io == "bf16" else 4
    unit_steps = wl.B * wl.N * wl.T
    ck = wl.B * wl.N * -(-wl.T // chunk) * wl.K * wl.V * 4 if wl.backward else 0
    if kind == "fwd":
        return unit_steps * ((2 * wl.K + 2 * wl.V) * io + 4) + ck
    return unit_steps * ((2 * wl.K + 2 * wl.V) * io + (2 * wl.K + wl.V) * io + 8) + ck


def alu_slots(kind):
    v, t = ALU_OPS[kind]
    return v + TRANS_SLOTS * t


def cpu_baseline(wl, inp):
    """The float64 oracle, as it stands, on a bounded sample of the workload
    (about 15 s of CPU work): whole (batch, head) recurrences of the first few
    heads, at full T where one head fits the budget."""
    import oracle
    from paper_2603_14360_amd.synth_inputs import select_heads
    threads = oracle.num_threads()
    # size the sample for roughly 15 s.  The oracle runs one (batch, head) recurrence per
    # thread, so the sample is a whole number of "rounds" of `threads` recurrences; if one
    # recurrence alone takes longer than ~25 s, a prefix of the sequence is used
    per_unit = lambda T: T * wl.K * wl.V * wl.V * (10 if wl.backward else 3) / 4e9   # seconds
    T = wl.T
    while per_unit(T) > 25.0 and T > 256:
        T //= 2
    rounds = max(1, int(15.0 // max(per_unit(T), 1e-9)))
    heads = int(max(1, min(wl.N, (rounds * max(1, threads)) // wl.B)))
    sub = select_heads(inp, list(range(heads)))
    for n in ("q", "k", "v", "f", "dy"):
        sub[n] = sub[n][:, :T]
    args = [sub[n] for n in ("q", "k", "v", "f", "W")]
    t0 = time.perf_counter()
    oracle.fwd(*args, sub["H0"])
    if wl.backward:
        oracle.bwd(*args, sub["H0"], sub["dy"], sub["dHT"])
    dt = time.perf_counter() - t0
    tokens_equiv = wl.B * T * heads / wl.N   # tokens span all N heads
    return {"value": tokens_equiv / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d of %d heads x all %d batch rows, T=%d of %d, fwd%s, %.1f s wall; "
                      "tokens scaled by heads/N" % (heads, wl.N, wl.B, T, wl.T,
                                                    "+bwd" if wl.backward else "", dt)}


def decode_latency():
    """One decode step (m2rnn_fwd with T = 1, state handed from call to call): microseconds per
    call issued eagerly and per step inside a replayed HIP graph of 16 steps."""
    import torch
    from paper_2603_14360_amd import binding as mb
    rows = []
    for (B, N, Nqk, K, V) in [(1, 16, 16, 64, 64), (8, 84, 1, 64, 16), (256, 16, 16, 64, 64)]:
        d = mb.make_desc(B, 1, N, K, V, mb.M2RNN_BF16, Nqk=Nqk)
        q = (torch.randn(B, 1, Nqk, K, device="cuda") * 0.125).bfloat16()
        k = (torch.randn(B, 1, Nqk, K, device="cuda") * 0.125).bfloat16()
        v = (torch.randn(B, 1, N, V, device="cuda") * 0.125).bfloat16()
        f = torch.rand(B, 1, N, device="cuda")
        W = (torch.randn(N, V, V, device="cuda") / V ** 0.5).bfloat16()
        H = [torch.randn(B, N, K, V, device="cuda") * 0.1, torch.empty(B, N, K, V, device="cuda")]
        y = torch.empty(B, 1, N, V, device="cuda", dtype=torch.bfloat16)
        ws = torch.empty(max(256, mb.m2rnn_workspace_bytes(d, 0)), dtype=torch.uint8, device="cuda")

        def step(i, stream):
            mb.m2rnn_fwd(d, q, k, v, f, W, H[i & 1], y, H[(i + 1) & 1], None, ws, stream=stream)
        st = torch.cuda.current_stream().cuda_stream
        for i in range(20):
            step(i, st)
        torch.cuda.synchronize()
        n = 2000
        t0 = time.perf_counter()
        for i in range(n):
            step(i, st)
        torch.cuda.synchronize()
        eager = (time.perf_counter() - t0) / n * 1e6
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for i in range(4):
                step(i, side.cuda_stream)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for i in range(16):
                step(i, torch.cuda.current_stream().cuda_stream)
        for _ in range(5):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(200):
            g.replay()
        torch.cuda.synchronize()
        graph = (time.perf_counter() - t0) / (200 * 16) * 1e6
        rows.append({"states": B * N, "K": K, "V": V, "route": mb.m2rnn_route_string(d, 0),
                     "eager_us_per_call": round(eager, 2), "graph_us_per_step": round(graph, 2),
                     "state_traffic_GBps_in_graph": round(2 * B * N * K * V * 4 / (graph * 1e-6) / 1e9, 1)})
    return rows


def block_kernels_bandwidth():
    """The scan's neighbours in the block at the C3 layer width (1024 channels): algorithmic
    HBM bytes (each tensor once) over the HIP-event time of the call, against 8 TB/s."""
    import numpy as np
    import torch
    from paper_2603_14360_amd import binding as mb
    B, T, C = 8, 4096, 1024
    bf = torch.bfloat16
    x = torch.randn(B, T, C, device="cuda").to(bf)
    a = torch.randn(B, T, C, device="cuda").to(bf)
    d = torch.randn(B, T, C, device="cuda").to(bf)
    w4 = (torch.randn(C, 4, device="cuda") * 0.5).to(bf)
    bias = torch.randn(C, device="cuda").to(bf)
    wn = torch.rand(C, device="cuda").to(bf)
    o1, o2 = torch.empty_like(x), torch.empty_like(x)
    dw4, db = torch.empty(C, 4, device="cuda"), torch.empty(C, device="cuda")
    dwn, sc = torch.empty(C, device="cuda"), torch.empty(B, T, device="cuda")
    ws = torch.empty(max(mb.m2rnn_conv_silu_workspace_bytes(B, T, C),
                         mb.m2rnn_gated_rmsnorm_workspace_bytes(B, T, C), 256), dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    n = B * T * C * 2   # bytes of one bf16 activation tensor
    calls = {
        "conv_silu_fwd": (lambda: mb.m2rnn_conv_silu_fwd(x, w4, bias, o1, stream=st), 2 * n),
        "conv_silu_bwd": (lambda: mb.m2rnn_conv_silu_bwd(x, w4, bias, d, o1, dw4, db, ws, stream=st), 3 * n),
        "gated_rmsnorm_fwd": (lambda: mb.m2rnn_gated_rmsnorm_fwd(x, a, wn, 1e-5, o1, sc, stream=st), 3 * n),
        "gated_rmsnorm_bwd": (lambda: mb.m2rnn_gated_rmsnorm_bwd(x, a, wn, 1e-5, sc, d, o1, o2, dwn, ws, stream=st), 5 * n),
    }
    out = {}
    for name, (fn, nbytes) in calls.items():
        for _ in range(3):
            fn()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        for e0, e1 in ev:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in ev]))
        out[name] = {"ms": round(ms, 4), "algorithmic_GB": round(nbytes / 1e9, 3),
                     "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1), "hbm_frac": round(nbytes / (ms * 1e-3) / HBM_PEAK, 3)}
    return {"shape": "B=%d T=%d C=D=%d bf16" % (B, T, C), "kernels": out}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", action="store_true",
                    help="instead of the headline line, print one JSON line with the decode-step "
                         "latency and the bandwidth of the block's neighbour kernels")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run a plain elementwise copy of this many MiB (read) + as many "
                         "(write) three times before the warm-up: the yardstick that scales "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the scan has no multi-GPU path); "
                 "--gpus %d is not supported" % args.gpus)

    import numpy as np
    import torch
    from paper_2603_14360_amd import binding as mb
    from paper_2603_14360_amd.synth_inputs import WORKLOADS, make_inputs

    mb.lib()  # fail loudly when the HIP library is missing
    if args.extras:
        print(json.dumps({"decode_step_latency": decode_latency(),
                          "block_neighbours": block_kernels_bandwidth()}))
        return
    wl = WORKLOADS[args.workload]
    inp = make_inputs(wl)
    io_dt = torch.bfloat16 if wl.io == "bf16" else torch.float32
    dev = {}
    for n in ("q", "k", "v", "W", "dy"):
        dev[n] = torch.from_numpy(inp[n]).to("cuda").to(io_dt)
    dev["f"] = torch.from_numpy(inp["f"]).to("cuda")
    for n in ("H0", "dHT"):
        dev[n] = None if inp[n] is None else torch.from_numpy(inp[n]).to("cuda")
    scan = mb.Scan(wl.B, wl.T, wl.N, wl.K, wl.V, wl.io, Nqk=(wl.Nqk or None), backward=wl.backward)

    def step():
        scan.fwd(dev["q"], dev["k"], dev["v"], dev["f"], dev["W"], dev["H0"])
        if wl.backward:
            scan.bwd(dev["q"], dev["k"], dev["v"], dev["f"], dev["W"], dev["H0"], dev["dy"],
                     dev["dHT"])

    if args.calib_copy_mib > 0:
        src = torch.ones(args.calib_copy_mib * (1 << 20) // 4, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # HIP events on the stream the library launches on (torch's current stream)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        scan.fwd(dev["q"], dev["k"], dev["v"], dev["f"], dev["W"], dev["H0"])
        ev[i][1].record()
        if wl.backward:
            scan.bwd(dev["q"], dev["k"], dev["v"], dev["f"], dev["W"], dev["H0"], dev["dy"],
                     dev["dHT"])
        ev[i][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    fwd_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    bwd_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in ev])) if wl.backward else 0.0

    ms_per_step = wall * 1e3 / args.steps
    tokens = wl.B * wl.T
    elem_steps = wl.B * wl.N * wl.T * wl.K * wl.V
    dom = "bwd" if wl.backward else "fwd"
    dom_ms = bwd_ms if wl.backward else fwd_ms
    achieved = elem_steps * alu_slots(dom) / (dom_ms * 1e-3)
    step_slots = alu_slots("fwd") + (alu_slots("bwd") if wl.backward else 0)
    chunk = mb.m2rnn_default_chunk(scan.desc)
    mfma_flops = elem_steps * wl.V * (2 + (6 if wl.backward else 0))
    alg_bytes = algorithmic_bytes(wl, chunk, "fwd") + (algorithmic_bytes(wl, chunk, "bwd") if wl.backward else 0)
    traffic = traffic_source = None
    if wl.name in MEASURED_TRAFFIC:
        fk, fs, wk, ws_, src = MEASURED_TRAFFIC[wl.name]
        traffic = (fk * fs + wk * ws_) * 1024.0
        traffic_source = src + " (a profiled run of this command, not this run)"
    out = {
        "metric": "M2RNN fwd+bwd tokens/s on 1 MI355X" if wl.backward else "M2RNN fwd tokens/s on 1 MI355X",
        "value": tokens / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 state, f16 matrix-core operands, bf16 io" if wl.io == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": "%s: B=%d N=%d%s K=%d V=%d T=%d %s io, fwd%s" % (
            wl.name, wl.B, wl.N, " (Nqk=%d)" % wl.Nqk if wl.Nqk else "", wl.K, wl.V, wl.T, wl.io,
            "+bwd" if wl.backward else ""),
            "tokens_per_step": tokens, "chunk": chunk,
            "routes": [mb.m2rnn_route_string(scan.desc, 0)] + ([mb.m2rnn_route_string(scan.desc, 1)] if wl.backward else [])},
        "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
        "roofline": {
            "bound": "alu",
            "kernel": "m2rnn_%s call: the %s scan kernel and its ordered-sum epilogues (the scan "
                      "kernel alone is ~98 %% of it: profiles/)" % (dom, "backward" if wl.backward else "forward"),
            "achieved": achieved / 1e12, "peak": PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s",
            "frac": achieved / PEAK_LANE_OPS,
            "traffic": traffic,
            "traffic_source": traffic_source,
            "step_frac": elem_steps * step_slots / (ms_per_step * 1e-3) / PEAK_LANE_OPS,
            "fwd_frac": elem_steps * alu_slots("fwd") / (fwd_ms * 1e-3) / PEAK_LANE_OPS,
            # the other two rooflines of the metric, for the whole step (small by construction:
            # the path is bound by tanh and gating on the vector ALUs)
            "mfma_tflops": mfma_flops / (ms_per_step * 1e-3) / 1e12,
            "mfma_frac": mfma_flops / (ms_per_step * 1e-3) / MFMA_PEAK,
            "hbm_algorithmic_GBps": alg_bytes / (ms_per_step * 1e-3) / 1e9,
            "hbm_frac": alg_bytes / (ms_per_step * 1e-3) / HBM_PEAK,
        },
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, inp)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
