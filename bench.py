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

# HBM bytes per launch of the dominant kernel, from two rocprofv3 --pmc runs of this script
# (FETCH_SIZE, then WRITE_SIZE; each scaled by what the same counter reads for the
# --calib-copy-mib copy: x2.000 and x1.000).  Summary: profiles/c3_fwd_bwd_pmc_counters.txt.
MEASURED_TRAFFIC_BYTES = {"C3": 440049 * 1024 * 2.000 + 672730 * 1024 * 1.000}


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
            "tokens_per_step": tokens, "chunk": mb.m2rnn_default_chunk(scan.desc)},
        "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
        "roofline": {
            "bound": "alu", "kernel": "m2rnn_%s (scan kernel of the %s call)" % (dom, dom),
            "achieved": achieved / 1e12, "peak": PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s",
            "frac": achieved / PEAK_LANE_OPS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name),
            "step_frac": elem_steps * step_slots / (ms_per_step * 1e-3) / PEAK_LANE_OPS,
            "fwd_frac": elem_steps * alu_slots("fwd") / (fwd_ms * 1e-3) / PEAK_LANE_OPS,
            "mfma_tflops": elem_steps * wl.V * (2 + (6 if wl.backward else 0)) / (ms_per_step * 1e-3) / 1e12,
        },
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, inp)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
