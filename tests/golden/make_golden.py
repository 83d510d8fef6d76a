"""Writes tests/golden/oracle_c1_samples.txt from the float64 oracle alone.

The paper prints no numeric worked example, so there is no value of the
paper's to store.  This file is a regression fixture: it freezes a few of the
oracle's own outputs on the tiny workload C1 (B=1, N=2, K=V=16, T=64, seed 0)
so that an accidental change to the oracle's arithmetic or to the input
recipe is noticed.  It calls only ``oracle/`` and the seeded input generator.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2603_14360_amd.synth_inputs import WORKLOADS, make_inputs  # noqa: E402

SAMPLES = 12


def compute():
    inp = make_inputs(WORKLOADS["C1"])
    args = [inp[n] for n in ("q", "k", "v", "f", "W")]
    y, HT = oracle.fwd(*args, inp["H0"])
    grads = oracle.bwd(*args, inp["H0"], inp["dy"], inp["dHT"])
    tensors = dict(zip(("y", "HT", "dq", "dk", "dv", "df", "dW", "dH0"), (y, HT) + tuple(grads)))
    rows = []
    for name, x in tensors.items():
        flat = x.ravel()
        step = max(1, flat.size // SAMPLES)
        for idx in range(0, flat.size, step)[:SAMPLES]:
            rows.append((name, idx, flat[idx]))
    return rows


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_c1_samples.txt")
    with open(out, "w") as fh:
        fh.write("# tensor flat_index value ; written by make_golden.py from the float64 oracle on workload C1\n")
        for name, idx, val in compute():
            fh.write("%s %d %.17g\n" % (name, idx, val))
    print("wrote", out)
