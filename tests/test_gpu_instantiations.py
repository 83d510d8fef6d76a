"""GPU parity for EVERY kernel variant the dispatcher can select for bf16 io: each tiling of
the matrix-core kernels and each shape of the one-wave-per-row-block forward, forward and
backward against the float64 oracle, with B*N chosen so that the call is really routed to
the variant named in the test id (m2rnn_route_string tells which one serves a descriptor).
Ragged T, H0 and dH_T set."""
import pytest

from paper_2603_14360_amd import binding as mb
from paper_2603_14360_amd.synth_inputs import Workload, make_inputs
import gpu_util as gu

pytestmark = pytest.mark.gpu

# (K, V, B, N, Nqk, forward route, backward route)
CASES = [
    # matrix-core tilings (forward and backward share the tiling)
    (64, 64, 8, 16, 0, "tile<64,64,2>", "tile<64,64,2>"),
    (64, 64, 3, 5, 0, "tile<64,64,1>", "tile<64,64,1>"),
    (128, 128, 2, 3, 0, "tile<128,128,1>", "tile<128,128,1>"),
    (32, 32, 16, 16, 0, "tile<32,32,2>", "tile<32,32,2>"),
    (32, 32, 16, 24, 4, "tile<32,32,2>", "tile<32,32,2>"),
    (32, 32, 3, 5, 0, "tile<32,32,1>", "tile<32,32,1>"),
    (16, 16, 3, 5, 0, "tile<16,16,1>", "rowwave_bwd<16,16>"),
    (64, 16, 3, 5, 0, "tile<64,16,1>", "rowwave_bwd<64,16>"),
    # one wave per row block (forward), paired with a matrix-core backward ...
    (64, 64, 32, 16, 0, "rowwave<64,64>", "tile<64,64,2>"),
    (32, 32, 32, 32, 0, "rowwave<32,32>", "tile<32,32,2>"),
    (16, 16, 32, 64, 0, "rowwave<16,16>", "rowwave_bwd<16,16>"),
    (64, 16, 8, 84, 1, "rowwave<64,16>", "rowwave_bwd<64,16>"),
    # ... V = 16 with any K: register-resident both ways
    (32, 16, 2, 3, 0, "rowwave<32,16>", "rowwave_bwd<32,16>"),
    (128, 16, 2, 3, 0, "rowwave<128,16>", "rowwave_bwd<128,16>"),
    # ... or with the fp32 vector-ALU backward where no matrix-core backward exists
    (16, 32, 2, 3, 0, "rowwave<16,32>", "generic<bf16>"),
    (64, 32, 2, 3, 0, "rowwave<64,32>", "generic<bf16>"),
    (128, 32, 2, 3, 0, "rowwave<128,32>", "generic<bf16>"),
    (16, 64, 2, 3, 0, "rowwave<16,64>", "generic<bf16>"),
    (32, 64, 2, 3, 0, "rowwave<32,64>", "generic<bf16>"),
    (128, 64, 2, 3, 0, "rowwave<128,64>", "generic<bf16>"),
    # shapes with V = 128 and K != V: vector-ALU kernels both ways
    (64, 128, 1, 2, 0, "generic<bf16>", "generic<bf16>"),
]


@pytest.mark.parametrize("K,V,B,N,Nqk,fwd_route,bwd_route", CASES,
                         ids=["%s+%s@K%dV%dB%dN%d" % (c[5], c[6], c[0], c[1], c[2], c[3]) for c in CASES])
def test_every_dispatch_route(K, V, B, N, Nqk, fwd_route, bwd_route):
    T = 35
    desc = mb.make_desc(B, T, N, K, V, mb.M2RNN_BF16, Nqk=(Nqk or None))
    assert mb.m2rnn_route_string(desc, 0) == fwd_route
    assert mb.m2rnn_route_string(desc, 1) == bwd_route
    label = "route %s / %s" % (fwd_route, bwd_route)
    print("case", label, "B%d N%d" % (B, N), flush=True)
    wl = Workload("t", B, T, N, K, V, "bf16", 900 + K + 3 * V + B, K ** -0.5, 1.0, use_H0=True,
                  use_dHT=True, Nqk=Nqk)
    inp = make_inputs(wl)
    got = gu.run_gpu(inp, "bf16")
    ref = gu.run_oracle(inp)
    errs = gu.compare(got, ref, gu.TOL["bf16"], label=label)
    print(label, {k: float("%.3g" % v) for k, v in errs.items()}, flush=True)
