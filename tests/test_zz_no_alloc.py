"""GPU: m2rnn_fwd_static (the forward on the library's own static scratch, for callers that
cannot allocate) against m2rnn_fwd_opt on a caller-allocated workspace, through the C ABI.
Both run the same kernels, so the outputs must be equal bit for bit; two calls in a row,
the second on a smaller input (the array keeps the first call's contents), and the first
call's result is also held against the float64 oracle at the bf16 tolerance."""
import numpy as np
import pytest

from paper_2603_14360_amd import binding as mb
from paper_2603_14360_amd.synth_inputs import Workload, make_inputs
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _run_both(B, T, N, K, V, seed):
    import torch
    wl = Workload("t", B, T, N, K, V, "bf16", seed, K ** -0.5, 1.0, use_H0=True)
    inp = make_inputs(wl)
    dev = gu.to_device(inp, "bf16")
    desc = mb.make_desc(B, T, N, K, V, mb.M2RNN_BF16)
    need = mb.m2rnn_workspace_bytes(desc, 0)
    assert 0 < need <= mb.M2RNN_STATIC_SCRATCH_BYTES, need   # the case must use the scratch
    stream = torch.cuda.current_stream().cuda_stream
    outs = []
    for static in (False, True):
        y = torch.full((B, T, N, V), float("nan"), dtype=torch.bfloat16, device="cuda")
        HT = torch.full((B, N, K, V), float("nan"), dtype=torch.float32, device="cuda")
        args = (dev["q"], dev["k"], dev["v"], dev["f"], dev["W"], dev["H0"], y, HT, None)
        if static:
            mb.m2rnn_fwd_static(desc, None, *args, stream=stream)
        else:
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            mb.m2rnn_fwd_opt(desc, None, *args, ws, stream=stream)
        torch.cuda.synchronize()
        outs.append((y, HT))
    (y0, H0_), (y1, H1_) = outs
    assert torch.equal(y0, y1) and torch.equal(H0_, H1_)
    ref = gu.run_oracle(inp, backward=False)
    errs = {"y": gu.rel_err(gu.to_np(y1), ref["y"]), "HT": gu.rel_err(gu.to_np(H1_), ref["HT"])}
    assert max(errs.values()) <= gu.TOL["bf16"], errs
    return errs


def test_static_scratch_forward_two_calls():
    print("case static scratch: first call B2 T45 N2 K64 V64", flush=True)
    e1 = _run_both(2, 45, 2, 64, 64, seed=301)
    print("case static scratch: second, smaller call B1 T17 N2 K64 V64", flush=True)
    e2 = _run_both(1, 17, 2, 64, 64, seed=302)
    print("static scratch", e1, e2, flush=True)
