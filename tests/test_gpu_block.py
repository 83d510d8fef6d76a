"""GPU parity of the scan's two neighbours in the block (conv1d(4) + SiLU prologue, gated
RMSNorm epilogue) against the float64 oracle, through the C ABI: 1e-5 for fp32 io, 2e-2 for
bf16 io, max|gpu - oracle| / max|oracle| per tensor, the oracle reading the storage-rounded
inputs.  Shapes span several work items with ragged tails, the paper's layer widths
(N K = 1024 query channels at C3; D = N V = 84 x 16 = 1344 at the layer shape P1), T = 0 / 1."""
import numpy as np
import pytest

import oracle
from paper_2603_14360_amd import binding as mb
from paper_2603_14360_amd.synth_inputs import round_to_bf16
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _store(x, io):
    return round_to_bf16(x)[0] if io == "bf16" else np.asarray(x, dtype=np.float32)


def _dev(x, io):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to("cuda")
    return t.to(torch.bfloat16) if io == "bf16" else t


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("B,T,C,bias", [(2, 1, 8, True), (3, 37, 24, False), (2, 70, 1024, True),
                                        (1, 4096, 64, True), (2, 0, 16, True)])
def test_conv_silu(io, B, T, C, bias):
    import torch
    rng = np.random.default_rng(B * 100 + T + C)
    x = _store(rng.standard_normal((B, T, C)), io)
    w = _store(rng.standard_normal((C, 4)) * 0.5, io)
    b = _store(rng.standard_normal(C) * 0.3, io) if bias else None
    dout = _store(rng.standard_normal((B, T, C)), io)
    label = "conv %s B%d T%d C%d bias%d" % (io, B, T, C, bias)
    print("case", label, flush=True)
    xd, wd, dd = _dev(x, io), _dev(w, io), _dev(dout, io)
    bd = _dev(b, io) if bias else None
    out, dx = torch.empty_like(xd), torch.empty_like(xd)
    dw = torch.full((C, 4), float("nan"), device="cuda")
    db = torch.full((C,), float("nan"), device="cuda") if bias else None
    ws = torch.empty(max(256, mb.m2rnn_conv_silu_workspace_bytes(B, T, C)), dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    mb.m2rnn_conv_silu_fwd(xd, wd, bd, out, stream=st)
    mb.m2rnn_conv_silu_bwd(xd, wd, bd, dd, dx, dw, db, ws, stream=st)
    torch.cuda.synchronize()
    ref = {"out": oracle.block.conv_silu_fwd(x, w, b)}
    ref["dx"], ref["dw"], rdb = oracle.block.conv_silu_bwd(x, w, b, dout)
    got = {"out": gu.to_np(out), "dx": gu.to_np(dx), "dw": gu.to_np(dw)}
    if bias:
        ref["dbias"], got["dbias"] = rdb, gu.to_np(db)
    errs = gu.compare(got, ref, gu.TOL[io], label=label)
    print(label, {k: float("%.3g" % v) for k, v in errs.items()}, flush=True)


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("B,T,D,eps,cache", [(2, 1, 8, 0.0, True), (3, 37, 1344, 1e-5, False),
                                             (2, 300, 1024, 1e-5, True), (1, 5, 4096, 0.0, True),
                                             (2, 0, 64, 1e-5, True)])
def test_gated_rmsnorm(io, B, T, D, eps, cache):
    import torch
    rng = np.random.default_rng(B * 100 + T + D)
    y = _store(rng.standard_normal((B, T, D)), io)
    a = _store(rng.standard_normal((B, T, D)) * 1.5, io)
    w = _store(rng.uniform(0.5, 1.5, D), io)
    dout = _store(rng.standard_normal((B, T, D)), io)
    label = "rmsnorm %s B%d T%d D%d eps%g cache%d" % (io, B, T, D, eps, cache)
    print("case", label, flush=True)
    yd, ad, wd, dd = _dev(y, io), _dev(a, io), _dev(w, io), _dev(dout, io)
    out, dy, da = torch.empty_like(yd), torch.empty_like(yd), torch.empty_like(yd)
    s = torch.full((B, T), float("nan"), device="cuda") if cache else None
    dw = torch.full((D,), float("nan"), device="cuda")
    ws = torch.empty(max(256, mb.m2rnn_gated_rmsnorm_workspace_bytes(B, T, D)), dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    mb.m2rnn_gated_rmsnorm_fwd(yd, ad, wd, eps, out, s, stream=st)
    mb.m2rnn_gated_rmsnorm_bwd(yd, ad, wd, eps, s, dd, dy, da, dw, ws, stream=st)
    torch.cuda.synchronize()
    ref = {}
    ref["out"], rs = oracle.block.gated_rmsnorm_fwd(y, a, w, eps)
    ref["dy"], ref["da"], ref["dw"] = oracle.block.gated_rmsnorm_bwd(y, a, w, eps, dout)
    got = {"out": gu.to_np(out), "dy": gu.to_np(dy), "da": gu.to_np(da), "dw": gu.to_np(dw)}
    if cache:
        ref["s"], got["s"] = rs, gu.to_np(s)
    errs = gu.compare(got, ref, gu.TOL[io], label=label)
    print(label, {k: float("%.3g" % v) for k, v in errs.items()}, flush=True)
