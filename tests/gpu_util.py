"""Helpers for the GPU parity tests: move a seeded input set to the device,
run the library through its C ABI, run the float64 oracle on the same values,
and compare tensor by tensor with  max|gpu - oracle| / max|oracle|."""
import numpy as np

import oracle
from paper_2603_14360_amd import binding as mb

TOL = {"f32": 1e-5, "bf16": 2e-2}
GRAD_NAMES = ("dq", "dk", "dv", "df", "dW", "dH0")


def to_device(inp, io):
    import torch
    dt = torch.bfloat16 if io == "bf16" else torch.float32
    dev = {}
    for name in ("q", "k", "v", "W", "dy"):
        dev[name] = torch.from_numpy(np.ascontiguousarray(inp[name], dtype=np.float32)).to("cuda").to(dt)
    dev["f"] = torch.from_numpy(np.ascontiguousarray(inp["f"], dtype=np.float32)).to("cuda")
    for name in ("H0", "dHT"):
        x = inp.get(name)
        dev[name] = None if x is None else torch.from_numpy(
            np.ascontiguousarray(x, dtype=np.float32)).to("cuda")
    return dev


def to_np(x):
    return x.detach().to("cpu").float().numpy().astype(np.float64)


def run_gpu(inp, io, chunk=0, backward=True, use_ckpt=True, grad_clip=0.0):
    """Returns dict of float64 numpy outputs from the HIP library.  An input set with a
    "w_r" entry runs with the residual (and returns dw_r)."""
    import torch
    B, T, Nqk, K = inp["q"].shape
    N, V = inp["v"].shape[2], inp["v"].shape[3]
    dev = to_device(inp, io)
    scan = mb.Scan(B, T, N, K, V, io, Nqk=Nqk, chunk=chunk, backward=backward)
    w_r = None
    if inp.get("w_r") is not None:
        w_r = torch.from_numpy(np.ascontiguousarray(inp["w_r"], dtype=np.float32)).to("cuda").to(
            torch.bfloat16 if io == "bf16" else torch.float32)
    gate = None
    if inp.get("gate") is not None:
        gate = tuple(torch.from_numpy(np.ascontiguousarray(g, dtype=np.float32)).to("cuda")
                     for g in inp["gate"])
    y, HT = scan.fwd(dev["q"], dev["k"], dev["v"], dev["f"], dev["W"], dev["H0"], w_r=w_r, gate=gate)
    out = {"y": to_np(y), "HT": to_np(HT)}
    if backward:
        g = scan.bwd(dev["q"], dev["k"], dev["v"], dev["f"], dev["W"], dev["H0"], dev["dy"],
                     dev["dHT"], use_ckpt=use_ckpt, w_r=w_r, grad_clip=grad_clip, gate=gate)
        extra = (("dw_r",) if w_r is not None else ()) + (("dalpha", "dbeta") if gate else ())
        for name, x in zip(GRAD_NAMES + extra, g):
            out[name] = to_np(x)
    torch.cuda.synchronize()
    return out


def run_oracle(inp, backward=True, grad_clip=0.0):
    args = [inp[n] for n in ("q", "k", "v", "f", "W")]
    y, HT = oracle.fwd(*args, inp.get("H0"), w_r=inp.get("w_r"), gate=inp.get("gate"))
    out = {"y": y, "HT": HT}
    if backward:
        g = oracle.bwd(*args, inp.get("H0"), inp["dy"], inp.get("dHT"), w_r=inp.get("w_r"),
                       clip=grad_clip, gate=inp.get("gate"))
        extra = ((("dw_r",) if inp.get("w_r") is not None else ())
                 + (("dalpha", "dbeta") if inp.get("gate") is not None else ()))
        out.update(dict(zip(GRAD_NAMES + extra, g)))
    return out


def rel_err(got, ref):
    den = np.abs(ref).max() if ref.size else 0.0
    num = np.abs(got - ref).max() if ref.size else 0.0
    return num / den if den > 0 else num


def compare(got, ref, tol, names=None, label=""):
    """Asserts every tensor is within tol; returns {name: err}."""
    errs = {}
    for name in (names or ref.keys()):
        assert got[name].shape == ref[name].shape, (label, name, got[name].shape, ref[name].shape)
        assert np.isfinite(got[name]).all(), (label, name, "non-finite values")
        errs[name] = rel_err(got[name], ref[name])
    bad = {n: e for n, e in errs.items() if not e <= tol}
    assert not bad, "%s: over tolerance %g: %s (all: %s)" % (label, tol, bad, errs)
    return errs
