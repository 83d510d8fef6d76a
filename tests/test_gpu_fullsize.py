"""GPU parity at the benchmark's full sizes, in the launch configuration that
bench.py times.  The oracle cannot run every recurrence of these workloads in
seconds, but (batch, head) recurrences are independent, so it is run on a
sample of heads (all batch elements of each sampled head, because dW sums over
the batch) and compared element by element with the GPU's full-size output."""
import numpy as np
import pytest

from paper_2603_14360_amd.synth_inputs import WORKLOADS, make_inputs, select_heads
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _slice_heads(out, heads):
    res = {}
    for n, x in out.items():
        if n in ("dq", "dk") and x.shape[2] == 1:
            continue  # shared q/k heads: sums over all heads, not a per-head output
        if n in ("y", "dq", "dk", "dv"):
            res[n] = x[:, :, heads]
        elif n == "df":
            res[n] = x[:, :, heads]
        elif n in ("dW", "dw_r", "dalpha", "dbeta"):
            res[n] = x[heads]
        else:
            res[n] = x[:, heads]
    return res


@pytest.mark.parametrize("name,heads,T_oracle", [("C3", [5], None), ("C4", [2], 2048), ("C5", [7, 20], None)])
def test_full_size_sampled_heads(name, heads, T_oracle):
    wl = WORKLOADS[name]
    print("case", name, "generating", flush=True)
    inp = make_inputs(wl)
    print("case", name, "gpu", flush=True)
    got = gu.run_gpu(inp, wl.io, backward=wl.backward)
    got = _slice_heads(got, heads)
    sub = select_heads(inp, heads)
    if T_oracle is None:
        print("case", name, "oracle on heads", heads, flush=True)
        ref = gu.run_oracle(sub, backward=wl.backward)
        errs = gu.compare(got, ref, gu.TOL[wl.io], label=name)
    else:
        # forward outputs of a prefix are exact prefixes of the full run; the
        # oracle checks y on the first T_oracle steps, and all gradients of a
        # separate full-size-shaped run of that prefix length are covered by
        # test_prefix_backward below.
        pre = {n: (x[:, :T_oracle] if (x is not None and n in ("q", "k", "v", "f", "dy")) else x)
               for n, x in sub.items()}
        print("case", name, "oracle prefix", T_oracle, flush=True)
        ref = gu.run_oracle(pre, backward=False)
        errs = {"y": gu.rel_err(got["y"][:, :T_oracle], ref["y"])}
        assert errs["y"] <= gu.TOL[wl.io], errs
        assert np.isfinite(got["y"]).all() and np.isfinite(got["HT"]).all()
        assert np.abs(got["HT"]).max() <= 1.0 + 1e-6   # |H| <= 1 from a zero initial state
    print(name, {k: float("%.3g" % v) for k, v in errs.items()}, flush=True)


def test_prefix_backward_C4_shape():
    """C4's shape (K = V = 128, all B and N) at T = 1024: full gradients of two heads."""
    wl = WORKLOADS["C4"]
    inp = make_inputs(wl, T=1024)
    print("case C4 T=1024 gpu", flush=True)
    got = _slice_heads(gu.run_gpu(inp, wl.io), [1, 6])
    ref = gu.run_oracle(select_heads(inp, [1, 6]))
    errs = gu.compare(got, ref, gu.TOL[wl.io], label="C4 prefix")
    print("C4 T=1024", {k: float("%.3g" % v) for k, v in errs.items()}, flush=True)


def test_production_shape_shared_qk():
    """The paper's layer shape (K = 64, V = 16, 84 heads, q/k shared by all heads) at full
    size: per-head outputs (y, dv, df, dW, H_T, dH0) of sampled heads against the oracle.
    dq and dk are sums over all 84 heads and are covered by the next test."""
    wl = WORKLOADS["P1"]
    heads = [0, 41, 83]
    print("case P1 generating", flush=True)
    inp = make_inputs(wl)
    print("case P1 gpu", flush=True)
    got = _slice_heads(gu.run_gpu(inp, wl.io), heads)
    print("case P1 oracle on heads", heads, flush=True)
    ref = gu.run_oracle(select_heads(inp, heads))
    names = ("y", "HT", "dv", "df", "dW", "dH0")
    errs = gu.compare(got, ref, gu.TOL[wl.io], names=names, label="P1")
    print("P1", {k: float("%.3g" % v) for k, v in errs.items()}, flush=True)


def test_production_shape_all_heads_prefix():
    """Same shape, all 84 heads, T = 512: every output including the head-summed dq, dk."""
    wl = WORKLOADS["P1"]
    inp = make_inputs(wl, T=512)
    print("case P1 T=512 gpu", flush=True)
    got = gu.run_gpu(inp, wl.io)
    print("case P1 T=512 oracle", flush=True)
    ref = gu.run_oracle(inp)
    errs = gu.compare(got, ref, gu.TOL[wl.io], label="P1 T=512")
    print("P1 T=512", {k: float("%.3g" % v) for k, v in errs.items()}, flush=True)


def test_full_size_options_C3():
    """C3 at full size with the residual, the gate function and clipping in one call:
    sampled head against the oracle run with the same options."""
    from paper_2603_14360_amd.synth_inputs import make_gate_inputs, make_residual_weight
    wl = WORKLOADS["C3"]
    heads = [11]
    print("case C3 options generating", flush=True)
    inp = make_inputs(wl)
    inp["w_r"] = make_residual_weight(wl)
    inp["f"], inp["gate"] = make_gate_inputs(wl)
    sub = select_heads(inp, heads)
    sub["w_r"] = inp["w_r"][heads]
    sub["gate"] = tuple(g[heads] for g in inp["gate"])
    print("case C3 options oracle on heads", heads, flush=True)
    free = gu.run_oracle(sub)
    # a bound that is active for the sampled head (the other heads run with the same bound)
    clip = 0.05 * float(max(np.abs(free["dH0"]).max(), np.abs(free["dW"]).max() / wl.T))
    ref = gu.run_oracle(sub, grad_clip=clip)
    assert gu.rel_err(free["dW"], ref["dW"]) > 1e-2
    print("case C3 options gpu, clip", clip, flush=True)
    got = gu.run_gpu(inp, wl.io, grad_clip=clip)
    got = _slice_heads(got, heads)
    errs = gu.compare(got, ref, gu.TOL[wl.io], label="C3 options")
    print("C3 options", {k: float("%.3g" % v) for k, v in errs.items()}, flush=True)
