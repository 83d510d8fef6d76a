"""GPU parity of the two options on the scan (m2rnn_fwd_opt / m2rnn_bwd_opt): the residual
w_r (.) v_t of the y equation with its gradients, and per-step clipping of the carried state
gradient, against the float64 oracle run with the same options.  Same tolerances and error
measure as the other parity tests.  The shapes cover every store site of y and dv: tilings
that split a state over workgroups (sums finished by an epilogue kernel), tilings that do
not, the register-resident forward, and the fp32 kernels."""
import numpy as np
import pytest

from paper_2603_14360_amd.synth_inputs import (WORKLOADS, Workload, make_gate_inputs, make_inputs,
                                                make_residual_weight)
import gpu_util as gu

pytestmark = pytest.mark.gpu

CASES = [
    # io, B, T, N, K, V, Nqk
    ("f32", 2, 37, 3, 16, 16, 0),
    ("f32", 2, 40, 4, 32, 32, 1),
    ("bf16", 2, 37, 3, 16, 16, 0),      # one workgroup per state
    ("bf16", 2, 70, 2, 32, 32, 0),      # one workgroup per state, two row blocks
    ("bf16", 2, 100, 3, 64, 64, 0),     # four workgroups per state
    ("bf16", 8, 45, 16, 64, 64, 0),     # two row blocks per workgroup, two workgroups per state
    ("bf16", 1, 45, 2, 128, 128, 0),
    ("bf16", 2, 50, 6, 64, 16, 1),      # shared q/k heads
    ("bf16", 8, 35, 64, 64, 16, 0),     # enough row blocks for the register-resident forward
]


def _wl(io, B, T, N, K, V, Nqk, seed):
    return Workload("t", B, T, N, K, V, io, seed, K ** -0.5, 1.0, use_H0=True, use_dHT=True, Nqk=Nqk)


def _report(label, errs):
    print("%s: %s" % (label, {k: float("%.3g" % v) for k, v in errs.items()}), flush=True)


@pytest.mark.parametrize("io,B,T,N,K,V,Nqk", CASES)
def test_residual(io, B, T, N, K, V, Nqk):
    label = "residual %s B%d T%d N%d K%d V%d Nqk%d" % (io, B, T, N, K, V, Nqk)
    print("case", label, flush=True)
    wl = _wl(io, B, T, N, K, V, Nqk, seed=B + T + K + V)
    inp = make_inputs(wl)
    inp["w_r"] = make_residual_weight(wl)
    got = gu.run_gpu(inp, io)
    ref = gu.run_oracle(inp)
    assert "dw_r" in got and "dw_r" in ref
    # the residual must matter in this case, or the comparison would not see it missing
    plain = gu.run_oracle({n: x for n, x in inp.items() if n != "w_r"}, backward=False)
    assert gu.rel_err(plain["y"], ref["y"]) > 0.1
    _report(label, gu.compare(got, ref, gu.TOL[io], label=label))


@pytest.mark.parametrize("io,B,T,N,K,V,Nqk", CASES[:8])
def test_clipped_backward(io, B, T, N, K, V, Nqk):
    label = "clip %s B%d T%d N%d K%d V%d Nqk%d" % (io, B, T, N, K, V, Nqk)
    print("case", label, flush=True)
    inp = make_inputs(_wl(io, B, T, N, K, V, Nqk, seed=B + T + K + V + 1))
    free = gu.run_oracle(inp)
    clip = 0.3 * float(np.abs(free["dH0"]).max())
    ref = gu.run_oracle(inp, grad_clip=clip)
    assert gu.rel_err(free["dW"], ref["dW"]) > 1e-2      # the bound is active in this case
    got = gu.run_gpu(inp, io, grad_clip=clip)
    assert np.abs(got["dH0"]).max() <= clip * (1 + 1e-6)
    _report(label, gu.compare(got, ref, gu.TOL[io], label=label))


@pytest.mark.parametrize("io,B,T,N,K,V,Nqk", CASES)
def test_gate_function(io, B, T, N, K, V, Nqk):
    """f holds the input of psi(x) = (1 + e^(x + beta))^(-alpha); df is the gradient of x."""
    label = "gate %s B%d T%d N%d K%d V%d Nqk%d" % (io, B, T, N, K, V, Nqk)
    print("case", label, flush=True)
    wl = _wl(io, B, T, N, K, V, Nqk, seed=B + T + K + V + 2)
    inp = make_inputs(wl)
    inp["f"], inp["gate"] = make_gate_inputs(wl)
    got = gu.run_gpu(inp, io)
    ref = gu.run_oracle(inp)
    assert "dalpha" in got and "dbeta" in ref
    _report(label, gu.compare(got, ref, gu.TOL[io], label=label))


def test_gate_function_without_checkpoints_bf16():
    """The backward's own checkpoint pass applies the gate function as well."""
    wl = _wl("bf16", 2, 50, 3, 64, 64, 0, seed=91)
    inp = make_inputs(wl)
    inp["f"], inp["gate"] = make_gate_inputs(wl)
    print("case gate, ckpt = NULL", flush=True)
    got = gu.run_gpu(inp, "bf16", use_ckpt=False)
    ref = gu.run_oracle(inp)
    _report("gate no ckpt", gu.compare(got, ref, gu.TOL["bf16"], label="gate no ckpt"))


def test_options_together_and_null_opts_bf16():
    """Residual, gate function and clipping in one call; a NULL options pointer and an all-zero options
    struct give exactly the plain entry points' results."""
    import torch
    from paper_2603_14360_amd import binding as mb
    wl = _wl("bf16", 2, 60, 4, 64, 64, 0, seed=77)
    inp = make_inputs(wl)
    print("case options together", flush=True)
    both = dict(inp, w_r=make_residual_weight(wl))
    both["f"], both["gate"] = make_gate_inputs(wl)
    free = gu.run_oracle(both)
    clip = 0.3 * float(np.abs(free["dH0"]).max())
    got = gu.run_gpu(both, "bf16", grad_clip=clip)
    ref = gu.run_oracle(both, grad_clip=clip)
    _report("both", gu.compare(got, ref, gu.TOL["bf16"], label="both"))

    print("case null options", flush=True)
    dev = gu.to_device(inp, "bf16")
    scan = mb.Scan(2, 60, 4, 64, 64, "bf16")
    scan.fwd(dev["q"], dev["k"], dev["v"], dev["f"], dev["W"], dev["H0"])
    g0 = [x.clone() for x in scan.bwd(dev["q"], dev["k"], dev["v"], dev["f"], dev["W"], dev["H0"],
                                      dev["dy"], dev["dHT"])]
    y0 = scan.y.clone()
    for opts in (None, mb.make_opts()):
        scan.y.zero_()
        mb.m2rnn_fwd_opt(scan.desc, opts, dev["q"], dev["k"], dev["v"], dev["f"], dev["W"],
                         dev["H0"], scan.y, scan.HT, scan.ckpt, scan.workspace,
                         stream=torch.cuda.current_stream().cuda_stream)
        mb.m2rnn_bwd_opt(scan.desc, opts, dev["q"], dev["k"], dev["v"], dev["f"], dev["W"],
                         dev["H0"], scan.ckpt, dev["dy"], dev["dHT"], scan.dq, scan.dk, scan.dv,
                         scan.df, scan.dW, scan.dH0, scan.workspace,
                         stream=torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert torch.equal(scan.y, y0)
        for a, b in zip((scan.dq, scan.dk, scan.dv, scan.df, scan.dW, scan.dH0), g0):
            assert torch.equal(a, b)


def test_residual_weight_without_gradient_buffer_is_an_error():
    import torch
    from paper_2603_14360_amd import binding as mb
    scan = mb.Scan(1, 4, 1, 16, 16, "bf16")
    z = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device="cuda")
    q, v, W = z(1, 4, 1, 16), z(1, 4, 1, 16), z(1, 16, 16)
    f = torch.zeros(1, 4, 1, device="cuda")
    w_r = z(1, 16)
    rc = mb.m2rnn_bwd_opt(scan.desc, mb.make_opts(w_r=w_r), q, q, v, f, W, None, None, v, None,
                          scan.dq, scan.dk, scan.dv, scan.df, scan.dW, scan.dH0, scan.workspace,
                          check=False)
    assert rc == 1  # M2RNN_ERR_NULL
