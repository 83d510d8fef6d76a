"""GPU parity: the HIP library (through its C ABI) against the float64 oracle,
element by element, on seeded synthetic inputs.  Tolerances: 1e-5 for float32
io, 2e-2 for bfloat16 io with fp32 state, measured as max|diff| / max|oracle|
per output tensor."""
import numpy as np
import pytest

from paper_2603_14360_amd.synth_inputs import WORKLOADS, Workload, make_inputs, select_heads
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _report(label, errs):
    print("%s: %s" % (label, {k: float("%.3g" % v) for k, v in errs.items()}), flush=True)


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_fp32_workloads(name):
    wl = WORKLOADS[name]
    inp = make_inputs(wl)
    print("case", name, flush=True)
    got = gu.run_gpu(inp, wl.io)
    ref = gu.run_oracle(inp)
    _report(name, gu.compare(got, ref, gu.TOL["f32"], label=name))


def _small(io, B, T, N, K, V, seed, Nqk=0, H0=True, dHT=True, logit_mean=1.0):
    return Workload("t", B, T, N, K, V, io, seed, K ** -0.5, logit_mean, use_H0=H0, use_dHT=dHT,
                    Nqk=Nqk)


SHAPES = [
    # io, B, T, N, K, V, Nqk
    ("f32", 2, 37, 3, 16, 16, 0),
    ("f32", 1, 50, 2, 64, 16, 0),
    ("f32", 1, 33, 2, 16, 64, 0),
    ("f32", 1, 21, 1, 128, 128, 0),
    ("f32", 2, 40, 4, 32, 32, 1),
    ("f32", 1, 40, 6, 32, 16, 2),
    ("f32", 1, 19, 2, 64, 32, 0),    # fp32 kernels with 2 state elements per thread
    ("f32", 1, 18, 2, 64, 64, 0),    # ... 4
    ("f32", 1, 17, 1, 128, 64, 0),   # ... 8 (16: the 128 x 128 case above)
    ("bf16", 2, 37, 3, 16, 16, 0),
    ("bf16", 2, 70, 2, 32, 32, 0),
    ("bf16", 2, 100, 3, 64, 64, 0),
    ("bf16", 1, 45, 2, 128, 128, 0),
    ("bf16", 1, 50, 2, 64, 16, 0),
    ("bf16", 1, 33, 2, 16, 64, 0),
    ("bf16", 2, 40, 4, 64, 64, 1),
    ("bf16", 1, 40, 6, 64, 16, 2),
]


@pytest.mark.parametrize("io,B,T,N,K,V,Nqk", SHAPES)
def test_shapes(io, B, T, N, K, V, Nqk):
    label = "%s B%d T%d N%d K%d V%d Nqk%d" % (io, B, T, N, K, V, Nqk)
    print("case", label, flush=True)
    inp = make_inputs(_small(io, B, T, N, K, V, seed=B * 1000 + T + K + V, Nqk=Nqk))
    got = gu.run_gpu(inp, io)
    ref = gu.run_oracle(inp)
    _report(label, gu.compare(got, ref, gu.TOL[io], label=label))


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("T", [0, 1, 2, 15, 16, 17, 31, 33])
def test_ragged_lengths_and_empty(io, T):
    K = V = 32 if io == "f32" else 64
    label = "%s T=%d" % (io, T)
    print("case", label, flush=True)
    inp = make_inputs(_small(io, 2, T, 2, K, V, seed=T + 5))
    got = gu.run_gpu(inp, io)
    ref = gu.run_oracle(inp)
    gu.compare(got, ref, gu.TOL[io], label=label)


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_null_optional_arguments(io):
    K = V = 32 if io == "f32" else 64
    inp = make_inputs(_small(io, 1, 40, 2, K, V, seed=3, H0=False, dHT=False))
    print("case null optionals", io, flush=True)
    got = gu.run_gpu(inp, io)
    ref = gu.run_oracle(inp)
    gu.compare(got, ref, gu.TOL[io], label="null H0/dHT " + io)


@pytest.mark.parametrize("io,K,V", [("f32", 32, 32), ("bf16", 64, 64), ("bf16", 64, 16), ("bf16", 16, 16)])
def test_checkpoint_interval_does_not_change_results(io, K, V):
    """The backward recomputes states from checkpoints; any interval C, and the
    backward's own pass 1 (ckpt = NULL), must give the same gradients.  (V = 16 runs the
    register-resident backward, whose unrolled 16-step chunk treats the steps beyond a
    shorter interval as identity steps.)"""
    inp = make_inputs(_small(io, 2, 75, 2, K, V, seed=17))
    ref = gu.run_oracle(inp)
    base = None
    from paper_2603_14360_amd import binding as mb
    cmax = mb.m2rnn_max_chunk(mb.make_desc(2, 75, 2, K, V, mb.M2RNN_BF16 if io == "bf16" else mb.M2RNN_F32))
    for chunk, use_ckpt in [(0, True), (1, True), (5, True), (min(cmax, 32), True), (0, False)]:
        print("case chunk", io, chunk, use_ckpt, flush=True)
        got = gu.run_gpu(inp, io, chunk=chunk, use_ckpt=use_ckpt)
        gu.compare(got, ref, gu.TOL[io], label="chunk=%d ckpt=%s" % (chunk, use_ckpt))
        if base is None:
            base = got
        else:
            # forward does not depend on C at all; gradients may differ only by
            # rounding (chunk boundaries move where states are re-derived)
            assert np.array_equal(got["y"], base["y"]) and np.array_equal(got["HT"], base["HT"])
            # (bf16 outputs may flip by one bf16 ulp = 2^-8 of the value)
            bound = 1e-6 if io == "f32" else 8e-3
            for n in gu.GRAD_NAMES:
                assert gu.rel_err(got[n], base[n]) <= bound, (n, chunk)


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_inference_mode_without_checkpoints(io):
    K = V = 32 if io == "f32" else 64
    inp = make_inputs(_small(io, 2, 50, 2, K, V, seed=23))
    a = gu.run_gpu(inp, io, backward=False)
    b = gu.run_gpu(inp, io, backward=True)
    assert np.array_equal(a["y"], b["y"]) and np.array_equal(a["HT"], b["HT"])


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_segment_chaining_and_determinism(io):
    """HT of one call fed as H0 of the next equals one long call (bitwise on the
    fp32 path, where the arithmetic per step is the same; the matrix-core path
    keeps a scaled state on chip, so the hand-off re-rounds it by one fp32 ulp),
    and repeated calls are bit-identical."""
    K = V = 32 if io == "f32" else 64
    wl = _small(io, 2, 64, 2, K, V, seed=29)
    inp = make_inputs(wl)
    full = gu.run_gpu(inp, io)
    again = gu.run_gpu(inp, io)
    for n in full:
        assert np.array_equal(full[n], again[n]), n
    T1 = 32
    first = {n: (x[:, :T1] if (x is not None and n in ("q", "k", "v", "f", "dy")) else x)
             for n, x in inp.items()}
    a = gu.run_gpu(first, io, backward=False)
    second = {n: (x[:, T1:] if (x is not None and n in ("q", "k", "v", "f", "dy")) else x)
              for n, x in inp.items()}
    second["H0"] = a["HT"].astype(np.float32)
    b = gu.run_gpu(second, io, backward=False)
    y2 = np.concatenate([a["y"], b["y"]], axis=1)
    if io == "f32":
        assert np.array_equal(y2, full["y"]) and np.array_equal(b["HT"], full["HT"])
    else:
        assert np.array_equal(a["y"], full["y"][:, :T1])
        assert gu.rel_err(y2, full["y"]) <= 5e-3 and gu.rel_err(b["HT"], full["HT"]) <= 1e-3


def test_gate_limits_bf16():
    """f = 1 keeps the state (dk = dv = dW = 0 exactly); f = 0 replaces it."""
    inp = make_inputs(_small("bf16", 1, 20, 2, 64, 64, seed=31))
    for val in (1.0, 0.0):
        inp2 = dict(inp)
        inp2["f"] = np.full_like(inp["f"], val)
        print("case gate", val, flush=True)
        got = gu.run_gpu(inp2, "bf16")
        ref = gu.run_oracle(inp2)
        gu.compare(got, ref, gu.TOL["bf16"], label="f=%g" % val)
        if val == 1.0:
            assert np.abs(got["dk"]).max() == 0 and np.abs(got["dv"]).max() == 0
            assert np.abs(got["dW"]).max() == 0
            assert gu.rel_err(got["HT"], inp["H0"].astype(np.float64)) <= 2e-7


def test_saturated_tanh_bf16():
    """Large pre-activations: tanh saturates to +-1 without NaN or overflow."""
    wl = Workload("sat", 1, 24, 2, 64, 64, "bf16", 41, 6.0, 0.0, use_H0=True, use_dHT=True)
    inp = make_inputs(wl)
    got = gu.run_gpu(inp, "bf16")
    ref = gu.run_oracle(inp)
    gu.compare(got, ref, gu.TOL["bf16"], label="saturated")


@pytest.mark.parametrize("K,V", [(64, 64), (32, 32), (64, 16), (16, 16), (128, 128)])
@pytest.mark.parametrize("scale", [2.0 ** -24, 2.0 ** 18])
def test_gradient_dynamic_range_bf16(K, V, scale):
    """dy and dH_T far outside the fp16 range (token-averaged losses give ~1e-7, loss scaling
    gives ~1e5): the backward is linear in (dy, dH_T), so every gradient must scale with
    them and keep its accuracy; nothing may overflow or flush to zero on the way."""
    wl = _small("bf16", 2, 70, 2, K, V, seed=77 + K + V)
    inp = make_inputs(wl)
    inp["dy"] = (inp["dy"] * np.float32(scale)).astype(np.float32)    # exact: power of two
    inp["dHT"] = (inp["dHT"] * np.float32(scale)).astype(np.float32)
    label = "range K%d V%d x%g" % (K, V, scale)
    print("case", label, flush=True)
    got = gu.run_gpu(inp, "bf16")
    ref = gu.run_oracle(inp)
    _report(label, gu.compare(got, ref, gu.TOL["bf16"], label=label))


@pytest.mark.parametrize("K,V", [(64, 64), (64, 16), (128, 128)])
@pytest.mark.parametrize("gain", [1.5, 3.0])
def test_growing_state_gradient_bf16(K, V, gain):
    """The regime the paper's gradient-clipping paragraph is about, without clipping: a small
    forget gate and a transition matrix of gain 1.5 or 3 make the carried state gradient grow
    by orders of magnitude, chunk after chunk (2^18 over 32 steps at gain 3).  The backward's
    fp16 dS operand must follow it: its power-of-two scale is chosen per chunk with headroom
    that widens when the previous chunk grew.  fp32 holds 3^32 easily, so the oracle stays
    finite and so must the library.  Such a recurrence is chaotic forward as well (H_T itself
    differs by percents between any two roundings).  At gain 1.5 the growth-aware bound
    holds; at gain 3 (expansion 1.4 per step) the chunk recompute's single fp16 state
    operand, 2^-12 per step amplified 1.4^16 within a chunk, adds errors of several percent:
    there the test asks for finite gradients within 25 %."""
    wl = Workload("grow", 2, 32, 2, K, V, "bf16", 55, K ** -0.5, -3.0, use_H0=True, use_dHT=True)
    inp = make_inputs(wl)
    from paper_2603_14360_amd.synth_inputs import round_to_bf16
    inp["W"] = round_to_bf16(inp["W"] * np.float32(gain))[0]
    label = "growing gradient K%d V%d gain %g" % (K, V, gain)
    print("case", label, flush=True)
    ref = gu.run_oracle(inp)
    got = gu.run_gpu(inp, "bf16")
    worst, info = gu.compare_units(got, ref, inp, gu.TOL["bf16"], label=label)
    errs = {n: float("%.3g" % gu.rel_err(got[n], ref[n])) for n in ref}
    print(label, ": worst error / bound %.3g" % worst, info, errs, flush=True)
    if gain < 2:
        assert worst <= 1.0, (worst, info)
    else:
        assert info["max_growth"] > 1e3      # the case really explodes
        assert max(errs.values()) <= 0.25, errs


def test_vanishing_gradient_after_large_late_dy_bf16():
    """dy is non-zero at the last step only and loss-scaled (x 2^22); the recurrence contracts
    (small W, small gate), so the carried gradient decays to nothing over the sequence.  The
    backward's internal scale then rises chunk by chunk while dW already holds large sums:
    rescaling the accumulated dW must not overflow."""
    wl = Workload("vanish", 1, 400, 2, 64, 64, "bf16", 56, 0.125, -2.0)
    inp = make_inputs(wl)
    from paper_2603_14360_amd.synth_inputs import round_to_bf16
    inp["W"] = round_to_bf16(inp["W"] * np.float32(0.25))[0]
    dy = np.zeros_like(inp["dy"])
    dy[:, -1] = inp["dy"][:, -1] * np.float32(2.0 ** 22)
    inp["dy"] = dy
    print("case vanishing gradient", flush=True)
    ref = gu.run_oracle(inp)
    print("oracle max |dW| %.3g, max |dH0| %.3g" % (np.abs(ref["dW"]).max(), np.abs(ref["dH0"]).max()),
          flush=True)
    got = gu.run_gpu(inp, "bf16")
    # the float64 oracle's dH0 (~1e-177) is below the smallest fp32 number: the fp32 result is 0
    assert np.abs(ref["dH0"]).max() < 1e-45 and np.abs(got["dH0"]).max() < 1e-30
    names = [n for n in ref if n != "dH0"]
    _report("vanishing gradient", gu.compare(got, ref, gu.TOL["bf16"], names=names,
                                             label="vanishing gradient"))


@pytest.mark.parametrize("K,V,Nqk", [(64, 64, 0), (64, 16, 1), (128, 64, 0), (16, 32, 2), (32, 16, 0)])
def test_single_step_decode_chain_bf16(K, V, Nqk):
    """Recurrent inference: T = 1 per call, the state handed from call to call (H_T -> H0),
    for a batch of sequences; every step's y and the final state against the oracle's one
    long run.  T = 1 is served by the single-launch decode kernel."""
    from paper_2603_14360_amd import binding as mb
    B, N, steps = 24, 4, 20
    assert mb.m2rnn_route_string(mb.make_desc(B, 1, N, K, V, mb.M2RNN_BF16, Nqk=(Nqk or None)), 0) \
        == "decode<%d,%d>" % (K, V)
    wl = Workload("t", B, steps, N, K, V, "bf16", 123 + V, K ** -0.5, 2.0, use_H0=True, Nqk=Nqk)
    inp = make_inputs(wl)
    ref = gu.run_oracle(inp, backward=False)
    H = inp["H0"]
    ys = []
    for t in range(steps):
        one = {n: (x[:, t:t + 1] if (x is not None and n in ("q", "k", "v", "f", "dy")) else x)
               for n, x in inp.items()}
        one["H0"] = H
        out = gu.run_gpu(one, "bf16", backward=False)
        ys.append(out["y"])
        H = out["HT"].astype(np.float32)
    y = np.concatenate(ys, axis=1)
    errs = {"y": gu.rel_err(y, ref["y"]), "HT": gu.rel_err(H.astype(np.float64), ref["HT"])}
    _report("decode K%d V%d" % (K, V), errs)
    assert errs["y"] <= gu.TOL["bf16"] and errs["HT"] <= gu.TOL["bf16"], errs


def test_decode_step_options_and_training_pair_bf16():
    """The decode kernel with the forward options (residual w_r, gate function), with a zero
    initial state (H0 = NULL), and as the forward of a T = 1 training pair (it then writes
    checkpoint 0 for m2rnn_bwd)."""
    from paper_2603_14360_amd.synth_inputs import make_gate_inputs, make_residual_weight
    wl = Workload("t", 5, 1, 6, 64, 32, "bf16", 77, 0.125, 1.0, use_H0=True, use_dHT=True, Nqk=3)
    inp = make_inputs(wl)
    inp["w_r"] = make_residual_weight(wl)
    inp["f"], inp["gate"] = make_gate_inputs(wl)
    print("case decode with options, training pair", flush=True)
    got = gu.run_gpu(inp, "bf16")
    ref = gu.run_oracle(inp)
    _report("decode options", gu.compare(got, ref, gu.TOL["bf16"], label="decode options"))
    inp2 = make_inputs(Workload("t", 3, 1, 2, 32, 64, "bf16", 78, 0.125, 1.0))
    got = gu.run_gpu(inp2, "bf16", backward=False)
    ref = gu.run_oracle(inp2, backward=False)
    _report("decode H0 = NULL", gu.compare(got, ref, gu.TOL["bf16"], label="decode null H0"))


def test_graph_capture_and_replay_bf16():
    """The calls allocate nothing and synchronise nothing, so a forward + backward pair can
    be captured into a HIP graph.  The graph is replayed three times on changing inputs, with
    eager work and synchronisations in between, and every replay must equal the eager
    result bit for bit (the kernels are deterministic)."""
    import torch
    from paper_2603_14360_amd import binding as mb
    wl = _small("bf16", 2, 45, 4, 64, 64, seed=21)
    sets = [gu.to_device(make_inputs(Workload("t", 2, 45, 4, 64, 64, "bf16", 21 + i, 0.125, 1.0,
                                              use_H0=True, use_dHT=True)), "bf16") for i in range(3)]
    names = ("q", "k", "v", "f", "W", "H0", "dy", "dHT")
    static = {n: sets[0][n].clone() for n in names}
    scan = mb.Scan(2, 45, 4, 64, 64, "bf16")

    def run():
        scan.fwd(static["q"], static["k"], static["v"], static["f"], static["W"], static["H0"])
        scan.bwd(static["q"], static["k"], static["v"], static["f"], static["W"], static["H0"],
                 static["dy"], static["dHT"])

    print("case graph: eager references", flush=True)
    eager = []
    for st in sets:
        for n in names:
            static[n].copy_(st[n])
        run()
        torch.cuda.synchronize()
        eager.append([x.clone() for x in (scan.y, scan.HT, scan.dq, scan.dk, scan.dv, scan.df,
                                          scan.dW, scan.dH0)])
    print("case graph: capture", flush=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run()
    for i in (2, 0, 1):
        print("case graph: replay on input set", i, flush=True)
        for n in names:
            static[n].copy_(sets[i][n])
        for x in (scan.y, scan.dq, scan.dW):  # eager work between replays
            x.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (scan.y, scan.HT, scan.dq, scan.dk, scan.dv, scan.df, scan.dW, scan.dH0)
        for a, b in zip(got, eager[i]):
            assert torch.equal(a, b)


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_empty_sequence_without_checkpoint_buffer(io):
    """T = 0 with ckpt = NULL: dH0 = dHT, dW = 0, H_T = H0, nothing else is touched."""
    K = V = 32 if io == "f32" else 64
    inp = make_inputs(_small(io, 2, 0, 2, K, V, seed=5))
    print("case T=0, ckpt NULL", io, flush=True)
    got = gu.run_gpu(inp, io, use_ckpt=False)
    ref = gu.run_oracle(inp)
    gu.compare(got, ref, gu.TOL[io], label="T=0 " + io)
    assert np.array_equal(got["dH0"], inp["dHT"].astype(np.float64))
    assert np.abs(got["dW"]).max() == 0.0
