"""Seeded synthetic inputs for the M2RNN scan (shared by tests, bench and smoke).

This module holds no arithmetic of the method itself: it only draws random
tensors, scales them, and rounds them to the storage type.  Both the float64
oracle and the GPU library are fed from here, so that they see bit-identical
values (the oracle receives the already-rounded values widened to float64).

The named workloads stand in for the paper's language-model activations
(training context 4096, K = 64, bf16 storage), which are not available here.

Recipe: one ``numpy.random.default_rng(seed)`` stream, standard-normal float64
draws in the fixed order  q, k, v, gate logits, W, H0, dy, dHT  (all drawn even
when a workload does not use one, so the streams stay aligned), then scaled:
q, k, v by ``qkv_scale``; optional L2 normalisation of every k_t; the gate is
f = sigmoid(logit_mean + logit) stored as float32; W by 1/sqrt(V); H0 and dHT
by 0.1; dy unscaled.  q, k, v, W, dy are rounded to the io dtype.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    T: int
    N: int
    K: int
    V: int
    io: str            # "f32" or "bf16"
    seed: int
    qkv_scale: float
    logit_mean: float
    normalise_k: bool = False
    use_H0: bool = False
    use_dHT: bool = False
    backward: bool = True
    Nqk: int = 0       # 0 -> one q/k head per head (Nqk = N)


WORKLOADS = {
    "C1": Workload("C1", 1, 64, 2, 16, 16, "f32", 0, 0.25, 0.0),
    "C2": Workload("C2", 4, 512, 8, 32, 32, "f32", 1, 32 ** -0.5, 0.0,
                   normalise_k=True, use_H0=True, use_dHT=True),
    "C3": Workload("C3", 8, 4096, 16, 64, 64, "bf16", 2, 0.125, 2.0),
    "C4": Workload("C4", 4, 8192, 8, 128, 128, "bf16", 3, 128 ** -0.5, 2.0),
    "C5": Workload("C5", 1, 65536, 32, 64, 64, "bf16", 4, 0.125, 3.0,
                   backward=False),
    # the paper's own layer shape (state-size appendix: K = 64, V = 16; 84 heads at the 410M
    # scale; q and k shared by all heads, i.e. the multi-value form of Algorithms 1 and 2)
    "P1": Workload("P1", 8, 4096, 84, 64, 16, "bf16", 5, 0.125, 2.0, Nqk=1),
    # a training shape with many states (B N = 512): the forward is then served by the
    # one-wave-per-row-block kernel, the backward by the tiled one
    "R1": Workload("R1", 32, 1024, 16, 64, 64, "bf16", 6, 0.125, 2.0),
}


def round_to_bf16(x):
    """Round float values to the nearest bfloat16 (ties to even); returns the
    rounded values as float32 and the raw 16-bit patterns as uint16."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    bits = x32.view(np.uint32)
    bias = ((bits >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    hi = ((bits + bias) >> np.uint32(16)).astype(np.uint16)
    back = (hi.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return back.reshape(x32.shape), hi.reshape(x32.shape)


def bf16_bits_to_f32(bits):
    """Widen raw bfloat16 bit patterns (uint16) to float32."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(b.shape)


def _store(x, io):
    """Round to the io dtype; the returned float32 array holds exactly the
    values the device buffer will hold."""
    if io == "bf16":
        return round_to_bf16(x)[0]
    if io == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError("io must be 'f32' or 'bf16'")


def make_inputs(wl, T=None, B=None, N=None):
    """Draw the tensors of a workload (optionally with a shorter T or fewer
    B / N: the generator then draws the reduced shapes directly).

    Returns a dict of float32 arrays holding storage-rounded values:
    q, k [B,T,Nqk,K]; v, dy [B,T,N,V]; f [B,T,N]; W [N,V,V];
    H0, dHT [B,N,K,V] or None.
    """
    B = wl.B if B is None else B
    T = wl.T if T is None else T
    N = wl.N if N is None else N
    Nqk = N if wl.Nqk == 0 else wl.Nqk
    K, V = wl.K, wl.V
    rng = np.random.default_rng(wl.seed)
    q = rng.standard_normal((B, T, Nqk, K))
    k = rng.standard_normal((B, T, Nqk, K))
    v = rng.standard_normal((B, T, N, V))
    logit = rng.standard_normal((B, T, N))
    W = rng.standard_normal((N, V, V))
    H0 = rng.standard_normal((B, N, K, V))
    dy = rng.standard_normal((B, T, N, V))
    dHT = rng.standard_normal((B, N, K, V))

    q *= wl.qkv_scale
    k *= wl.qkv_scale
    v *= wl.qkv_scale
    if wl.normalise_k:
        k /= np.linalg.norm(k, axis=-1, keepdims=True)
    f = 1.0 / (1.0 + np.exp(-(logit + wl.logit_mean)))
    W *= V ** -0.5
    out = {
        "q": _store(q, wl.io), "k": _store(k, wl.io), "v": _store(v, wl.io),
        "f": f.astype(np.float32), "W": _store(W, wl.io),
        "H0": (0.1 * H0).astype(np.float32) if wl.use_H0 else None,
        "dy": _store(dy, wl.io),
        "dHT": (0.1 * dHT).astype(np.float32) if wl.use_dHT else None,
    }
    return out


def make_residual_weight(wl, N=None):
    """w_r [N,V]: weights of the residual term w_r (.) v_t, N(0,1), from a generator stream
    of its own (so that the tensors of make_inputs do not change), rounded to the io dtype."""
    N = wl.N if N is None else N
    rng = np.random.default_rng([wl.seed, 7919])
    return _store(rng.standard_normal((N, wl.V)), wl.io)


def make_gate_inputs(wl, B=None, T=None, N=None):
    """Inputs of the forget-gate function: x [B,T,N] ~ N(0, 2^2) (float32) in place of the gate
    value, alpha ~ Uniform(0.3, 2.5) and beta ~ N(0, 1) per head, from a generator stream of
    their own.  Returns (x, (alpha, beta))."""
    B = wl.B if B is None else B
    T = wl.T if T is None else T
    N = wl.N if N is None else N
    rng = np.random.default_rng([wl.seed, 104729])
    x = (2.0 * rng.standard_normal((B, T, N))).astype(np.float32)
    alpha = rng.uniform(0.3, 2.5, N).astype(np.float32)
    beta = rng.standard_normal(N).astype(np.float32)
    return x, (alpha, beta)


def select_heads(inp, heads):
    """Restrict workload tensors to a list of heads; the recurrences of
    different heads are independent, so the oracle can be run on the selection
    alone.  With one q/k head per head (Nqk = N) q and k are restricted too;
    with shared q/k (Nqk = 1) they are kept whole, and dq, dk of the selection
    are then sums over the selected heads only."""
    heads = list(heads)
    out = {}
    per_head_qk = inp["q"].shape[2] == inp["v"].shape[2]
    for name in ("q", "k"):
        if per_head_qk:
            out[name] = np.ascontiguousarray(inp[name][:, :, heads])
        else:
            assert inp[name].shape[2] == 1, "select_heads: Nqk must be N or 1"
            out[name] = inp[name]
    for name in ("v", "dy"):
        out[name] = np.ascontiguousarray(inp[name][:, :, heads])
    out["f"] = np.ascontiguousarray(inp["f"][:, :, heads])
    out["W"] = np.ascontiguousarray(inp["W"][heads])
    for name in ("H0", "dHT"):
        out[name] = None if inp[name] is None else np.ascontiguousarray(inp[name][:, heads])
    return out
