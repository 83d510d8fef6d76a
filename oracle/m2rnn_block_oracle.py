"""ctypes front end of the float64 oracle of the scan's two neighbours in the M2RNN block
(``m2rnn_block_oracle.c``): the conv1d(4) + SiLU prologue of q, k, v and the gated RMSNorm
epilogue of y.

TEST INFRASTRUCTURE ONLY: argument marshalling; all arithmetic is in the C file.  Nothing in
this module is shared with, or imported by, the GPU library.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "m2rnn_block_oracle.c")
_LIB = os.path.join(_HERE, "libm2rnn_block_oracle.so")
_lib = None
_DP = ctypes.POINTER(ctypes.c_double)


def build(force=False):
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-fno-fast-math", "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


def _bind(path):
    lib = ctypes.CDLL(path)
    i = ctypes.c_int
    lib.m2rnn_oracle_conv_silu_fwd.restype = i
    lib.m2rnn_oracle_conv_silu_fwd.argtypes = [i, i, i] + [_DP] * 4
    lib.m2rnn_oracle_conv_silu_bwd.restype = i
    lib.m2rnn_oracle_conv_silu_bwd.argtypes = [i, i, i] + [_DP] * 7
    lib.m2rnn_oracle_gated_rmsnorm_fwd.restype = i
    lib.m2rnn_oracle_gated_rmsnorm_fwd.argtypes = [i, i, i] + [_DP] * 3 + [ctypes.c_double] + [_DP] * 2
    lib.m2rnn_oracle_gated_rmsnorm_bwd.restype = i
    lib.m2rnn_oracle_gated_rmsnorm_bwd.argtypes = [i, i, i] + [_DP] * 3 + [ctypes.c_double] + [_DP] * 4
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(build())
    return _lib


def _in(a, shape):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.shape != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (tuple(shape), a.shape))
    return a, a.ctypes.data_as(_DP)


def conv_silu_fwd(x, w, bias=None, _lib=None):
    """out [B,T,C] = SiLU(depthwise causal conv1d of kernel size 4 of x [B,T,C]); w [C,4]."""
    B, T, C = np.shape(x)
    xa, xp = _in(x, (B, T, C))
    wa, wp = _in(w, (C, 4))
    ba, bp = _in(bias, (C,))
    out = np.zeros((B, T, C))
    rc = (_lib or _load()).m2rnn_oracle_conv_silu_fwd(B, T, C, xp, wp, bp, out.ctypes.data_as(_DP))
    assert rc == 0
    return out


def conv_silu_bwd(x, w, bias, dout, _lib=None):
    """(dx, dw, dbias) of sum(out * dout); dbias is None when bias is None."""
    B, T, C = np.shape(x)
    xa, xp = _in(x, (B, T, C))
    wa, wp = _in(w, (C, 4))
    ba, bp = _in(bias, (C,))
    da, dp_ = _in(dout, (B, T, C))
    dx = np.zeros((B, T, C))
    dw = np.zeros((C, 4))
    db = np.zeros(C) if bias is not None else None
    rc = (_lib or _load()).m2rnn_oracle_conv_silu_bwd(
        B, T, C, xp, wp, bp, dp_, dx.ctypes.data_as(_DP), dw.ctypes.data_as(_DP),
        None if db is None else db.ctypes.data_as(_DP))
    assert rc == 0
    return dx, dw, db


def gated_rmsnorm_fwd(y, a, w, eps=0.0, _lib=None):
    """(out [B,T,D], s [B,T]) with out = w (.) x s, x = y (.) SiLU(a), s = 1/sqrt(mean x^2 + eps)."""
    B, T, D = np.shape(y)
    ya, yp = _in(y, (B, T, D))
    aa, ap = _in(a, (B, T, D))
    wa, wp = _in(w, (D,))
    out = np.zeros((B, T, D))
    s = np.zeros((B, T))
    rc = (_lib or _load()).m2rnn_oracle_gated_rmsnorm_fwd(
        B, T, D, yp, ap, wp, float(eps), out.ctypes.data_as(_DP), s.ctypes.data_as(_DP))
    assert rc == 0
    return out, s


def gated_rmsnorm_bwd(y, a, w, eps, dout, _lib=None):
    """(dy, da, dw) of sum(out * dout)."""
    B, T, D = np.shape(y)
    ya, yp = _in(y, (B, T, D))
    aa, ap = _in(a, (B, T, D))
    wa, wp = _in(w, (D,))
    da_, dop = _in(dout, (B, T, D))
    dy = np.zeros((B, T, D))
    da = np.zeros((B, T, D))
    dw = np.zeros(D)
    rc = (_lib or _load()).m2rnn_oracle_gated_rmsnorm_bwd(
        B, T, D, yp, ap, wp, float(eps), dop, dy.ctypes.data_as(_DP), da.ctypes.data_as(_DP),
        dw.ctypes.data_as(_DP))
    assert rc == 0
    return dy, da, dw


class Variant:
    """The four functions bound to another build of the same C interface (the tests use this to
    run the pins against deliberately broken copies)."""

    def __init__(self, path):
        lib = _bind(path)
        self.conv_silu_fwd = lambda *a, **k: conv_silu_fwd(*a, _lib=lib, **k)
        self.conv_silu_bwd = lambda *a, **k: conv_silu_bwd(*a, _lib=lib, **k)
        self.gated_rmsnorm_fwd = lambda *a, **k: gated_rmsnorm_fwd(*a, _lib=lib, **k)
        self.gated_rmsnorm_bwd = lambda *a, **k: gated_rmsnorm_bwd(*a, _lib=lib, **k)
