"""ctypes front end of the float64 oracle (``m2rnn_oracle.c``).

TEST INFRASTRUCTURE ONLY: argument marshalling for the plain-C oracle.  All of
the recurrence's arithmetic is in the C file, which follows the paper's
recurrence equations (forward) and its backward algorithm (BPTT).  Nothing in
this module is shared with, or imported by, the GPU library.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "m2rnn_oracle.c")
_LIB = os.path.join(_HERE, "libm2rnn_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP over independent (b, n) units)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared",
                           "-fno-fast-math", "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


def _bind(path):
    lib = ctypes.CDLL(path)
    dp = ctypes.POINTER(ctypes.c_double)
    lib.m2rnn_oracle_fwd.restype = ctypes.c_int
    lib.m2rnn_oracle_fwd.argtypes = [ctypes.c_int] * 6 + [dp] * 11
    lib.m2rnn_oracle_bwd.restype = ctypes.c_int
    lib.m2rnn_oracle_bwd.argtypes = ([ctypes.c_int] * 6 + [dp] * 7 + [ctypes.c_double]
                                     + [dp] * 13)
    lib.m2rnn_oracle_num_threads.restype = ctypes.c_int
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(build())
    return _lib


def num_threads():
    return int(_load().m2rnn_oracle_num_threads())


def _in(a, shape):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.shape != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (tuple(shape), a.shape))
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _shapes(q, v):
    B, T, Nqk, K = q.shape
    B2, T2, N, V = v.shape
    if (B, T) != (B2, T2):
        raise ValueError("q and v disagree on (B, T)")
    return B, T, N, Nqk, K, V


def fwd(q, k, v, f, W, H0=None, w_r=None, gate=None, _lib=None):
    """y [B,T,N,V], HT [B,N,K,V] from q,k [B,T,Nqk,K], v [B,T,N,V], f [B,T,N],
    W [N,V,V], H0 [B,N,K,V] or None (zero state); w_r [N,V] or None adds the
    residual w_r (.) v_t to y_t; gate = (alpha [N], beta [N]) makes f the input of
    the forget-gate function psi instead of the gate value."""
    q = np.asarray(q)
    v = np.asarray(v)
    B, T, N, Nqk, K, V = _shapes(q, v)
    qa, qp = _in(q, (B, T, Nqk, K))
    ka, kp = _in(k, (B, T, Nqk, K))
    va, vp = _in(v, (B, T, N, V))
    fa, fp = _in(f, (B, T, N))
    Wa, Wp = _in(W, (N, V, V))
    Ha, Hp = _in(H0, (B, N, K, V))
    ra, rp = _in(w_r, (N, V))
    aa, ap = _in(None if gate is None else gate[0], (N,))
    ba, bp = _in(None if gate is None else gate[1], (N,))
    y = np.zeros((B, T, N, V))
    HT = np.zeros((B, N, K, V))
    dp = ctypes.POINTER(ctypes.c_double)
    rc = (_lib or _load()).m2rnn_oracle_fwd(
        B, T, N, Nqk, K, V, qp, kp, vp, fp, Wp, Hp, rp, ap, bp,
        y.ctypes.data_as(dp), HT.ctypes.data_as(dp))
    if rc != 0:
        raise RuntimeError("m2rnn_oracle_fwd failed with code %d" % rc)
    return y, HT


def bwd(q, k, v, f, W, H0, dy, dHT=None, w_r=None, clip=0.0, gate=None, _lib=None):
    """Gradients (dq, dk, dv, df, dW, dH0) of  sum(y*dy) + sum(HT*dHT); with
    w_r [N,V] the residual is part of y and dw_r is appended to the result;
    clip > 0 clamps the state gradient handed from each step to the one before;
    gate = (alpha, beta): f is the gate function's input, df is the gradient with
    respect to it, and (dalpha, dbeta) are appended to the result."""
    q = np.asarray(q)
    v = np.asarray(v)
    B, T, N, Nqk, K, V = _shapes(q, v)
    qa, qp = _in(q, (B, T, Nqk, K))
    ka, kp = _in(k, (B, T, Nqk, K))
    va, vp = _in(v, (B, T, N, V))
    fa, fp = _in(f, (B, T, N))
    Wa, Wp = _in(W, (N, V, V))
    Ha, Hp = _in(H0, (B, N, K, V))
    dya, dyp = _in(dy, (B, T, N, V))
    dHa, dHp = _in(dHT, (B, N, K, V))
    ra, rp = _in(w_r, (N, V))
    dw_r = np.zeros((N, V))
    aa, ap = _in(None if gate is None else gate[0], (N,))
    ba, bp = _in(None if gate is None else gate[1], (N,))
    dalpha = np.zeros(N)
    dbeta = np.zeros(N)
    dq = np.zeros((B, T, Nqk, K))
    dk = np.zeros((B, T, Nqk, K))
    dv = np.zeros((B, T, N, V))
    df = np.zeros((B, T, N))
    dW = np.zeros((N, V, V))
    dH0 = np.zeros((B, N, K, V))
    dp = ctypes.POINTER(ctypes.c_double)
    rc = (_lib or _load()).m2rnn_oracle_bwd(
        B, T, N, Nqk, K, V, qp, kp, vp, fp, Wp, Hp, rp, float(clip), ap, bp, dyp, dHp,
        dq.ctypes.data_as(dp), dk.ctypes.data_as(dp), dv.ctypes.data_as(dp),
        df.ctypes.data_as(dp), dW.ctypes.data_as(dp), dH0.ctypes.data_as(dp),
        dw_r.ctypes.data_as(dp), dalpha.ctypes.data_as(dp), dbeta.ctypes.data_as(dp))
    if rc != 0:
        raise RuntimeError("m2rnn_oracle_bwd failed with code %d" % rc)
    out = (dq, dk, dv, df, dW, dH0)
    if w_r is not None:
        out = out + (dw_r,)
    if gate is not None:
        out = out + (dalpha, dbeta)
    return out


def variant(path):
    """(fwd, bwd) bound to another build of the same C interface (the tests
    use this to run the pins against deliberately broken copies)."""
    lib = _bind(path)
    return (lambda *a, **kw: fwd(*a, _lib=lib, **kw),
            lambda *a, **kw: bwd(*a, _lib=lib, **kw))
