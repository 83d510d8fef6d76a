"""Thin ctypes binding of libm2rnn.so (the C ABI in include/m2rnn.h).

Same entry-point names as the header; this layer only marshals arguments:
torch tensors own the device memory and supply the stream, every step of the
scan runs inside the library's HIP kernels.  If the library is missing the
import of any entry point raises -- there is no fallback.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libm2rnn.so")

M2RNN_F32 = 0
M2RNN_BF16 = 1

EXPORTS = ("m2rnn_status_string", "m2rnn_default_chunk", "m2rnn_max_chunk",
           "m2rnn_ckpt_bytes", "m2rnn_workspace_bytes", "m2rnn_fwd", "m2rnn_bwd",
           "m2rnn_fwd_opt", "m2rnn_bwd_opt", "m2rnn_fwd_static", "m2rnn_route_string",
           "m2rnn_conv_silu_workspace_bytes", "m2rnn_conv_silu_fwd", "m2rnn_conv_silu_bwd",
           "m2rnn_gated_rmsnorm_workspace_bytes", "m2rnn_gated_rmsnorm_fwd",
           "m2rnn_gated_rmsnorm_bwd")
M2RNN_STATIC_SCRATCH_BYTES = 8 << 20


class m2rnn_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T", ctypes.c_int32), ("N", ctypes.c_int32),
                ("Nqk", ctypes.c_int32), ("K", ctypes.c_int32), ("V", ctypes.c_int32),
                ("io", ctypes.c_int32), ("chunk", ctypes.c_int32), ("flags", ctypes.c_uint32)]


class m2rnn_opts(ctypes.Structure):
    _fields_ = [("w_r", ctypes.c_void_p), ("dw_r", ctypes.c_void_p), ("grad_clip", ctypes.c_float),
                ("gate_alpha", ctypes.c_void_p), ("gate_beta", ctypes.c_void_p),
                ("dgate_alpha", ctypes.c_void_p), ("dgate_beta", ctypes.c_void_p)]


class M2RNNError(RuntimeError):
    def __init__(self, code, where):
        self.code = int(code)
        super().__init__("%s failed: [%d] %s" % (where, self.code, m2rnn_status_string(self.code)))


_lib = None


def lib():
    """Loads libm2rnn.so once; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libm2rnn.so is not built (%s); run `python -m paper_2603_14360_amd.build`. "
                "There is no fallback path." % LIB_PATH)
        # torch first: it ships its own HIP runtime, and the library must bind to that copy
        # (the one that owns the tensors and streams passed in), not load a second one
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, dp = ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(m2rnn_desc)
        L.m2rnn_status_string.restype = ctypes.c_char_p
        L.m2rnn_status_string.argtypes = [ctypes.c_int]
        L.m2rnn_default_chunk.restype = ctypes.c_int32
        L.m2rnn_default_chunk.argtypes = [dp]
        L.m2rnn_max_chunk.restype = ctypes.c_int32
        L.m2rnn_max_chunk.argtypes = [dp]
        L.m2rnn_ckpt_bytes.restype = sz
        L.m2rnn_ckpt_bytes.argtypes = [dp]
        L.m2rnn_workspace_bytes.restype = sz
        L.m2rnn_workspace_bytes.argtypes = [dp, ctypes.c_int]
        L.m2rnn_fwd.restype = ctypes.c_int
        L.m2rnn_fwd.argtypes = [dp] + [vp] * 10 + [sz, vp]
        L.m2rnn_bwd.restype = ctypes.c_int
        L.m2rnn_bwd.argtypes = [dp] + [vp] * 16 + [sz, vp]
        op = ctypes.POINTER(m2rnn_opts)
        L.m2rnn_fwd_opt.restype = ctypes.c_int
        L.m2rnn_fwd_opt.argtypes = [dp, op] + [vp] * 10 + [sz, vp]
        L.m2rnn_bwd_opt.restype = ctypes.c_int
        L.m2rnn_bwd_opt.argtypes = [dp, op] + [vp] * 16 + [sz, vp]
        L.m2rnn_route_string.restype = ctypes.c_char_p
        L.m2rnn_route_string.argtypes = [dp, ctypes.c_int]
        L.m2rnn_fwd_static.restype = ctypes.c_int
        L.m2rnn_fwd_static.argtypes = [dp, op] + [vp] * 9 + [vp]
        i32, fl = ctypes.c_int32, ctypes.c_float
        L.m2rnn_conv_silu_workspace_bytes.restype = sz
        L.m2rnn_conv_silu_workspace_bytes.argtypes = [i32] * 3
        L.m2rnn_conv_silu_fwd.restype = ctypes.c_int
        L.m2rnn_conv_silu_fwd.argtypes = [i32] * 4 + [vp] * 5
        L.m2rnn_conv_silu_bwd.restype = ctypes.c_int
        L.m2rnn_conv_silu_bwd.argtypes = [i32] * 4 + [vp] * 8 + [sz, vp]
        L.m2rnn_gated_rmsnorm_workspace_bytes.restype = sz
        L.m2rnn_gated_rmsnorm_workspace_bytes.argtypes = [i32] * 3
        L.m2rnn_gated_rmsnorm_fwd.restype = ctypes.c_int
        L.m2rnn_gated_rmsnorm_fwd.argtypes = [i32] * 4 + [vp] * 3 + [fl] + [vp] * 3
        L.m2rnn_gated_rmsnorm_bwd.restype = ctypes.c_int
        L.m2rnn_gated_rmsnorm_bwd.argtypes = [i32] * 4 + [vp] * 3 + [fl] + [vp] * 6 + [sz, vp]
        _lib = L
    return _lib


def make_desc(B, T, N, K, V, io, Nqk=None, chunk=0, flags=0):
    return m2rnn_desc(B, T, N, N if Nqk is None else Nqk, K, V, io, chunk, flags)


def m2rnn_status_string(code):
    return lib().m2rnn_status_string(int(code)).decode()


def m2rnn_default_chunk(desc):
    return int(lib().m2rnn_default_chunk(ctypes.byref(desc)))


def m2rnn_max_chunk(desc):
    return int(lib().m2rnn_max_chunk(ctypes.byref(desc)))


def m2rnn_route_string(desc, bwd):
    return lib().m2rnn_route_string(ctypes.byref(desc), int(bwd)).decode()


def m2rnn_ckpt_bytes(desc):
    return int(lib().m2rnn_ckpt_bytes(ctypes.byref(desc)))


def m2rnn_workspace_bytes(desc, bwd):
    return int(lib().m2rnn_workspace_bytes(ctypes.byref(desc), int(bwd)))


def _ptr(x):
    """Device (or raw integer) address of a tensor; None -> NULL."""
    if x is None:
        return None
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    return ctypes.c_void_p(x.data_ptr())


def _nbytes(x):
    return 0 if x is None else x.numel() * x.element_size()


def m2rnn_fwd(desc, q, k, v, f, W, H0, y, HT, ckpt, workspace, stream=None, check=True):
    """Raw call: every argument is a torch tensor on the GPU (or None where the
    header allows NULL); `stream` is a raw hipStream_t handle (int) or None."""
    rc = lib().m2rnn_fwd(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(f), _ptr(W),
                         _ptr(H0), _ptr(y), _ptr(HT), _ptr(ckpt), _ptr(workspace),
                         _nbytes(workspace), ctypes.c_void_p(stream or 0))
    if check and rc != 0:
        raise M2RNNError(rc, "m2rnn_fwd")
    return rc


def m2rnn_bwd(desc, q, k, v, f, W, H0, ckpt, dy, dHT, dq, dk, dv, df, dW, dH0, workspace,
              stream=None, check=True):
    rc = lib().m2rnn_bwd(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(f), _ptr(W),
                         _ptr(H0), _ptr(ckpt), _ptr(dy), _ptr(dHT), _ptr(dq), _ptr(dk), _ptr(dv),
                         _ptr(df), _ptr(dW), _ptr(dH0), _ptr(workspace), _nbytes(workspace),
                         ctypes.c_void_p(stream or 0))
    if check and rc != 0:
        raise M2RNNError(rc, "m2rnn_bwd")
    return rc


def make_opts(w_r=None, dw_r=None, grad_clip=0.0, gate=None, dgate=None):
    """m2rnn_opts from torch tensors (or None); gate = (alpha, beta), dgate = (dalpha, dbeta)."""
    p = lambda x: None if x is None else x.data_ptr()
    ga, gb = gate if gate is not None else (None, None)
    da, db = dgate if dgate is not None else (None, None)
    return m2rnn_opts(p(w_r), p(dw_r), float(grad_clip), p(ga), p(gb), p(da), p(db))


def m2rnn_fwd_opt(desc, opts, q, k, v, f, W, H0, y, HT, ckpt, workspace, stream=None, check=True):
    """m2rnn_fwd with an m2rnn_opts (None = no options)."""
    rc = lib().m2rnn_fwd_opt(ctypes.byref(desc), None if opts is None else ctypes.byref(opts),
                             _ptr(q), _ptr(k), _ptr(v), _ptr(f), _ptr(W), _ptr(H0), _ptr(y),
                             _ptr(HT), _ptr(ckpt), _ptr(workspace), _nbytes(workspace),
                             ctypes.c_void_p(stream or 0))
    if check and rc != 0:
        raise M2RNNError(rc, "m2rnn_fwd_opt")
    return rc


def m2rnn_fwd_static(desc, opts, q, k, v, f, W, H0, y, HT, ckpt, stream=None, check=True):
    """m2rnn_fwd_opt on the library's own static scratch (no workspace argument)."""
    rc = lib().m2rnn_fwd_static(ctypes.byref(desc), None if opts is None else ctypes.byref(opts),
                                _ptr(q), _ptr(k), _ptr(v), _ptr(f), _ptr(W), _ptr(H0), _ptr(y),
                                _ptr(HT), _ptr(ckpt), ctypes.c_void_p(stream or 0))
    if check and rc != 0:
        raise M2RNNError(rc, "m2rnn_fwd_static")
    return rc


def m2rnn_bwd_opt(desc, opts, q, k, v, f, W, H0, ckpt, dy, dHT, dq, dk, dv, df, dW, dH0,
                  workspace, stream=None, check=True):
    rc = lib().m2rnn_bwd_opt(ctypes.byref(desc), None if opts is None else ctypes.byref(opts),
                             _ptr(q), _ptr(k), _ptr(v), _ptr(f), _ptr(W), _ptr(H0), _ptr(ckpt),
                             _ptr(dy), _ptr(dHT), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(df),
                             _ptr(dW), _ptr(dH0), _ptr(workspace), _nbytes(workspace),
                             ctypes.c_void_p(stream or 0))
    if check and rc != 0:
        raise M2RNNError(rc, "m2rnn_bwd_opt")
    return rc


def _io_code(t):
    import torch
    return M2RNN_BF16 if t.dtype == torch.bfloat16 else M2RNN_F32


def _check(rc, where, check):
    if check and rc != 0:
        raise M2RNNError(rc, where)
    return rc


def m2rnn_conv_silu_workspace_bytes(B, T, C):
    return int(lib().m2rnn_conv_silu_workspace_bytes(B, T, C))


def m2rnn_conv_silu_fwd(x, w, bias, out, stream=None, check=True):
    """out = SiLU(causal depthwise conv1d(4) of x [B,T,C]); w [C,4], bias [C] or None."""
    B, T, C = x.shape
    rc = lib().m2rnn_conv_silu_fwd(B, T, C, _io_code(x), _ptr(x), _ptr(w), _ptr(bias), _ptr(out),
                                   ctypes.c_void_p(stream or 0))
    return _check(rc, "m2rnn_conv_silu_fwd", check)


def m2rnn_conv_silu_bwd(x, w, bias, dout, dx, dw, dbias, workspace, stream=None, check=True):
    B, T, C = x.shape
    rc = lib().m2rnn_conv_silu_bwd(B, T, C, _io_code(x), _ptr(x), _ptr(w), _ptr(bias), _ptr(dout),
                                   _ptr(dx), _ptr(dw), _ptr(dbias), _ptr(workspace),
                                   _nbytes(workspace), ctypes.c_void_p(stream or 0))
    return _check(rc, "m2rnn_conv_silu_bwd", check)


def m2rnn_gated_rmsnorm_workspace_bytes(B, T, D):
    return int(lib().m2rnn_gated_rmsnorm_workspace_bytes(B, T, D))


def m2rnn_gated_rmsnorm_fwd(y, a, w, eps, out, s, stream=None, check=True):
    """out = RMSNorm(y (.) SiLU(a)) over the last axis of [B,T,D]; s [B,T] fp32 or None."""
    B, T, D = y.shape
    rc = lib().m2rnn_gated_rmsnorm_fwd(B, T, D, _io_code(y), _ptr(y), _ptr(a), _ptr(w), float(eps),
                                       _ptr(out), _ptr(s), ctypes.c_void_p(stream or 0))
    return _check(rc, "m2rnn_gated_rmsnorm_fwd", check)


def m2rnn_gated_rmsnorm_bwd(y, a, w, eps, s, dout, dy, da, dw, workspace, stream=None, check=True):
    B, T, D = y.shape
    rc = lib().m2rnn_gated_rmsnorm_bwd(B, T, D, _io_code(y), _ptr(y), _ptr(a), _ptr(w), float(eps),
                                       _ptr(s), _ptr(dout), _ptr(dy), _ptr(da), _ptr(dw),
                                       _ptr(workspace), _nbytes(workspace),
                                       ctypes.c_void_p(stream or 0))
    return _check(rc, "m2rnn_gated_rmsnorm_bwd", check)


# --------------------------------------------------------------------------
# Buffer plumbing for callers that hold torch tensors: allocates outputs,
# checkpoints and workspace with torch and calls the raw entry points on
# torch's current stream.  No arithmetic happens here.
class Scan:
    """Owns the outputs / checkpoint / workspace buffers of one problem shape."""

    def __init__(self, B, T, N, K, V, io, Nqk=None, chunk=0, backward=True, device="cuda"):
        import torch
        self.torch = torch
        self.desc = make_desc(B, T, N, K, V, M2RNN_BF16 if io in ("bf16", M2RNN_BF16) else M2RNN_F32,
                              Nqk=Nqk, chunk=chunk)
        d = self.desc
        self.io_dtype = torch.bfloat16 if d.io == M2RNN_BF16 else torch.float32
        dev = device
        self.y = torch.empty((B, T, N, V), dtype=self.io_dtype, device=dev)
        self.HT = torch.empty((B, N, K, V), dtype=torch.float32, device=dev)
        self.backward = backward
        ws = m2rnn_workspace_bytes(d, 0)
        if backward:
            # (2: also room for the backward's own checkpoint pass, used by bwd(use_ckpt=False))
            ws = max(ws, m2rnn_workspace_bytes(d, 2))
            self.ckpt = torch.empty(max(1, m2rnn_ckpt_bytes(d) // 4), dtype=torch.float32, device=dev)
            self.dq = torch.empty((B, T, d.Nqk, K), dtype=self.io_dtype, device=dev)
            self.dk = torch.empty((B, T, d.Nqk, K), dtype=self.io_dtype, device=dev)
            self.dv = torch.empty((B, T, N, V), dtype=self.io_dtype, device=dev)
            self.df = torch.empty((B, T, N), dtype=torch.float32, device=dev)
            self.dW = torch.empty((N, V, V), dtype=torch.float32, device=dev)
            self.dH0 = torch.empty((B, N, K, V), dtype=torch.float32, device=dev)
        else:
            self.ckpt = None
        self.workspace = torch.empty(max(ws, 256), dtype=torch.uint8, device=dev)

    def _stream(self):
        return self.torch.cuda.current_stream().cuda_stream

    def fwd(self, q, k, v, f, W, H0=None, w_r=None, gate=None):
        """w_r [N,V] (io dtype): adds the residual w_r (.) v_t to y_t.  gate = (alpha, beta)
        [N] fp32 each: f is the input of the forget-gate function."""
        if w_r is None and gate is None:
            m2rnn_fwd(self.desc, q, k, v, f, W, H0, self.y, self.HT, self.ckpt, self.workspace,
                      stream=self._stream())
        else:
            m2rnn_fwd_opt(self.desc, make_opts(w_r=w_r, gate=gate), q, k, v, f, W, H0, self.y,
                          self.HT, self.ckpt, self.workspace, stream=self._stream())
        return self.y, self.HT

    def bwd(self, q, k, v, f, W, H0, dy, dHT=None, use_ckpt=True, w_r=None, grad_clip=0.0,
            gate=None):
        """With w_r the result has a further entry, dw_r [N,V] fp32; with gate two more,
        dalpha and dbeta [N] fp32 (and df is the gradient of the gate's input)."""
        ck = self.ckpt if use_ckpt else None
        if w_r is None and gate is None and not grad_clip > 0:
            m2rnn_bwd(self.desc, q, k, v, f, W, H0, ck, dy, dHT, self.dq, self.dk, self.dv,
                      self.df, self.dW, self.dH0, self.workspace, stream=self._stream())
            return self.dq, self.dk, self.dv, self.df, self.dW, self.dH0
        dw_r = None
        if w_r is not None:
            dw_r = self.torch.empty((self.desc.N, self.desc.V), dtype=self.torch.float32,
                                    device=self.dW.device)
        dgate = None
        if gate is not None:
            dgate = tuple(self.torch.empty((self.desc.N,), dtype=self.torch.float32,
                                           device=self.dW.device) for _ in range(2))
        m2rnn_bwd_opt(self.desc, make_opts(w_r, dw_r, grad_clip, gate, dgate), q, k, v, f, W, H0,
                      ck, dy, dHT, self.dq, self.dk, self.dv, self.df, self.dW, self.dH0,
                      self.workspace, stream=self._stream())
        out = (self.dq, self.dk, self.dv, self.df, self.dW, self.dH0)
        if dw_r is not None:
            out = out + (dw_r,)
        if dgate is not None:
            out = out + dgate
        return out
