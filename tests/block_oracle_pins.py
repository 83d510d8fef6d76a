"""Checks that pin the float64 oracle of the scan's neighbours (conv1d(4) + SiLU prologue,
gated RMSNorm epilogue) to things other than itself: a library convolution and reverse-mode
autodiff (torch, float64), closed forms, invariants, finite differences.  Every check takes
the oracle as an object with the four functions, so that the same checks can be pointed at
deliberately broken copies (test_block_oracle.py)."""
import numpy as np


def relerr(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.abs(b).max()
    return np.abs(a - b).max() / (den if den > 0 else 1.0)


def _conv_case(seed, B=2, T=9, C=5, bias=True):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, T, C)), rng.standard_normal((C, 4)) * 0.7,
            rng.standard_normal(C) * 0.3 if bias else None, rng.standard_normal((B, T, C)))


def check_conv_against_library_conv1d(o, tol=1e-12):
    """Layer equations for q_t, k_t, v_t: depthwise causal conv1d (kernel 4) + SiLU, against
    torch's conv1d on a left-padded sequence and its autograd."""
    import torch
    import torch.nn.functional as F
    for bias in (True, False):
        x, w, b, dout = _conv_case(3, bias=bias)
        xt = torch.tensor(x, requires_grad=True)
        wt = torch.tensor(w, requires_grad=True)
        bt = torch.tensor(b, requires_grad=True) if bias else None
        pre = F.conv1d(F.pad(xt.transpose(1, 2), (3, 0)), wt[:, None, :], bt, groups=x.shape[2])
        out = F.silu(pre).transpose(1, 2)
        (out * torch.tensor(dout)).sum().backward()
        assert relerr(o.conv_silu_fwd(x, w, b), out.detach().numpy()) < tol
        dx, dw, db = o.conv_silu_bwd(x, w, b, dout)
        assert relerr(dx, xt.grad.numpy()) < tol
        assert relerr(dw, wt.grad.numpy()) < tol
        if bias:
            assert relerr(db, bt.grad.numpy()) < tol
        else:
            assert db is None


def check_conv_closed_forms(o, tol=1e-14):
    """T = 1: only the last tap sees data.  A one-hot kernel is a delay line."""
    silu = lambda u: u / (1.0 + np.exp(-u))
    x, w, b, _ = _conv_case(4, T=1)
    assert relerr(o.conv_silu_fwd(x, w, b), silu(w[None, None, :, 3] * x + b)) < tol
    x, w, b, _ = _conv_case(5, T=8)
    for tap in range(4):
        w1 = np.zeros_like(w)
        w1[:, tap] = 1.0
        out = o.conv_silu_fwd(x, w1, None)
        delayed = np.zeros_like(x)
        d = 3 - tap
        delayed[:, d:] = x[:, :x.shape[1] - d]
        assert relerr(out, silu(delayed)) < tol


def check_conv_is_causal(o):
    x, w, b, _ = _conv_case(6, T=12)
    base = o.conv_silu_fwd(x, w, b)
    x2 = x.copy()
    x2[:, 5] += 1.0
    out = o.conv_silu_fwd(x2, w, b)
    assert np.array_equal(out[:, :5], base[:, :5])          # nothing before the change
    assert np.array_equal(out[:, 9:], base[:, 9:])          # nothing more than 3 steps after
    assert np.abs(out[:, 5:9] - base[:, 5:9]).min() > 0     # every step in between


def check_conv_finite_differences(o, h=1e-6, tol=1e-7):
    x, w, b, dout = _conv_case(7, B=1, T=6, C=3)
    dx, dw, db = o.conv_silu_bwd(x, w, b, dout)
    L = lambda x_, w_, b_: float((o.conv_silu_fwd(x_, w_, b_) * dout).sum())
    rng = np.random.default_rng(0)
    for arr, grad, which in ((x, dx, 0), (w, dw, 1), (b, db, 2)):
        for _ in range(6):
            idx = tuple(rng.integers(0, s) for s in arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[idx] += h
            am[idx] -= h
            args_p = [x, w, b]
            args_m = [x, w, b]
            args_p[which], args_m[which] = ap, am
            fd = (L(*args_p) - L(*args_m)) / (2 * h)
            assert abs(fd - grad[idx]) <= tol * max(1.0, abs(fd)), (which, idx, fd, grad[idx])


def _norm_case(seed, B=2, T=3, D=12):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, T, D)), rng.standard_normal((B, T, D)),
            rng.uniform(0.5, 1.5, D), rng.standard_normal((B, T, D)))


def check_rmsnorm_invariants(o, tol=1e-13):
    """RMSNorm appendix: with w = 1, eps = 0 the output has unit mean square per token, does not
    change when y is rescaled, s is the inverse root mean square of y (.) SiLU(a), and the
    gradient with respect to x = y (.) g is orthogonal to x."""
    y, a, w, dout = _norm_case(8)
    one = np.ones_like(w)
    out, s = o.gated_rmsnorm_fwd(y, a, one, 0.0)
    assert relerr((out ** 2).mean(axis=-1), np.ones(out.shape[:2])) < tol
    out2, s2 = o.gated_rmsnorm_fwd(3.7 * y, a, one, 0.0)
    assert relerr(out2, out) < tol and relerr(s2 * 3.7, s) < tol
    g = a / (1.0 + np.exp(-a))
    assert relerr(s, 1.0 / np.sqrt(((y * g) ** 2).mean(axis=-1))) < tol
    dy, da, dw = o.gated_rmsnorm_bwd(y, a, w, 0.0, dout)
    # dy = dx g  =>  sum_i dx_i x_i = sum_i dy_i y_i = 0 (scale invariance of the output)
    assert np.abs((dy * y).sum(axis=-1)).max() < 1e-12 * np.abs(dy * y).max() * y.shape[-1]


def check_rmsnorm_one_feature_closed_form(o, tol=1e-13):
    """d = 1, eps = 0: out = w sign(x)."""
    rng = np.random.default_rng(9)
    y = rng.standard_normal((2, 4, 1))
    a = rng.standard_normal((2, 4, 1))
    w = np.array([1.7])
    out, _ = o.gated_rmsnorm_fwd(y, a, w, 0.0)
    g = a / (1.0 + np.exp(-a))
    assert relerr(out, 1.7 * np.sign(y * g)) < tol


def check_rmsnorm_against_autodiff(o, tol=1e-12):
    import torch
    import torch.nn.functional as F
    for eps in (0.0, 1e-3):
        y, a, w, dout = _norm_case(10)
        yt, at, wt = (torch.tensor(v, requires_grad=True) for v in (y, a, w))
        x = yt * F.silu(at)
        out = wt * x * torch.rsqrt((x * x).mean(dim=-1, keepdim=True) + eps)
        (out * torch.tensor(dout)).sum().backward()
        got, _ = o.gated_rmsnorm_fwd(y, a, w, eps)
        assert relerr(got, out.detach().numpy()) < tol
        dy, da, dw = o.gated_rmsnorm_bwd(y, a, w, eps, dout)
        assert relerr(dy, yt.grad.numpy()) < tol
        assert relerr(da, at.grad.numpy()) < tol
        assert relerr(dw, wt.grad.numpy()) < tol


def check_rmsnorm_finite_differences(o, h=1e-6, tol=1e-7):
    y, a, w, dout = _norm_case(11, B=1, T=2, D=6)
    eps = 1e-2
    dy, da, dw = o.gated_rmsnorm_bwd(y, a, w, eps, dout)
    L = lambda y_, a_, w_: float((o.gated_rmsnorm_fwd(y_, a_, w_, eps)[0] * dout).sum())
    rng = np.random.default_rng(1)
    for which, (arr, grad) in enumerate(((y, dy), (a, da), (w, dw))):
        for _ in range(6):
            idx = tuple(rng.integers(0, s) for s in arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[idx] += h
            am[idx] -= h
            args_p, args_m = [y, a, w], [y, a, w]
            args_p[which], args_m[which] = ap, am
            fd = (L(*args_p) - L(*args_m)) / (2 * h)
            assert abs(fd - grad[idx]) <= tol * max(1.0, abs(fd)), (which, idx, fd, grad[idx])


ALL_CHECKS = [check_conv_against_library_conv1d, check_conv_closed_forms, check_conv_is_causal,
              check_conv_finite_differences, check_rmsnorm_invariants,
              check_rmsnorm_one_feature_closed_form, check_rmsnorm_against_autodiff,
              check_rmsnorm_finite_differences]
