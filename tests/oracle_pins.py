"""Checks that pin the float64 oracle to things other than itself.

Every check takes the oracle as a pair of callables ``(fwd, bwd)`` so that the
same checks can be pointed at deliberately broken copies of the oracle (see
``test_oracle_mutations.py``) to show that they would notice a mistake.

Each check follows from the paper's recurrence equations
  Z_t = tanh(H_{t-1} W + k_t v_t^T),  H_t = f_t H_{t-1} + (1 - f_t) Z_t,
  y_t = H_t^T q_t
or from Theorem 1 (the Elman-RNN special case).  None of them re-types the
oracle's loops: they use closed forms, a reverse-mode autodiff library on an
independently written unrolled forward, finite differences, or invariants.
"""
import numpy as np


def rand_case(seed, B, T, N, K, V, Nqk=None, H0=True, scale=0.7):
    rng = np.random.default_rng(seed)
    Nqk = N if Nqk is None else Nqk
    c = {
        "q": rng.standard_normal((B, T, Nqk, K)) * scale,
        "k": rng.standard_normal((B, T, Nqk, K)) * scale,
        "v": rng.standard_normal((B, T, N, V)) * scale,
        "f": rng.uniform(0.05, 0.95, (B, T, N)),
        "W": rng.standard_normal((N, V, V)) * V ** -0.5,
        "H0": rng.standard_normal((B, N, K, V)) * 0.3 if H0 else None,
        "dy": rng.standard_normal((B, T, N, V)),
        "dHT": rng.standard_normal((B, N, K, V)),
    }
    return c


def _args(c):
    return c["q"], c["k"], c["v"], c["f"], c["W"], c["H0"]


def relerr(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.abs(b).max()
    return np.abs(a - b).max() / (den if den > 0 else 1.0)


# --------------------------------------------------------------------------
# T = 1 closed form (forward and every gradient), from the three equations.
def check_T1_closed_form(fwd, bwd, tol=1e-13):
    c = rand_case(11, 2, 1, 3, 4, 5)
    q, k, v, f, W, H0 = _args(c)
    y, HT = fwd(q, k, v, f, W, H0)
    dq, dk, dv, df, dW, dH0 = bwd(q, k, v, f, W, H0, c["dy"], c["dHT"])
    dW_ref = np.zeros_like(W)
    for b in range(2):
        for n in range(3):
            Z = np.tanh(H0[b, n] @ W[n] + np.outer(k[b, 0, n], v[b, 0, n]))
            H1 = f[b, 0, n] * H0[b, n] + (1 - f[b, 0, n]) * Z
            assert relerr(HT[b, n], H1) < tol
            assert relerr(y[b, 0, n], H1.T @ q[b, 0, n]) < tol
            G = np.outer(q[b, 0, n], c["dy"][b, 0, n]) + c["dHT"][b, n]
            dS = (1 - f[b, 0, n]) * G * (1 - Z * Z)
            assert relerr(dq[b, 0, n], H1 @ c["dy"][b, 0, n]) < tol
            assert abs(df[b, 0, n] - np.sum(G * (H0[b, n] - Z))) < tol * 10
            assert relerr(dk[b, 0, n], dS @ v[b, 0, n]) < tol
            assert relerr(dv[b, 0, n], dS.T @ k[b, 0, n]) < tol
            assert relerr(dH0[b, n], f[b, 0, n] * G + dS @ W[n].T) < tol
            dW_ref[n] += H0[b, n].T @ dS
    assert relerr(dW, dW_ref) < tol
    # zero initial state: H_1 = (1 - f) tanh(k v^T)
    y0, HT0 = fwd(q, k, v, f, W, None)
    for b in range(2):
        for n in range(3):
            H1 = (1 - f[b, 0, n]) * np.tanh(np.outer(k[b, 0, n], v[b, 0, n]))
            assert relerr(HT0[b, n], H1) < tol
            assert relerr(y0[b, 0, n], H1.T @ q[b, 0, n]) < tol


# --------------------------------------------------------------------------
# Brute force: the forward unrolled with torch float64 tensor expressions and
# differentiated by torch.autograd (a library's reverse mode, independent of
# the hand-derived backward).
def torch_unrolled(c, need_grad=True, clip=0.0):
    """With "w_r" in the case the residual w_r (.) v_t is added to y_t.  clip > 0 clamps
    the gradient that autograd sends along every recurrent edge (state handed from one
    step to the next, and H0 to the first step); the readout of a state is not on it."""
    import torch
    names = (("q", "k", "v", "f", "W", "H0") + (("w_r",) if "w_r" in c else ())
             + (("alpha", "beta") if "alpha" in c else ()))
    t = {n: (None if c[n] is None else
             torch.tensor(c[n], dtype=torch.float64, requires_grad=need_grad))
         for n in names}

    def edge(H):
        if clip <= 0 or not need_grad or not H.requires_grad:
            return H
        Hc = H.clone()
        Hc.register_hook(lambda g: g.clamp(-clip, clip))
        return Hc
    B, T, Nqk, K = c["q"].shape
    N, V = c["v"].shape[2], c["v"].shape[3]
    per = N // Nqk
    ys, HTs = [], []
    for b in range(B):
        yb, Hb = [], []
        for n in range(N):
            g = n // per
            H = t["H0"][b, n] if t["H0"] is not None else torch.zeros(K, V, dtype=torch.float64)
            yn = []
            for s in range(T):
                Hp = edge(H)
                Z = torch.tanh(Hp @ t["W"][n] + torch.outer(t["k"][b, s, g], t["v"][b, s, n]))
                fs = t["f"][b, s, n]
                if "alpha" in t:  # the forget-gate function in its printed (power) form
                    fs = (1 + torch.exp(fs + t["beta"][n])) ** (-t["alpha"][n])
                H = fs * Hp + (1 - fs) * Z
                yt = H.T @ t["q"][b, s, g]
                if "w_r" in t:
                    yt = yt + t["w_r"][n] * t["v"][b, s, n]
                yn.append(yt)
            yb.append(torch.stack(yn) if T > 0 else torch.zeros(0, V, dtype=torch.float64))
            Hb.append(H)
        ys.append(torch.stack(yb, dim=1))       # [T, N, V]
        HTs.append(torch.stack(Hb))             # [N, K, V]
    y = torch.stack(ys)
    HT = torch.stack(HTs)
    if not need_grad:
        return y.detach().numpy(), HT.detach().numpy(), None
    loss = (y * torch.tensor(c["dy"])).sum() + (HT * torch.tensor(c["dHT"])).sum()
    loss.backward()
    grads = {n: (None if t[n] is None else t[n].grad.numpy()) for n in t}
    return y.detach().numpy(), HT.detach().numpy(), grads


def check_unrolled_autograd(fwd, bwd, shapes=None, tol=1e-11):
    shapes = shapes or [(1, 1, 3, 2, 2, None), (2, 1, 4, 3, 5, None),
                        (2, 4, 3, 4, 3, 2), (1, 4, 5, 3, 4, 1),
                        (1, 2, 3, 16, 16, None)]
    for (B, N, T, K, V, Nqk) in shapes:
        for with_H0 in (True, False):
            c = rand_case(100 + T + K, B, T, N, K, V, Nqk=Nqk, H0=with_H0)
            y_t, HT_t, g = torch_unrolled(c)
            y, HT = fwd(*_args(c))
            assert relerr(y, y_t) < tol and relerr(HT, HT_t) < tol
            dq, dk, dv, df, dW, dH0 = bwd(*_args(c), c["dy"], c["dHT"])
            assert relerr(dq, g["q"]) < tol, "dq"
            assert relerr(dk, g["k"]) < tol, "dk"
            assert relerr(dv, g["v"]) < tol, "dv"
            assert relerr(df, g["f"]) < tol, "df"
            assert relerr(dW, g["W"]) < tol, "dW"
            if with_H0:
                assert relerr(dH0, g["H0"]) < tol, "dH0"


# --------------------------------------------------------------------------
# The residual w_r (.) v_t of the y equation and per-step clipping of the state gradient.
def check_residual_T1_closed_form(fwd, bwd, tol=1e-13):
    c = rand_case(12, 2, 1, 3, 4, 5)
    q, k, v, f, W, H0 = _args(c)
    w_r = np.random.default_rng(5).standard_normal((3, 5))
    y0, HT0 = fwd(q, k, v, f, W, H0)
    y, HT = fwd(q, k, v, f, W, H0, w_r=w_r)
    assert np.array_equal(HT, HT0)
    assert relerr(y, y0 + w_r[None, None] * v) < tol
    g0 = bwd(q, k, v, f, W, H0, c["dy"], c["dHT"])
    g = bwd(q, k, v, f, W, H0, c["dy"], c["dHT"], w_r=w_r)
    assert len(g) == 7
    for i in (0, 1, 3, 4, 5):
        assert np.array_equal(g[i], g0[i])
    assert relerr(g[2], g0[2] + w_r[None, None] * c["dy"]) < tol
    assert relerr(g[6], (c["dy"] * v).sum(axis=(0, 1))) < tol


def check_residual_autograd(fwd, bwd, tol=1e-11):
    for (B, N, T, K, V, Nqk) in [(2, 4, 3, 4, 3, 2), (1, 2, 5, 3, 4, None)]:
        c = rand_case(300 + T, B, T, N, K, V, Nqk=Nqk)
        c["w_r"] = np.random.default_rng(6).standard_normal((N, V))
        y_t, HT_t, g = torch_unrolled(c)
        y, HT = fwd(*_args(c), w_r=c["w_r"])
        assert relerr(y, y_t) < tol and relerr(HT, HT_t) < tol
        got = bwd(*_args(c), c["dy"], c["dHT"], w_r=c["w_r"])
        for x, n in zip(got, ("q", "k", "v", "f", "W", "H0", "w_r")):
            assert relerr(x, g[n]) < tol, n


def check_clipped_backward(fwd, bwd, tol=1e-11):
    for (B, N, T, K, V, Nqk) in [(2, 2, 6, 3, 4, None), (1, 4, 5, 4, 3, 1)]:
        c = rand_case(400 + T, B, T, N, K, V, Nqk=Nqk)
        c["dy"] = c["dy"] * 3.0
        free = bwd(*_args(c), c["dy"], c["dHT"])
        # a bound above every carried gradient changes nothing
        same = bwd(*_args(c), c["dy"], c["dHT"], clip=1e6)
        for a, b in zip(free, same):
            assert np.array_equal(a, b)
        clip = 0.25 * float(np.abs(free[5]).max())
        got = bwd(*_args(c), c["dy"], c["dHT"], clip=clip)
        assert np.abs(got[5]).max() <= clip          # dH0 is a clamped value
        assert relerr(got[4], free[4]) > 1e-3        # and the bound was active
        _, _, g = torch_unrolled(c, clip=clip)
        for x, n in zip(got, ("q", "k", "v", "f", "W", "H0")):
            assert relerr(x, g[n]) < tol, n


# --------------------------------------------------------------------------
# The forget-gate function psi(x) = (1 + e^(x + beta))^(-alpha) in front of the scan.
def check_gate_function(fwd, bwd, tol=1e-11):
    for (B, N, T, K, V, Nqk) in [(2, 3, 4, 3, 4, None), (1, 4, 5, 4, 3, 2)]:
        c = rand_case(500 + T, B, T, N, K, V, Nqk=Nqk)
        rng = np.random.default_rng(7)
        x = rng.standard_normal((B, T, N)) * 2.0
        beta = rng.standard_normal(N)
        alpha = rng.uniform(0.3, 2.5, N)
        q, k, v, _, W, H0 = _args(c)
        # the gate value in the printed power form, then the plain scan on it
        f = (1.0 + np.exp(x + beta)) ** (-alpha)
        y0, HT0 = fwd(q, k, v, f, W, H0)
        y, HT = fwd(q, k, v, x, W, H0, gate=(alpha, beta))
        assert relerr(y, y0) < 1e-13 and relerr(HT, HT0) < 1e-13
        # alpha = 1 is a sigmoid of the reflected, shifted input
        one = np.ones(N)
        y1, _ = fwd(q, k, v, x, W, H0, gate=(one, beta))
        y2, _ = fwd(q, k, v, 1.0 / (1.0 + np.exp(x + beta)), W, H0)
        assert relerr(y1, y2) < 1e-13
        # far out in both tails the gate is 0 or 1 and stays finite
        yb, _ = fwd(q, k, v, np.where(x > 0, 800.0, -800.0), W, H0, gate=(alpha, beta))
        yc, _ = fwd(q, k, v, np.where(x > 0, 0.0, 1.0), W, H0)
        assert np.isfinite(yb).all() and relerr(yb, yc) < 1e-13
        # gradients by reverse-mode autodiff through the power form
        c2 = dict(c, f=x, alpha=alpha, beta=beta)
        _, _, g = torch_unrolled(c2)
        got = bwd(q, k, v, x, W, H0, c["dy"], c["dHT"], gate=(alpha, beta))
        assert len(got) == 8
        for xg, n in zip(got, ("q", "k", "v", "f", "W", "H0", "alpha", "beta")):
            assert relerr(xg, g[n]) < tol, n


# --------------------------------------------------------------------------
# Central finite differences of  L = <y, dy> + <HT, dHT>  in every input.
def check_finite_differences(fwd, bwd, tol=2e-7, h=1e-6):
    c = rand_case(5, 2, 5, 2, 3, 4)
    names = ["q", "k", "v", "f", "W", "H0"]
    grads = dict(zip(names, bwd(*_args(c), c["dy"], c["dHT"])))

    def loss(cc):
        y, HT = fwd(*_args(cc))
        return np.sum(y * cc["dy"]) + np.sum(HT * cc["dHT"])

    rng = np.random.default_rng(0)
    for name in names:
        x = c[name]
        flat_idx = rng.choice(x.size, size=min(x.size, 25), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, x.shape)
            cp = dict(c)
            cm = dict(c)
            xp = x.copy()
            xm = x.copy()
            xp[idx] += h
            xm[idx] -= h
            cp[name] = xp
            cm[name] = xm
            fd = (loss(cp) - loss(cm)) / (2 * h)
            an = grads[name][idx]
            assert abs(fd - an) <= tol * max(1.0, abs(an)), (name, idx, fd, an)


# Adjoint identity at a larger size: for a random direction d in input space,
# the directional derivative of L (by differences of the forward alone) must
# equal <gradient, d>.
def check_adjoint_identity(fwd, bwd, tol=1e-6):
    c = rand_case(77, 2, 48, 3, 16, 16, scale=0.4)
    names = ["q", "k", "v", "f", "W", "H0"]
    grads = dict(zip(names, bwd(*_args(c), c["dy"], c["dHT"])))
    rng = np.random.default_rng(3)
    d = {n: rng.standard_normal(c[n].shape) for n in names}
    d["f"] *= 0.01

    def loss(eps):
        cc = dict(c)
        for n in names:
            cc[n] = c[n] + eps * d[n]
        y, HT = fwd(*_args(cc))
        return np.sum(y * c["dy"]) + np.sum(HT * c["dHT"])

    e = 1e-6
    fd = (loss(e) - loss(-e)) / (2 * e)
    an = sum(np.sum(grads[n] * d[n]) for n in names)
    assert abs(fd - an) <= tol * max(1.0, abs(an)), (fd, an)


# --------------------------------------------------------------------------
# Theorem 1: f = 0, q = k = e_1, H0 = 0 makes row 1 of the state an Elman RNN
# h_t = tanh(W^T h_{t-1} + v_t) and y_t = h_t; all other rows stay zero.
def check_elman_reduction(fwd, bwd, tol=1e-14):
    rng = np.random.default_rng(21)
    B, T, N, K, V = 1, 40, 2, 5, 6
    e1 = np.zeros(K)
    e1[0] = 1.0
    q = np.broadcast_to(e1, (B, T, N, K)).copy()
    v = rng.standard_normal((B, T, N, V))
    f = np.zeros((B, T, N))
    W = rng.standard_normal((N, V, V)) * 0.5
    y, HT = fwd(q, q.copy(), v, f, W, None)
    for n in range(N):
        h = np.zeros(V)
        for t in range(T):
            h = np.tanh(W[n].T @ h + v[0, t, n])
            assert relerr(y[0, t, n], h) < tol
        assert np.abs(HT[0, n, 1:, :]).max() == 0.0
        assert relerr(HT[0, n, 0], h) < tol


# W = 0: Z_t = tanh(k_t v_t^T) does not depend on the state, so
# H_T = (prod f) H0 + sum_s (prod_{r>s} f_r)(1 - f_s) tanh(k_s v_s^T).
def check_W_zero_closed_form(fwd, bwd, tol=1e-13):
    c = rand_case(31, 2, 12, 2, 3, 4)
    q, k, v, f, W, H0 = _args(c)
    W = np.zeros_like(W)
    y, HT = fwd(q, k, v, f, W, H0)
    T = 12
    for b in range(2):
        for n in range(2):
            fs = f[b, :, n]
            Zs = np.tanh(np.einsum("ti,tj->tij", k[b, :, n], v[b, :, n]))
            for t_end in range(1, T + 1):
                # suffix products prod_{r=s+1}^{t_end-1} f_r
                tail = np.array([np.prod(fs[s + 1:t_end]) for s in range(t_end)])
                Ht = np.prod(fs[:t_end]) * H0[b, n] + np.einsum(
                    "s,sij->ij", tail * (1 - fs[:t_end]), Zs[:t_end])
                assert relerr(y[b, t_end - 1, n], Ht.T @ q[b, t_end - 1, n]) < tol
            assert relerr(HT[b, n], Ht) < tol


# f = 1 keeps the state; f = 0 replaces it by Z_t.
def check_gate_limits(fwd, bwd, tol=1e-13):
    c = rand_case(41, 2, 6, 2, 3, 4)
    q, k, v, f, W, H0 = _args(c)
    one = np.ones_like(f)
    y, HT = fwd(q, k, v, one, W, H0)
    assert relerr(HT, H0) == 0.0
    assert relerr(y, np.einsum("bnij,btni->btnj", H0, q)) < tol
    dq, dk, dv, df, dW, dH0 = bwd(q, k, v, one, W, H0, c["dy"], c["dHT"])
    assert np.abs(dk).max() == 0.0 and np.abs(dv).max() == 0.0 and np.abs(dW).max() == 0.0
    assert relerr(dH0, c["dHT"] + np.einsum("btni,btnj->bnij", q, c["dy"])) < tol
    assert relerr(dq, np.einsum("bnij,btnj->btni", H0, c["dy"])) < tol
    # df_t = sum G_t (.) (H0 - Z_t),  G_t = dHT + sum_{s>=t} q_s dy_s^T
    for b in range(2):
        for n in range(2):
            G = c["dHT"][b, n].copy()
            for t in range(5, -1, -1):
                G = G + np.outer(q[b, t, n], c["dy"][b, t, n])
                Z = np.tanh(H0[b, n] @ W[n] + np.outer(k[b, t, n], v[b, t, n]))
                assert abs(df[b, t, n] - np.sum(G * (H0[b, n] - Z))) < 1e-12
    # f = 0: the state after each step is Z_t of the previous state
    zero = np.zeros_like(f)
    y, HT = fwd(q, k, v, zero, W, H0)
    for b in range(2):
        for n in range(2):
            H = H0[b, n]
            for t in range(6):
                H = np.tanh(H @ W[n] + np.outer(k[b, t, n], v[b, t, n]))
                assert relerr(y[b, t, n], H.T @ q[b, t, n]) < tol
            assert relerr(HT[b, n], H) < tol


# Running [0,T) equals running [0,T1) then [T1,T) from the carried state; the
# backward chains through dHT <- dH0.
def check_segment_chaining(fwd, bwd):
    c = rand_case(51, 2, 9, 2, 3, 4)
    q, k, v, f, W, H0 = _args(c)
    T1 = 4
    y, HT = fwd(q, k, v, f, W, H0)
    ya, Ha = fwd(q[:, :T1], k[:, :T1], v[:, :T1], f[:, :T1], W, H0)
    yb, Hb = fwd(q[:, T1:], k[:, T1:], v[:, T1:], f[:, T1:], W, Ha)
    assert np.array_equal(np.concatenate([ya, yb], axis=1), y)
    assert np.array_equal(Hb, HT)
    full = bwd(q, k, v, f, W, H0, c["dy"], c["dHT"])
    gb = bwd(q[:, T1:], k[:, T1:], v[:, T1:], f[:, T1:], W, Ha, c["dy"][:, T1:], c["dHT"])
    ga = bwd(q[:, :T1], k[:, :T1], v[:, :T1], f[:, :T1], W, H0, c["dy"][:, :T1], gb[5])
    for i in range(4):   # dq, dk, dv, df
        assert relerr(np.concatenate([ga[i], gb[i]], axis=1), full[i]) < 1e-14
    assert relerr(ga[4] + gb[4], full[4]) < 1e-13
    assert relerr(ga[5], full[5]) < 1e-14


# Rows of the state are independent recurrences that share W, v, f: running a
# subset of rows gives partial outputs that add up; permuting rows changes
# nothing; permuting columns (with W -> P^T W P) permutes y.
def check_row_and_column_structure(fwd, bwd, tol=1e-13):
    c = rand_case(61, 1, 7, 2, 6, 4)
    q, k, v, f, W, H0 = _args(c)
    y, HT = fwd(q, k, v, f, W, H0)
    rows_a, rows_b = [0, 2, 3], [1, 4, 5]
    ya, Ha = fwd(q[..., rows_a], k[..., rows_a], v, f, W, H0[:, :, rows_a])
    yb, Hb = fwd(q[..., rows_b], k[..., rows_b], v, f, W, H0[:, :, rows_b])
    assert relerr(ya + yb, y) < tol
    assert relerr(Ha, HT[:, :, rows_a]) < tol and relerr(Hb, HT[:, :, rows_b]) < tol
    perm = np.array([3, 0, 5, 1, 4, 2])
    yp, Hp = fwd(q[..., perm], k[..., perm], v, f, W, H0[:, :, perm])
    assert relerr(yp, y) < tol and relerr(Hp, HT[:, :, perm]) < tol
    cp = np.array([2, 0, 3, 1])
    Wp = W[:, cp][:, :, cp]
    yc, Hc = fwd(q, k, v[..., cp], f, Wp, H0[..., cp])
    assert relerr(yc, y[..., cp]) < tol and relerr(Hc, HT[..., cp]) < tol


# |H0| <= 1 implies |H_t| <= 1 (a convex combination of the state and a tanh).
def check_state_bound(fwd, bwd):
    c = rand_case(71, 1, 60, 2, 4, 4, scale=3.0)
    q, k, v, f, W, H0 = _args(c)
    H0 = np.clip(H0 * 5, -1, 1)
    W = W * 4
    for T in (1, 7, 60):
        _, HT = fwd(q[:, :T], k[:, :T], v[:, :T], f[:, :T], W, H0)
        assert np.abs(HT).max() <= 1.0


# The backward is linear in (dy, dHT).
def check_backward_linearity(fwd, bwd, tol=1e-12):
    c = rand_case(81, 2, 6, 2, 3, 4)
    rng = np.random.default_rng(9)
    dy2 = rng.standard_normal(c["dy"].shape)
    dH2 = rng.standard_normal(c["dHT"].shape)
    g1 = bwd(*_args(c), c["dy"], c["dHT"])
    g2 = bwd(*_args(c), dy2, dH2)
    g3 = bwd(*_args(c), 2.0 * c["dy"] - 3.0 * dy2, 2.0 * c["dHT"] - 3.0 * dH2)
    for a, b, s in zip(g1, g2, g3):
        assert relerr(2.0 * a - 3.0 * b, s) < tol
    gz = bwd(*_args(c), c["dy"], None)
    gz2 = bwd(*_args(c), c["dy"], np.zeros_like(c["dHT"]))
    for a, b in zip(gz, gz2):
        assert np.array_equal(a, b)


# T = 0: nothing happens, HT = H0.
def check_empty_sequence(fwd, bwd):
    c = rand_case(91, 2, 0, 2, 3, 4)
    y, HT = fwd(*_args(c))
    assert y.shape == (2, 0, 2, 4) and np.array_equal(HT, c["H0"])
    g = bwd(*_args(c), c["dy"], c["dHT"])
    assert np.array_equal(g[5], c["dHT"]) and np.abs(g[4]).max() == 0.0


ALL_CHECKS = [
    check_T1_closed_form, check_unrolled_autograd, check_finite_differences,
    check_adjoint_identity, check_elman_reduction, check_W_zero_closed_form,
    check_gate_limits, check_segment_chaining, check_row_and_column_structure,
    check_state_bound, check_backward_linearity, check_empty_sequence,
    check_residual_T1_closed_form, check_residual_autograd, check_clipped_backward,
    check_gate_function,
]
