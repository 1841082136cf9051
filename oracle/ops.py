"""Float64 reference operators with their tangent (R-op) forms.

TEST INFRASTRUCTURE ONLY: a slow, plain numpy float64 restatement of the
calculus behind the paper's Hessian-vector product (Algorithm 1 computes
d/dp <grad L, v>, which equals d/de grad L(p + e v) at e = 0).  Nothing in the
product path may import this package.

Notation.  For a forward quantity a, `a_t` is its directional derivative along
the parameter direction v ("tangent").  `da` is the adjoint dL/da and `da_t`
is the directional derivative of that adjoint.  Every operator below comes as

    fwd(x, x_t, params, params_t)   -> y, y_t, cache
    bwd(dy, dy_t, cache)            -> dx, dx_t, (dparam, dparam_t ...)

where dparam is the ordinary gradient block and dparam_t the block of H v.
All formulas are the product / chain rule applied to the operator's definition;
each is checked by finite differences in tests/test_oracle_ops.py.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf

# ---------------------------------------------------------------- linear ----


def linear_fwd(X, X_t, W, W_t, b=None, b_t=None):
    """Y = X W + b (Algorithm 1's model forward is built from these)."""
    Y = X @ W
    Y_t = X_t @ W + X @ W_t
    if b is not None:
        Y = Y + b
        Y_t = Y_t + b_t
    return Y, Y_t, (X, X_t, W, W_t, b is not None)


def linear_bwd(dY, dY_t, cache):
    X, X_t, W, W_t, has_b = cache
    dX = dY @ W.T
    dX_t = dY_t @ W.T + dY @ W_t.T
    dW = X.T @ dY
    dW_t = X_t.T @ dY + X.T @ dY_t
    if has_b:
        return dX, dX_t, dW, dW_t, dY.sum(0), dY_t.sum(0)
    return dX, dX_t, dW, dW_t


# ------------------------------------------------------------- pointwise ----


def tanh_fwd(a, a_t):
    t = np.tanh(a)
    return t, (1.0 - t * t) * a_t, (t, a_t)


def tanh_bwd(dy, dy_t, cache):
    t, a_t = cache
    f1 = 1.0 - t * t
    f2 = -2.0 * t * f1
    return f1 * dy, f1 * dy_t + f2 * a_t * dy


_SQRT2 = np.sqrt(2.0)
_INV_SQRT_2PI = 1.0 / np.sqrt(2.0 * np.pi)


def gelu_fwd(a, a_t):
    """Exact (erf) GELU: f(a) = a Phi(a)."""
    Phi = 0.5 * (1.0 + erf(a / _SQRT2))
    phi = _INV_SQRT_2PI * np.exp(-0.5 * a * a)
    f1 = Phi + a * phi
    return a * Phi, f1 * a_t, (a, a_t, f1, phi)


def gelu_bwd(dy, dy_t, cache):
    a, a_t, f1, phi = cache
    f2 = phi * (2.0 - a * a)
    return f1 * dy, f1 * dy_t + f2 * a_t * dy


_GT_C = np.sqrt(2.0 / np.pi)
_GT_A = 0.044715


def gelu_tanh_fwd(a, a_t):
    """tanh-form GELU: f(a) = a/2 (1 + tanh u), u = sqrt(2/pi) (a + 0.044715 a^3)."""
    t = np.tanh(_GT_C * (a + _GT_A * a ** 3))
    u1 = _GT_C * (1.0 + 3.0 * _GT_A * a * a)
    t1 = (1.0 - t * t) * u1
    f1 = 0.5 * (1.0 + t) + 0.5 * a * t1
    return 0.5 * a * (1.0 + t), f1 * a_t, (a, a_t, f1, t, u1, t1)


def gelu_tanh_bwd(dy, dy_t, cache):
    a, a_t, f1, t, u1, t1 = cache
    u2 = 6.0 * _GT_A * _GT_C * a
    t2 = (1.0 - t * t) * (u2 - 2.0 * t * u1 * u1)
    f2 = t1 + 0.5 * a * t2
    return f1 * dy, f1 * dy_t + f2 * a_t * dy


def swiglu_fwd(g, g_t, u, u_t):
    """y = silu(g) * u, silu(g) = g sigmoid(g)."""
    sg = 1.0 / (1.0 + np.exp(-g))
    s = g * sg
    s1 = sg + g * sg * (1.0 - sg)
    y = s * u
    y_t = s1 * g_t * u + s * u_t
    return y, y_t, (g, g_t, u, u_t, sg, s, s1)


def swiglu_bwd(dy, dy_t, cache):
    g, g_t, u, u_t, sg, s, s1 = cache
    dsg = sg * (1.0 - sg)
    s2 = dsg * (2.0 + g * (1.0 - 2.0 * sg))
    dg = s1 * u * dy
    du = s * dy
    dg_t = s2 * g_t * u * dy + s1 * u_t * dy + s1 * u * dy_t
    du_t = s1 * g_t * dy + s * dy_t
    return dg, dg_t, du, du_t


# ----------------------------------------------------------------- norms ----


def layernorm_fwd(x, x_t, gam, gam_t, bet, bet_t, eps):
    """Row-wise LayerNorm with biased variance."""
    mu = x.mean(-1, keepdims=True)
    xc = x - mu
    sig = np.sqrt((xc * xc).mean(-1, keepdims=True) + eps)
    xh = xc / sig
    sig_t_over = (xh * x_t).mean(-1, keepdims=True)           # = sigma_t
    xh_t = (x_t - x_t.mean(-1, keepdims=True) - xh * sig_t_over) / sig
    y = gam * xh + bet
    y_t = gam_t * xh + gam * xh_t + bet_t
    return y, y_t, (xh, xh_t, sig, sig_t_over, gam, gam_t)


def layernorm_bwd(dy, dy_t, cache):
    xh, xh_t, sig, sig_t, gam, gam_t = cache
    g = gam * dy
    g_t = gam_t * dy + gam * dy_t
    m1 = g.mean(-1, keepdims=True)
    m2 = (g * xh).mean(-1, keepdims=True)
    dx = (g - m1 - xh * m2) / sig
    m1_t = g_t.mean(-1, keepdims=True)
    m2_t = (g_t * xh + g * xh_t).mean(-1, keepdims=True)
    dx_t = (g_t - m1_t - xh_t * m2 - xh * m2_t) / sig - dx * sig_t / sig
    red = tuple(range(dy.ndim - 1))
    dgam = (dy * xh).sum(red)
    dgam_t = (dy_t * xh + dy * xh_t).sum(red)
    dbet = dy.sum(red)
    dbet_t = dy_t.sum(red)
    return dx, dx_t, dgam, dgam_t, dbet, dbet_t


def rmsnorm_fwd(x, x_t, gam, gam_t, eps):
    r = np.sqrt((x * x).mean(-1, keepdims=True) + eps)
    xh = x / r
    r_t = (xh * x_t).mean(-1, keepdims=True)
    xh_t = (x_t - xh * r_t) / r
    return gam * xh, gam_t * xh + gam * xh_t, (xh, xh_t, r, r_t, gam, gam_t)


def rmsnorm_bwd(dy, dy_t, cache):
    xh, xh_t, r, r_t, gam, gam_t = cache
    g = gam * dy
    g_t = gam_t * dy + gam * dy_t
    m2 = (g * xh).mean(-1, keepdims=True)
    dx = (g - xh * m2) / r
    m2_t = (g_t * xh + g * xh_t).mean(-1, keepdims=True)
    dx_t = (g_t - xh_t * m2 - xh * m2_t) / r - dx * r_t / r
    red = tuple(range(dy.ndim - 1))
    return dx, dx_t, (dy * xh).sum(red), (dy_t * xh + dy * xh_t).sum(red)


# ------------------------------------------------------------------ RoPE ----


def rope_tables(S, dh, theta):
    """cos/sin [S, dh/2] for positions 0..S-1; pair (i, i + dh/2) rotates by
    pos * theta^(-2i/dh)."""
    half = dh // 2
    inv = theta ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = np.arange(S, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang), np.sin(ang)


def rope_apply(x, cos, sin, inverse=False):
    """x: [B, H, S, dh].  A fixed orthogonal map, so tangents use the same map
    and adjoints the inverse (transpose) rotation."""
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    s = -sin if inverse else sin
    return np.concatenate([x1 * cos - x2 * s, x2 * cos + x1 * s], axis=-1)


# ------------------------------------------------------------- attention ----


def _T(a):
    return np.swapaxes(a, -1, -2)


def attention_fwd(q, q_t, k, k_t, v, v_t):
    """Causal softmax attention per batch and head.  q,k,v: [B, H, S, dh];
    `@` is the batched matrix product over the last two axes."""
    S, dh = q.shape[-2], q.shape[-1]
    c = 1.0 / np.sqrt(dh)
    mask = np.tril(np.ones((S, S), dtype=bool))
    sc = c * (q @ _T(k))
    sc_t = c * (q_t @ _T(k) + q @ _T(k_t))
    sc = np.where(mask, sc, -np.inf)
    sc = sc - sc.max(-1, keepdims=True)
    e = np.exp(sc)
    P = e / e.sum(-1, keepdims=True)
    sc_t = np.where(mask, sc_t, 0.0)
    P_t = P * (sc_t - (P * sc_t).sum(-1, keepdims=True))
    o = P @ v
    o_t = P_t @ v + P @ v_t
    return o, o_t, (q, q_t, k, k_t, v, v_t, P, P_t, c)


def attention_bwd(do, do_t, cache):
    q, q_t, k, k_t, v, v_t, P, P_t, c = cache
    dv = _T(P) @ do
    dv_t = _T(P_t) @ do + _T(P) @ do_t
    dP = do @ _T(v)
    dP_t = do_t @ _T(v) + do @ _T(v_t)
    delta = (P * dP).sum(-1, keepdims=True)
    delta_t = (P_t * dP + P * dP_t).sum(-1, keepdims=True)
    dS = P * (dP - delta)
    dS_t = P_t * (dP - delta) + P * (dP_t - delta_t)
    dq = c * (dS @ k)
    dq_t = c * (dS_t @ k + dS @ k_t)
    dk = c * (_T(dS) @ q)
    dk_t = c * (_T(dS_t) @ q + _T(dS) @ q_t)
    return dq, dq_t, dk, dk_t, dv, dv_t


# -------------------------------------------------- softmax cross-entropy ----


def cross_entropy_fwd(z, z_t, labels):
    """Mean cross-entropy over positions whose label is >= 0.

    z, z_t: [T, V]; labels: [T] int, -1 = ignored.  Returns the loss, its
    tangent, and dz, dz_t (the adjoint seeds of the backward pass):
      dz = (p - onehot)/N,  dz_t = p * (z_t - <p, z_t>)/N."""
    valid = labels >= 0
    N = int(valid.sum())
    zs = z - z.max(-1, keepdims=True)
    lse = np.log(np.exp(zs).sum(-1, keepdims=True))
    logp = zs - lse
    p = np.exp(logp)
    rows = np.nonzero(valid)[0]
    lab = labels[rows]
    loss = -logp[rows, lab].sum() / N
    pz = (p * z_t).sum(-1, keepdims=True)
    loss_t = (pz[rows, 0] - z_t[rows, lab]).sum() / N
    dz = p.copy()
    dz[rows, lab] -= 1.0
    dz_t = p * (z_t - pz)
    dz[~valid] = 0.0
    dz_t[~valid] = 0.0
    return loss, loss_t, dz / N, dz_t / N
