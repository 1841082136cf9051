"""Pins for oracle/ops.py: each operator's forward against an independent
library routine or closed form, and its tangent / adjoint / tangent-of-adjoint
against central finite differences and the transposition identity."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ops

RNG = np.random.default_rng(7)


def rnd(*s):
    return RNG.standard_normal(s)


def fd(f, h=1e-6):
    return (f(h) - f(-h)) / (2 * h)


def check_op(fwd, bwd, xs, xts, n_out=1):
    """xs: list of input arrays (activations and parameters), xts: tangents.
    fwd(*xs, *xts interleaved by caller) is wrapped by the caller as
    run(xs, xts) -> (ys, yts, cache); bwd(dys, dyts, cache) -> (dxs, dxts)."""
    ys, yts, cache = fwd(xs, xts)
    # 1. tangent-forward == d/de f(x + e x_t)
    for i in range(len(ys)):
        num = fd(lambda e: fwd([x + e * t for x, t in zip(xs, xts)], xts)[0][i])
        np.testing.assert_allclose(yts[i], num, rtol=1e-6, atol=1e-8)
    dys = [rnd(*y.shape) for y in ys]
    dyts = [rnd(*y.shape) for y in ys]
    dxs, dxts = bwd(dys, dyts, cache)
    # 2. adjoint identity: <dy, J x_t> == <J^T dy, x_t>
    lhs = sum((dy * yt).sum() for dy, yt in zip(dys, yts))
    rhs = sum((dx * xt).sum() for dx, xt in zip(dxs, xts))
    assert abs(lhs - rhs) <= 1e-9 * max(1.0, abs(lhs))
    # 3. tangent of the adjoint == d/de bwd(dy + e dy_t; x + e x_t)
    for i in range(len(dxs)):
        def g(e, i=i):
            xs_e = [x + e * t for x, t in zip(xs, xts)]
            _, _, c = fwd(xs_e, xts)
            return bwd([dy + e * dt for dy, dt in zip(dys, dyts)], dyts, c)[0][i]
        np.testing.assert_allclose(dxts[i], fd(g), rtol=1e-5, atol=1e-7)


def test_linear():
    def fwd(xs, xts):
        y, yt, c = ops.linear_fwd(xs[0], xts[0], xs[1], xts[1], xs[2], xts[2])
        return [y], [yt], c

    def bwd(dys, dyts, c):
        dX, dXt, dW, dWt, db, dbt = ops.linear_bwd(dys[0], dyts[0], c)
        return [dX, dW, db], [dXt, dWt, dbt]
    xs = [rnd(5, 4), rnd(4, 3), rnd(3)]
    check_op(fwd, bwd, xs, [rnd(*x.shape) for x in xs])
    y = ops.linear_fwd(xs[0], xs[0], xs[1], xs[1], xs[2], xs[2])[0]
    ref = F.linear(torch.tensor(xs[0]), torch.tensor(xs[1]).T, torch.tensor(xs[2])).numpy()
    np.testing.assert_allclose(y, ref, rtol=1e-13)


@pytest.mark.parametrize("name", ["tanh", "gelu", "gelu_tanh"])
def test_pointwise(name):
    f, b = {"tanh": (ops.tanh_fwd, ops.tanh_bwd), "gelu": (ops.gelu_fwd, ops.gelu_bwd),
            "gelu_tanh": (ops.gelu_tanh_fwd, ops.gelu_tanh_bwd)}[name]

    def fwd(xs, xts):
        y, yt, c = f(xs[0], xts[0])
        return [y], [yt], c

    def bwd(dys, dyts, c):
        dx, dxt = b(dys[0], dyts[0], c)
        return [dx], [dxt]
    x = rnd(6, 7) * 2
    check_op(fwd, bwd, [x], [rnd(6, 7)])
    tfn = {"tanh": torch.tanh, "gelu": F.gelu, "gelu_tanh": lambda t: F.gelu(t, approximate="tanh")}[name]
    ref = tfn(torch.tensor(x)).numpy()
    np.testing.assert_allclose(f(x, x)[0], ref, rtol=1e-12, atol=1e-15)


def test_swiglu():
    def fwd(xs, xts):
        y, yt, c = ops.swiglu_fwd(xs[0], xts[0], xs[1], xts[1])
        return [y], [yt], c

    def bwd(dys, dyts, c):
        dg, dgt, du, dut = ops.swiglu_bwd(dys[0], dyts[0], c)
        return [dg, du], [dgt, dut]
    xs = [rnd(5, 6) * 2, rnd(5, 6)]
    check_op(fwd, bwd, xs, [rnd(5, 6), rnd(5, 6)])
    ref = (F.silu(torch.tensor(xs[0])) * torch.tensor(xs[1])).numpy()
    np.testing.assert_allclose(fwd(xs, xs)[0][0], ref, rtol=1e-12)


def test_layernorm():
    eps = 1e-5

    def fwd(xs, xts):
        y, yt, c = ops.layernorm_fwd(xs[0], xts[0], xs[1], xts[1], xs[2], xts[2], eps)
        return [y], [yt], c

    def bwd(dys, dyts, c):
        dx, dxt, dg, dgt, db, dbt = ops.layernorm_bwd(dys[0], dyts[0], c)
        return [dx, dg, db], [dxt, dgt, dbt]
    xs = [rnd(6, 8) * 3 + 1, rnd(8) + 1, rnd(8)]
    check_op(fwd, bwd, xs, [rnd(*x.shape) for x in xs])
    ref = F.layer_norm(torch.tensor(xs[0]), (8,), torch.tensor(xs[1]), torch.tensor(xs[2]), eps).numpy()
    np.testing.assert_allclose(fwd(xs, xs)[0][0], ref, rtol=1e-12)


def test_rmsnorm():
    eps = 1e-5

    def fwd(xs, xts):
        y, yt, c = ops.rmsnorm_fwd(xs[0], xts[0], xs[1], xts[1], eps)
        return [y], [yt], c

    def bwd(dys, dyts, c):
        dx, dxt, dg, dgt = ops.rmsnorm_bwd(dys[0], dyts[0], c)
        return [dx, dg], [dxt, dgt]
    xs = [rnd(6, 8) * 3 + 1, rnd(8) + 1]
    check_op(fwd, bwd, xs, [rnd(*x.shape) for x in xs])
    x = xs[0]
    ref = x / np.sqrt((x ** 2).mean(-1, keepdims=True) + eps) * xs[1]
    np.testing.assert_allclose(fwd(xs, xs)[0][0], ref, rtol=1e-13)
    reft = F.rms_norm(torch.tensor(x), (8,), torch.tensor(xs[1]), eps).numpy()
    np.testing.assert_allclose(ref, reft, rtol=1e-12)


def test_rope_is_rotation_by_position():
    S, dh = 5, 8
    cos, sin = ops.rope_tables(S, dh, 10000.0)
    x = rnd(2, 3, S, dh)
    y = ops.rope_apply(x, cos, sin)
    # closed form with complex numbers: (x_i + i x_{i+dh/2}) * exp(i pos w_i)
    w = 10000.0 ** (-2.0 * np.arange(dh // 2) / dh)
    z = (x[..., :dh // 2] + 1j * x[..., dh // 2:]) * np.exp(1j * np.arange(S)[:, None] * w[None, :])
    np.testing.assert_allclose(y, np.concatenate([z.real, z.imag], -1), rtol=1e-13, atol=1e-15)
    # inverse is the transpose: norms preserved and round trip exact
    np.testing.assert_allclose(ops.rope_apply(y, cos, sin, inverse=True), x, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose((y * y).sum(-1), (x * x).sum(-1), rtol=1e-13)
    # position 0 is the identity
    np.testing.assert_allclose(y[:, :, 0], x[:, :, 0], rtol=0, atol=0)


def test_attention():
    def fwd(xs, xts):
        o, ot, c = ops.attention_fwd(xs[0], xts[0], xs[1], xts[1], xs[2], xts[2])
        return [o], [ot], c

    def bwd(dys, dyts, c):
        dq, dqt, dk, dkt, dv, dvt = ops.attention_bwd(dys[0], dyts[0], c)
        return [dq, dk, dv], [dqt, dkt, dvt]
    xs = [rnd(2, 2, 6, 4), rnd(2, 2, 6, 4), rnd(2, 2, 6, 4)]
    check_op(fwd, bwd, xs, [rnd(*x.shape) for x in xs])
    with torch.nn.attention.sdpa_kernel(torch.nn.attention.SDPBackend.MATH):
        ref = F.scaled_dot_product_attention(*[torch.tensor(x) for x in xs], is_causal=True).numpy()
    np.testing.assert_allclose(fwd(xs, xs)[0][0], ref, rtol=1e-12)
    # causality: output at position i must not depend on keys/values after i
    xs2 = [x.copy() for x in xs]
    xs2[1][:, :, 4:] += 1.0
    xs2[2][:, :, 4:] -= 2.0
    np.testing.assert_allclose(fwd(xs2, xs)[0][0][:, :, :4], fwd(xs, xs)[0][0][:, :, :4], rtol=0, atol=0)


def test_cross_entropy():
    T, V = 7, 5
    z, zt = rnd(T, V) * 2, rnd(T, V)
    lab = np.array([0, 3, -1, 4, 1, -1, 2])
    loss, loss_t, dz, dzt = ops.cross_entropy_fwd(z, zt, lab)
    ref = F.cross_entropy(torch.tensor(z), torch.tensor(lab), ignore_index=-1).item()
    assert abs(loss - ref) < 1e-13
    f = lambda e: ops.cross_entropy_fwd(z + e * zt, zt, lab)[0]
    assert abs(loss_t - fd(f)) < 1e-8
    # dz is the gradient of the loss in z
    num = np.zeros_like(z)
    for i in range(T):
        for j in range(V):
            e = np.zeros_like(z); e[i, j] = 1
            num[i, j] = fd(lambda h: ops.cross_entropy_fwd(z + h * e, zt, lab)[0])
    np.testing.assert_allclose(dz, num, atol=1e-8)
    # dz_t is (diag(p) - p p^T) z_t / N per valid row (closed-form CE Hessian)
    N = (lab >= 0).sum()
    p = torch.softmax(torch.tensor(z), -1).numpy()
    for i in range(T):
        Hz = (np.diag(p[i]) - np.outer(p[i], p[i])) / N if lab[i] >= 0 else np.zeros((V, V))
        np.testing.assert_allclose(dzt[i], Hz @ zt[i], atol=1e-14)
