"""Pins for the oracle's operator definitions (CPU only).

The paper prints no worked numeric example and defines none of these
operators, so nothing here is a value taken from the paper.  Each oracle
function is pinned to something other than itself:
  * brute force: pure-Python loops written from the formulas on tiny
    integer-valued inputs (exact in floating point);
  * closed forms (all-ones convolution counts taps, delta kernels shift,
    identity weights copy, constant pooling, LSTM with zero weights);
  * invariants (linearity, 1x1 conv == dense, stride-2 == subsampled
    stride-1, explicit padding, batch independence, split GEMM);
  * a library routine: the same arrays through PyTorch's CPU float64
    conv2d / matmul / max_pool2d (cross-check of the oracle only).
"""
import math

import numpy as np
import pytest
import torch

import oracle as O

RNG = np.random.default_rng(12345)


def ints(shape, lo=-3, hi=4):
    return RNG.integers(lo, hi, size=shape).astype(np.float64)


# ---------------------------------------------------------------- brute force
def brute_conv(x, w, s, p):
    N, C, H, W = x.shape
    Oc, _, KH, KW = w.shape
    OH = (H + 2 * p[0] - KH) // s[0] + 1
    OW = (W + 2 * p[1] - KW) // s[1] + 1
    y = [[[[0.0] * OW for _ in range(OH)] for _ in range(Oc)] for _ in range(N)]
    for n in range(N):
        for o in range(Oc):
            for i in range(OH):
                for j in range(OW):
                    acc = 0.0
                    for c in range(C):
                        for a in range(KH):
                            for b in range(KW):
                                ih, iw = i * s[0] - p[0] + a, j * s[1] - p[1] + b
                                if 0 <= ih < H and 0 <= iw < W:
                                    acc += float(x[n, c, ih, iw]) * float(w[o, c, a, b])
                    y[n][o][i][j] = acc
    return np.array(y)


@pytest.mark.parametrize("s,p,k", [((1, 1), (0, 0), (3, 3)), ((1, 1), (1, 1), (3, 3)), ((2, 2), (1, 1), (3, 3)),
                                   ((2, 1), (0, 2), (3, 2)), ((2, 2), (3, 3), (7, 7)), ((2, 2), (0, 0), (1, 1))])
def test_conv2d_brute_force(s, p, k):
    x, w = ints((2, 3, 9, 8)), ints((2, 3) + k)
    np.testing.assert_array_equal(O.conv2d(x, w, s, p), brute_conv(x, w, s, p))


def test_dense_brute_force():
    x, w = ints((3, 5)), ints((4, 5))
    ref = [[sum(float(x[m, k]) * float(w[n, k]) for k in range(5)) for n in range(4)] for m in range(3)]
    np.testing.assert_array_equal(O.dense(x, w), np.array(ref))


def test_dense_is_not_transposed():
    # W is [out, in]: a one-hot row n of W picks column k of x into output column n
    x = ints((2, 3))
    w = np.zeros((4, 3)); w[2, 1] = 1.0
    y = O.dense(x, w)
    assert y.shape == (2, 4)
    np.testing.assert_array_equal(y[:, 2], x[:, 1])
    assert np.all(y[:, [0, 1, 3]] == 0)


def test_maxpool_brute_force():
    x = ints((2, 2, 7, 6), -9, 9)
    k, s, p = (3, 3), (2, 2), (1, 1)
    got = O.maxpool2d(x, k, s, p)
    N, C, H, W = x.shape
    OH, OW = (H + 2 - 3) // 2 + 1, (W + 2 - 3) // 2 + 1
    assert got.shape == (N, C, OH, OW)
    for n in range(N):
        for c in range(C):
            for i in range(OH):
                for j in range(OW):
                    taps = [x[n, c, ih, iw] for ih in range(i * 2 - 1, i * 2 + 2) for iw in range(j * 2 - 1, j * 2 + 2)
                            if 0 <= ih < H and 0 <= iw < W]
                    assert got[n, c, i, j] == max(taps)


def test_maxpool_ignores_padding_on_negative_inputs():
    x = -np.ones((1, 1, 4, 4))
    assert np.all(O.maxpool2d(x, (3, 3), (2, 2), (1, 1)) == -1.0)   # zero padding would give 0


def test_bias_add_axes():
    x = ints((2, 3, 4, 5))
    b = ints((3,))
    np.testing.assert_array_equal(O.bias_add(x, b, 1), x + b[None, :, None, None])
    b = ints((5,))
    np.testing.assert_array_equal(O.bias_add(x, b, 3), x + b)
    b = ints((2,))
    np.testing.assert_array_equal(O.bias_add(x, b, 0), x + b[:, None, None, None])


def test_elementwise_definitions():
    a, b = RNG.standard_normal(50), RNG.uniform(1, 2, 50)
    for i in range(50):
        assert O.binary("add", a, b)[i] == a[i] + b[i]
        assert O.binary("sub", a, b)[i] == a[i] - b[i]   # operand order
        assert O.binary("mul", a, b)[i] == a[i] * b[i]
        assert O.binary("div", a, b)[i] == a[i] / b[i]
        assert O.unary("neg", a)[i] == -a[i]
        assert O.unary("sq", a)[i] == a[i] * a[i]
        assert O.unary("relu", a)[i] == max(a[i], 0.0)
        assert abs(O.unary("sigmoid", a)[i] - 1.0 / (1.0 + math.exp(-a[i]))) < 1e-15
        assert abs(O.unary("tanh", a)[i] - math.tanh(a[i])) < 1e-15
    # special values
    assert O.unary("sigmoid", np.zeros(1))[0] == 0.5
    assert O.unary("tanh", np.zeros(1))[0] == 0.0
    s = O.unary("sigmoid", a)
    np.testing.assert_allclose(s + O.unary("sigmoid", -a), 1.0, atol=1e-15)   # sigma(x)+sigma(-x)=1
    np.testing.assert_allclose(O.unary("tanh", a), 2 * O.unary("sigmoid", 2 * a) - 1, atol=1e-15)


# ---------------------------------------------------------------- closed forms
def test_conv_all_ones_counts_taps():
    C = 5
    y = O.conv2d(np.ones((1, C, 6, 7)), np.ones((2, C, 3, 3)), (1, 1), (1, 1))
    assert y.shape == (1, 2, 6, 7)
    assert np.all(y[:, :, 1:-1, 1:-1] == 9 * C)
    assert np.all(y[:, :, 0, 1:-1] == 6 * C) and np.all(y[:, :, 1:-1, 0] == 6 * C)
    for i, j in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.all(y[:, :, i, j] == 4 * C)


def test_conv_delta_kernel_shifts_without_flip():
    x = ints((1, 1, 6, 6))
    w = np.zeros((1, 1, 3, 3)); w[0, 0, 0, 2] = 1.0     # tap at (a=0, b=2)
    y = O.conv2d(x, w, (1, 1), (1, 1))
    # y[i,j] = x[i-1+0, j-1+2] = x[i-1, j+1]: cross-correlation (a flipped kernel would give x[i+1, j-1])
    for i in range(6):
        for j in range(6):
            exp = x[0, 0, i - 1, j + 1] if (i - 1 >= 0 and j + 1 < 6) else 0.0
            assert y[0, 0, i, j] == exp


def test_dense_identity_copies():
    x = ints((4, 6))
    np.testing.assert_array_equal(O.dense(x, np.eye(6)), x)


def test_global_avgpool_constant_and_mean():
    assert np.all(O.global_avgpool(np.full((2, 3, 7, 7), 2.5)) == 2.5)
    x = ints((2, 3, 4, 5))
    np.testing.assert_allclose(O.global_avgpool(x)[:, :, 0, 0], x.sum(axis=(2, 3)) / 20.0, rtol=0, atol=1e-15)


def test_lstm_zero_weights_closed_form():
    # W = 0: c_t = alpha c_{t-1} + beta with alpha = sigma(b_f), beta = sigma(b_i) tanh(b_g)
    # => c_t = beta (1 - alpha^t)/(1 - alpha) from c_0 = 0;  h_t = sigma(b_o) tanh(c_t)
    B, I, H, T = 2, 3, 4, 6
    b = RNG.uniform(-1, 1, 4 * H)
    x = RNG.standard_normal((T, B, I))
    w = np.zeros((4 * H, I + H))
    hs, c = O.lstm_sequence(x, w, b, np.zeros((B, H)), np.zeros((B, H)), h_dtype="f32")
    sig = lambda v: 1 / (1 + np.exp(-v))
    alpha, beta = sig(b[H:2 * H]), sig(b[:H]) * np.tanh(b[2 * H:3 * H])
    for t in range(1, T + 1):
        ct = beta * (1 - alpha ** t) / (1 - alpha)
        np.testing.assert_allclose(hs[t - 1], np.broadcast_to(sig(b[3 * H:]) * np.tanh(ct), (B, H)), rtol=1e-6)
    np.testing.assert_allclose(c, np.broadcast_to(beta * (1 - alpha ** T) / (1 - alpha), (B, H)), rtol=1e-6)
    # b = 0 as well: g = tanh(0) = 0 so c stays 0 and h == 0
    hs, c = O.lstm_sequence(x, w, np.zeros(4 * H), np.zeros((B, H)), np.zeros((B, H)), h_dtype="f32")
    assert np.all(hs == 0) and np.all(c == 0)


def test_lstm_gate_order_is_i_f_g_o():
    H = 3
    c = np.full((1, H), 0.7)
    big = 50.0
    # only f open: c' = c, h' = 0 (o closed)
    z = np.concatenate([np.full(H, -big), np.full(H, big), np.zeros(H), np.full(H, -big)])[None]
    c2, h2 = O.lstm_gates(z, c)
    np.testing.assert_allclose(c2, c, atol=1e-12); np.testing.assert_allclose(h2, 0, atol=1e-12)
    # i and o open, g saturated at +1, f closed: c' = 1, h' = tanh(1)
    z = np.concatenate([np.full(H, big), np.full(H, -big), np.full(H, big), np.full(H, big)])[None]
    c2, h2 = O.lstm_gates(z, c)
    np.testing.assert_allclose(c2, 1.0, atol=1e-12); np.testing.assert_allclose(h2, math.tanh(1.0), atol=1e-12)


# ---------------------------------------------------------------- invariants
def test_conv_linearity():
    x, y, w = RNG.standard_normal((1, 3, 6, 6)), RNG.standard_normal((1, 3, 6, 6)), RNG.standard_normal((4, 3, 3, 3))
    lhs = O.conv2d(2.5 * x - 0.5 * y, w, (1, 1), (1, 1))
    rhs = 2.5 * O.conv2d(x, w, (1, 1), (1, 1)) - 0.5 * O.conv2d(y, w, (1, 1), (1, 1))
    np.testing.assert_allclose(lhs, rhs, atol=1e-12)


def test_conv_1x1_equals_dense():
    x, w = RNG.standard_normal((2, 5, 4, 3)), RNG.standard_normal((6, 5, 1, 1))
    y = O.conv2d(x, w)
    d = O.dense(x.transpose(0, 2, 3, 1).reshape(-1, 5), w.reshape(6, 5)).reshape(2, 4, 3, 6).transpose(0, 3, 1, 2)
    np.testing.assert_allclose(y, d, atol=1e-13)


def test_conv_stride2_is_subsampled_stride1():
    x, w = RNG.standard_normal((1, 2, 9, 9)), RNG.standard_normal((3, 2, 3, 3))
    np.testing.assert_array_equal(O.conv2d(x, w, (2, 2), (1, 1)), O.conv2d(x, w, (1, 1), (1, 1))[:, :, ::2, ::2])


def test_conv_padding_equals_explicit_zero_pad():
    x, w = RNG.standard_normal((1, 2, 5, 6)), RNG.standard_normal((3, 2, 3, 3))
    xp = np.pad(x, ((0, 0), (0, 0), (2, 2), (1, 1)))
    np.testing.assert_array_equal(O.conv2d(x, w, (1, 1), (2, 1)), O.conv2d(xp, w, (1, 1), (0, 0)))


def test_conv_translation_equivariance_interior():
    x, w = RNG.standard_normal((1, 2, 8, 8)), RNG.standard_normal((2, 2, 3, 3))
    xs = np.roll(x, 1, axis=3)
    y, ys = O.conv2d(x, w, (1, 1), (1, 1)), O.conv2d(xs, w, (1, 1), (1, 1))
    np.testing.assert_array_equal(ys[:, :, :, 2:-1], y[:, :, :, 1:-2])


def test_batch_independence():
    x, w = RNG.standard_normal((3, 2, 5, 5)), RNG.standard_normal((2, 2, 3, 3))
    y = O.conv2d(x, w, (1, 1), (1, 1))
    np.testing.assert_array_equal(y[1:2], O.conv2d(x[1:2], w, (1, 1), (1, 1)))


def test_dense_split_inner_dim():
    x, h, w = RNG.standard_normal((3, 4)), RNG.standard_normal((3, 5)), RNG.standard_normal((6, 9))
    whole = O.dense(np.concatenate([x, h], 1), w)
    np.testing.assert_allclose(whole, O.dense(x, w[:, :4]) + O.dense(h, w[:, 4:]), atol=1e-13)


def test_folded_batchnorm_equals_explicit():
    x, w = RNG.standard_normal((2, 3, 6, 6)), RNG.standard_normal((4, 3, 3, 3))
    g, b, m, v = RNG.uniform(.5, 1.5, 4), RNG.uniform(-.1, .1, 4), RNG.standard_normal(4) * .1, RNG.uniform(.5, 1.5, 4)
    explicit = O.batchnorm(O.conv2d(x, w, (1, 1), (1, 1)), g, b, m, v, 1e-5)
    wf, bf = O.fold_batchnorm(w, g, b, m, v, 1e-5)
    np.testing.assert_allclose(O.bias_add(O.conv2d(x, wf, (1, 1), (1, 1)), bf, 1), explicit, atol=1e-12)
    # batch-norm itself against its formula on one element
    y = O.batchnorm(x[:, :3], g[:3], b[:3], m[:3], v[:3], 1e-5)
    assert abs(y[1, 2, 3, 4] - (g[2] * (x[1, 2, 3, 4] - m[2]) / math.sqrt(v[2] + 1e-5) + b[2])) < 1e-14


def test_batchnorm_closed_forms():
    # gamma = sqrt(var + eps), beta = mean  =>  y = x;   x = mean  =>  y = beta  (whatever the other statistics are)
    x = RNG.standard_normal((3, 4, 5, 2))
    g, b, m, v = RNG.uniform(.5, 1.5, 4), RNG.uniform(-1, 1, 4), RNG.standard_normal(4), RNG.uniform(.5, 1.5, 4)
    np.testing.assert_allclose(O.batchnorm(x, np.sqrt(v + 1e-5), m, m, v, 1e-5), x, atol=1e-14)
    xm = np.broadcast_to(m[None, :, None, None], x.shape)
    np.testing.assert_array_equal(O.batchnorm(xm, g, b, m, v, 1e-5), np.broadcast_to(b[None, :, None, None], x.shape))
    # eps sits under the root, next to the variance: numbers worked by hand (all exactly representable).
    # channel 0: (5 - 1) / sqrt(3.75 + .25) * 1 + 0 = 2;  channel 1: (5 - 2) / sqrt(.75 + .25) * 3 - 1 = 8
    y = O.batchnorm(np.full((2, 2, 1, 3), 5.0), [1.0, 3.0], [0.0, -1.0], [1.0, 2.0], [3.75, 0.75], 0.25)
    np.testing.assert_array_equal(y, np.broadcast_to(np.array([2.0, 8.0])[None, :, None, None], (2, 2, 1, 3)))
    # zero variance: only eps is left in the denominator: 2 * (3 - 1) / sqrt(.25) + .5 = 8.5
    assert O.batchnorm(np.full((1, 1, 1, 1), 3.0), [2.0], [0.5], [1.0], [0.0], 0.25)[0, 0, 0, 0] == 8.5
    # the folded form on the same hand numbers: scale = 3 / sqrt(.75 + .25) = 3, w' = 3 w, b' = -1 - 2 * 3 = -7
    wf, bf = O.fold_batchnorm(np.array([[2.0, 4.0], [1.0, -1.0]]), [3.0, 1.0], [-1.0, 0.0], [2.0, 1.0], [0.75, 3.75], 0.25)
    np.testing.assert_array_equal(wf, [[6.0, 12.0], [0.5, -0.5]])
    np.testing.assert_array_equal(bf, [-7.0, -0.5])


# ---------------------------------------------------------------- partial derivatives of the contractions
GRAD_GEOMS = [
    # n  c  h  w  o  k  s  p
    (2, 3, 5, 4, 2, 3, 1, 1),
    (1, 2, 7, 6, 3, 3, 2, 1),          # (H + 2p - K) % s = 0 for H, 1 for W: the last input column gets no gradient from some taps
    (2, 2, 6, 6, 2, 1, 2, 0),          # the 1x1 / stride 2 projection: odd rows and columns get none at all
    (1, 1, 8, 5, 2, 5, 1, 2),
    (1, 2, 6, 7, 2, 2, 3, 0),          # stride larger than the kernel: gaps
]


def _brute_conv_grads(dy, x, w, s, p):
    """Gather formulation, pure Python: each result element collects the forward terms that contain it."""
    N, C, H, W = x.shape
    O, _, KH, KW = w.shape
    _, _, OH, OW = dy.shape
    dx = np.zeros(x.shape); dw = np.zeros(w.shape)
    for n in range(N):
        for c in range(C):
            for h in range(H):
                for ww in range(W):
                    acc = 0.0
                    for o in range(O):
                        for a in range(KH):
                            for b in range(KW):
                                ti, tj = h + p - a, ww + p - b
                                if ti % s or tj % s:
                                    continue
                                i, j = ti // s, tj // s
                                if 0 <= i < OH and 0 <= j < OW:
                                    acc += dy[n, o, i, j] * w[o, c, a, b]
                    dx[n, c, h, ww] = acc
    for o in range(O):
        for c in range(C):
            for a in range(KH):
                for b in range(KW):
                    acc = 0.0
                    for n in range(N):
                        for i in range(OH):
                            for j in range(OW):
                                ih, iw = i * s - p + a, j * s - p + b
                                if 0 <= ih < H and 0 <= iw < W:
                                    acc += dy[n, o, i, j] * x[n, c, ih, iw]
                    dw[o, c, a, b] = acc
    return dx, dw


@pytest.mark.parametrize("geom", GRAD_GEOMS, ids=[f"g{i}" for i in range(len(GRAD_GEOMS))])
def test_conv_gradients_brute_force_and_adjoint(geom):
    n, c, h, w_, o, k, s, p = geom
    x = RNG.integers(-3, 4, (n, c, h, w_)).astype(np.float64)
    w = RNG.integers(-3, 4, (o, c, k, k)).astype(np.float64)
    y = O.conv2d(x, w, (s, s), (p, p))
    dy = RNG.integers(-3, 4, y.shape).astype(np.float64)
    dx = O.conv2d_grad_x(dy, w, x.shape, (s, s), (p, p))
    dw = O.conv2d_grad_w(dy, x, (k, k), (s, s), (p, p))
    bx, bw = _brute_conv_grads(dy, x, w, s, p)
    np.testing.assert_array_equal(dx, bx)          # integer-valued: exact
    np.testing.assert_array_equal(dw, bw)
    # the convolution is linear in x and in w, and the gradients are its adjoints: <conv(x; w), dy> = <x, dx> = <w, dw>
    lhs = float((y * dy).sum())
    assert lhs == float((x * dx).sum()) == float((w * dw).sum())


def test_conv_gradients_by_finite_differences():
    # L = <conv(x; w), g> is linear in x and in w, so a central difference gives its partial derivatives up to rounding
    n, c, h, w_, o, k, s, p = 1, 2, 5, 6, 2, 3, 2, 1
    x, w = RNG.standard_normal((n, c, h, w_)), RNG.standard_normal((o, c, k, k))
    L = lambda xx, ww: float((O.conv2d(xx, ww, (s, s), (p, p)) * g).sum())
    g = RNG.standard_normal(O.conv2d(x, w, (s, s), (p, p)).shape)
    dx = O.conv2d_grad_x(g, w, x.shape, (s, s), (p, p))
    dw = O.conv2d_grad_w(g, x, (k, k), (s, s), (p, p))
    eps = 0.5
    for idx in [(0, 0, 0, 0), (0, 1, 4, 5), (0, 0, 2, 3), (0, 1, 3, 0)]:
        e = np.zeros_like(x); e[idx] = eps
        assert abs((L(x + e, w) - L(x - e, w)) / (2 * eps) - dx[idx]) < 1e-12
    for idx in [(0, 0, 0, 0), (1, 1, 2, 2), (0, 1, 1, 2), (1, 0, 2, 0)]:
        e = np.zeros_like(w); e[idx] = eps
        assert abs((L(x, w + e) - L(x, w - e)) / (2 * eps) - dw[idx]) < 1e-12


def test_conv_gradient_closed_forms():
    # all-ones dy and weights, 3x3 / stride 1 / pad 1: dx counts the outputs whose window holds the pixel, times O:
    # 9 O inside, 6 O on an edge, 4 O in a corner; all-ones dy and x: dw counts the window positions inside the image
    dy, w = np.ones((1, 5, 6, 7)), np.ones((5, 2, 3, 3))
    dx = O.conv2d_grad_x(dy, w, (1, 2, 6, 7), (1, 1), (1, 1))
    assert dx[0, 0, 3, 3] == 45 and dx[0, 1, 0, 3] == 30 and dx[0, 0, 5, 6] == 20 and dx[0, 1, 2, 0] == 30
    dw = O.conv2d_grad_w(dy, np.ones((1, 2, 6, 7)), (3, 3), (1, 1), (1, 1))
    assert dw[0, 0, 1, 1] == 42 and dw[4, 1, 0, 1] == 35 and dw[2, 0, 0, 0] == 30 and dw[0, 1, 1, 2] == 36
    # a one-hot dy puts the (unflipped) kernel into dx at the window's place, and the window of x into dw
    w = RNG.standard_normal((1, 1, 3, 3)); x = RNG.standard_normal((1, 1, 6, 6))
    dy = np.zeros((1, 1, 2, 2)); dy[0, 0, 1, 0] = 1.0            # stride 2, pad 0: window rows 2..4, columns 0..2
    dx = O.conv2d_grad_x(dy, w, x.shape, (2, 2), (0, 0))
    np.testing.assert_array_equal(dx[0, 0, 2:5, 0:3], w[0, 0])
    assert abs(dx.sum() - w.sum()) < 1e-12 and np.count_nonzero(dx) == 9
    np.testing.assert_array_equal(O.conv2d_grad_w(dy, x, (3, 3), (2, 2), (0, 0))[0, 0], x[0, 0, 2:5, 0:3])


def test_dense_gradients():
    dy, w, x = RNG.integers(-3, 4, (4, 3)).astype(float), RNG.integers(-3, 4, (3, 5)).astype(float), RNG.integers(-3, 4, (4, 5)).astype(float)
    dx, dw = O.dense_grad_x(dy, w), O.dense_grad_w(dy, x)
    for m in range(4):
        for k in range(5):
            assert dx[m, k] == sum(dy[m, n] * w[n, k] for n in range(3))
    for n in range(3):
        for k in range(5):
            assert dw[n, k] == sum(dy[m, n] * x[m, k] for m in range(4))
    # adjoints of y = dense(x, W): <y, dy> = <x, dx> = <W, dW>; a one-hot dy picks a row of W / a row of x
    y = O.dense(x, w)
    assert float((y * dy).sum()) == float((x * dx).sum()) == float((w * dw).sum())
    e = np.zeros((4, 3)); e[2, 1] = 1.0
    np.testing.assert_array_equal(O.dense_grad_x(e, w)[2], w[1])
    np.testing.assert_array_equal(O.dense_grad_w(e, x)[1], x[2])
    # the 1x1 convolution's gradients are the dense ones on the [N*H*W, C] view
    xc, wc = RNG.standard_normal((2, 5, 4, 3)), RNG.standard_normal((6, 5, 1, 1))
    g = RNG.standard_normal((2, 6, 4, 3))
    gm, xm = g.transpose(0, 2, 3, 1).reshape(-1, 6), xc.transpose(0, 2, 3, 1).reshape(-1, 5)
    np.testing.assert_allclose(O.conv2d_grad_x(g, wc, xc.shape), O.dense_grad_x(gm, wc.reshape(6, 5)).reshape(2, 4, 3, 5).transpose(0, 3, 1, 2), atol=1e-13)
    np.testing.assert_allclose(O.conv2d_grad_w(g, xc, (1, 1)).reshape(6, 5), O.dense_grad_w(gm, xm), atol=1e-13)


def test_gradients_against_library_autograd_float64():
    for (n, c, h, w_, o, k, s, p) in [(2, 3, 9, 8, 4, 3, 1, 1), (1, 4, 11, 10, 3, 3, 2, 1), (2, 2, 8, 8, 3, 1, 2, 0), (1, 3, 12, 12, 2, 7, 2, 3)]:
        x = torch.from_numpy(RNG.standard_normal((n, c, h, w_))).requires_grad_(True)
        w = torch.from_numpy(RNG.standard_normal((o, c, k, k))).requires_grad_(True)
        y = torch.nn.functional.conv2d(x, w, stride=s, padding=p)
        g = torch.from_numpy(RNG.standard_normal(tuple(y.shape)))
        gx, gw = torch.autograd.grad(y, (x, w), g)
        np.testing.assert_allclose(O.conv2d_grad_x(g.numpy(), w.detach().numpy(), x.shape, (s, s), (p, p)), gx.numpy(), atol=1e-12)
        np.testing.assert_allclose(O.conv2d_grad_w(g.numpy(), x.detach().numpy(), (k, k), (s, s), (p, p)), gw.numpy(), atol=1e-12)
    a = torch.from_numpy(RNG.standard_normal((7, 33))).requires_grad_(True)
    b = torch.from_numpy(RNG.standard_normal((9, 33))).requires_grad_(True)
    g = torch.from_numpy(RNG.standard_normal((7, 9)))
    ga, gb = torch.autograd.grad(a @ b.T, (a, b), g)
    np.testing.assert_allclose(O.dense_grad_x(g.numpy(), b.detach().numpy()), ga.numpy(), atol=1e-12)
    np.testing.assert_allclose(O.dense_grad_w(g.numpy(), a.detach().numpy()), gb.numpy(), atol=1e-12)


# ---------------------------------------------------------------- library cross-check
def test_against_library_float64():
    x, w = RNG.standard_normal((2, 8, 13, 11)), RNG.standard_normal((5, 8, 3, 3))
    for s, p in [((1, 1), (1, 1)), ((2, 2), (1, 1)), ((2, 2), (0, 0))]:
        ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w), stride=s, padding=p).numpy()
        np.testing.assert_allclose(O.conv2d(x, w, s, p), ref, atol=1e-12)
    x7, w7 = RNG.standard_normal((1, 3, 20, 20)), RNG.standard_normal((4, 3, 7, 7))
    ref = torch.nn.functional.conv2d(torch.from_numpy(x7), torch.from_numpy(w7), stride=2, padding=3).numpy()
    np.testing.assert_allclose(O.conv2d(x7, w7, (2, 2), (3, 3)), ref, atol=1e-12)
    a, b = RNG.standard_normal((7, 33)), RNG.standard_normal((9, 33))
    np.testing.assert_allclose(O.dense(a, b), a @ b.T, atol=1e-12)
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(x), 3, 2, 1).numpy()
    np.testing.assert_array_equal(O.maxpool2d(x, (3, 3), (2, 2), (1, 1)), ref)


# ---------------------------------------------------------------- rounding helpers
def test_round_bf16_ties_and_exactness():
    v = np.array([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -7, -(1 + 2.0 ** -8 + 2.0 ** -20), 0.0, 255.5, 3.0e-5])
    r = O.round_to(v, "bf16")
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1 + 2.0 ** -6 and r[3] == 1 + 2.0 ** -7
    assert r[4] == -(1 + 2.0 ** -7) and r[5] == 0.0 and r[6] == 256.0
    # a bf16 value has at most 8 significant bits and is a fixed point of the rounding
    np.testing.assert_array_equal(O.round_to(r, "bf16"), r)
    m, e = np.frexp(r[r != 0])
    assert np.all(m * 256 == np.round(m * 256))
    # agrees with the bit-pattern definition (upper 16 bits of float32 after RNE) on float32 inputs
    x = RNG.standard_normal(2000).astype(np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    bits = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint32) << 16
    np.testing.assert_array_equal(O.round_to(x.astype(np.float64), "bf16"), bits.astype(np.uint32).view(np.float32).astype(np.float64))
    # half an ulp of an 8-bit significand: 2^-8 relative
    y = RNG.standard_normal(2000)
    assert np.max(np.abs(O.round_to(y, "bf16") - y) / np.abs(y)) <= 2.0 ** -8


def test_round_f32():
    y = RNG.standard_normal(100)
    np.testing.assert_array_equal(O.round_to(y, "f32"), y.astype(np.float32).astype(np.float64))


def test_widen_is_exact():
    x = RNG.standard_normal(100).astype(np.float32)
    np.testing.assert_array_equal(O.widen(x, "f32"), x.astype(np.float64))
    bits = np.array([0x3F80, 0x3FC0, 0xC000, 0x0000, 0x4049], dtype=np.uint16)
    np.testing.assert_array_equal(O.widen(bits, "bf16"), [1.0, 1.5, -2.0, 0.0, 3.140625])
