"""Pins for the CPU oracle's layer functions: hand cases, closed forms, adjoint identities,
finite differences, brute force, and torch-CPU-fp64 library routines as an independent
witness.  A wrong sign, index, transposition or dropped term in the oracle fails here."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ops

GOLD = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(12345)


def _read_rows(name):
    rows = []
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append([float(v) for v in line.split()])
    return rows


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a))


CONV_CASES = [
    # N, Cin, H, W, Cout, k, stride, pad
    (2, 3, 7, 6, 4, 3, 1, 1),
    (2, 5, 9, 8, 3, 3, 2, 1),
    (1, 4, 8, 8, 6, 1, 1, 0),
    (2, 4, 9, 7, 6, 1, 2, 0),
    (1, 2, 6, 6, 2, 3, 1, 0),
    (1, 2, 10, 11, 3, 7, 2, 3),
    (1, 1, 1, 1, 2, 3, 1, 1),
]


# ------------------------------------------------------------------ conv forward
def test_conv_hand_ones():
    want = np.array(_read_rows("conv3x3_ones.txt"))
    y = ops.conv2d_fwd(np.ones((1, 1, 3, 3)), np.ones((1, 1, 3, 3)), None, 1, 1)
    assert np.array_equal(y[0, 0], want)


def test_conv_delta_kernel_is_identity():
    x = RNG.standard_normal((2, 3, 5, 6))
    w = np.zeros((3, 3, 3, 3))
    for c in range(3):
        w[c, c, 1, 1] = 1.0
    assert np.array_equal(ops.conv2d_fwd(x, w, None, 1, 1), x)


def test_conv_shifted_delta_reads_the_right_neighbour():
    # kernel with a single 1 at (r,s) must return x shifted by (r-pad, s-pad): pins the
    # direction of the correlation (no kernel flip) and the row/column roles.
    x = RNG.standard_normal((1, 1, 5, 5))
    w = np.zeros((1, 1, 3, 3))
    w[0, 0, 0, 2] = 1.0                      # up one row, right one column
    y = ops.conv2d_fwd(x, w, None, 1, 1)
    want = np.zeros_like(x)
    want[0, 0, 1:, :-1] = x[0, 0, :-1, 1:]
    assert np.array_equal(y, want)


def test_conv_full_kernel_is_dot_product_and_bias():
    x = RNG.standard_normal((3, 4, 5, 5))
    w = RNG.standard_normal((2, 4, 5, 5))
    b = RNG.standard_normal(2)
    y = ops.conv2d_fwd(x, w, b, 1, 0)
    want = np.einsum("nchw,ochw->no", x, w) + b
    assert y.shape == (3, 2, 1, 1)
    np.testing.assert_allclose(y[:, :, 0, 0], want, rtol=1e-13, atol=1e-13)


def test_conv_1x1_on_1x1_equals_linear():
    x = RNG.standard_normal((5, 7))
    w = RNG.standard_normal((3, 7))
    b = RNG.standard_normal(3)
    y = ops.conv2d_fwd(x.reshape(5, 7, 1, 1), w.reshape(3, 7, 1, 1), b, 1, 0)
    np.testing.assert_allclose(y.reshape(5, 3), ops.linear_fwd(x, w, b), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(y.reshape(5, 3), x @ w.T + b, rtol=1e-13, atol=1e-13)


def _im2col_conv(x, w, b, st, pad):
    """Independent brute force: explicit patch matrix times flattened filters."""
    N, Cin, H, W = x.shape
    Cout, _, kh, kw = w.shape
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    Ho, Wo = (H + 2 * pad - kh) // st + 1, (W + 2 * pad - kw) // st + 1
    cols = np.empty((N, Ho, Wo, Cin * kh * kw))
    for p in range(Ho):
        for q in range(Wo):
            cols[:, p, q, :] = xp[:, :, p * st:p * st + kh, q * st:q * st + kw].reshape(N, -1)
    y = cols @ w.reshape(Cout, -1).T
    if b is not None:
        y = y + b
    return y.transpose(0, 3, 1, 2)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd_vs_bruteforce_and_torch(case):
    N, Cin, H, W, Cout, k, st, pad = case
    x = RNG.standard_normal((N, Cin, H, W))
    w = RNG.standard_normal((Cout, Cin, k, k))
    b = RNG.standard_normal(Cout)
    y = ops.conv2d_fwd(x, w, b, st, pad)
    np.testing.assert_allclose(y, _im2col_conv(x, w, b, st, pad), rtol=1e-12, atol=1e-12)
    yt = F.conv2d(_t(x), _t(w), _t(b), stride=st, padding=pad).numpy()
    np.testing.assert_allclose(y, yt, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------ conv backward
@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_dgrad_adjoint_identity(case):
    N, Cin, H, W, Cout, k, st, pad = case
    x = RNG.standard_normal((N, Cin, H, W))
    w = RNG.standard_normal((Cout, Cin, k, k))
    y = ops.conv2d_fwd(x, w, None, st, pad)
    g = RNG.standard_normal(y.shape)
    dx = ops.conv2d_dgrad(g, w, x.shape, st, pad)
    lhs, rhs = np.sum(y * g), np.sum(x * dx)
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_wgrad_adjoint_identity_and_bias(case):
    N, Cin, H, W, Cout, k, st, pad = case
    x = RNG.standard_normal((N, Cin, H, W))
    w = RNG.standard_normal((Cout, Cin, k, k))
    y = ops.conv2d_fwd(x, w, None, st, pad)
    g = RNG.standard_normal(y.shape)
    dw = np.zeros_like(w)
    db = np.zeros(Cout)
    ops.conv2d_wgrad(x, g, dw, db, st, pad)
    lhs, rhs = np.sum(y * g), np.sum(w * dw)          # conv is linear in w
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
    np.testing.assert_allclose(db, g.sum(axis=(0, 2, 3)), rtol=1e-12, atol=1e-12)
    # accumulation: a second call adds the same amount again
    ops.conv2d_wgrad(x, g, dw, db, st, pad)
    dw1 = np.zeros_like(w)
    ops.conv2d_wgrad(x, g, dw1, None, st, pad)
    np.testing.assert_allclose(dw, 2 * dw1, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db, 2 * g.sum(axis=(0, 2, 3)), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("case", CONV_CASES[:4])
def test_conv_grads_vs_torch_autograd(case):
    N, Cin, H, W, Cout, k, st, pad = case
    x = RNG.standard_normal((N, Cin, H, W))
    w = RNG.standard_normal((Cout, Cin, k, k))
    xt = _t(x).requires_grad_()
    wt = _t(w).requires_grad_()
    yt = F.conv2d(xt, wt, None, stride=st, padding=pad)
    g = RNG.standard_normal(tuple(yt.shape))
    yt.backward(_t(g))
    dx = ops.conv2d_dgrad(g, w, x.shape, st, pad)
    dw = np.zeros_like(w)
    ops.conv2d_wgrad(x, g, dw, None, st, pad)
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=1e-11, atol=1e-11)


def _fd(f, a, idxs, h=1e-5):
    out = []
    for ix in idxs:
        old = a[ix]
        a[ix] = old + h
        fp = f()
        a[ix] = old - h
        fm = f()
        a[ix] = old
        out.append((fp - fm) / (2 * h))
    return np.array(out)


def _some_indices(shape, n=6):
    return [tuple(int(RNG.integers(0, s)) for s in shape) for _ in range(n)]


@pytest.mark.parametrize("case", [CONV_CASES[0], CONV_CASES[1], CONV_CASES[3]])
def test_conv_finite_differences(case):
    N, Cin, H, W, Cout, k, st, pad = case
    x = RNG.standard_normal((N, Cin, H, W))
    w = RNG.standard_normal((Cout, Cin, k, k))
    b = RNG.standard_normal(Cout)
    g = RNG.standard_normal(ops.conv2d_fwd(x, w, b, st, pad).shape)
    f = lambda: float(np.sum(ops.conv2d_fwd(x, w, b, st, pad) * g))
    dx = ops.conv2d_dgrad(g, w, x.shape, st, pad)
    dw = np.zeros_like(w)
    db = np.zeros_like(b)
    ops.conv2d_wgrad(x, g, dw, db, st, pad)
    for arr, grad in ((x, dx), (w, dw), (b, db)):
        idxs = _some_indices(arr.shape)
        num = _fd(f, arr, idxs)
        ana = np.array([grad[i] for i in idxs])
        np.testing.assert_allclose(num, ana, rtol=1e-7, atol=1e-8)


# ------------------------------------------------------------------ ReLU / max-pool
def test_relu_hand():
    x = np.array([-2.0, -0.0, 0.0, 1e-30, 3.0])
    y = ops.relu_fwd(x)
    assert np.array_equal(y, [0, 0, 0, 1e-30, 3.0])
    dy = np.array([1.0, 2.0, 3.0, 4.0, 5.0])
    assert np.array_equal(ops.relu_bwd(y, dy), [0, 0, 0, 4.0, 5.0])   # strict > 0


def test_maxpool_hand_ties():
    rows = _read_rows("maxpool_ties.txt")
    x = np.array(rows[:4]).reshape(1, 1, 4, 4)
    y, idx = ops.maxpool_fwd(x)
    assert np.array_equal(y[0, 0], np.array(rows[4:6]))
    assert np.array_equal(idx[0, 0], np.array(rows[6:8]).astype(np.uint8))
    dy = np.array([[10.0, 20.0], [30.0, 40.0]]).reshape(1, 1, 2, 2)
    dx = ops.maxpool_bwd(dy, idx, x.shape)
    want = np.zeros((4, 4))
    want[0, 0], want[0, 3], want[2, 0], want[2, 2] = 10, 20, 30, 40
    assert np.array_equal(dx[0, 0], want)


def test_maxpool_all_zero_window_gives_index_zero():
    y, idx = ops.maxpool_fwd(np.zeros((1, 2, 4, 6)))
    assert not idx.any() and not y.any()


@pytest.mark.parametrize("shape", [(2, 3, 8, 6), (1, 2, 7, 9)])
def test_maxpool_vs_torch_and_conservation(shape):
    x = RNG.standard_normal(shape)
    y, idx = ops.maxpool_fwd(x)
    yt, it = F.max_pool2d(_t(x), 2, 2, return_indices=True)
    assert np.array_equal(y, yt.numpy())
    N, C, H, W = shape
    Ho, Wo = y.shape[2:]
    p, q = np.meshgrid(np.arange(Ho), np.arange(Wo), indexing="ij")
    flat = (2 * p + idx // 2) * W + (2 * q + idx % 2)                # window index -> plane index
    assert np.array_equal(flat, it.numpy())
    assert idx.max() < 4
    dy = RNG.standard_normal(y.shape)
    dx = ops.maxpool_bwd(dy, idx, shape)
    assert abs(dx.sum() - dy.sum()) < 1e-12
    assert np.count_nonzero(dx) == dy.size                          # one landing spot each
    xt = _t(x).requires_grad_()
    F.max_pool2d(xt, 2, 2).backward(_t(dy))
    assert np.array_equal(dx, xt.grad.numpy())


def test_maxpool_3x3_s2_pad1_vs_torch():
    x = RNG.standard_normal((2, 3, 9, 10))
    y, idx = ops.maxpool_fwd(x, 3, 2, 1)
    yt = F.max_pool2d(_t(x), 3, 2, 1)
    assert np.array_equal(y, yt.numpy())
    dy = RNG.standard_normal(y.shape)
    xt = _t(x).requires_grad_()
    F.max_pool2d(xt, 3, 2, 1).backward(_t(dy))
    assert np.allclose(ops.maxpool_bwd(dy, idx, x.shape, 3, 2, 1), xt.grad.numpy(), atol=1e-14)


def test_maxpool_overlapping_windows_add_their_gradients():
    # 1x5 row, 3-wide windows at stride 2 with one pad: windows cover {-,0,1}, {1,2,3}, {3,4,-};
    # the peak at position 1 wins the first two windows, position 4 the last
    x = np.array([0.0, 9.0, 1.0, 2.0, 5.0]).reshape(1, 1, 1, 5)
    y, idx = ops.maxpool_fwd(x, 3, 2, 1)
    assert y.shape == (1, 1, 1, 3) and np.array_equal(y.ravel(), [9.0, 9.0, 5.0])
    # window row 0 is the padding row, so the in-window index is 3 + column
    assert np.array_equal(idx.ravel(), [3 + 2, 3 + 0, 3 + 1])
    dx = ops.maxpool_bwd(np.array([1.0, 10.0, 100.0]).reshape(1, 1, 1, 3), idx, x.shape, 3, 2, 1)
    assert np.array_equal(dx.ravel(), [0.0, 11.0, 0.0, 0.0, 100.0])


def test_avgpool_hand_global_and_torch():
    x = np.arange(16.0).reshape(1, 1, 4, 4)
    assert np.array_equal(ops.avgpool_fwd(x, 2)[0, 0], [[2.5, 4.5], [10.5, 12.5]])
    assert ops.avgpool_fwd(x, 4).ravel()[0] == 7.5                      # global: the plain mean
    x = RNG.standard_normal((3, 5, 7, 7))
    y = ops.avgpool_fwd(x, 7)
    assert np.allclose(y[:, :, 0, 0], x.mean(axis=(2, 3)), atol=1e-15)
    x = RNG.standard_normal((2, 3, 9, 6))                               # 9 rows: the last is in no window
    y = ops.avgpool_fwd(x, 2)
    assert np.allclose(y, F.avg_pool2d(_t(x), 2).numpy(), atol=1e-15)
    dy = RNG.standard_normal(y.shape)
    dx = ops.avgpool_bwd(dy, x.shape, 2)
    assert abs(np.sum(y * dy) - np.sum(x * dx)) < 1e-12                 # adjoint of a linear map
    assert not dx[:, :, 8].any()
    xt = _t(x).requires_grad_()
    F.avg_pool2d(xt, 2).backward(_t(dy))
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-15)


# ------------------------------------------------------------------ LSTM
def _torch_lstm(x, w, b, In, Hd):
    """torch.nn.LSTM (CPU, fp64) loaded with the same weights: x [N][In][T][1] -> module, sequence-first view."""
    m = torch.nn.LSTM(In, Hd, batch_first=True).double()
    with torch.no_grad():
        m.weight_ih_l0.copy_(_t(w[:, :In]))
        m.weight_hh_l0.copy_(_t(w[:, In:]))
        m.bias_ih_l0.copy_(_t(b))
        m.bias_hh_l0.zero_()
    return m


def test_lstm_one_step_closed_form_and_saturated_forget_gate():
    # zero weights: every gate sees only its bias
    Hd, In = 3, 2
    w = np.zeros((4 * Hd, In + Hd))
    b = RNG.standard_normal(4 * Hd)
    x = RNG.standard_normal((2, In, 1, 1))
    y, _ = ops.lstm_fwd(x, w, b)
    sg = lambda v: 1 / (1 + np.exp(-v))
    want = sg(b[3 * Hd:]) * np.tanh(sg(b[:Hd]) * np.tanh(b[2 * Hd:3 * Hd]))
    assert np.allclose(y[:, :, 0, 0], want[None, :], atol=1e-15)
    # forget gate held at 1 (bias +40), constant input gate and candidate: c_t grows by i*g per step
    b2 = b.copy()
    b2[Hd:2 * Hd] = 40.0
    T = 6
    y, (gates, cells) = ops.lstm_fwd(np.zeros((1, In, T, 1)), w, b2)
    step = sg(b2[:Hd]) * np.tanh(b2[2 * Hd:3 * Hd])
    for t in range(T):
        assert np.allclose(cells[0, t], (t + 1) * step, atol=1e-12)
        assert np.allclose(y[0, :, t, 0], sg(b2[3 * Hd:]) * np.tanh((t + 1) * step), atol=1e-12)


@pytest.mark.parametrize("N,In,Hd,T", [(3, 4, 5, 7), (2, 6, 3, 1), (1, 2, 2, 9)])
def test_lstm_vs_torch_autograd_and_finite_differences(N, In, Hd, T):
    x = RNG.standard_normal((N, In, T, 1))
    w = RNG.standard_normal((4 * Hd, In + Hd)) * 0.5
    b = RNG.standard_normal(4 * Hd) * 0.5
    dy = RNG.standard_normal((N, Hd, T, 1))
    y, saved = ops.lstm_fwd(x, w, b)
    dw, db = np.zeros_like(w), np.zeros_like(b)
    dx = ops.lstm_bwd(x, y, w, saved, dy, dw, db)
    m = _torch_lstm(x, w, b, In, Hd)
    xt = _t(x[:, :, :, 0].transpose(0, 2, 1).copy()).requires_grad_()       # [N][T][In]
    yt, _ = m(xt)
    assert np.allclose(y[:, :, :, 0].transpose(0, 2, 1), yt.detach().numpy(), atol=1e-13)
    yt.backward(_t(dy[:, :, :, 0].transpose(0, 2, 1).copy()))
    assert np.allclose(dx[:, :, :, 0].transpose(0, 2, 1), xt.grad.numpy(), atol=1e-12)
    assert np.allclose(dw[:, :In], m.weight_ih_l0.grad.numpy(), atol=1e-12)
    assert np.allclose(dw[:, In:], m.weight_hh_l0.grad.numpy(), atol=1e-12)
    assert np.allclose(db, m.bias_ih_l0.grad.numpy(), atol=1e-12)
    # central differences of <lstm(x), dy> in a few random directions
    f = lambda x_, w_, b_: float(np.sum(ops.lstm_fwd(x_, w_, b_)[0] * dy))
    h = 1e-6
    for _ in range(3):
        ex, ew, eb = RNG.standard_normal(x.shape), RNG.standard_normal(w.shape), RNG.standard_normal(b.shape)
        fd = (f(x + h * ex, w + h * ew, b + h * eb) - f(x - h * ex, w - h * ew, b - h * eb)) / (2 * h)
        an = np.sum(dx * ex) + np.sum(dw * ew) + np.sum(db * eb)
        assert abs(fd - an) <= 1e-7 * max(1.0, abs(an)), (fd, an)


def test_lstm_gradients_accumulate_and_rounding_points():
    N, In, Hd, T = 2, 3, 4, 5
    x = ops.round_bf16(RNG.standard_normal((N, In, T, 1)))
    w = ops.round_bf16(RNG.standard_normal((4 * Hd, In + Hd)) * 0.5)
    b = RNG.standard_normal(4 * Hd) * 0.5
    y, saved = ops.lstm_fwd(x, w, b, round16=True)
    assert np.array_equal(y, ops.round_bf16(y))                     # the layer output is a stored tensor
    y_exact, _ = ops.lstm_fwd(x, w, b)
    assert 0 < np.max(np.abs(y - y_exact)) < 2e-2
    dy = RNG.standard_normal(y.shape)
    dw, db = np.ones_like(w), np.ones_like(b)
    ops.lstm_bwd(x, y, w, saved, dy, dw, db)
    dw2, db2 = np.zeros_like(w), np.zeros_like(b)
    ops.lstm_bwd(x, y, w, saved, dy, dw2, db2)
    assert np.allclose(dw, 1 + dw2, atol=1e-13) and np.allclose(db, 1 + db2, atol=1e-13)
    assert ops.lstm_bwd(x, y, w, saved, dy, dw2, db2, want_dx=False) is None


# ------------------------------------------------------------------ batch-norm
def test_bn_forward_invariants():
    x = 3.0 + 2.0 * RNG.standard_normal((4, 5, 6, 7))
    eps = 1e-5
    y, mean, invstd = ops.bn_fwd(x, np.ones(5), np.zeros(5), eps)
    np.testing.assert_allclose(mean, x.mean(axis=(0, 2, 3)), rtol=1e-13)
    var = x.var(axis=(0, 2, 3))                                       # biased
    np.testing.assert_allclose(invstd, 1 / np.sqrt(var + eps), rtol=1e-13)
    np.testing.assert_allclose(y.mean(axis=(0, 2, 3)), 0, atol=1e-13)
    np.testing.assert_allclose(y.var(axis=(0, 2, 3)), var / (var + eps), rtol=1e-12)
    gamma, beta = RNG.standard_normal(5), RNG.standard_normal(5)
    y2, _, _ = ops.bn_fwd(x, gamma, beta, eps)
    np.testing.assert_allclose(y2.mean(axis=(0, 2, 3)), beta, atol=1e-13)
    np.testing.assert_allclose(y2.var(axis=(0, 2, 3)), gamma ** 2 * var / (var + eps), rtol=1e-12)


def test_bn_backward_invariants_fd_and_torch():
    x = 1.0 + RNG.standard_normal((3, 4, 5, 5))
    gamma, beta = 1 + 0.3 * RNG.standard_normal(4), RNG.standard_normal(4)
    eps = 1e-5
    y, mean, invstd = ops.bn_fwd(x, gamma, beta, eps)
    g = RNG.standard_normal(y.shape)
    dgamma, dbeta = np.zeros(4), np.zeros(4)
    dx = ops.bn_bwd(x, g, gamma, mean, invstd, dgamma, dbeta)
    xhat = (x - mean[None, :, None, None]) * invstd[None, :, None, None]
    np.testing.assert_allclose(dx.sum(axis=(0, 2, 3)), 0, atol=1e-12)
    # sum(dx*xhat) = gamma*inv*s2*(1 - sum(xhat^2)/m) = gamma*inv^3*eps*s2 (zero only for eps=0)
    s2 = (g * xhat).sum(axis=(0, 2, 3))
    np.testing.assert_allclose((dx * xhat).sum(axis=(0, 2, 3)), gamma * invstd ** 3 * eps * s2,
                               rtol=1e-6, atol=1e-12)
    np.testing.assert_allclose(dbeta, g.sum(axis=(0, 2, 3)), rtol=1e-13)
    f = lambda: float(np.sum(ops.bn_fwd(x, gamma, beta, eps)[0] * g))
    for arr, grad in ((x, dx), (gamma, dgamma), (beta, dbeta)):
        idxs = _some_indices(arr.shape)
        np.testing.assert_allclose(_fd(f, arr, idxs), [grad[i] for i in idxs], rtol=1e-6, atol=1e-8)
    xt, gt, bt = _t(x).requires_grad_(), _t(gamma).requires_grad_(), _t(beta).requires_grad_()
    yt = F.batch_norm(xt, None, None, gt, bt, training=True, eps=eps)
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=1e-11, atol=1e-11)
    yt.backward(_t(g))
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(dgamma, gt.grad.numpy(), rtol=1e-10, atol=1e-11)


# ------------------------------------------------------------------ linear
def test_linear_vs_matmul_and_fd():
    x, w, b = RNG.standard_normal((5, 11)), RNG.standard_normal((7, 11)), RNG.standard_normal(7)
    y = ops.linear_fwd(x, w, b)
    np.testing.assert_allclose(y, x @ w.T + b, rtol=1e-13, atol=1e-13)
    g = RNG.standard_normal(y.shape)
    dx = ops.linear_dgrad(g, w)
    dw, db = np.zeros_like(w), np.zeros_like(b)
    ops.linear_wgrad(x, g, dw, db)
    np.testing.assert_allclose(dx, g @ w, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dw, g.T @ x, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(db, g.sum(0), rtol=1e-13, atol=1e-13)
    ops.linear_wgrad(x, g, dw, db)
    np.testing.assert_allclose(dw, 2 * g.T @ x, rtol=1e-13, atol=1e-13)
    f = lambda: float(np.sum(ops.linear_fwd(x, w, b) * g))
    idxs = _some_indices(w.shape)
    np.testing.assert_allclose(_fd(f, w, idxs), [(g.T @ x)[i] for i in idxs], rtol=1e-7, atol=1e-9)


# ------------------------------------------------------------------ softmax cross-entropy
def test_xent_uniform_logits_closed_form():
    K, want = _read_rows("xent_uniform.txt")[0]
    K = int(K)
    z = np.full((3, K), 0.7)
    labels = np.array([0, 17, K - 1], np.int32)
    s = 0.25
    loss, dz = ops.xent_bwd(z, labels, s)
    assert abs(loss - s * 3 * want) < 1e-12
    expect = np.full((3, K), s / K)
    expect[np.arange(3), labels] -= s
    np.testing.assert_allclose(dz, expect, rtol=0, atol=1e-15)
    np.testing.assert_allclose(ops.softmax_fwd(z), 1.0 / K, rtol=1e-14)


def test_xent_invariants_and_fd():
    z = 4 * RNG.standard_normal((6, 13))
    labels = RNG.integers(0, 13, 6).astype(np.int32)
    s = 1 / 6
    loss, dz = ops.xent_bwd(z, labels, s)
    np.testing.assert_allclose(dz.sum(axis=1), 0, atol=1e-15)
    loss2, dz2 = ops.xent_bwd(z + RNG.standard_normal((6, 1)) * 50, labels, s)
    assert abs(loss - loss2) < 1e-12
    np.testing.assert_allclose(dz, dz2, atol=1e-13)
    p = ops.softmax_fwd(z)
    np.testing.assert_allclose(p.sum(axis=1), 1, rtol=1e-14)
    f = lambda: ops.xent_bwd(z, labels, s)[0]
    idxs = _some_indices(z.shape, 8)
    np.testing.assert_allclose(_fd(f, z, idxs), [dz[i] for i in idxs], rtol=1e-6, atol=1e-9)
    lt = F.cross_entropy(_t(z), _t(labels.astype(np.int64)), reduction="sum") * s
    assert abs(loss - float(lt)) < 1e-12
    # huge logits must not overflow
    big, _ = ops.xent_bwd(np.array([[1000.0, 0.0]]), np.array([0], np.int32), 1.0)
    assert abs(big) < 1e-300 or big == 0.0


# ------------------------------------------------------------------ SGD
def test_sgd_closed_form():
    w, g = RNG.standard_normal(50), RNG.standard_normal(50)
    want = w - 0.05 * g
    ops.sgd_step(w, g, 0.05)
    np.testing.assert_allclose(w, want, rtol=0, atol=1e-16)


# ------------------------------------------------------------------ bf16 rounding
def test_bf16_all_values_are_fixed_points_and_midpoints_tie_to_even():
    bits = np.arange(1 << 16, dtype=np.uint32) << 16
    vals = bits.view(np.float32).astype(np.float64)
    finite = np.isfinite(vals)
    r = ops.round_bf16(vals[finite])
    assert np.array_equal(r, vals[finite])
    # positive finite bf16 numbers in increasing order; check midpoints and near-midpoints
    pos = np.sort(vals[finite & (vals >= 0)])
    lo, hi = pos[:-1], pos[1:]
    mid = (lo + hi) / 2                                   # exact in double
    lo_bits = (lo.astype(np.float32).view(np.uint32) >> 16)
    even_is_lo = (lo_bits & 1) == 0
    rm = ops.round_bf16(mid)
    assert np.array_equal(rm, np.where(even_is_lo, lo, hi))
    assert np.array_equal(ops.round_bf16(-mid), -np.where(even_is_lo, lo, hi))
    just_above = mid + (hi - lo) * 2.0 ** -40
    just_below = mid - (hi - lo) * 2.0 ** -40
    assert np.array_equal(ops.round_bf16(just_above), hi)
    assert np.array_equal(ops.round_bf16(just_below), lo)


def test_bf16_vs_torch_cast_and_input_snap():
    from stage_inputs import gen
    x = (RNG.standard_normal(200000) * np.exp(RNG.uniform(-30, 30, 200000))).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(ops.round_bf16(x.astype(np.float64)), want)
    assert np.array_equal(gen.snap_bf16(x).astype(np.float64), want)
    assert ops.round_bf16(np.array([3.4e38]))[0] == np.inf
