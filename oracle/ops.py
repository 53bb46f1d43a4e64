"""ctypes access to the CPU oracle's layer functions (oracle/bapipe_oracle.c).

TEST INFRASTRUCTURE ONLY.  Arrays are float64 numpy, activations NCHW."""
import ctypes as ct
import os

import numpy as np

from . import build as _build

_lib = None
_D = ct.POINTER(ct.c_double)


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ct.CDLL(path)
        _lib.orc_xent_bwd.restype = ct.c_double
        _lib.orc_num_threads.restype = ct.c_int
    return _lib


def _p(a):
    if a is None:
        return None
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"], (a.dtype, a.flags)
    return a.ctypes.data_as(_D)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads():
    return lib().orc_num_threads()


def round_bf16(a):
    """Round every element to the nearest-even bf16 value (returns a new float64 array)."""
    out = _f64(a).copy()
    lib().orc_round_bf16(_p(out), ct.c_size_t(out.size))
    return out


def _out_hw(H, W, k, st, pad):
    return (H + 2 * pad - k[0]) // st + 1, (W + 2 * pad - k[1]) // st + 1


def conv2d_fwd(x, w, b, stride, pad):
    x, w = _f64(x), _f64(w)
    b = None if b is None else _f64(b)
    N, Cin, H, W = x.shape
    Cout, Cin2, kh, kw = w.shape
    assert Cin == Cin2
    Ho, Wo = _out_hw(H, W, (kh, kw), stride, pad)
    y = np.empty((N, Cout, Ho, Wo))
    lib().orc_conv2d_fwd(_p(x), _p(w), _p(b), _p(y), N, Cin, H, W, Cout, kh, kw, stride, pad)
    return y


def conv2d_dgrad(dy, w, x_shape, stride, pad):
    dy, w = _f64(dy), _f64(w)
    N, Cin, H, W = x_shape
    Cout, _, kh, kw = w.shape
    assert dy.shape == (N, Cout) + _out_hw(H, W, (kh, kw), stride, pad)
    dx = np.empty(x_shape)
    lib().orc_conv2d_dgrad(_p(dy), _p(w), _p(dx), N, Cin, H, W, Cout, kh, kw, stride, pad)
    return dx


def conv2d_wgrad(x, dy, dw, db, stride, pad):
    """Accumulates into dw (OIHW float64) and db (may be None)."""
    x, dy = _f64(x), _f64(dy)
    N, Cin, H, W = x.shape
    Cout, _, kh, kw = dw.shape
    assert dy.shape == (N, Cout) + _out_hw(H, W, (kh, kw), stride, pad)
    lib().orc_conv2d_wgrad(_p(x), _p(dy), _p(dw), _p(db), N, Cin, H, W, Cout, kh, kw, stride, pad)


def relu_fwd(x):
    x = _f64(x)
    y = np.empty_like(x)
    lib().orc_relu_fwd(_p(x), _p(y), ct.c_size_t(x.size))
    return y


def relu_bwd(y, dy):
    y, dy = _f64(y), _f64(dy)
    dx = np.empty_like(y)
    lib().orc_relu_bwd(_p(y), _p(dy), _p(dx), ct.c_size_t(y.size))
    return dx


def maxpool_fwd(x, k=2, stride=2, pad=0):
    x = _f64(x)
    N, C, H, W = x.shape
    Ho, Wo = _out_hw(H, W, (k, k), stride, pad)
    y = np.empty((N, C, Ho, Wo))
    idx = np.empty((N, C, Ho, Wo), np.uint8)
    lib().orc_maxpool_fwd(_p(x), _p(y), idx.ctypes.data_as(ct.POINTER(ct.c_uint8)),
                          N, C, H, W, k, k, stride, pad)
    return y, idx


def maxpool_bwd(dy, idx, x_shape, k=2, stride=2, pad=0):
    dy = _f64(dy)
    idx = np.ascontiguousarray(idx, np.uint8)
    N, C, H, W = x_shape
    dx = np.empty(x_shape)
    lib().orc_maxpool_bwd(_p(dy), idx.ctypes.data_as(ct.POINTER(ct.c_uint8)), _p(dx),
                          N, C, H, W, k, k, stride, pad)
    return dx


def avgpool_fwd(x, k):
    x = _f64(x)
    N, C, H, W = x.shape
    y = np.empty((N, C, H // k, W // k))
    lib().orc_avgpool_fwd(_p(x), _p(y), N, C, H, W, k, k)
    return y


def avgpool_bwd(dy, x_shape, k):
    dy = _f64(dy)
    N, C, H, W = x_shape
    assert dy.shape == (N, C, H // k, W // k)
    dx = np.empty(x_shape)
    lib().orc_avgpool_bwd(_p(dy), _p(dx), N, C, H, W, k, k)
    return dx


def bn_fwd(x, gamma, beta, eps):
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    N, C, H, W = x.shape
    y = np.empty_like(x)
    mean = np.empty(C)
    invstd = np.empty(C)
    lib().orc_bn_fwd(_p(x), _p(gamma), _p(beta), ct.c_double(eps), _p(y), _p(mean), _p(invstd),
                     N, C, H * W)
    return y, mean, invstd


def bn_bwd(x, dy, gamma, mean, invstd, dgamma, dbeta):
    """Returns dx; accumulates into dgamma, dbeta."""
    x, dy, gamma = _f64(x), _f64(dy), _f64(gamma)
    N, C, H, W = x.shape
    dx = np.empty_like(x)
    lib().orc_bn_bwd(_p(x), _p(dy), _p(gamma), _p(mean), _p(invstd), _p(dx), _p(dgamma),
                     _p(dbeta), N, C, H * W)
    return dx


def lstm_fwd(x, w, b, round16=False):
    """x [N][In][T][1], w [4*Hd][In+Hd], b [4*Hd] or None -> (y [N][Hd][T][1], (gates, cells))."""
    x, w = _f64(x), _f64(w)
    b = None if b is None else _f64(b)
    N, In, T, one = x.shape
    assert one == 1 and w.shape[0] % 4 == 0
    Hd = w.shape[0] // 4
    assert w.shape[1] == In + Hd
    y = np.empty((N, Hd, T, 1))
    gates = np.empty((N, T, 4 * Hd))
    cells = np.empty((N, T, Hd))
    lib().orc_lstm_fwd(_p(x), _p(w), _p(b), _p(y), _p(gates), _p(cells), N, In, Hd, T, int(bool(round16)))
    return y, (gates, cells)


def lstm_bwd(x, y, w, saved, dy, dw, db, want_dx=True, round16=False):
    """Returns dx (or None); accumulates into dw, db."""
    x, y, w, dy = _f64(x), _f64(y), _f64(w), _f64(dy)
    gates, cells = saved
    N, In, T, _ = x.shape
    Hd = w.shape[0] // 4
    dx = np.empty_like(x) if want_dx else None
    D = np.empty((N, T, 4 * Hd))
    lib().orc_lstm_bwd(_p(x), _p(y), _p(w), _p(gates), _p(cells), _p(dy), _p(dx), _p(dw), _p(db), _p(D),
                       N, In, Hd, T, int(bool(round16)))
    return dx


def linear_fwd(x, w, b):
    x, w = _f64(x), _f64(w)
    b = None if b is None else _f64(b)
    N, In = x.shape
    Out = w.shape[0]
    assert w.shape[1] == In
    y = np.empty((N, Out))
    lib().orc_linear_fwd(_p(x), _p(w), _p(b), _p(y), N, In, Out)
    return y


def linear_dgrad(dy, w):
    dy, w = _f64(dy), _f64(w)
    N, Out = dy.shape
    In = w.shape[1]
    dx = np.empty((N, In))
    lib().orc_linear_dgrad(_p(dy), _p(w), _p(dx), N, In, Out)
    return dx


def linear_wgrad(x, dy, dw, db):
    x, dy = _f64(x), _f64(dy)
    N, In = x.shape
    Out = dy.shape[1]
    assert dw.shape == (Out, In)
    lib().orc_linear_wgrad(_p(x), _p(dy), _p(dw), _p(db), N, In, Out)


def softmax_fwd(z):
    z = _f64(z)
    p = np.empty_like(z)
    lib().orc_softmax_fwd(_p(z), _p(p), z.shape[0], z.shape[1])
    return p


def xent_bwd(z, labels, scale):
    """Returns (loss, dz) with loss = -scale*sum_n log softmax(z)[n,label_n]."""
    z = _f64(z)
    labels = np.ascontiguousarray(labels, np.int32)
    dz = np.empty_like(z)
    loss = lib().orc_xent_bwd(_p(z), labels.ctypes.data_as(ct.POINTER(ct.c_int32)),
                              ct.c_double(scale), _p(dz), z.shape[0], z.shape[1])
    return loss, dz


def sgd_step(w, g, lr):
    """In place: w <- w - lr*g."""
    lib().orc_sgd_step(_p(w), _p(_f64(g)), ct.c_double(lr), ct.c_size_t(w.size))
