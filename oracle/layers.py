"""numpy-facing wrappers around the plain-C oracle (test infrastructure only).

Each function takes and returns C-contiguous float64 arrays in NCHW.  The arithmetic is in
vdnn_oracle.c; this file only marshals arguments.  The product path never imports this.
"""
import ctypes as C

import numpy as np

from .build import build

_lib = C.CDLL(build())
_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int)


def _p(a):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_dp)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


_lib.oracle_out_dim.restype = C.c_int
_lib.oracle_softmax_ce.restype = C.c_double
_lib.oracle_relu_fwd.argtypes = [_dp, C.c_size_t]
_lib.oracle_relu_bwd.argtypes = [_dp, _dp, C.c_size_t]
_conv_args = [_dp, _dp, _dp] + [C.c_int] * 9
_lib.oracle_conv_fwd.argtypes = _conv_args
_lib.oracle_conv_bwd_data.argtypes = _conv_args
_lib.oracle_conv_bwd_filter.argtypes = _conv_args
_lib.oracle_maxpool_fwd.argtypes = [_dp, _dp] + [C.c_int] * 7
_lib.oracle_avgpool_fwd.argtypes = [_dp, _dp] + [C.c_int] * 7
_lib.oracle_maxpool_bwd.argtypes = [_dp, _dp, _dp] + [C.c_int] * 7
_lib.oracle_avgpool_bwd.argtypes = [_dp, _dp] + [C.c_int] * 7
_lib.oracle_fc_fwd.argtypes = [_dp, _dp, _dp] + [C.c_int] * 3
_lib.oracle_fc_bwd_data.argtypes = [_dp, _dp, _dp] + [C.c_int] * 3
_lib.oracle_fc_bwd_filter.argtypes = [_dp, _dp, _dp] + [C.c_int] * 3
_lib.oracle_softmax_ce.argtypes = [_dp, _ip, _dp, C.c_int, C.c_int]


def out_dim(size, k, stride, pad):
    return int(_lib.oracle_out_dim(size, k, stride, pad))


def conv_fwd(x, w, stride=1, pad=0):
    x, w = _f64(x), _f64(w)
    n, c, h, wd = x.shape
    k, c2, r, s = w.shape
    assert c == c2
    y = np.empty((n, k, out_dim(h, r, stride, pad), out_dim(wd, s, stride, pad)), np.float64)
    _lib.oracle_conv_fwd(_p(x), _p(w), _p(y), n, c, h, wd, k, r, s, stride, pad)
    return y


def conv_bwd_data(dy, w, x_shape, stride=1, pad=0):
    dy, w = _f64(dy), _f64(w)
    n, c, h, wd = x_shape
    k, c2, r, s = w.shape
    assert c == c2 and dy.shape == (n, k, out_dim(h, r, stride, pad), out_dim(wd, s, stride, pad))
    dx = np.empty(x_shape, np.float64)
    _lib.oracle_conv_bwd_data(_p(dy), _p(w), _p(dx), n, c, h, wd, k, r, s, stride, pad)
    return dx


def conv_bwd_filter(x, dy, w_shape, stride=1, pad=0):
    x, dy = _f64(x), _f64(dy)
    n, c, h, wd = x.shape
    k, c2, r, s = w_shape
    assert c == c2 and dy.shape == (n, k, out_dim(h, r, stride, pad), out_dim(wd, s, stride, pad))
    dw = np.empty(w_shape, np.float64)
    _lib.oracle_conv_bwd_filter(_p(x), _p(dy), _p(dw), n, c, h, wd, k, r, s, stride, pad)
    return dw


def relu_fwd(x):
    y = _f64(x).copy()
    _lib.oracle_relu_fwd(_p(y), y.size)
    return y


def relu_bwd(y, dy):
    y = _f64(y)
    dx = _f64(dy).copy()
    _lib.oracle_relu_bwd(_p(y), _p(dx), dx.size)
    return dx


def _pool_shape(x, k, stride, pad):
    n, c, h, w = x.shape
    return (n, c, out_dim(h, k, stride, pad), out_dim(w, k, stride, pad))


def maxpool_fwd(x, k, stride, pad=0):
    x = _f64(x)
    y = np.empty(_pool_shape(x, k, stride, pad), np.float64)
    _lib.oracle_maxpool_fwd(_p(x), _p(y), *x.shape, k, stride, pad)
    return y


def maxpool_bwd(x, dy, k, stride, pad=0):
    x, dy = _f64(x), _f64(dy)
    assert dy.shape == _pool_shape(x, k, stride, pad)
    dx = np.empty(x.shape, np.float64)
    _lib.oracle_maxpool_bwd(_p(x), _p(dy), _p(dx), *x.shape, k, stride, pad)
    return dx


def avgpool_fwd(x, k, stride, pad=0):
    x = _f64(x)
    y = np.empty(_pool_shape(x, k, stride, pad), np.float64)
    _lib.oracle_avgpool_fwd(_p(x), _p(y), *x.shape, k, stride, pad)
    return y


def avgpool_bwd(dy, x_shape, k, stride, pad=0):
    dy = _f64(dy)
    dx = np.empty(x_shape, np.float64)
    _lib.oracle_avgpool_bwd(_p(dy), _p(dx), *x_shape, k, stride, pad)
    return dx


def fc_fwd(x, w):
    x, w = _f64(x), _f64(w)
    n = x.shape[0]
    x2 = x.reshape(n, -1)
    o, i = w.shape
    assert x2.shape[1] == i
    y = np.empty((n, o), np.float64)
    _lib.oracle_fc_fwd(_p(x2), _p(w), _p(y), n, i, o)
    return y


def fc_bwd_data(dy, w, x_shape):
    dy, w = _f64(dy), _f64(w)
    n, o = dy.shape
    i = w.shape[1]
    dx = np.empty((n, i), np.float64)
    _lib.oracle_fc_bwd_data(_p(dy), _p(w), _p(dx), n, i, o)
    return dx.reshape(x_shape)


def fc_bwd_filter(x, dy):
    x, dy = _f64(x), _f64(dy)
    n, o = dy.shape
    x2 = np.ascontiguousarray(x.reshape(n, -1))
    i = x2.shape[1]
    dw = np.empty((o, i), np.float64)
    _lib.oracle_fc_bwd_filter(_p(x2), _p(dy), _p(dw), n, i, o)
    return dw


def softmax_ce(z, labels):
    """Returns (loss, dz)."""
    z = _f64(z)
    n, classes = z.shape
    lab = np.ascontiguousarray(labels, dtype=np.int32)
    assert lab.shape == (n,) and lab.min() >= 0 and lab.max() < classes
    dz = np.empty_like(z)
    loss = _lib.oracle_softmax_ce(_p(z), lab.ctypes.data_as(_ip), _p(dz), n, classes)
    return float(loss), dz
