"""ctypes binding of the C oracle (test infrastructure; see ``conv_oracle.c``).

The definitions it evaluates -- forward, backward-data and backward-filter of a
convolutional layer as used by back-propagation through the ConvNet that the
paper trains (its data-parallelism and model-parallelism paragraphs) -- are
written out in the header comment of ``conv_oracle.c``.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "libconv_oracle.so")

_lib = None

_c_dp = ctypes.POINTER(ctypes.c_double)
_c_ip = ctypes.POINTER(ctypes.c_int64)
_c_i32p = ctypes.POINTER(ctypes.c_int32)


def build(force=False):
    """Compile ``conv_oracle.c`` into ``libconv_oracle.so`` next to it."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-std=c99", "-Wall", "-Wextra", "-shared",
           "-fPIC", "-o", _LIB, _SRC]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        dims = [ctypes.c_int] * 9
        for name in ("oracle_conv_fwd", "oracle_conv_bwd_data", "oracle_conv_bwd_filter"):
            f = getattr(_lib, name)
            f.argtypes = [_c_dp, _c_dp, _c_dp] + dims
            f.restype = None
        for name in ("oracle_conv_fwd_at", "oracle_conv_bwd_data_at",
                     "oracle_conv_bwd_filter_at"):
            f = getattr(_lib, name)
            f.argtypes = [_c_dp, _c_dp] + dims + [_c_ip, ctypes.c_int64, _c_dp]
            f.restype = None
        _lib.oracle_relu_fwd.argtypes = [_c_dp, _c_dp, ctypes.c_int64]
        _lib.oracle_relu_bwd.argtypes = [_c_dp, _c_dp, _c_dp, ctypes.c_int64]
        _lib.oracle_maxpool3x3s2_fwd.argtypes = [_c_dp, _c_dp, _c_i32p, ctypes.c_int64,
                                                 ctypes.c_int, ctypes.c_int]
        _lib.oracle_maxpool3x3s2_bwd.argtypes = [_c_dp, _c_dp, _c_dp, ctypes.c_int64,
                                                 ctypes.c_int, ctypes.c_int]
        _lib.oracle_out_extent.argtypes = [ctypes.c_int] * 4
        _lib.oracle_out_extent.restype = ctypes.c_int
        _lib.oracle_pool_extent.argtypes = [ctypes.c_int]
        _lib.oracle_pool_extent.restype = ctypes.c_int
        _lib.oracle_num_threads.restype = ctypes.c_int
        _lib.oracle_round_bf16.argtypes = [ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint16),
                                           ctypes.c_int64]
        _lib.oracle_round_bf16.restype = None
        _lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _p(a):
    return a.ctypes.data_as(_c_dp)


def num_threads():
    return int(_load().oracle_num_threads())


def set_num_threads(t):
    _load().oracle_set_num_threads(int(t))


def out_extent(size, filt, stride, pad):
    return int(_load().oracle_out_extent(size, filt, stride, pad))


def pool_extent(size):
    return int(_load().oracle_pool_extent(size))


def conv_fwd(x, w, stride, pad):
    x, w = _f64(x), _f64(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    P, Q = out_extent(H, R, stride, pad), out_extent(W, S, stride, pad)
    y = np.empty((N, K, P, Q), dtype=np.float64)
    _load().oracle_conv_fwd(_p(x), _p(w), _p(y), N, C, H, W, K, R, S, stride, pad)
    return y


def conv_bwd_data(dy, w, H, W, stride, pad):
    dy, w = _f64(dy), _f64(w)
    N, K, P, Q = dy.shape
    K2, C, R, S = w.shape
    assert K == K2
    assert P == out_extent(H, R, stride, pad) and Q == out_extent(W, S, stride, pad)
    dx = np.empty((N, C, H, W), dtype=np.float64)
    _load().oracle_conv_bwd_data(_p(dy), _p(w), _p(dx), N, C, H, W, K, R, S, stride, pad)
    return dx


def conv_bwd_filter(x, dy, R, S, stride, pad):
    x, dy = _f64(x), _f64(dy)
    N, C, H, W = x.shape
    N2, K, P, Q = dy.shape
    assert N == N2
    assert P == out_extent(H, R, stride, pad) and Q == out_extent(W, S, stride, pad)
    dw = np.empty((K, C, R, S), dtype=np.float64)
    _load().oracle_conv_bwd_filter(_p(x), _p(dy), _p(dw), N, C, H, W, K, R, S, stride, pad)
    return dw


# Grouped (multi-column) layers: the two-column architecture of the paper's
# model-parallelism paragraph splits a layer's filters into `groups` columns, and
# where the columns are not cross-connected the filters of column g read only
# the input channels of column g.  x [N, C, H, W] with C = groups * Cg, w
# [K, Cg, R, S] with K = groups * Kg (filters g*Kg .. (g+1)*Kg-1 form column g):
# every column is an ordinary layer on its channel slice, written out as such.
def _column(t, g, groups, axis):
    size = t.shape[axis] // groups
    sl = [slice(None)] * t.ndim
    sl[axis] = slice(g * size, (g + 1) * size)
    return t[tuple(sl)]


def _check_groups(C, K, Cw, groups):
    assert groups >= 1 and C % groups == 0 and K % groups == 0 and Cw == C // groups


def conv_fwd_grouped(x, w, stride, pad, groups):
    _check_groups(x.shape[1], w.shape[0], w.shape[1], groups)
    return np.concatenate([conv_fwd(_column(x, g, groups, 1), _column(w, g, groups, 0), stride, pad)
                           for g in range(groups)], axis=1)


def conv_bwd_data_grouped(dy, w, H, W, stride, pad, groups):
    _check_groups(w.shape[1] * groups, w.shape[0], w.shape[1], groups)
    assert dy.shape[1] == w.shape[0]
    return np.concatenate([conv_bwd_data(_column(dy, g, groups, 1), _column(w, g, groups, 0), H, W, stride, pad)
                           for g in range(groups)], axis=1)


def conv_bwd_filter_grouped(x, dy, R, S, stride, pad, groups):
    assert x.shape[1] % groups == 0 and dy.shape[1] % groups == 0
    return np.concatenate([conv_bwd_filter(_column(x, g, groups, 1), _column(dy, g, groups, 1), R, S, stride, pad)
                           for g in range(groups)], axis=0)


def _idx(idx):
    return np.ascontiguousarray(np.asarray(idx, dtype=np.int64).ravel())


def conv_fwd_at(x, w, stride, pad, idx):
    """y.ravel()[idx] by the forward definition, one element at a time."""
    x, w, idx = _f64(x), _f64(w), _idx(idx)
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    out = np.empty(idx.shape, dtype=np.float64)
    _load().oracle_conv_fwd_at(_p(x), _p(w), N, C, H, W, K, R, S, stride, pad,
                               idx.ctypes.data_as(_c_ip), idx.size, _p(out))
    return out


def conv_bwd_data_at(dy, w, H, W, stride, pad, idx):
    """dx.ravel()[idx] by the backward-data definition, one element at a time."""
    dy, w, idx = _f64(dy), _f64(w), _idx(idx)
    N, K, _, _ = dy.shape
    _, C, R, S = w.shape
    out = np.empty(idx.shape, dtype=np.float64)
    _load().oracle_conv_bwd_data_at(_p(dy), _p(w), N, C, H, W, K, R, S, stride, pad,
                                    idx.ctypes.data_as(_c_ip), idx.size, _p(out))
    return out


def conv_bwd_filter_at(x, dy, R, S, stride, pad, idx):
    """dw.ravel()[idx] by the backward-filter definition, one element at a time."""
    x, dy, idx = _f64(x), _f64(dy), _idx(idx)
    N, C, H, W = x.shape
    _, K, _, _ = dy.shape
    out = np.empty(idx.shape, dtype=np.float64)
    _load().oracle_conv_bwd_filter_at(_p(x), _p(dy), N, C, H, W, K, R, S, stride, pad,
                                      idx.ctypes.data_as(_c_ip), idx.size, _p(out))
    return out


def relu_fwd(x):
    x = _f64(x)
    y = np.empty_like(x)
    _load().oracle_relu_fwd(_p(x), _p(y), x.size)
    return y


def relu_bwd(x, dy):
    x, dy = _f64(x), _f64(dy)
    dx = np.empty_like(x)
    _load().oracle_relu_bwd(_p(x), _p(dy), _p(dx), x.size)
    return dx


def maxpool3x3s2_fwd(x, return_arg=False):
    x = _f64(x)
    N, C, H, W = x.shape
    PH, PW = pool_extent(H), pool_extent(W)
    y = np.empty((N, C, PH, PW), dtype=np.float64)
    arg = np.empty((N, C, PH, PW), dtype=np.int32)
    _load().oracle_maxpool3x3s2_fwd(_p(x), _p(y), arg.ctypes.data_as(_c_i32p), N * C, H, W)
    return (y, arg) if return_arg else y


def maxpool3x3s2_bwd(x, dy):
    x, dy = _f64(x), _f64(dy)
    N, C, H, W = x.shape
    dx = np.empty_like(x)
    _load().oracle_maxpool3x3s2_bwd(_p(x), _p(dy), _p(dx), N * C, H, W)
    return dx


# Bias of a convolutional layer (one value per filter, the same at every
# output position): forward adds it, its gradient is the sum of the output
# gradient over samples and positions.
def bias_fwd(y, b):
    y, b = _f64(y), _f64(b)
    assert y.ndim == 4 and b.shape == (y.shape[1],)
    out = np.empty_like(y)
    for k in range(y.shape[1]):
        out[:, k] = y[:, k] + b[k]
    return out


def bias_bwd(dy):
    dy = _f64(dy)
    db = np.zeros(dy.shape[1], dtype=np.float64)
    for k in range(dy.shape[1]):
        db[k] = np.sum(dy[:, k])
    return db


# A convolutional layer with the element-wise layers that follow it, as the
# chain of their definitions: bias, then ReLU (forward); the gradient through
# a ReLU, then nothing else (backward-data: the ReLU in question is the one
# that FEEDS the layer, so its mask multiplies the layer's input gradient).
def conv_fwd_bias_relu(x, w, b, stride, pad, relu=True):
    y = conv_fwd(x, w, stride, pad)
    if b is not None:
        y = bias_fwd(y, b)
    return relu_fwd(y) if relu else y


def conv_bwd_data_relu(dy, w, act, stride, pad):
    act = _f64(act)
    H, W = act.shape[2], act.shape[3]
    return relu_bwd(act, conv_bwd_data(dy, w, H, W, stride, pad))


# ---------------------------------------------------------------------------
# Fully connected layers (the top layers of the network; model-parallelism
# paragraph) and the synchronous mini-batch SGD update (training-procedure
# paragraph).  The paper names both without formulas; these are the textbook
# definitions.  x [N, I] (a sample per row), w [O, I] (a neuron per row).
# ---------------------------------------------------------------------------
def fc_fwd(x, w, b=None, relu=False):
    x, w = _f64(x), _f64(w)
    assert x.ndim == 2 and w.ndim == 2 and x.shape[1] == w.shape[1]
    y = np.matmul(x, w.T)                       # y[n, o] = sum_i x[n, i] * w[o, i]
    if b is not None:
        y = y + _f64(b)[None, :]
    return np.where(y > 0, y, 0.0) if relu else y


def fc_bwd_data(dy, w):
    dy, w = _f64(dy), _f64(w)
    assert dy.shape[1] == w.shape[0]
    return np.matmul(dy, w)                     # dx[n, i] = sum_o dy[n, o] * w[o, i]


def fc_bwd_filter(x, dy):
    x, dy = _f64(x), _f64(dy)
    assert x.shape[0] == dy.shape[0]
    return np.matmul(dy.T, x)                   # dw[o, i] = sum_n dy[n, o] * x[n, i]


def sgd_update(w, dw, v, lr, momentum=0.0, weight_decay=0.0, grad_scale=1.0):
    """One step of mini-batch SGD with momentum and L2 weight decay:
        v' = momentum * v - lr * (weight_decay * w + grad_scale * dw),   w' = w + v'
    (grad_scale = 1 / mini-batch size turns a summed gradient into the mean).  Returns (w', v')."""
    w, dw, v = _f64(w), _f64(dw), _f64(v)
    v2 = momentum * v - lr * (weight_decay * w + grad_scale * dw)
    return w + v2, v2


# ---------------------------------------------------------------------------
# bfloat16 storage of the reduced-precision variant: a value is kept as the
# upper 16 bits of its IEEE binary32 pattern, rounded to nearest, ties to even.
# ---------------------------------------------------------------------------
def bf16_bits(a):
    """uint16 bfloat16 patterns of a float32 array, round to nearest even (NaN stays NaN)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).ravel()
    out = np.empty(bits.shape, dtype=np.uint16)
    _load().oracle_round_bf16(bits.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)),
                              out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), bits.size)
    return out.reshape(a.shape)


def bf16_round(a):
    """The float32 array rounded onto the bfloat16 grid, returned as float32 (exactly representable)."""
    b = bf16_bits(a)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)
