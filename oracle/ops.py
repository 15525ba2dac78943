"""numpy-facing wrappers of the oracle's C operators (ops.c) plus the output
shape of each primitive operator.

TEST INFRASTRUCTURE ONLY (parity anchor of the GPU library); imported by the
tests, the smoke check and the benchmark's cpu_baseline leg, never by the
product path.  Each function is the plain definition of one operator of the
evaluated workloads (paper Sec. 5.1: transformer layers are batch matmul,
layer norm, softmax; vision models are convolutions and activations), fp32 in
and out with double accumulation inside.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import build

_lib = C.CDLL(build())
_f = C.POINTER(C.c_float)
_i = C.POINTER(C.c_int32)


def _p(a):
    return a.ctypes.data_as(_f)


def _sig(name, argtypes, restype=None):
    fn = getattr(_lib, name)
    fn.argtypes = argtypes
    fn.restype = restype
    return fn


_conv2d = _sig("orc_conv2d", [_f, _f, _f] + [C.c_int] * 12)
_conv3d = _sig("orc_conv3d", [_f, _f, _f] + [C.c_int] * 15)
_maxpool3d = _sig("orc_max_pool3d", [_f, _f] + [C.c_int] * 13)
_convt = _sig("orc_conv2d_transpose", [_f, _f, _f] + [C.c_int] * 11)
_dense = _sig("orc_dense", [_f, _f, _f] + [C.c_int] * 3)
_bmm = _sig("orc_batch_matmul", [_f, _f, _f] + [C.c_int] * 5)
_bias = _sig("orc_bias_add", [_f, _f, _f] + [C.c_int64] * 3)
_add = _sig("orc_add", [_f, _f, _f, C.c_int64])
_mul = _sig("orc_mul_scalar", [_f, C.c_double, _f, C.c_int64])
_relu = _sig("orc_relu", [_f, _f, C.c_int64])
_gelu = _sig("orc_gelu", [_f, _f, C.c_int64])
_tanh = _sig("orc_tanh", [_f, _f, C.c_int64])
_softmax = _sig("orc_softmax", [_f, _f, C.c_int64, C.c_int64])
_ln = _sig("orc_layer_norm", [_f, _f, _f, _f, C.c_int64, C.c_int64, C.c_double])
_maxpool = _sig("orc_max_pool2d", [_f, _f] + [C.c_int] * 10)
_avgpool = _sig("orc_avg_pool2d", [_f, _f] + [C.c_int] * 10)
_gap = _sig("orc_global_avg_pool2d", [_f, _f, C.c_int, C.c_int])
_take = _sig("orc_take", [_f, _i, _f, C.c_int64, C.c_int64, C.c_int64], C.c_int)
_set_threads = _sig("orc_set_threads", [C.c_int])
_max_threads = _sig("orc_max_threads", [], C.c_int)


def set_threads(n: int) -> None:
    _set_threads(int(n))


def max_threads() -> int:
    return int(_max_threads())


def _f32(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float32, a.dtype
    return a


def _pair(v):
    return (int(v[0]), int(v[1])) if np.ndim(v) else (int(v), int(v))


# ---- output shapes -----------------------------------------------------------
def conv2d_shape(xs, ws, stride, pad, groups):
    n, c, h, w = xs
    o, cg, kh, kw = ws
    (sh, sw), (ph, pw) = _pair(stride), _pair(pad)
    if c % groups or o % groups or cg != c // groups:
        raise ValueError(f"conv2d: channels {xs} {ws} groups {groups}")
    ho, wo = (h + 2 * ph - kh) // sh + 1, (w + 2 * pw - kw) // sw + 1
    if ho <= 0 or wo <= 0:
        raise ValueError("conv2d: empty output")
    return (n, o, ho, wo)


def conv2d_transpose_shape(xs, ws, stride, pad):
    n, c, h, w = xs
    ci, o, kh, kw = ws
    (sh, sw), (ph, pw) = _pair(stride), _pair(pad)
    if ci != c:
        raise ValueError("conv2d_transpose: channels")
    return (n, o, (h - 1) * sh - 2 * ph + kh, (w - 1) * sw - 2 * pw + kw)


# ---- operators -----------------------------------------------------------------
def conv2d(x, w, stride=(1, 1), pad=(0, 0), groups=1):
    x, w = _f32(x), _f32(w)
    shp = conv2d_shape(x.shape, w.shape, stride, pad, groups)
    (sh, sw), (ph, pw) = _pair(stride), _pair(pad)
    y = np.empty(shp, np.float32)
    n, c, h, wd = x.shape
    _conv2d(_p(x), _p(w), _p(y), n, c, h, wd, w.shape[0], w.shape[2],
            w.shape[3], sh, sw, ph, pw, int(groups))
    return y


def _triple(v):
    return (int(v[0]), int(v[1]), int(v[2]))


def conv3d(x, w, stride=(1, 1, 1), pad=(0, 0, 0)):
    x, w = _f32(x), _f32(w)
    n, c, d, h, wd = x.shape
    o, ci, kd, kh, kw = w.shape
    if ci != c:
        raise ValueError("conv3d: channels")
    (sd, sh, sw), (pd, ph, pw) = _triple(stride), _triple(pad)
    do, ho, wo = (d + 2 * pd - kd) // sd + 1, (h + 2 * ph - kh) // sh + 1, (wd + 2 * pw - kw) // sw + 1
    if min(do, ho, wo) <= 0:
        raise ValueError("conv3d: empty output")
    y = np.empty((n, o, do, ho, wo), np.float32)
    _conv3d(_p(x), _p(w), _p(y), n, c, d, h, wd, o, kd, kh, kw, sd, sh, sw, pd, ph, pw)
    return y


def max_pool3d(x, kernel=(3, 3, 3), stride=(2, 2, 2), pad=(1, 1, 1)):
    x = _f32(x)
    n, c, d, h, w = x.shape
    (kd, kh, kw), (sd, sh, sw), (pd, ph, pw) = _triple(kernel), _triple(stride), _triple(pad)
    do, ho, wo = (d + 2 * pd - kd) // sd + 1, (h + 2 * ph - kh) // sh + 1, (w + 2 * pw - kw) // sw + 1
    y = np.empty((n, c, do, ho, wo), np.float32)
    _maxpool3d(_p(x), _p(y), n * c, d, h, w, kd, kh, kw, sd, sh, sw, pd, ph, pw)
    return y


def global_avg_pool3d(x):
    """Mean over D, H and W; output [N, C]."""
    x = _f32(x)
    n, c, d, h, w = x.shape
    y = np.empty((n, c), np.float32)
    _gap(_p(x), _p(y), n * c, d * h * w)
    return y


def conv2d_transpose(x, w, stride=(2, 2), pad=(1, 1)):
    x, w = _f32(x), _f32(w)
    shp = conv2d_transpose_shape(x.shape, w.shape, stride, pad)
    (sh, sw), (ph, pw) = _pair(stride), _pair(pad)
    y = np.empty(shp, np.float32)
    n, c, h, wd = x.shape
    _convt(_p(x), _p(w), _p(y), n, c, h, wd, w.shape[1], w.shape[2],
           w.shape[3], sh, sw, ph, pw)
    return y


def dense(x, w):
    x, w = _f32(x), _f32(w)
    if x.ndim != 2 or w.ndim != 2 or x.shape[1] != w.shape[1]:
        raise ValueError(f"dense: {x.shape} {w.shape}")
    y = np.empty((x.shape[0], w.shape[0]), np.float32)
    _dense(_p(x), _p(w), _p(y), x.shape[0], x.shape[1], w.shape[0])
    return y


def batch_matmul(a, b, transpose_b=True):
    a, b = _f32(a), _f32(b)
    if a.ndim != 3 or b.ndim != 3 or a.shape[0] != b.shape[0]:
        raise ValueError(f"batch_matmul: {a.shape} {b.shape}")
    bt, m, k = a.shape
    if transpose_b:
        n, kb = b.shape[1], b.shape[2]
    else:
        kb, n = b.shape[1], b.shape[2]
    if kb != k:
        raise ValueError(f"batch_matmul: {a.shape} {b.shape}")
    y = np.empty((bt, m, n), np.float32)
    _bmm(_p(a), _p(b), _p(y), bt, m, n, k, 1 if transpose_b else 0)
    return y


def bias_add(x, b, axis=1):
    x, b = _f32(x), _f32(b)
    ax = axis if axis >= 0 else x.ndim + axis
    if b.ndim != 1 or not (0 <= ax < x.ndim) or x.shape[ax] != b.shape[0]:
        raise ValueError(f"bias_add: {x.shape} {b.shape} axis {axis}")
    outer = int(np.prod(x.shape[:ax], dtype=np.int64))
    inner = int(np.prod(x.shape[ax + 1:], dtype=np.int64))
    y = np.empty_like(x)
    _bias(_p(x), _p(b), _p(y), outer, x.shape[ax], inner)
    return y


def add(x, z):
    x, z = _f32(x), _f32(z)
    if x.shape != z.shape:
        raise ValueError(f"add: {x.shape} {z.shape}")
    y = np.empty_like(x)
    _add(_p(x), _p(z), _p(y), x.size)
    return y


def mul_scalar(x, scalar):
    x = _f32(x)
    y = np.empty_like(x)
    _mul(_p(x), float(scalar), _p(y), x.size)
    return y


def _unary(fn):
    def f(x):
        x = _f32(x)
        y = np.empty_like(x)
        fn(_p(x), _p(y), x.size)
        return y
    return f


relu = _unary(_relu)
gelu = _unary(_gelu)
tanh = _unary(_tanh)


def softmax(x):
    x = _f32(x)
    y = np.empty_like(x)
    _softmax(_p(x), _p(y), x.size // x.shape[-1], x.shape[-1])
    return y


def layer_norm(x, gamma, beta, eps=1e-12):
    x, gamma, beta = _f32(x), _f32(gamma), _f32(beta)
    L = x.shape[-1]
    if gamma.shape != (L,) or beta.shape != (L,):
        raise ValueError("layer_norm: gamma/beta")
    y = np.empty_like(x)
    _ln(_p(x), _p(gamma), _p(beta), _p(y), x.size // L, L, float(eps))
    return y


def max_pool2d(x, kernel=(3, 3), stride=(2, 2), pad=(1, 1)):
    x = _f32(x)
    (kh, kw), (sh, sw), (ph, pw) = _pair(kernel), _pair(stride), _pair(pad)
    n, c, h, w = x.shape
    ho, wo = (h + 2 * ph - kh) // sh + 1, (w + 2 * pw - kw) // sw + 1
    y = np.empty((n, c, ho, wo), np.float32)
    _maxpool(_p(x), _p(y), n, c, h, w, kh, kw, sh, sw, ph, pw)
    return y


def avg_pool2d(x, kernel=(3, 3), stride=(1, 1), pad=(1, 1)):
    """Mean over the window's pixels inside the image (padding not counted)."""
    x = _f32(x)
    (kh, kw), (sh, sw), (ph, pw) = _pair(kernel), _pair(stride), _pair(pad)
    n, c, h, w = x.shape
    ho, wo = (h + 2 * ph - kh) // sh + 1, (w + 2 * pw - kw) // sw + 1
    y = np.empty((n, c, ho, wo), np.float32)
    _avgpool(_p(x), _p(y), n, c, h, w, kh, kw, sh, sw, ph, pw)
    return y


def concat(xs, axis=1):
    """Tensors joined along `axis`; every other extent equal."""
    xs = [_f32(x) for x in xs]
    nd = xs[0].ndim
    ax = axis + nd if axis < 0 else axis
    for x in xs:
        if x.ndim != nd or any(x.shape[d] != xs[0].shape[d] for d in range(nd) if d != ax):
            raise ValueError("concat: shapes differ outside the axis")
    outer = int(np.prod(xs[0].shape[:ax], dtype=np.int64))
    shape = list(xs[0].shape)
    shape[ax] = sum(x.shape[ax] for x in xs)
    y = np.empty(shape, np.float32)
    yf = y.reshape(outer, -1)
    at = 0
    for x in xs:                      # plain copies, block by block
        xf = x.reshape(outer, -1)
        yf[:, at:at + xf.shape[1]] = xf
        at += xf.shape[1]
    return y


def global_avg_pool2d(x):
    x = _f32(x)
    n, c, h, w = x.shape
    y = np.empty((n, c), np.float32)
    _gap(_p(x), _p(y), n * c, h * w)
    return y


def take(table, ids):
    table = _f32(table)
    ids = np.ascontiguousarray(ids)
    assert ids.dtype == np.int32 and ids.ndim == 1 and table.ndim == 2
    y = np.empty((ids.shape[0], table.shape[1]), np.float32)
    rc = _take(_p(table), ids.ctypes.data_as(_i), _p(y), ids.shape[0],
               table.shape[1], table.shape[0])
    if rc != 0:
        raise IndexError("take: id out of range")
    return y


def reshape(x, dims):
    return np.ascontiguousarray(np.reshape(x, tuple(int(d) for d in dims)))


def transpose(x, dims):
    return np.ascontiguousarray(np.transpose(x, tuple(int(d) for d in dims)))
