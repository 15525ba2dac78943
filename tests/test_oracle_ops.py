"""Pins of the oracle's operators against what mathematics and independent
library routines fix (CPU only).  The paper prints no worked numeric example
(its DP walk-through is a figure), so the pins are closed forms, invariants,
brute force in a different formulation, and PyTorch-CPU float64 routines.
"""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ops

RNG = np.random.default_rng(1234)
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rnd(*shape):
    return RNG.standard_normal(shape).astype(np.float32)


def t64(a):
    return torch.from_numpy(np.asarray(a, np.float64))


def close(got, ref64, rtol=2e-6):
    """got is fp32 rounded once from a double sum; ref64 is an fp64 library
    result: they agree to fp32 rounding of the result's own magnitude."""
    ref64 = np.asarray(ref64, np.float64)
    scale = np.maximum(np.abs(ref64), 1e-30)
    tol = rtol * np.maximum(scale, float(np.max(np.abs(ref64))) * 1e-3)
    assert got.dtype == np.float32
    assert got.shape == ref64.shape
    assert np.all(np.abs(got.astype(np.float64) - ref64) <= tol)


# ---------------------------------------------------------------- conv2d
CONV_CASES = [
    # N, C, H, W, O, k, stride, pad, groups
    (1, 3, 9, 9, 4, 3, 1, 1, 1),
    (2, 4, 8, 7, 6, 3, 2, 1, 2),
    (1, 8, 6, 6, 8, 1, 1, 0, 1),
    (1, 8, 7, 7, 8, 1, 2, 0, 1),
    (1, 3, 15, 15, 5, 7, 2, 3, 1),
    (1, 8, 6, 6, 16, 3, 1, 1, 4),
    (1, 6, 5, 5, 6, 3, 2, 1, 6),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv2d_vs_torch_float64(case):
    n, c, h, w, o, k, s, p, g = case
    x, wt = rnd(n, c, h, w), rnd(o, c // g, k, k)
    y = ops.conv2d(x, wt, (s, s), (p, p), g)
    ref = F.conv2d(t64(x), t64(wt), stride=s, padding=p, groups=g).numpy()
    close(y, ref)


def _conv_brute_padded(x, w, s, p, g):
    """Different formulation from the oracle's: pad the input physically and
    take window * kernel sums with numpy; python loops over outputs."""
    n, c, h, wd = x.shape
    o, cg, kh, kw = w.shape
    xp = np.zeros((n, c, h + 2 * p, wd + 2 * p), np.float64)
    xp[:, :, p:p + h, p:p + wd] = x
    ho, wo = (h + 2 * p - kh) // s + 1, (wd + 2 * p - kw) // s + 1
    y = np.zeros((n, o, ho, wo), np.float64)
    og = o // g
    for b in range(n):
        for co in range(o):
            grp = co // og
            for i in range(ho):
                for j in range(wo):
                    win = xp[b, grp * cg:(grp + 1) * cg, i * s:i * s + kh, j * s:j * s + kw]
                    y[b, co, i, j] = np.sum(win * w[co].astype(np.float64))
    return y


@pytest.mark.parametrize("case", [(1, 2, 5, 4, 3, 3, 1, 1, 1), (1, 4, 5, 5, 4, 3, 2, 1, 2),
                                  (2, 2, 4, 4, 2, 2, 2, 0, 1)])
def test_conv2d_vs_brute_force_tiny(case):
    n, c, h, w, o, k, s, p, g = case
    x, wt = rnd(n, c, h, w), rnd(o, c // g, k, k)
    close(ops.conv2d(x, wt, (s, s), (p, p), g), _conv_brute_padded(x, wt, s, p, g))


def test_conv2d_all_ones_closed_form():
    cin = 5
    x = np.ones((1, cin, 6, 7), np.float32)
    w = np.ones((2, cin, 3, 3), np.float32)
    y = ops.conv2d(x, w, (1, 1), (1, 1), 1)
    assert y.shape == (1, 2, 6, 7)
    assert np.all(y[:, :, 1:-1, 1:-1] == 9 * cin)
    assert np.all(y[:, :, 0, 1:-1] == 6 * cin) and np.all(y[:, :, 1:-1, 0] == 6 * cin)
    for i, j in ((0, 0), (0, -1), (-1, 0), (-1, -1)):
        assert np.all(y[:, :, i, j] == 4 * cin)


def test_conv2d_delta_kernel_is_a_shift_not_a_flip():
    # cross-correlation: w[.,.,kh,kw] = 1 picks x[oh-p+kh, ow-p+kw]
    x = rnd(1, 1, 6, 6)
    w = np.zeros((1, 1, 3, 3), np.float32)
    w[0, 0, 0, 2] = 1.0          # kh=0, kw=2 -> x[oh-1, ow+1]
    y = ops.conv2d(x, w, (1, 1), (1, 1), 1)
    assert np.array_equal(y[0, 0, 1:, :-1], x[0, 0, :-1, 1:])
    assert np.all(y[0, 0, 0, :] == 0) and np.all(y[0, 0, :, -1] == 0)


def test_conv2d_depthwise_1x1_is_channel_scale():
    x = rnd(1, 6, 4, 4)
    s = rnd(6, 1, 1, 1)
    y = ops.conv2d(x, s, (1, 1), (0, 0), 6)
    assert np.array_equal(y, x * s.reshape(1, 6, 1, 1))


def test_conv2d_rejects_bad_channels():
    with pytest.raises(ValueError):
        ops.conv2d(rnd(1, 3, 4, 4), rnd(2, 4, 1, 1))


# ------------------------------------------------------- conv2d_transpose
@pytest.mark.parametrize("case", [(1, 4, 4, 4, 3, 4, 2, 1), (2, 3, 5, 3, 2, 4, 2, 1),
                                  (1, 2, 3, 3, 2, 3, 1, 1), (1, 2, 3, 4, 3, 2, 2, 0)])
def test_conv2d_transpose_vs_torch_float64(case):
    n, c, h, w, o, k, s, p = case
    x, wt = rnd(n, c, h, w), rnd(c, o, k, k)
    y = ops.conv2d_transpose(x, wt, (s, s), (p, p))
    ref = F.conv_transpose2d(t64(x), t64(wt), stride=s, padding=p).numpy()
    close(y, ref)


def test_conv2d_transpose_is_adjoint_of_conv2d():
    # <conv(a, w), b> == <a, convT(b, w)> with w read as OIHW by conv (O = channels of b)
    # and as IOHW by convT (I = channels of b)
    a, wt = rnd(1, 3, 8, 8), rnd(5, 3, 4, 4)
    ca = ops.conv2d(a, wt, (2, 2), (1, 1), 1)           # [1,5,4,4]
    b = rnd(*ca.shape)
    tb = ops.conv2d_transpose(b, wt, (2, 2), (1, 1))    # [1,3,8,8]
    assert tb.shape == a.shape
    lhs = float(np.sum(ca.astype(np.float64) * b))
    rhs = float(np.sum(a.astype(np.float64) * tb))
    assert abs(lhs - rhs) <= 1e-5 * max(1.0, abs(lhs))


def test_conv2d_transpose_equals_zero_stuffed_flipped_conv():
    x, wt = rnd(1, 3, 4, 4), rnd(3, 2, 4, 4)
    s, p, k = 2, 1, 4
    y = ops.conv2d_transpose(x, wt, (s, s), (p, p))
    z = np.zeros((1, 3, (4 - 1) * s + 1, (4 - 1) * s + 1), np.float32)
    z[:, :, ::s, ::s] = x
    wf = np.ascontiguousarray(np.flip(wt, (2, 3)).transpose(1, 0, 2, 3))
    ref = ops.conv2d(z, wf, (1, 1), (k - 1 - p, k - 1 - p), 1)
    close(y, ref.astype(np.float64))


def test_dcgan_upsampling_shape():
    assert ops.conv2d_transpose(rnd(1, 2, 4, 4), rnd(2, 1, 4, 4), (2, 2), (1, 1)).shape == (1, 1, 8, 8)


# ------------------------------------------------------------ dense / bmm
def test_dense_vs_float64_matmul_and_identity():
    x, w = rnd(5, 17), rnd(9, 17)
    close(ops.dense(x, w), x.astype(np.float64) @ w.astype(np.float64).T)
    assert np.array_equal(ops.dense(x, np.eye(17, dtype=np.float32)), x)
    # a non-square selector pins the [units, in] orientation of the weight
    sel = np.zeros((2, 17), np.float32)
    sel[0, 3] = 1
    sel[1, 11] = 1
    assert np.array_equal(ops.dense(x, sel), x[:, [3, 11]])


@pytest.mark.parametrize("tb", [True, False])
def test_batch_matmul_vs_float64(tb):
    a = rnd(3, 4, 6)
    b = rnd(3, 5, 6) if tb else rnd(3, 6, 5)
    ref = np.einsum("bmk,bnk->bmn" if tb else "bmk,bkn->bmn",
                    a.astype(np.float64), b.astype(np.float64))
    close(ops.batch_matmul(a, b, tb), ref)


def test_double_accumulation_survives_cancellation():
    # 2^24 + 1 - 2^24 is 1 in double, 0 if the sum were carried in float
    x = np.array([[16777216.0, 1.0, -16777216.0]], np.float32)
    w = np.ones((1, 3), np.float32)
    assert ops.dense(x, w)[0, 0] == 1.0


# ---------------------------------------------------------- elementwise
def test_bias_add_axes():
    x, b = rnd(2, 3, 4, 5), rnd(3)
    assert np.array_equal(ops.bias_add(x, b, 1), x + b.reshape(1, 3, 1, 1))
    x2, b2 = rnd(4, 7), rnd(7)
    assert np.array_equal(ops.bias_add(x2, b2, -1), x2 + b2)
    with pytest.raises(ValueError):
        ops.bias_add(x, rnd(4), 1)


def test_add_mul_relu():
    x, z = rnd(3, 5), rnd(3, 5)
    assert np.array_equal(ops.add(x, z), x + z)
    assert np.array_equal(ops.mul_scalar(x, 0.125), x * np.float32(0.125))
    assert np.array_equal(ops.relu(x), np.maximum(x, 0))
    with pytest.raises(ValueError):
        ops.add(x, rnd(5, 3))


def test_gelu_table_symmetry_and_library():
    rows = [l.split() for l in open(os.path.join(GOLD, "normal_cdf.txt"))
            if l.strip() and not l.startswith("#")]
    xs = np.array([float(r[0]) for r in rows], np.float32)
    phi = np.array([float(r[1]) for r in rows])
    assert np.allclose(ops.gelu(xs), xs * phi, rtol=0, atol=2e-7)
    v = rnd(1000) * 3
    # x*Phi(x) - (-x)*Phi(-x) = x
    assert np.allclose(ops.gelu(v) - ops.gelu(-v), v, atol=1e-6)
    close(ops.gelu(v), F.gelu(t64(v)).numpy())
    assert ops.gelu(np.zeros(1, np.float32))[0] == 0.0


def test_tanh_values_and_oddness():
    v = rnd(1000) * 2
    assert np.array_equal(ops.tanh(-v), -ops.tanh(v))
    ref = np.array([math.tanh(float(t)) for t in v])
    close(ops.tanh(v), ref)
    assert abs(float(ops.tanh(np.array([0.5], np.float32))[0]) - 0.46211715726) < 1e-7


# --------------------------------------------------------- softmax / LN
def test_softmax_invariants_and_library():
    x = rnd(7, 33) * 4
    y = ops.softmax(x)
    assert np.allclose(y.sum(-1, dtype=np.float64), 1.0, atol=1e-6)
    assert np.all(y > 0)
    assert np.allclose(ops.softmax(x + np.float32(3.0)), y, rtol=1e-5, atol=1e-9)
    assert np.allclose(ops.softmax(np.full((2, 8), 5.0, np.float32)), 1 / 8)
    close(y, F.softmax(t64(x), -1).numpy())
    big = np.array([[1000.0, 999.0]], np.float32)   # max-subtraction keeps it finite
    assert np.allclose(ops.softmax(big), [[1 / (1 + math.exp(-1)), 1 / (1 + math.e)]], atol=1e-7)
    # 3-d input normalises the last axis only
    x3 = rnd(2, 3, 5)
    close(ops.softmax(x3), F.softmax(t64(x3), -1).numpy())


def test_layer_norm_invariants_and_library():
    x, g, b = rnd(6, 48) * 3 + 1, rnd(48), rnd(48)
    ones, zeros = np.ones(48, np.float32), np.zeros(48, np.float32)
    y = ops.layer_norm(x, ones, zeros, 1e-12).astype(np.float64)
    assert np.allclose(y.mean(-1), 0, atol=1e-6)
    assert np.allclose((y ** 2).mean(-1), 1, atol=1e-5)       # biased variance
    const = np.full((2, 48), 2.5, np.float32)
    assert np.allclose(ops.layer_norm(const, g, b, 1e-5), b, atol=1e-6)
    ref = F.layer_norm(t64(x), (48,), t64(g), t64(b), 1e-12).numpy()
    close(ops.layer_norm(x, g, b, 1e-12), ref, rtol=1e-5)
    ref = F.layer_norm(t64(x), (48,), t64(g), t64(b), 0.1).numpy()   # eps is inside the sqrt
    close(ops.layer_norm(x, g, b, 0.1), ref, rtol=1e-5)


# ------------------------------------------------------------- pools, take
def test_max_pool_vs_torch_and_padding_is_minus_inf():
    x = rnd(2, 3, 9, 8)
    y = ops.max_pool2d(x, (3, 3), (2, 2), (1, 1))
    ref = F.max_pool2d(torch.from_numpy(x), 3, 2, 1).numpy()
    assert np.array_equal(y, ref)
    neg = -np.abs(rnd(1, 1, 4, 4)) - 1
    assert np.all(ops.max_pool2d(neg, (3, 3), (2, 2), (1, 1)) < 0)


@pytest.mark.parametrize("k,s,p", [(3, 1, 1), (3, 2, 1), (2, 2, 0), (5, 1, 2), (1, 2, 0)])
def test_avg_pool_vs_torch_padding_not_counted(k, s, p):
    x = rnd(2, 3, 9, 8)
    y = ops.avg_pool2d(x, (k, k), (s, s), (p, p))
    ref = F.avg_pool2d(t64(x), k, s, p, count_include_pad=False).numpy()
    close(y, ref, rtol=1e-6)
    # a constant image stays constant up to the border (it would not if padding were counted)
    assert np.all(ops.avg_pool2d(np.full((1, 2, 6, 7), 2.5, np.float32), (k, k), (s, s), (p, p)) == 2.5)


def test_avg_pool_corner_divisor_by_hand():
    # 3x3 window, pad 1, on a 3x3 ramp 0..8: the corner window holds 0 1 3 4 (mean 2),
    # the top edge window 0 1 2 3 4 5 (mean 2.5), the centre all nine (mean 4)
    x = np.arange(9, dtype=np.float32).reshape(1, 1, 3, 3)
    y = ops.avg_pool2d(x, (3, 3), (1, 1), (1, 1))
    assert y[0, 0, 0, 0] == 2.0 and y[0, 0, 0, 1] == 2.5 and y[0, 0, 1, 1] == 4.0 and y[0, 0, 2, 2] == 6.0


def test_concat_vs_torch_and_by_hand():
    a, b, c = rnd(2, 3, 4, 5), rnd(2, 1, 4, 5), rnd(2, 6, 4, 5)
    assert np.array_equal(ops.concat([a, b, c], 1), torch.cat([torch.from_numpy(t) for t in (a, b, c)], 1).numpy())
    u, v = rnd(3, 4), rnd(3, 2)
    assert np.array_equal(ops.concat([u, v], -1), np.concatenate([u, v], 1))
    y = ops.concat([np.zeros((1, 1, 2, 2), np.float32), np.ones((1, 2, 2, 2), np.float32)], 1)
    assert y.shape == (1, 3, 2, 2) and y[0, 0].sum() == 0 and y[0, 1:].sum() == 8
    with pytest.raises(ValueError):
        ops.concat([a, rnd(2, 3, 4, 6)], 1)


@pytest.mark.parametrize("k,s,p", [((3, 3, 3), (1, 1, 1), (1, 1, 1)), ((3, 3, 3), (2, 2, 2), (1, 1, 1)),
                                   ((7, 7, 7), (1, 2, 2), (3, 3, 3)), ((1, 1, 1), (2, 2, 2), (0, 0, 0)),
                                   ((3, 1, 2), (1, 2, 1), (0, 0, 1))])
def test_conv3d_vs_torch(k, s, p):
    x, w = rnd(2, 3, 6, 9, 8), rnd(5, 3, *k)
    ref = F.conv3d(t64(x), t64(w), stride=s, padding=p).numpy()
    close(ops.conv3d(x, w, s, p), ref, rtol=1e-5)


def test_conv3d_closed_forms():
    # all-ones kernel on an all-ones volume counts the taps inside: 27 in the middle, 8 in a corner
    y = ops.conv3d(np.ones((1, 2, 4, 4, 4), np.float32), np.ones((1, 2, 3, 3, 3), np.float32), (1, 1, 1), (1, 1, 1))
    assert y[0, 0, 1, 1, 1] == 54 and y[0, 0, 0, 0, 0] == 16 and y[0, 0, 0, 1, 1] == 36
    # a delta at tap (kd, kh, kw) = (2, 0, 1) reads x at (d + 1, h - 1, w): the three axes are not interchangeable
    x = rnd(1, 1, 5, 5, 5)
    w = np.zeros((1, 1, 3, 3, 3), np.float32)
    w[0, 0, 2, 0, 1] = 1
    y = ops.conv3d(x, w, (1, 1, 1), (1, 1, 1))
    assert np.array_equal(y[0, 0, 1:4, 1:5, :], x[0, 0, 2:5, 0:4, :]) and np.all(y[0, 0, 4] == 0) and np.all(y[0, 0, :, 0] == 0)
    # depth 1, kernel depth 1: the 2-D convolution
    x2, w2 = rnd(2, 3, 7, 6), rnd(4, 3, 3, 3)
    y3 = ops.conv3d(x2[:, :, None], w2[:, :, None], (1, 2, 1), (0, 1, 1))
    assert np.array_equal(y3[:, :, 0], ops.conv2d(x2, w2, (2, 1), (1, 1)))


def test_max_pool3d_and_global_avg_pool3d():
    x = rnd(2, 3, 6, 9, 8)
    assert np.array_equal(ops.max_pool3d(x, (3, 3, 3), (2, 2, 2), (1, 1, 1)), F.max_pool3d(torch.from_numpy(x), 3, 2, 1).numpy())
    assert np.array_equal(ops.max_pool3d(x, (1, 3, 2), (1, 2, 2), (0, 1, 0)),
                          F.max_pool3d(torch.from_numpy(x), (1, 3, 2), (1, 2, 2), (0, 1, 0)).numpy())
    close(ops.global_avg_pool3d(x), x.astype(np.float64).mean((2, 3, 4)))


def test_global_avg_pool():
    x = rnd(2, 5, 3, 4)
    close(ops.global_avg_pool2d(x), x.astype(np.float64).mean((2, 3)))
    assert np.all(ops.global_avg_pool2d(np.full((1, 2, 3, 3), 1.5, np.float32)) == 1.5)
    assert ops.global_avg_pool2d(x).shape == (2, 5)


def test_take_reshape_transpose():
    tab = rnd(11, 6)
    ids = np.array([3, 0, 10, 3], np.int32)
    assert np.array_equal(ops.take(tab, ids), tab[ids])
    with pytest.raises(IndexError):
        ops.take(tab, np.array([11], np.int32))
    x = rnd(4, 6)
    assert np.array_equal(ops.reshape(x, (4, 2, 3)).ravel(), x.ravel())
    t = ops.transpose(ops.reshape(x, (4, 2, 3)), (1, 0, 2))
    assert t.shape == (2, 4, 3) and t[1, 2, 0] == x[2, 3] and t.flags["C_CONTIGUOUS"]
