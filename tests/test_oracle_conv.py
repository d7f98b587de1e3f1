"""Pins of the oracle's convolutions: hand-worked values, library matmul on the 1x1 special case,
brute force written from the definition in pure Python, structural special cases (identity / shift
filters, subsampling), finite differences and the adjoint identities."""
import itertools

import numpy as np
import pytest

from oracle import ops


def brute_conv_fwd(x, w, stride, pad):
    n, c, h, ww = x.shape
    k, _, r, s = w.shape
    p, q = (h + 2 * pad - r) // stride + 1, (ww + 2 * pad - s) // stride + 1
    y = np.zeros((n, k, p, q))
    for ni, ki, pi, qi in itertools.product(range(n), range(k), range(p), range(q)):
        acc = 0.0
        for ci, ri, si in itertools.product(range(c), range(r), range(s)):
            hi, wi = pi * stride + ri - pad, qi * stride + si - pad
            if 0 <= hi < h and 0 <= wi < ww:
                acc += x[ni, ci, hi, wi] * w[ki, ci, ri, si]
        y[ni, ki, pi, qi] = acc
    return y


def brute_conv_bwd_data(dy, w, stride, pad, h, ww):
    """Gather form: each dx element collects the taps that land on it."""
    n, k, p, q = dy.shape
    _, c, r, s = w.shape
    dx = np.zeros((n, c, h, ww))
    for ni, ci, hi, wi in itertools.product(range(n), range(c), range(h), range(ww)):
        acc = 0.0
        for ki, ri, si in itertools.product(range(k), range(r), range(s)):
            a, b = hi + pad - ri, wi + pad - si
            if a % stride or b % stride:
                continue
            pi, qi = a // stride, b // stride
            if 0 <= pi < p and 0 <= qi < q:
                acc += dy[ni, ki, pi, qi] * w[ki, ci, ri, si]
        dx[ni, ci, hi, wi] = acc
    return dx


def test_hand_worked_1x1():
    # 2 input channels, 2 output channels, 1x2 image, one sample; worked by hand:
    # y[k,q] = w[k,0]*x[0,q] + w[k,1]*x[1,q]
    x = np.array([[[[1.0, 2.0]], [[3.0, -1.0]]]])          # N=1,C=2,H=1,W=2
    w = np.array([[[[2.0]], [[0.5]]], [[[-1.0]], [[4.0]]]])  # K=2,C=2
    y = ops.conv2d_fwd(x, w, 1, 0)
    assert y.shape == (1, 2, 1, 2)
    np.testing.assert_array_equal(y[0, :, 0, :], [[2 * 1 + 0.5 * 3, 2 * 2 + 0.5 * -1], [-1 + 12, -2 - 4]])
    # gradient of L = sum(y*dy): dx[c,q] = sum_k dy[k,q] w[k,c]; dw[k,c] = sum_q dy[k,q] x[c,q]
    dy = np.array([[[[1.0, -2.0]], [[0.5, 3.0]]]])
    dx = ops.conv2d_bwd_data(dy, w, 1, 0, 1, 2)
    np.testing.assert_array_equal(dx[0, :, 0, :], [[1 * 2 + 0.5 * -1, -2 * 2 + 3 * -1], [1 * 0.5 + 0.5 * 4, -2 * 0.5 + 3 * 4]])
    dw = ops.conv2d_bwd_weight(x, dy, 1, 1, 1, 0)
    np.testing.assert_array_equal(dw[:, :, 0, 0], [[1 * 1 + -2 * 2, 1 * 3 + -2 * -1], [0.5 * 1 + 3 * 2, 0.5 * 3 + 3 * -1]])


def test_hand_worked_3x3_pad():
    # single channel 2x2 image, 3x3 filter, pad 1: y[p,q] = sum_{r,s} x[p+r-1,q+s-1] w[r,s]
    x = np.array([[[[1.0, 2.0], [3.0, 4.0]]]])
    w = np.arange(1.0, 10.0).reshape(1, 1, 3, 3)
    y = ops.conv2d_fwd(x, w, 1, 1)
    # y[0,0] = x00*w11 + x01*w12 + x10*w21 + x11*w22 = 1*5+2*6+3*8+4*9
    # y[0,1] = x00*w10 + x01*w11 + x10*w20 + x11*w21 = 1*4+2*5+3*7+4*8
    # y[1,0] = x00*w01 + x01*w02 + x10*w11 + x11*w12 = 1*2+2*3+3*5+4*6
    # y[1,1] = x00*w00 + x01*w01 + x10*w10 + x11*w11 = 1*1+2*2+3*4+4*5
    np.testing.assert_array_equal(y[0, 0], [[77.0, 67.0], [47.0, 37.0]])


def test_1x1_is_matmul():
    g = np.random.default_rng(1)
    x, w = g.standard_normal((3, 5, 4, 6)), g.standard_normal((7, 5, 1, 1))
    y = ops.conv2d_fwd(x, w, 1, 0)
    ref = (w[:, :, 0, 0] @ x.transpose(1, 0, 2, 3).reshape(5, -1)).reshape(7, 3, 4, 6).transpose(1, 0, 2, 3)
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-13)


def test_identity_shift_and_subsample():
    g = np.random.default_rng(2)
    x = g.standard_normal((2, 3, 6, 7))
    w = np.zeros((3, 3, 3, 3))
    for c in range(3):
        w[c, c, 1, 1] = 1.0
    np.testing.assert_array_equal(ops.conv2d_fwd(x, w, 1, 1), x)
    # tap (r,s)=(0,2): y[p,q] = x[p-1,q+1]
    w = np.zeros((3, 3, 3, 3))
    for c in range(3):
        w[c, c, 0, 2] = 1.0
    y = ops.conv2d_fwd(x, w, 1, 1)
    np.testing.assert_array_equal(y[:, :, 1:, :-1], x[:, :, :-1, 1:])
    assert np.all(y[:, :, 0, :] == 0) and np.all(y[:, :, :, -1] == 0)
    # 1x1 stride 2 with unit weights = subsampling
    w = np.eye(3).reshape(3, 3, 1, 1)
    np.testing.assert_array_equal(ops.conv2d_fwd(x, w, 2, 0), x[:, :, ::2, ::2])


CASES = [  # n, c, h, w, k, r, stride, pad
    (2, 3, 5, 6, 4, 3, 1, 1),
    (1, 2, 7, 7, 3, 1, 2, 0),
    (2, 2, 9, 8, 2, 3, 2, 1),
    (1, 3, 11, 10, 2, 7, 2, 3),
    (1, 1, 4, 4, 1, 3, 1, 0),
]


@pytest.mark.parametrize("case", CASES)
def test_brute_force(case):
    n, c, h, ww, k, r, stride, pad = case
    g = np.random.default_rng(sum(case))
    x, w = g.standard_normal((n, c, h, ww)), g.standard_normal((k, c, r, r))
    y = ops.conv2d_fwd(x, w, stride, pad)
    np.testing.assert_allclose(y, brute_conv_fwd(x, w, stride, pad), rtol=0, atol=1e-12)
    dy = g.standard_normal(y.shape)
    np.testing.assert_allclose(ops.conv2d_bwd_data(dy, w, stride, pad, h, ww),
                               brute_conv_bwd_data(dy, w, stride, pad, h, ww), rtol=0, atol=1e-12)


@pytest.mark.parametrize("case", CASES)
def test_adjoint_and_finite_differences(case):
    n, c, h, ww, k, r, stride, pad = case
    g = np.random.default_rng(100 + sum(case))
    x, w = g.standard_normal((n, c, h, ww)), g.standard_normal((k, c, r, r))
    y = ops.conv2d_fwd(x, w, stride, pad)
    dy = g.standard_normal(y.shape)
    dx = ops.conv2d_bwd_data(dy, w, stride, pad, h, ww)
    dw = ops.conv2d_bwd_weight(x, dy, r, r, stride, pad)
    lhs = np.sum(y * dy)
    assert abs(lhs - np.sum(x * dx)) <= 1e-11 * max(1.0, abs(lhs))
    assert abs(lhs - np.sum(w * dw)) <= 1e-11 * max(1.0, abs(lhs))
    # central differences of L = <conv(x,w), dy> element by element (L is linear in x and in w,
    # so the difference quotient is exact up to rounding)
    eps = 1e-3
    for _ in range(10):
        i = tuple(g.integers(0, s) for s in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[i] += eps
        xm[i] -= eps
        fd = (np.sum(ops.conv2d_fwd(xp, w, stride, pad) * dy) - np.sum(ops.conv2d_fwd(xm, w, stride, pad) * dy)) / (2 * eps)
        assert abs(fd - dx[i]) < 1e-8
        j = tuple(g.integers(0, s) for s in w.shape)
        wp, wm = w.copy(), w.copy()
        wp[j] += eps
        wm[j] -= eps
        fd = (np.sum(ops.conv2d_fwd(x, wp, stride, pad) * dy) - np.sum(ops.conv2d_fwd(x, wm, stride, pad) * dy)) / (2 * eps)
        assert abs(fd - dw[j]) < 1e-8


def test_bwd_data_stride2_writes_zeros():
    # 1x1 stride 2: three quarters of dx receive no tap and must be exactly zero (not left unwritten)
    g = np.random.default_rng(5)
    w = g.standard_normal((3, 2, 1, 1))
    dy = g.standard_normal((1, 3, 3, 3))
    dx = ops.conv2d_bwd_data(dy, w, 2, 0, 6, 6)
    assert np.all(dx[:, :, 1::2, :] == 0) and np.all(dx[:, :, :, 1::2] == 0)
    np.testing.assert_allclose(dx[0, :, ::2, ::2], np.einsum("kpq,kc->cpq", dy[0], w[:, :, 0, 0]), atol=1e-13)
