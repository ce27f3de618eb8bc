"""Pins for the reference operators (oracle/conv_ref.c via oracle/subnet_eval.py).

The paper prints no worked numerical example, so the operators are pinned by what the
mathematics fixes: brute force on tiny inputs, closed forms, invariants, and agreement with
library routines (numpy matmul, torch CPU conv2d) that share no code with the oracle.
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import subnet_eval as E
from workloads import rng
from workloads.arch import ACT_HSWISH, ACT_NONE, ACT_RELU
from workloads.tensors import round_to_bf16


def _rand(seed, shape):
    return rng.normal(seed, int(np.prod(shape))).astype(np.float32).reshape(shape)


def _brute_conv(x, w, stride, pad, depthwise=False):
    """Nested loops over every index, double accumulation — the definition itself."""
    n_, c_, h_, w_ = x.shape
    k_, cw, r_, s_ = w.shape
    p_ = (h_ + 2 * pad - r_) // stride + 1
    q_ = (w_ + 2 * pad - s_) // stride + 1
    y = np.zeros((n_, k_, p_, q_), dtype=np.float64)
    for n, k, p, q in itertools.product(range(n_), range(k_), range(p_), range(q_)):
        acc = 0.0
        chans = [k] if depthwise else range(c_)
        for c in chans:
            for r in range(r_):
                for s in range(s_):
                    hh, ww = p * stride + r - pad, q * stride + s - pad
                    if 0 <= hh < h_ and 0 <= ww < w_:
                        acc += float(w[k, 0 if depthwise else c, r, s]) * float(x[n, c, hh, ww])
        y[n, k, p, q] = acc
    return y


@pytest.mark.parametrize("r,stride,h,w", [(1, 1, 5, 4), (1, 2, 5, 6), (3, 1, 5, 5), (3, 2, 6, 7), (3, 2, 7, 5),
                                          (5, 1, 6, 6), (7, 2, 9, 8)])
def test_conv_matches_brute_force(r, stride, h, w):
    x = _rand(11 + r, (2, 3, h, w))
    wt = _rand(12 + stride, (4, 3, r, r))
    got = E.conv2d(x, wt, stride)
    want = _brute_conv(x, wt, stride, (r - 1) // 2)
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-6)


@pytest.mark.parametrize("r,stride,h,w", [(3, 1, 5, 5), (3, 2, 6, 7), (5, 1, 7, 6), (5, 2, 8, 8), (7, 1, 7, 9),
                                          (7, 2, 10, 9)])
def test_dwconv_matches_brute_force(r, stride, h, w):
    x = _rand(21 + r, (2, 5, h, w))
    wt = _rand(22 + stride, (5, 1, r, r))
    got = E.dwconv2d(x, wt, stride)
    want = _brute_conv(x, wt, stride, (r - 1) // 2, depthwise=True)
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-6)


def test_maxpool_matches_brute_force():
    x = _rand(31, (2, 3, 9, 8))
    got = E.maxpool3x3s2(x)
    n_, c_, h_, w_ = x.shape
    p_, q_ = (h_ - 1) // 2 + 1, (w_ - 1) // 2 + 1
    assert got.shape == (n_, c_, p_, q_)
    for n, c, p, q in itertools.product(range(n_), range(c_), range(p_), range(q_)):
        vals = [x[n, c, hh, ww] for hh in range(2 * p - 1, 2 * p + 2) for ww in range(2 * q - 1, 2 * q + 2)
                if 0 <= hh < h_ and 0 <= ww < w_]
        assert got[n, c, p, q] == max(vals)


def test_identity_kernel_returns_input():
    x = _rand(41, (1, 4, 6, 7))
    for r in (1, 3, 5):
        w = np.zeros((4, 4, r, r), dtype=np.float32)
        for c in range(4):
            w[c, c, r // 2, r // 2] = 1.0
        np.testing.assert_array_equal(E.conv2d(x, w, 1), x)
    w = np.zeros((4, 1, 7, 7), dtype=np.float32)
    w[:, 0, 3, 3] = 1.0
    np.testing.assert_array_equal(E.dwconv2d(x, w, 1), x)


def test_shifted_tap_shifts_image():
    """A single off-centre tap moves the image by that offset (catches a flipped kernel or a
    transposed r/s index, which the centred identity kernel would not)."""
    x = _rand(42, (1, 1, 6, 6))
    w = np.zeros((1, 1, 3, 3), dtype=np.float32)
    w[0, 0, 0, 2] = 1.0          # r=0 (one row up), s=2 (one column right)
    y = E.conv2d(x, w, 1)
    want = np.zeros_like(x)
    want[0, 0, 1:, :-1] = x[0, 0, :-1, 1:]
    np.testing.assert_array_equal(y, want)
    y = E.dwconv2d(x, w, 1)
    np.testing.assert_array_equal(y, want)


@pytest.mark.parametrize("k", [3, 5, 7])
def test_ones_depthwise_counts_window_cells(k):
    """All-ones k x k depthwise kernel on a constant image c: output = c * (#window cells inside
    the image) = c * rows(p) * cols(q), rows(p) = min(p+h,H-1) - max(p-h,0) + 1 with h = k//2."""
    H, W, cval = 9, 11, 0.5
    x = np.full((1, 2, H, W), cval, dtype=np.float32)
    w = np.ones((2, 1, k, k), dtype=np.float32)
    y = E.dwconv2d(x, w, 1)
    h = k // 2
    rows = np.array([min(p + h, H - 1) - max(p - h, 0) + 1 for p in range(H)])
    cols = np.array([min(q + h, W - 1) - max(q - h, 0) + 1 for q in range(W)])
    want = cval * rows[:, None] * cols[None, :]
    np.testing.assert_allclose(y[0, 0], want, rtol=0, atol=1e-6)
    assert y[0, 1, H // 2, W // 2] == cval * k * k


def test_conv_is_linear():
    a, b = _rand(51, (1, 3, 6, 6)), _rand(52, (1, 3, 6, 6))
    w = _rand(53, (5, 3, 3, 3))
    np.testing.assert_allclose(E.conv2d(a + b, w, 2), E.conv2d(a, w, 2) + E.conv2d(b, w, 2), atol=1e-5)


def test_pointwise_conv_is_matmul():
    x = _rand(61, (2, 7, 4, 5))
    w = _rand(62, (6, 7, 1, 1))
    got = E.conv2d(x, w, 1)
    want = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0].astype(np.float64), x.astype(np.float64))
    np.testing.assert_allclose(got, want, atol=2e-6)


@pytest.mark.parametrize("r,stride", [(1, 1), (1, 2), (3, 1), (3, 2)])
def test_conv_matches_torch_cpu(r, stride):
    x = _rand(71, (2, 24, 15, 14))
    w = _rand(72, (16, 24, r, r))
    got = E.conv2d(x, w, stride)
    want = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), stride=stride, padding=(r - 1) // 2)
    np.testing.assert_allclose(got, want.numpy(), atol=2e-5)


@pytest.mark.parametrize("r,stride", [(3, 1), (5, 2), (7, 1), (7, 2)])
def test_dwconv_matches_torch_cpu(r, stride):
    x = _rand(81, (2, 24, 15, 14))
    w = _rand(82, (24, 1, r, r))
    got = E.dwconv2d(x, w, stride)
    want = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), stride=stride, padding=(r - 1) // 2,
                    groups=24)
    np.testing.assert_allclose(got, want.numpy(), atol=2e-5)


def test_maxpool_matches_torch_cpu():
    x = _rand(91, (2, 8, 17, 16))
    want = F.max_pool2d(torch.from_numpy(x), 3, 2, 1).numpy()
    np.testing.assert_array_equal(E.maxpool3x3s2(x), want)


def test_activation_closed_forms():
    v = np.array([-4.0, -3.0, -1.0, 0.0, 1.0, 3.0, 5.0], dtype=np.float32)
    np.testing.assert_allclose(E.activation(v, ACT_HSWISH), [0, 0, -1 * 2 / 6, 0, 1 * 4 / 6, 3, 5], atol=1e-7)
    np.testing.assert_allclose(E.hsigmoid(v), [0, 0, 2 / 6, 0.5, 4 / 6, 1, 1], atol=1e-7)
    np.testing.assert_array_equal(E.activation(v, ACT_RELU), [0, 0, 0, 0, 1, 3, 5])
    np.testing.assert_array_equal(E.activation(v, ACT_NONE), v)
    np.testing.assert_allclose(E.activation(v, ACT_HSWISH), F.hardswish(torch.from_numpy(v)).numpy(), atol=1e-7)
    np.testing.assert_allclose(E.hsigmoid(v), F.hardsigmoid(torch.from_numpy(v)).numpy(), atol=1e-7)


def test_affine_then_activation_order():
    y = np.array([[[[-2.0]], [[2.0]]]], dtype=np.float32)          # [1,2,1,1]
    out = E.affine_act(y, np.array([-1.0, 0.5], np.float32), np.array([0.25, -2.0], np.float32), ACT_RELU)
    np.testing.assert_array_equal(out.ravel(), [2.25, 0.0])        # relu(-1*-2+0.25), relu(0.5*2-2)


def test_global_avg_and_linear():
    x = np.arange(2 * 3 * 2 * 2, dtype=np.float32).reshape(2, 3, 2, 2)
    g = E.global_avg(x)
    np.testing.assert_array_equal(g, [[1.5, 5.5, 9.5], [13.5, 17.5, 21.5]])
    w = np.array([[1, 0, -1], [2, 2, 2]], dtype=np.float32)
    b = np.array([0.5, -1], dtype=np.float32)
    np.testing.assert_array_equal(E.linear(g, w, b), [[1.5 - 9.5 + 0.5, 33 - 1], [13.5 - 21.5 + 0.5, 105 - 1]])


def test_channel_rounding_rule():
    # multiples of 8 are fixed points; halves round up; the 0.9 guard bumps a too-small result
    assert [E.ch(v) for v in (8, 16, 2048)] == [8, 16, 2048]
    assert E.ch(2048 * 0.35) == 720          # 716.8 -> 89.6 -> 90
    assert E.ch(256 * 0.65) == 168           # 166.4 -> 20.8 -> 21
    assert E.ch(1024 * 0.65) == 664          # 665.6 -> 83.2 -> 83
    assert E.ch(52) == 56                    # 6.5 rounds half up
    assert E.ch(3) == 8                      # floor of 8
    assert E.ch(12) == 16 and E.ch(11.9) == 16   # 8 would be below 0.9*x
    assert E.ch(20.8) == 24                  # 2.6 -> 3


def test_bf16_rounding_matches_torch():
    x = _rand(101, (4096,)) * 37.0
    x[:4] = [1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -1.0 - 2 ** -8, 0.0]     # exact ties -> even
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(round_to_bf16(x), want)
    assert round_to_bf16(x)[0] == 1.0 and round_to_bf16(x)[1] == 1.0 + 2 ** -6
