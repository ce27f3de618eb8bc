"""Pins of the int8 reference evaluator (oracle/int8_eval.py) and of the int8 model generator.

The paper fixes the number formats of its accelerator (int8 weights, activations and zero points, int32 scale:
Section 5.1 footnote, Section 4.2.2) and prints no worked example, so nothing here is a paper value; the pins are
brute force in Python integers, closed forms of the rounding rule, a library float64 convolution on the same
integers, exact rational arithmetic for the classifier, structural invariants of slicing, and the closeness of the
whole int8 forward pass to the float evaluator.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import int8_eval as Q
from oracle import subnet_eval as E
from workloads import arch as A
from workloads import quant, streams, tensors as T
from workloads.rng import Stream


def _rand_i8(rs, shape, lo=-128, hi=127):
    return rs.randint(lo, hi + 1, size=shape).astype(np.int8)


@pytest.mark.parametrize("r,stride", [(1, 1), (1, 2), (3, 1), (3, 2)])
def test_integer_conv_against_nested_python_loops(r, stride):
    rs = np.random.RandomState(r * 10 + stride)
    n, c, h, w, k, zx = 2, 3, 6, 5, 4, -7
    x, wt = _rand_i8(rs, (n, c, h, w)), _rand_i8(rs, (k, c, r, r), -127, 127)
    got = Q.conv2d_i8(x, wt, zx, stride)
    pad = (r - 1) // 2
    p, q = (h + 2 * pad - r) // stride + 1, (w + 2 * pad - r) // stride + 1
    assert got.shape == (n, k, p, q) and got.dtype == np.int32
    for ni in range(n):
        for ki in range(k):
            for pi in range(p):
                for qi in range(q):
                    acc = 0
                    for ci in range(c):
                        for a in range(r):
                            for b in range(r):
                                hh, ww = pi * stride + a - pad, qi * stride + b - pad
                                if 0 <= hh < h and 0 <= ww < w:
                                    acc += int(wt[ki, ci, a, b]) * (int(x[ni, ci, hh, ww]) - zx)
                    assert int(got[ni, ki, pi, qi]) == acc


def test_integer_conv_against_a_library_float64_convolution():
    """The same integers through torch's CPU conv2d in float64 (exact below 2^53): the zero point is subtracted
    first, so torch's zero padding is the padding of the definition."""
    rs = np.random.RandomState(3)
    for (c, k, r, stride, hw, zx) in [(16, 24, 3, 1, 9, -128), (40, 8, 1, 2, 8, 0), (8, 8, 3, 2, 11, 5)]:
        x, wt = _rand_i8(rs, (2, c, hw, hw)), _rand_i8(rs, (k, c, r, r), -127, 127)
        want = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64) - zx), torch.from_numpy(wt.astype(np.float64)),
                                          stride=stride, padding=(r - 1) // 2).numpy()
        np.testing.assert_array_equal(Q.conv2d_i8(x, wt, zx, stride).astype(np.float64), want)


def test_a_padded_position_holds_the_zero_point():
    """An image that is the zero point everywhere convolves to zero whatever the weights, borders included; with
    another constant the borders differ from the interior by the closed-form window counts."""
    wt = np.ones((1, 1, 3, 3), dtype=np.int8)
    np.testing.assert_array_equal(Q.conv2d_i8(np.full((1, 1, 5, 5), -128, np.int8), wt, -128), 0)
    got = Q.conv2d_i8(np.full((1, 1, 4, 4), 10, np.int8), wt, 7)[0, 0]
    counts = np.array([[4, 6, 6, 4], [6, 9, 9, 6], [6, 9, 9, 6], [4, 6, 6, 4]])
    np.testing.assert_array_equal(got, 3 * counts)


def test_max_pool_on_codes():
    rs = np.random.RandomState(5)
    x = _rand_i8(rs, (2, 3, 7, 6))
    want = torch.nn.functional.max_pool2d(torch.from_numpy(x.astype(np.float32)), 3, 2, 1).numpy()
    np.testing.assert_array_equal(Q.maxpool3x3s2_i8(x).astype(np.float32), want)
    assert Q.maxpool3x3s2_i8(np.full((1, 1, 4, 4), -128, np.int8)).min() == -128   # padding takes no part


def test_rounding_shift_is_round_half_up_of_the_exact_quotient():
    assert [int(Q.rr(v, 1)) for v in (1, -1, 3, -3, 2, -2, 0)] == [1, 0, 2, -1, 1, -1, 0]
    rs = np.random.RandomState(7)
    for _ in range(2000):
        v = int(rs.randint(-2 ** 62, 2 ** 62, dtype=np.int64)) >> int(rs.randint(0, 40))
        s = int(rs.randint(1, 40))
        exact = Fraction(v, 2 ** s) + Fraction(1, 2)
        assert int(Q.rr(v, s)) == exact.numerator // exact.denominator


def test_requantisation_against_python_integers_and_its_saturation():
    rs = np.random.RandomState(11)
    acc = rs.randint(-3_000_000, 3_000_000, size=(2, 5, 3, 3)).astype(np.int32)
    mult = rs.randint(1 << 30, (1 << 31) - 1, size=5).astype(np.int64).astype(np.int32)
    rshift = rs.randint(40, 52, size=5).astype(np.int32)
    bias = rs.randint(-5000, 5000, size=5).astype(np.int32)
    res = _rand_i8(rs, acc.shape)
    m_res, sh_res, z_res, z_y = 1518500250, 30, -128, -128
    for relu in (False, True):
        for with_res in (False, True):
            got = Q.requant(acc, mult, rshift, bias, z_y, relu, res=res if with_res else None, m_res=m_res, sh_res=sh_res, z_res=z_res)
            for idx in np.ndindex(acc.shape):
                k = idx[1]
                t = ((int(acc[idx]) + int(bias[k])) * int(mult[k]) + (1 << (int(rshift[k]) - 1))) >> int(rshift[k])
                if with_res:
                    t += ((int(res[idx]) - z_res) * m_res + (1 << (sh_res - 1))) >> sh_res
                want = min(max(t + z_y, z_y if relu else -128), 127)
                assert int(got[idx]) == want
    one = np.array([1 << 30], dtype=np.int32)          # mult 2^30, shift 30: the identity
    big = np.array([[[[100000]]], [[[-100000]]], [[[5]]]], dtype=np.int32)
    np.testing.assert_array_equal(Q.requant(big, one, np.array([30]), np.array([0]), 0, False).ravel(), [127, -128, 5])
    np.testing.assert_array_equal(Q.requant(big, one, np.array([30]), np.array([0]), -128, True).ravel(), [127, -128, -123])


def test_fixed_point_multipliers_represent_their_factor():
    rs = np.random.RandomState(13)
    for m in list(10.0 ** rs.uniform(-9, 1, size=300)) + [1.0, 0.5, 2.0 ** -20, 0.99999999]:
        mult, shift = quant.fixed_point(m)
        assert (1 << 30) <= mult < (1 << 31)
        assert abs(mult * 2.0 ** -shift - m) <= m * 2.0 ** -30


def test_classifier_is_the_exact_rational_rounded_within_the_two_stated_roundings():
    rs = np.random.RandomState(17)
    sums = rs.randint(-12000, 12000, size=(3, 64)).astype(np.int32)
    wq = _rand_i8(rs, (10, 64), -127, 127)
    base = (10.0 ** rs.uniform(-6, -3, size=10)).astype(np.float32)
    bias = rs.randint(-3000, 3000, size=10).astype(np.int32)
    for hw in (1, 4, 49, 1024):
        got = Q.classifier(sums, hw, wq, base.view(np.int32), bias)
        for n in range(3):
            for k in range(10):
                acc = sum(int(wq[k, c]) * int(sums[n, c]) for c in range(64)) + hw * int(bias[k])
                exact = Fraction(acc) * Fraction(float(base[k])) / hw
                if exact == 0:
                    assert got[n, k] == 0
                else:
                    assert abs(Fraction(float(got[n, k])) - exact) <= abs(exact) * Fraction(1, 2 ** 22)
        if hw in (1, 4, 1024):      # a power of two: the division is exact, one rounding of the product remains
            acc = sums.astype(np.int64) @ wq.astype(np.int64).T + hw * bias.astype(np.int64)[None, :]
            np.testing.assert_array_equal(got, (acc.astype(np.float64) * (base.astype(np.float64) / hw)).astype(np.float32))


def _model(arch, seed):
    table = E.supernet_tensors(arch)
    tens = T.make_weights([(s, k) for _, s, k in table], seed, False)
    return table, tens, quant.make_int8_model(table, tens, quant.layer_roles(arch))


def test_generated_weights_are_the_rounded_float_weights():
    arch = A.tiny_arch()
    table, tens, model = _model(arch, 3)
    w = E.name_weights(arch, tens)
    for m in model:
        wf = w[m["name"] + ".w"].astype(np.float64)
        s_w = np.abs(wf.reshape(wf.shape[0], -1)).max(axis=1) / 127.0
        back = m["wq"].astype(np.float64) * s_w.reshape((-1,) + (1,) * (wf.ndim - 1))
        assert np.abs(back - wf).max() <= s_w.max() * 0.5 + 1e-12
        assert m["wq"].min() >= -127 and np.abs(m["wq"]).reshape(wf.shape[0], -1).max(axis=1).min() == 127


@pytest.mark.parametrize("fam", ["tiny", "resnet"])
def test_int8_forward_tracks_the_float_evaluator(fam):
    """The whole int8 forward pass lands near the float forward pass of the same SubNet (quantisation noise only):
    a dropped term, a wrong sign, a transposed operand or a mis-sliced parameter word moves the logits by O(1)."""
    arch = A.tiny_arch() if fam == "tiny" else A.small_resnet_arch()
    table, tens, model = _model(arch, 5)
    wts, qm = E.name_weights(arch, tens), Q.name_model(model)
    st = Stream(19)
    res = arch.res_choices[0]
    cfgs = [A.min_cfg(arch, res), A.max_cfg(arch, res)] + [streams.uniform_cfg(arch, st, res) for _ in range(3)]
    for t, cfg in enumerate(cfgs):
        x = T.make_input(5, t, 2, res, 3, False)
        xq = quant.quantize_input(x)
        want = E.forward(arch, wts, cfg, np.ascontiguousarray(x.transpose(0, 3, 1, 2)))
        got = Q.forward_int8(arch, qm, cfg, np.ascontiguousarray(xq.transpose(0, 3, 1, 2)))
        assert got.dtype == np.float32 and got.shape == want.shape
        err = np.linalg.norm(got.astype(np.float64) - want) / np.linalg.norm(want)
        assert err < 0.15, (fam, t, err)


def test_zero_mask_equivalence_of_int8_slicing():
    """The widest network at the SubNet's depth with every weight and bias outside the slice set to zero computes
    the SubNet's logits: an inactive channel is stored as the code of the real value 0 and adds nothing downstream."""
    arch = A.small_resnet_arch()
    table, tens, model = _model(arch, 7)
    qm = Q.name_model(model)
    st = Stream(23)
    res = arch.res_choices[0]
    cfg = streams.uniform_cfg(arch, st, res)
    wide = A.max_cfg(arch, res)
    wide.depth = list(cfg.depth)
    box = {n: (k, c, r) for (n, k, c, r) in E.active_layers(arch, cfg)}
    masked = {}
    for name, m in qm.items():
        k, c, r = box[name]
        wq = np.zeros_like(m["wq"])
        bias = np.zeros_like(m["bias"])
        if k:
            if wq.ndim == 4:
                wq[:k, :c] = m["wq"][:k, :c]
            else:
                wq[:k, :c] = m["wq"][:k, :c]
            bias[:k] = m["bias"][:k]
        masked[name] = dict(m, wq=wq, bias=bias)
    xq = quant.quantize_input(T.make_input(7, 0, 1, res, 3, False)).transpose(0, 3, 1, 2)
    a = Q.forward_int8(arch, qm, cfg, xq)
    b = Q.forward_int8(arch, masked, wide, xq)
    np.testing.assert_array_equal(a, b)
    # a planted mistake: slicing the parameter words from the wrong end must break the equality
    wrong = {n: dict(m, mult=m["mult"][::-1].copy()) for n, m in qm.items()}
    assert not np.array_equal(Q.forward_int8(arch, wrong, cfg, xq), a)
