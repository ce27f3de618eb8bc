"""Reference evaluator of the int8 path — TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper's accelerator computes in int8: weights, input activations and zero points are int8, the quantisation
scale is an int32 (Section 5.1, footnote on number formats; Section 4.2.2, the zero-point / scale buffer).  It
gives the formats, not the arithmetic; the reading taken here (the design doc lists it) is the usual integer-only
scheme, written out with exact integers so that every step has ONE right answer:

  conv       acc[k] = sum_taps,c w_q[k,c,tap] * (x_q[c,tap] - z_x)            exact int32 (conv_ref.c)
  requant    t = rr((acc[k] + bias[k]) * mult[k], rshift[k])                  64-bit product,
             rr(v, s) = (v + 2^(s-1)) >> s  (arithmetic shift: round half up)
  residual   t += rr((res_q - z_res) * m_res, sh_res)
  store      y_q = clamp(z_y + t, lo, 127),  lo = z_y after a ReLU (the code of the real value 0) else -128
  max-pool   maximum of the codes
  pooling    sum[c] = sum_pixels (x_q - z_x)                                  exact int32
  classifier acc64[k] = sum_c w_q[k,c] * sum[c] + HW * bias[k]                exact int64
             logit[k] = float32( float64(acc64[k]) * (float64(base[k]) / float64(HW)) ),
             base[k] = the float32 whose bit pattern is mult[k]

A SubNet is sliced exactly as in subnet_eval.py (leading filters, leading input channels, first blocks); the
parameter words of a layer are sliced by the same filter prefix.  Families: the Tiny conv chain and the
bottleneck (ResNet50-shaped) SuperNet; the inverted-residual family (depthwise, squeeze-excite, h-swish) has no
int8 reading here.

Parity note: the paper prints no worked example of its integer arithmetic, so this file is pinned by brute
force in Python integers, closed forms of the rounding rule, a library float64 convolution on the same integers
and the closeness of the whole int8 forward pass to the float evaluator (tests/test_oracle_int8.py).
"""
import ctypes

import numpy as np

from workloads.arch import FAMILY_RESNET, FAMILY_TINY

from . import subnet_eval as E

_lib = None


def _clib():
    global _lib
    if _lib is None:
        _lib = E._clib()
        i8 = ctypes.POINTER(ctypes.c_int8)
        i32 = ctypes.POINTER(ctypes.c_int32)
        _lib.ref_conv2d_i8.argtypes = [i8, i8, i32] + [ctypes.c_int] * 10
        _lib.ref_maxpool2d_i8.argtypes = [i8, i8] + [ctypes.c_int] * 7
    return _lib


def conv2d_i8(x, w, zx, stride=1):
    """x int8 [N,C,H,W], w int8 [K,C,r,r] -> int32 [N,K,P,Q], pad (r-1)/2."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    w = np.ascontiguousarray(w, dtype=np.int8)
    n, c, h, wd = x.shape
    k, c2, r, s = w.shape
    assert c == c2 and r == s and r % 2 == 1
    pad = (r - 1) // 2
    p = (h + 2 * pad - r) // stride + 1
    q = (wd + 2 * pad - r) // stride + 1
    acc = np.empty((n, k, p, q), dtype=np.int32)
    rc = _clib().ref_conv2d_i8(x.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)), w.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)),
                               acc.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), n, c, h, wd, k, r, s, stride, pad, int(zx))
    assert rc == 0, rc
    return acc


def maxpool3x3s2_i8(x):
    x = np.ascontiguousarray(x, dtype=np.int8)
    n, c, h, wd = x.shape
    p, q = (h + 2 - 3) // 2 + 1, (wd + 2 - 3) // 2 + 1
    y = np.empty((n, c, p, q), dtype=np.int8)
    rc = _clib().ref_maxpool2d_i8(x.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)), y.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)),
                                  n, c, h, wd, 3, 2, 1)
    assert rc == 0, rc
    return y


def rr(v, s):
    """Rounding right shift of int64 values: (v + 2^(s-1)) >> s, s >= 1 (per-element s allowed)."""
    v = np.asarray(v, dtype=np.int64)
    s = np.asarray(s, dtype=np.int64)
    return (v + (np.int64(1) << (s - 1))) >> s


def requant(acc, mult, rshift, bias, z_y, relu, res=None, m_res=0, sh_res=1, z_res=0):
    """acc int32 [N,K,P,Q]; per-filter mult / rshift / bias [K]; optional residual codes res int8 [N,K,P,Q]."""
    k = acc.shape[1]
    bc = (1, k, 1, 1)
    t = rr((acc.astype(np.int64) + bias.astype(np.int64).reshape(bc)) * mult.astype(np.int64).reshape(bc),
           rshift.astype(np.int64).reshape(bc))
    if res is not None:
        t = t + rr((res.astype(np.int64) - int(z_res)) * int(m_res), int(sh_res))
    lo = int(z_y) if relu else -128
    return np.clip(t + int(z_y), lo, 127).astype(np.int8)


def pooled_sums(x, z_x):
    """[N,C,H,W] int8 -> exact int32 sums of (x - z_x) over H, W."""
    return (x.astype(np.int64) - int(z_x)).sum(axis=(2, 3)).astype(np.int32)


def classifier(sums, hw, wq, mult_bits, bias):
    """sums int32 [N,C]; wq int8 [K,C]; mult_bits int32 [K] = bit patterns of float32 base[k]; bias int32 [K]."""
    acc = sums.astype(np.int64) @ wq.astype(np.int64).T + np.int64(hw) * bias.astype(np.int64)[None, :]
    base = mult_bits.astype(np.int32).view(np.float32).astype(np.float64)
    return (acc.astype(np.float64) * (base / np.float64(hw))[None, :]).astype(np.float32)


def name_model(model):
    """List of layer dicts (workloads.quant.make_int8_model) -> dict by layer name."""
    return {m["name"]: m for m in model}


def _conv(qm, name, x, k, r, stride, relu, res=None):
    """Layer `name` sliced to k leading filters and x's channels; conv, requantise, store."""
    L = qm[name]
    c = x.shape[1]
    w = E.centre_crop(L["wq"][:k, :c], r)
    sc = L["scalars"]
    acc = conv2d_i8(x, w, sc[0], stride)
    return requant(acc, L["mult"][:k], L["rshift"][:k], L["bias"][:k], sc[1], relu,
                   res=res, m_res=sc[2], sh_res=max(int(sc[3]), 1), z_res=sc[4])


def forward_int8(arch, qm, cfg, x_q):
    """float32 logits [N, n_classes] of SubNet `cfg` on the int8 input x_q [N,3,res,res] (zero point 0)."""
    assert E.check_cfg(arch, cfg), "invalid SubNet configuration"
    W, Ex = arch.width_choices, arch.expand_choices
    x = np.ascontiguousarray(x_q, dtype=np.int8)
    if arch.family == FAMILY_TINY:
        for l in range(cfg.depth[0]):
            x = _conv(qm, "conv%d" % l, x, E.ch(arch.stage_base_out[l] * W[cfg.width_idx[1 + l]]), 3, 1, True)
    elif arch.family == FAMILY_RESNET:
        w0 = W[cfg.width_idx[0]]
        mid, o = E.ch(arch.stem_mid * w0), E.ch(arch.stem_out * w0)
        x = _conv(qm, "stem0", x, mid, 3, 2, True)
        x = _conv(qm, "stem1", x, mid, 3, 1, True)
        x = _conv(qm, "stem2", x, o, 3, 1, True)
        x = maxpool3x3s2_i8(x)
        for s in range(arch.n_stages):
            cout = E.ch(arch.stage_base_out[s] * W[cfg.width_idx[1 + s]])
            for j in range(cfg.depth[s]):
                n = "s%db%d" % (s, j)
                stride = arch.stage_stride[s] if j == 0 else 1
                cmid = E.ch(cout * Ex[cfg.expand_idx[arch.slot(s, j)]])
                h = _conv(qm, n + ".conv1", x, cmid, 1, 1, True)
                h = _conv(qm, n + ".conv2", h, cmid, 3, stride, True)
                sc = _conv(qm, n + ".proj", x, cout, 1, stride, False) if j == 0 else x
                x = _conv(qm, n + ".conv3", h, cout, 1, 1, True, res=sc)
    else:
        raise ValueError("the int8 evaluator covers the Tiny and the bottleneck families")
    fc = qm["fc"]
    c = x.shape[1]
    hw = x.shape[2] * x.shape[3]
    sums = pooled_sums(x, fc["scalars"][0])
    k = arch.n_classes
    return classifier(sums, hw, fc["wq"][:k, :c], fc["mult"][:k], fc["bias"][:k])
