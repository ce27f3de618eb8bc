"""Reference SubNet evaluator — TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

What it computes: the forward pass of one SubNet of a weight-shared SuperNet
(paper Section 2.1).  A SubNet is picked by elastic choices; its weights are
*slices* of the SuperNet tensors:

  * depth      - the first d blocks of a stage run, the rest are skipped;
  * width /    - a conv keeps its leading K' output filters and the leading C'
    expand       input channels ("top k kernels", Section 2.1);
  * kernel     - a k x k depthwise kernel is the centred k x k crop of the
                 largest one (the paper names the dimension but gives no rule;
                 the centred crop keeps every SubNet an exact slice).

For a fixed slice the result is the textbook CNN forward pass, so this file is
that definition written out: numpy slicing, direct convolutions from
conv_ref.c (double accumulation), float32 activations in NCHW.

Channel rounding (the paper is silent): ch(x) = max(8, floor(x/8 + 0.5) * 8),
plus 8 if that is below 0.9 x.

Parity note: the paper prints no numerical example of a forward pass, so the
evaluator is pinned by brute force, library cross-checks and structural
invariants in tests/test_oracle_*.py, not by paper values.
"""
import ctypes
import math
import os

import numpy as np

from workloads.arch import (ACT_HSWISH, ACT_NONE, ACT_RELU, FAMILY_MBV3, FAMILY_RESNET, FAMILY_TINY)
from workloads.tensors import (KIND_BIAS, KIND_CONV, KIND_DWCONV, KIND_FC, KIND_SCALE, KIND_SCALE_RES,
                               KIND_SHIFT)

from . import build as _build

_lib = None


def _clib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build.build())
        fp = ctypes.POINTER(ctypes.c_float)
        _lib.ref_conv2d.argtypes = [fp, fp, fp] + [ctypes.c_int] * 9
        _lib.ref_dwconv2d.argtypes = [fp, fp, fp] + [ctypes.c_int] * 8
        _lib.ref_maxpool2d.argtypes = [fp, fp] + [ctypes.c_int] * 7
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


# ---------------------------------------------------------------- operators

def conv2d(x, w, stride=1):
    """Dense conv, 'same'-style zero padding pad=(r-1)/2.  x [N,C,H,W], w [K,C,r,r]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    n, c, h, wd = x.shape
    k, c2, r, s = w.shape
    assert c == c2 and r == s and r % 2 == 1
    pad = (r - 1) // 2
    p = (h + 2 * pad - r) // stride + 1
    q = (wd + 2 * pad - r) // stride + 1
    y = np.empty((n, k, p, q), dtype=np.float32)
    rc = _clib().ref_conv2d(_ptr(x), _ptr(w), _ptr(y), n, c, h, wd, k, r, s, stride, pad)
    assert rc == 0
    return y


def dwconv2d(x, w, stride=1):
    """Depthwise conv.  x [N,C,H,W], w [C,1,r,r]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    n, c, h, wd = x.shape
    c2, one, r, s = w.shape
    assert c == c2 and one == 1 and r == s and r % 2 == 1
    pad = (r - 1) // 2
    p = (h + 2 * pad - r) // stride + 1
    q = (wd + 2 * pad - r) // stride + 1
    y = np.empty((n, c, p, q), dtype=np.float32)
    rc = _clib().ref_dwconv2d(_ptr(x), _ptr(w), _ptr(y), n, c, h, wd, r, s, stride, pad)
    assert rc == 0
    return y


def maxpool3x3s2(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    n, c, h, wd = x.shape
    p = (h + 2 - 3) // 2 + 1
    q = (wd + 2 - 3) // 2 + 1
    y = np.empty((n, c, p, q), dtype=np.float32)
    rc = _clib().ref_maxpool2d(_ptr(x), _ptr(y), n, c, h, wd, 3, 2, 1)
    assert rc == 0
    return y


def activation(v, act):
    if act == ACT_NONE:
        return v
    if act == ACT_RELU:
        return np.maximum(v, np.float32(0))
    if act == ACT_HSWISH:                      # x * min(max(x+3,0),6) / 6
        return (v * np.minimum(np.maximum(v + np.float32(3), np.float32(0)), np.float32(6)) / np.float32(6)).astype(np.float32)
    raise ValueError(act)


def hsigmoid(v):                               # min(max(x+3,0),6) / 6
    return (np.minimum(np.maximum(v + np.float32(3), np.float32(0)), np.float32(6)) / np.float32(6)).astype(np.float32)


def affine_act(y, scale, shift, act):
    """Per-output-channel y*scale+shift then activation (batch norm reduced to one pair)."""
    return activation(y * scale[None, :, None, None] + shift[None, :, None, None], act).astype(np.float32)


def global_avg(x):
    """Mean over H, W in double, rounded to float32.  [N,C,H,W] -> [N,C]."""
    return x.astype(np.float64).mean(axis=(2, 3)).astype(np.float32)


def linear(g, w, b):
    """g [N,C] @ w[K,C]^T + b in double, rounded to float32."""
    return (g.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)).astype(np.float32)


# ---------------------------------------------------------------- structure

def ch(x):
    """Channel rounding rule (see module docstring)."""
    v = max(8, int(math.floor(x / 8.0 + 0.5)) * 8)
    if v < 0.9 * x:
        v += 8
    return v


def centre_crop(w, r):
    """Centred r x r crop of a [K,C,R,R] tensor."""
    o = (w.shape[2] - r) // 2
    return w[:, :, o:o + r, o:o + r]


def supernet_tensors(arch):
    """Canonical list of (name, shape, kind) of every SuperNet tensor, in blob order."""
    t = []

    def conv(name, k, c, r, res_scale=False, dw=False):
        t.append((name + ".w", (k, 1 if dw else c, r, r), KIND_DWCONV if dw else KIND_CONV))
        t.append((name + ".scale", (k,), KIND_SCALE_RES if res_scale else KIND_SCALE))
        t.append((name + ".shift", (k,), KIND_SHIFT))

    def fc(name, k, c):
        t.append((name + ".w", (k, c), KIND_FC))
        t.append((name + ".b", (k,), KIND_BIAS))

    wmax, emax, kmax = max(arch.width_choices), max(arch.expand_choices), max(arch.kernel_choices)
    if arch.family == FAMILY_TINY:
        cin = arch.in_channels
        for l in range(arch.n_stages):
            cout = ch(arch.stage_base_out[l] * wmax)
            conv("conv%d" % l, cout, cin, 3)
            cin = cout
        fc("fc", arch.n_classes, cin)
    elif arch.family == FAMILY_RESNET:
        mid, out = ch(arch.stem_mid * wmax), ch(arch.stem_out * wmax)
        conv("stem0", mid, arch.in_channels, 3)
        conv("stem1", mid, mid, 3)
        conv("stem2", out, mid, 3)
        cin = out
        for s in range(arch.n_stages):
            cout = ch(arch.stage_base_out[s] * wmax)
            cmid = ch(cout * emax)
            for j in range(arch.stage_max_depth[s]):
                n = "s%db%d" % (s, j)
                conv(n + ".conv1", cmid, cin, 1)
                conv(n + ".conv2", cmid, cmid, 3)
                conv(n + ".conv3", cout, cmid, 1, res_scale=True)
                if j == 0:
                    conv(n + ".proj", cout, cin, 1)
                cin = cout
        fc("fc", arch.n_classes, cin)
    elif arch.family == FAMILY_MBV3:
        c0 = arch.stem_out
        conv("stem", c0, arch.in_channels, 3)
        conv("first.dw", c0, 1, 3, dw=True)
        conv("first.pw", c0, c0, 1, res_scale=True)
        cin = c0
        for s in range(arch.n_stages):
            cout = arch.stage_base_out[s]
            for j in range(arch.stage_max_depth[s]):
                n = "s%db%d" % (s, j)
                stride = arch.stage_stride[s] if j == 0 else 1
                cmid = ch(cin * emax)
                conv(n + ".expand", cmid, cin, 1)
                conv(n + ".dw", cmid, 1, kmax, dw=True)
                if arch.stage_se[s]:
                    red = ch(cmid / 4.0)
                    fc(n + ".se1", red, cmid)
                    fc(n + ".se2", cmid, red)
                conv(n + ".project", cout, cmid, 1, res_scale=(stride == 1 and cin == cout))
                cin = cout
        conv("head", arch.head_mid, cin, 1)
        fc("feat", arch.head_feat, arch.head_mid)
        fc("fc", arch.n_classes, arch.head_feat)
    else:
        raise ValueError("family")
    return t


def name_weights(arch, tensors):
    """Zip a list of arrays (blob order) with the canonical names."""
    table = supernet_tensors(arch)
    assert len(table) == len(tensors)
    out = {}
    for (name, shape, _), a in zip(table, tensors):
        assert tuple(a.shape) == tuple(shape), (name, a.shape, shape)
        out[name] = a
    return out


def check_cfg(arch, cfg):
    """True iff every choice index is in range and the depths are allowed."""
    if cfg.resolution not in arch.res_choices:
        return False
    if arch.family == FAMILY_TINY:
        if len(cfg.depth) < 1 or (arch.n_stages - cfg.depth[0]) not in arch.depth_drop_choices:
            return False
    else:
        for s in range(arch.n_stages):
            if (arch.stage_max_depth[s] - cfg.depth[s]) not in arch.depth_drop_choices:
                return False
    if any(not (0 <= i < len(arch.width_choices)) for i in cfg.width_idx[:arch.n_stages + 1]):
        return False
    nb = arch.n_block_slots
    if any(not (0 <= i < len(arch.expand_choices)) for i in cfg.expand_idx[:nb]):
        return False
    if any(not (0 <= i < len(arch.kernel_choices)) for i in cfg.kernel_idx[:nb]):
        return False
    return True


def active_layers(arch, cfg):
    """Structure only: for EVERY weight-bearing SuperNet layer, in canonical order,
    (name, K', C', r') of the slice the SubNet uses; a skipped layer has (name, 0, 0, 0).
    Depthwise layers report C' = 1.  Fully connected layers report r' = 1."""
    out = []
    W, E, Kc = arch.width_choices, arch.expand_choices, arch.kernel_choices
    if arch.family == FAMILY_TINY:
        cin = arch.in_channels
        for l in range(arch.n_stages):
            if l < cfg.depth[0]:
                cout = ch(arch.stage_base_out[l] * W[cfg.width_idx[1 + l]])
                out.append(("conv%d" % l, cout, cin, 3))
                cin = cout
            else:
                out.append(("conv%d" % l, 0, 0, 0))
        out.append(("fc", arch.n_classes, cin, 1))
    elif arch.family == FAMILY_RESNET:
        w0 = W[cfg.width_idx[0]]
        mid, o = ch(arch.stem_mid * w0), ch(arch.stem_out * w0)
        out += [("stem0", mid, arch.in_channels, 3), ("stem1", mid, mid, 3), ("stem2", o, mid, 3)]
        cin = o
        for s in range(arch.n_stages):
            cout = ch(arch.stage_base_out[s] * W[cfg.width_idx[1 + s]])
            for j in range(arch.stage_max_depth[s]):
                n = "s%db%d" % (s, j)
                names = [n + ".conv1", n + ".conv2", n + ".conv3"] + ([n + ".proj"] if j == 0 else [])
                if j >= cfg.depth[s]:
                    out += [(x, 0, 0, 0) for x in names]
                    continue
                cmid = ch(cout * E[cfg.expand_idx[arch.slot(s, j)]])
                out += [(names[0], cmid, cin, 1), (names[1], cmid, cmid, 3), (names[2], cout, cmid, 1)]
                if j == 0:
                    out.append((names[3], cout, cin, 1))
                cin = cout
        out.append(("fc", arch.n_classes, cin, 1))
    elif arch.family == FAMILY_MBV3:
        c0 = arch.stem_out
        out += [("stem", c0, arch.in_channels, 3), ("first.dw", c0, 1, 3), ("first.pw", c0, c0, 1)]
        cin = c0
        for s in range(arch.n_stages):
            cout = arch.stage_base_out[s]
            for j in range(arch.stage_max_depth[s]):
                n = "s%db%d" % (s, j)
                names = [n + ".expand", n + ".dw"] + ([n + ".se1", n + ".se2"] if arch.stage_se[s] else []) \
                    + [n + ".project"]
                if j >= cfg.depth[s]:
                    out += [(x, 0, 0, 0) for x in names]
                    continue
                b = arch.slot(s, j)
                cmid = ch(cin * E[cfg.expand_idx[b]])
                k = Kc[cfg.kernel_idx[b]]
                out += [(n + ".expand", cmid, cin, 1), (n + ".dw", cmid, 1, k)]
                if arch.stage_se[s]:
                    red = ch(cmid / 4.0)
                    out += [(n + ".se1", red, cmid, 1), (n + ".se2", cmid, red, 1)]
                out.append((n + ".project", cout, cmid, 1))
                cin = cout
        out += [("head", arch.head_mid, cin, 1), ("feat", arch.head_feat, arch.head_mid, 1),
                ("fc", arch.n_classes, arch.head_feat, 1)]
    return out


# ---------------------------------------------------------------- forward

class _Run:
    """Carries the weights and the per-layer record through one forward pass."""

    def __init__(self, wts, act_round):
        self.w = wts
        self.layers = []
        self.round = act_round if act_round is not None else (lambda a: a)

    def conv(self, name, x, k, r, stride, act, dw=False):
        """Slice layer `name` to k leading filters, x's channel count, centred r x r; conv + affine + act."""
        c = x.shape[1]
        wfull = self.w[name + ".w"]
        if dw:
            w = centre_crop(wfull[:k], r)
            y = dwconv2d(x, w, stride)
            self.layers.append((name, k, 1, r))
        else:
            w = centre_crop(wfull[:k, :c], r)
            y = conv2d(x, w, stride)
            self.layers.append((name, k, c, r))
        return affine_act(y, self.w[name + ".scale"][:k], self.w[name + ".shift"][:k], act)

    def fc(self, name, g, k):
        c = g.shape[1]
        self.layers.append((name, k, c, 1))
        return linear(g, self.w[name + ".w"][:k, :c], self.w[name + ".b"][:k])


def forward(arch, wts, cfg, x, act_round=None, return_layers=False):
    """Logits [N, n_classes] (float32) of SubNet `cfg` on input x [N,3,res,res].

    wts: dict name -> full SuperNet tensor.  act_round: optional function applied to every
    stored activation (diagnostic: emulates a lower-precision activation store)."""
    assert check_cfg(arch, cfg), "invalid SubNet configuration"
    assert x.shape[2] == cfg.resolution and x.shape[3] == cfg.resolution
    run = _Run(wts, act_round)
    rd = run.round
    W, E, Kc = arch.width_choices, arch.expand_choices, arch.kernel_choices
    x = np.ascontiguousarray(x, dtype=np.float32)

    if arch.family == FAMILY_TINY:
        for l in range(cfg.depth[0]):
            x = rd(run.conv("conv%d" % l, x, ch(arch.stage_base_out[l] * W[cfg.width_idx[1 + l]]), 3, 1, ACT_RELU))
        logits = run.fc("fc", global_avg(x), arch.n_classes)

    elif arch.family == FAMILY_RESNET:
        w0 = W[cfg.width_idx[0]]
        mid, o = ch(arch.stem_mid * w0), ch(arch.stem_out * w0)
        x = rd(run.conv("stem0", x, mid, 3, 2, ACT_RELU))
        x = rd(run.conv("stem1", x, mid, 3, 1, ACT_RELU))
        x = rd(run.conv("stem2", x, o, 3, 1, ACT_RELU))
        x = maxpool3x3s2(x)
        for s in range(arch.n_stages):
            cout = ch(arch.stage_base_out[s] * W[cfg.width_idx[1 + s]])
            for j in range(cfg.depth[s]):
                n = "s%db%d" % (s, j)
                stride = arch.stage_stride[s] if j == 0 else 1
                cmid = ch(cout * E[cfg.expand_idx[arch.slot(s, j)]])
                h = rd(run.conv(n + ".conv1", x, cmid, 1, 1, ACT_RELU))
                h = rd(run.conv(n + ".conv2", h, cmid, 3, stride, ACT_RELU))
                h = run.conv(n + ".conv3", h, cout, 1, 1, ACT_NONE)
                if j == 0:
                    sc = rd(run.conv(n + ".proj", x, cout, 1, stride, ACT_NONE))
                else:
                    sc = x
                x = rd(activation(h + sc, ACT_RELU).astype(np.float32))
        logits = run.fc("fc", global_avg(x), arch.n_classes)

    elif arch.family == FAMILY_MBV3:
        c0 = arch.stem_out
        x = rd(run.conv("stem", x, c0, 3, 2, ACT_HSWISH))
        h = rd(run.conv("first.dw", x, c0, 3, 1, ACT_RELU, dw=True))
        x = rd((run.conv("first.pw", h, c0, 1, 1, ACT_NONE) + x).astype(np.float32))
        for s in range(arch.n_stages):
            cout = arch.stage_base_out[s]
            act = arch.stage_act[s]
            for j in range(cfg.depth[s]):
                n = "s%db%d" % (s, j)
                b = arch.slot(s, j)
                stride = arch.stage_stride[s] if j == 0 else 1
                cin = x.shape[1]
                cmid = ch(cin * E[cfg.expand_idx[b]])
                h = rd(run.conv(n + ".expand", x, cmid, 1, 1, act))
                h = rd(run.conv(n + ".dw", h, cmid, Kc[cfg.kernel_idx[b]], stride, act, dw=True))
                if arch.stage_se[s]:
                    red = ch(cmid / 4.0)
                    z = activation(run.fc(n + ".se1", global_avg(h), red), ACT_RELU)
                    gate = hsigmoid(run.fc(n + ".se2", z, cmid))
                    h = rd((h * gate[:, :, None, None]).astype(np.float32))
                y = run.conv(n + ".project", h, cout, 1, 1, ACT_NONE)
                if stride == 1 and cin == cout:
                    y = (y + x).astype(np.float32)
                x = rd(y)
        x = rd(run.conv("head", x, arch.head_mid, 1, 1, ACT_HSWISH))
        f = activation(run.fc("feat", global_avg(x), arch.head_feat), ACT_HSWISH)
        logits = run.fc("fc", f, arch.n_classes)
    else:
        raise ValueError("family")

    if return_layers:
        return logits, run.layers
    return logits


# ---------------------------------------------------------------- encodings and sizes

def encode_vector(arch, cfg):
    """The scheduler's vector [K_1, C_1, ..., K_N, C_N] over all N SuperNet layers
    (paper Section 3.3, 'Encoding SubGraph NN Architecture'); a skipped layer contributes (0, 0)."""
    v = []
    for (_, k, c, _) in active_layers(arch, cfg):
        v += [k, c]
    return v


def subnet_box(arch, cfg):
    """Per-layer (K, C, r) triples of the SubNet (the box of weights it touches)."""
    return [(k, c, r) for (_, k, c, r) in active_layers(arch, cfg)]


def weight_count(box):
    return sum(k * c * r * r for (k, c, r) in box)


def intersect(box_a, box_b):
    """Weights common to two prefix boxes: per layer the elementwise minimum."""
    return [(min(a[0], b[0]), min(a[1], b[1]), min(a[2], b[2])) if (a[0] and b[0]) else (0, 0, 0)
            for a, b in zip(box_a, box_b)]


def hit_ratio(vec_sn, vec_g):
    """Cache hit ratio ||SN ∩ G||_2 / ||SN||_2 on the [K,C] vectors (paper Appendix A.4)."""
    a = np.asarray(vec_sn, dtype=np.float64)
    b = np.asarray(vec_g, dtype=np.float64)
    return float(np.linalg.norm(np.minimum(a, b)) / np.linalg.norm(a))
