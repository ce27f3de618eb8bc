"""Pins for the reference SubNet evaluator (oracle/subnet_eval.py).

  1. the largest SubNet equals the whole SuperNet, evaluated by a separate straight-line
     routine written with torch CPU operators on the *unsliced* tensors;
  2. every SubNet's weights are exact slices: running the widest network of the same depth with
     everything outside the slice set to zero gives the same logits (zero-mask equivalence), and
     the slices the evaluator takes are literally W[:K', :C', o:o+r, o:o+r];
  3. elastic depth: a trailing block whose residual branch is switched off does not change the
     result, so dropping it (depth - 1) gives identical logits;
  4. structure of Section 2.1: the smallest SubNet's weights are in every SubNet, every SubNet
     is inside the largest.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import subnet_eval as E
from workloads import arch as A
from workloads import streams, tensors as T
from workloads.rng import Stream

ARCHS = {"tiny": A.tiny_arch, "resnet": A.small_resnet_arch, "mbv3": A.small_mbv3_arch}


def _weights(arch, seed=5, bf16=False):
    table = E.supernet_tensors(arch)
    return E.name_weights(arch, T.make_weights([(s, k) for _, s, k in table], seed, bf16))


def _input(cfg, seed=9, batch=2):
    return T.make_input(seed, 0, batch, cfg.resolution).transpose(0, 3, 1, 2).copy()


def _rel(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b))


# ---- 1. straight-line SuperNet with torch operators on the full tensors ----------------------

def _t(w, name):
    return torch.from_numpy(w[name]).double()


def _cba(w, name, x, stride, act, groups=1):
    wt = _t(w, name + ".w")
    y = F.conv2d(x, wt, stride=stride, padding=(wt.shape[-1] - 1) // 2, groups=groups)
    y = y * _t(w, name + ".scale")[None, :, None, None] + _t(w, name + ".shift")[None, :, None, None]
    return {A.ACT_NONE: lambda v: v, A.ACT_RELU: F.relu, A.ACT_HSWISH: F.hardswish}[act](y)


def _full_supernet_torch(arch, w, x):
    x = torch.from_numpy(x).double()
    if arch.family == A.FAMILY_TINY:
        for l in range(4):
            x = _cba(w, "conv%d" % l, x, 1, A.ACT_RELU)
        return (x.mean((2, 3)) @ _t(w, "fc.w").T + _t(w, "fc.b")).numpy()
    if arch.family == A.FAMILY_RESNET:
        x = _cba(w, "stem0", x, 2, A.ACT_RELU)
        x = _cba(w, "stem1", x, 1, A.ACT_RELU)
        x = _cba(w, "stem2", x, 1, A.ACT_RELU)
        x = F.max_pool2d(x, 3, 2, 1)
        for s in range(arch.n_stages):
            for j in range(arch.stage_max_depth[s]):
                n = "s%db%d" % (s, j)
                st = arch.stage_stride[s] if j == 0 else 1
                h = _cba(w, n + ".conv1", x, 1, A.ACT_RELU)
                h = _cba(w, n + ".conv2", h, st, A.ACT_RELU)
                h = _cba(w, n + ".conv3", h, 1, A.ACT_NONE)
                sc = _cba(w, n + ".proj", x, st, A.ACT_NONE) if j == 0 else x
                x = F.relu(h + sc)
        return (x.mean((2, 3)) @ _t(w, "fc.w").T + _t(w, "fc.b")).numpy()
    x = _cba(w, "stem", x, 2, A.ACT_HSWISH)
    h = _cba(w, "first.dw", x, 1, A.ACT_RELU, groups=x.shape[1])
    x = _cba(w, "first.pw", h, 1, A.ACT_NONE) + x
    for s in range(arch.n_stages):
        for j in range(arch.stage_max_depth[s]):
            n = "s%db%d" % (s, j)
            st = arch.stage_stride[s] if j == 0 else 1
            h = _cba(w, n + ".expand", x, 1, arch.stage_act[s])
            h = _cba(w, n + ".dw", h, st, arch.stage_act[s], groups=h.shape[1])
            if arch.stage_se[s]:
                z = F.relu(h.mean((2, 3)) @ _t(w, n + ".se1.w").T + _t(w, n + ".se1.b"))
                g = F.hardsigmoid(z @ _t(w, n + ".se2.w").T + _t(w, n + ".se2.b"))
                h = h * g[:, :, None, None]
            y = _cba(w, n + ".project", h, 1, A.ACT_NONE)
            x = y + x if (st == 1 and y.shape[1] == x.shape[1]) else y
    x = _cba(w, "head", x, 1, A.ACT_HSWISH)
    f = F.hardswish(x.mean((2, 3)) @ _t(w, "feat.w").T + _t(w, "feat.b"))
    return (f @ _t(w, "fc.w").T + _t(w, "fc.b")).numpy()


@pytest.mark.parametrize("fam", ["tiny", "resnet", "mbv3"])
def test_max_subnet_is_the_supernet(fam):
    arch = ARCHS[fam]()
    w = _weights(arch)
    cfg = A.max_cfg(arch, min(arch.res_choices))
    x = _input(cfg)
    got = E.forward(arch, w, cfg, x)
    want = _full_supernet_torch(arch, w, x)
    assert got.shape == want.shape == (2, arch.n_classes)
    assert _rel(got, want) < 2e-6
    # and the largest SubNet touches every weight of every tensor
    n_w = sum(int(np.prod(s)) for n, s, k in E.supernet_tensors(arch) if k in (T.KIND_CONV, T.KIND_DWCONV, T.KIND_FC))
    assert E.weight_count(E.subnet_box(arch, cfg)) == n_w


def test_max_subnet_is_the_supernet_full_size_mbv3():
    arch = A.mbv3_arch()
    w = _weights(arch)
    cfg = A.max_cfg(arch, 160)
    x = _input(cfg, batch=1)
    assert _rel(E.forward(arch, w, cfg, x), _full_supernet_torch(arch, w, x)) < 2e-6


# ---- 2. slices ------------------------------------------------------------------------------

def _masked_weights(arch, w, cfg):
    """Copy of the SuperNet with every weight, scale, shift and bias outside cfg's slice zeroed."""
    out = {k: np.zeros_like(v) for k, v in w.items()}
    for name, k, c, r in E.active_layers(arch, cfg):
        if k == 0:
            continue
        full = w[name + ".w"]
        if full.ndim == 4:
            R = full.shape[2]
            o = (R - r) // 2
            cc = 1 if full.shape[1] == 1 else c
            out[name + ".w"][:k, :cc, o:o + r, o:o + r] = full[:k, :cc, o:o + r, o:o + r]
            out[name + ".scale"][:k] = w[name + ".scale"][:k]
            out[name + ".shift"][:k] = w[name + ".shift"][:k]
        else:
            out[name + ".w"][:k, :c] = full[:k, :c]
            out[name + ".b"][:k] = w[name + ".b"][:k]
    return out


def _widest_same_depth(arch, cfg):
    m = A.max_cfg(arch, cfg.resolution)
    m.depth = list(cfg.depth)
    return m


@pytest.mark.parametrize("fam", ["tiny", "resnet", "mbv3"])
def test_zero_mask_equivalence(fam):
    arch = ARCHS[fam]()
    w = _weights(arch)
    st = Stream(1234)
    cfgs = [A.min_cfg(arch, min(arch.res_choices))] + \
        [streams.uniform_cfg(arch, st, min(arch.res_choices)) for _ in range(4)]
    for cfg in cfgs:
        x = _input(cfg, batch=1)
        sliced = E.forward(arch, w, cfg, x)
        masked = E.forward(arch, _masked_weights(arch, w, cfg), _widest_same_depth(arch, cfg), x)
        # MBV3's SE reduction width depends on the active mid width, so the widest net's SE
        # uses more (all-zero) rows: still the same function.
        assert _rel(sliced, masked) < 1e-6, cfg


def test_zero_mask_detects_a_wrong_crop():
    """The equivalence really depends on the centred crop: an off-centre crop breaks it."""
    arch = A.small_mbv3_arch()
    w = _weights(arch)
    cfg = A.min_cfg(arch, 64)              # kernel 3 everywhere, tensors are 7x7
    x = _input(cfg, batch=1)
    good = E.forward(arch, w, cfg, x)
    bad_w = dict(w)
    name = "s0b0.dw.w"
    bad_w[name] = np.roll(w[name], 1, axis=3)      # shifts which taps sit in the centre
    assert _rel(E.forward(arch, bad_w, cfg, x), good) > 1e-4


def test_slices_are_prefixes_and_centre_crops():
    wfull = np.arange(6 * 5 * 7 * 7, dtype=np.float32).reshape(6, 5, 7, 7)
    np.testing.assert_array_equal(E.centre_crop(wfull, 7), wfull)
    np.testing.assert_array_equal(E.centre_crop(wfull, 3), wfull[:, :, 2:5, 2:5])
    np.testing.assert_array_equal(E.centre_crop(wfull, 5), wfull[:, :, 1:6, 1:6])


@pytest.mark.parametrize("fam", ["tiny", "resnet", "mbv3"])
def test_forward_touches_exactly_the_listed_layers(fam):
    arch = ARCHS[fam]()
    w = _weights(arch)
    st = Stream(77)
    for _ in range(3):
        cfg = streams.uniform_cfg(arch, st, min(arch.res_choices))
        _, layers = E.forward(arch, w, cfg, _input(cfg, batch=1), return_layers=True)
        assert layers == [l for l in E.active_layers(arch, cfg) if l[1] > 0]
        names = [n for n, _, _, _ in E.active_layers(arch, cfg)]
        assert names == [n[:-2] for n, s, k in E.supernet_tensors(arch) if n.endswith(".w")]


# ---- 3. elastic depth -----------------------------------------------------------------------

def test_dropping_a_switched_off_block_changes_nothing():
    arch = A.small_resnet_arch()
    w = _weights(arch)
    cfg = A.max_cfg(arch, 64)
    x = _input(cfg, batch=1)
    w2 = dict(w)
    last = "s1b%d" % (arch.stage_max_depth[1] - 1)
    w2[last + ".conv3.scale"] = np.zeros_like(w[last + ".conv3.scale"])
    w2[last + ".conv3.shift"] = np.zeros_like(w[last + ".conv3.shift"])
    shallower = A.max_cfg(arch, 64)
    shallower.depth[1] -= 1
    # block output = relu(0 + x) = x because x is already a relu output
    np.testing.assert_array_equal(E.forward(arch, w2, cfg, x), E.forward(arch, w2, shallower, x))
    assert _rel(E.forward(arch, w, cfg, x), E.forward(arch, w, shallower, x)) > 1e-3

    arch = A.small_mbv3_arch()
    w = _weights(arch)
    cfg = A.max_cfg(arch, 64)
    x = _input(cfg, batch=1)
    w2 = dict(w)
    last = "s2b%d" % (arch.stage_max_depth[2] - 1)
    w2[last + ".project.scale"] = np.zeros_like(w[last + ".project.scale"])
    w2[last + ".project.shift"] = np.zeros_like(w[last + ".project.shift"])
    shallower = A.max_cfg(arch, 64)
    shallower.depth[2] -= 1
    np.testing.assert_array_equal(E.forward(arch, w2, cfg, x), E.forward(arch, w2, shallower, x))


# ---- 4. structure of the weight-shared SuperNet (Section 2.1) -------------------------------

@pytest.mark.parametrize("mk", [A.tiny_arch, A.resnet_arch, A.mbv3_arch])
def test_min_subnet_is_shared_and_max_contains_all(mk):
    arch = mk()
    res = max(arch.res_choices)
    bmin, bmax = E.subnet_box(arch, A.min_cfg(arch, res)), E.subnet_box(arch, A.max_cfg(arch, res))
    st = Stream(99)
    inter, union = bmax, bmin
    for _ in range(24):
        b = E.subnet_box(arch, streams.uniform_cfg(arch, st, res))
        assert E.intersect(b, bmin) == bmin          # smallest SubNet inside every SubNet
        assert E.intersect(b, bmax) == b             # every SubNet inside the largest
        inter = E.intersect(inter, b)
        union = [tuple(max(u, v) for u, v in zip(p, q)) for p, q in zip(union, b)]
    assert E.intersect(inter, bmin) == bmin
    assert E.intersect(union, bmax) == union


def test_full_size_weight_counts():
    """Sizes of the synthetic SuperNets (shape stand-ins for Section 5.1's SubNet size ranges:
    same order of magnitude at one byte per weight, not the same numbers)."""
    r, m = A.resnet_arch(), A.mbv3_arch()
    assert E.weight_count(E.subnet_box(r, A.max_cfg(r))) == 48037856
    assert E.weight_count(E.subnet_box(r, A.min_cfg(r))) == 6520648
    assert E.weight_count(E.subnet_box(m, A.max_cfg(m))) == 7613280
    assert E.weight_count(E.subnet_box(m, A.min_cfg(m))) == 3395856
    assert len(E.subnet_box(r, A.max_cfg(r))) == 62


def test_encoding_and_hit_ratio():
    arch = A.tiny_arch()
    cfg = A.SubnetCfg(32, [3], [0, 0, 2, 1, 0], [0] * 4, [0] * 4)     # widths 16, 32, 24; layer 3 skipped
    assert E.encode_vector(arch, cfg) == [16, 3, 32, 16, 24, 32, 0, 0, 10, 24]
    v = E.encode_vector(arch, cfg)
    assert E.hit_ratio(v, v) == 1.0                                   # G ⊇ SN  ->  1
    assert E.hit_ratio(v, [x + 5 for x in v]) == 1.0
    assert E.hit_ratio(v, [0] * len(v)) == 0.0                        # nothing cached -> 0
    g = [16, 3, 16, 16, 16, 16, 16, 16, 0, 0]
    want = np.sqrt(16 ** 2 + 9 + 16 ** 2 + 16 ** 2 + 16 ** 2 + 16 ** 2) / np.sqrt(sum(x * x for x in v))
    assert abs(E.hit_ratio(v, g) - want) < 1e-12
    box_g = [(16, 3, 3), (16, 16, 3), (16, 16, 3), (16, 16, 3), (0, 0, 0)]
    assert E.weight_count(E.intersect(E.subnet_box(arch, cfg), box_g)) == 16 * 3 * 9 + 2 * 16 * 16 * 9


def test_invalid_cfg_rejected():
    arch = A.resnet_arch()
    cfg = A.max_cfg(arch)
    assert E.check_cfg(arch, cfg)
    cfg.depth[2] = 7
    assert not E.check_cfg(arch, cfg)
    cfg = A.max_cfg(arch)
    cfg.expand_idx[3] = 3
    assert not E.check_cfg(arch, cfg)
    cfg = A.max_cfg(arch)
    cfg.resolution = 200
    assert not E.check_cfg(arch, cfg)
