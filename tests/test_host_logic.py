"""CPU-only checks of the library's host side: it loads, exports what include/sushi.h declares,
lists the same SuperNet tensors and SubNet slices as the oracle, and its scheduler takes exactly
the oracle scheduler's decisions.  No compute call is made."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2306_17266_amd as S
from oracle import subnet_eval as E
from oracle.sched_ref import STRICT_ACCURACY, STRICT_LATENCY, SchedRef
from paper_2306_17266_amd import binding
from workloads import arch as A
from workloads import streams
from workloads import tensors as T
from workloads.rng import Stream

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ALL_ARCHS = [A.tiny_arch, A.small_resnet_arch, A.small_mbv3_arch, A.resnet_arch, A.mbv3_arch]


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "sushi.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = sorted(set(re.findall(r"\b(sushi_[a-z_]+)\s*\(", header)))
    assert len(names) >= 12 and "sushi_infer" in names and "sushi_load_supernet" in names
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


@pytest.mark.parametrize("mk", ALL_ARCHS)
def test_tensor_table_and_slices_match_the_oracle(mk):
    arch = mk()
    assert S.sushi_describe_supernet(arch) == [(n, tuple(s), k) for n, s, k in E.supernet_tensors(arch)]
    st = Stream(5)
    cfgs = [A.min_cfg(arch), A.max_cfg(arch)] + [streams.uniform_cfg(arch, st) for _ in range(40)]
    for cfg in cfgs:
        assert S.sushi_subnet_layers(arch, cfg) == E.subnet_box(arch, cfg)


def test_invalid_subnets_are_rejected():
    arch = A.resnet_arch()
    for mutate in (lambda c: c.depth.__setitem__(2, 7), lambda c: c.depth.__setitem__(0, 1),
                   lambda c: c.expand_idx.__setitem__(3, 3), lambda c: c.width_idx.__setitem__(0, -1),
                   lambda c: setattr(c, "resolution", 200)):
        cfg = A.max_cfg(arch)
        mutate(cfg)
        assert not E.check_cfg(arch, cfg)
        with pytest.raises(S.SushiError) as e:
            S.sushi_subnet_layers(arch, cfg)
        assert e.value.code == -1
    bad = A.resnet_arch()
    bad.stage_base_out[1] = 4
    with pytest.raises(S.SushiError):
        S.sushi_describe_supernet(bad)


def test_host_only_context_refuses_device_work():
    ctx = S.Sushi(-1)
    with pytest.raises(S.SushiError) as e:
        ctx.sushi_load_supernet(A.tiny_arch(), np.zeros(29098, np.float32), S.FP32)
    assert e.value.code == -3
    with pytest.raises(S.SushiError) as e:
        ctx.sushi_sched_step(0.0, 0.0)
    assert e.value.code == -3
    ctx.close()


def _random_problem(seed, n, m, length):
    st = Stream(seed)
    v = [[8 * st.randint(9) for _ in range(length)] for _ in range(n)]
    g = [[8 * st.randint(9) for _ in range(length)] for _ in range(m)]
    acc = [float(np.float32(0.6 + 0.3 * st.next_uniform())) for _ in range(n)]
    table = [[float(np.float32(1.0 + 9.0 * st.next_uniform())) for _ in range(m + 1)] for _ in range(n)]
    return v, acc, g, table


@pytest.mark.parametrize("policy", [STRICT_ACCURACY, STRICT_LATENCY])
@pytest.mark.parametrize("Q", [1, 3, 8])
def test_scheduler_decisions_match_the_oracle_exactly(policy, Q):
    for seed in range(4):
        v, acc, g, table = _random_problem(seed, 7, 9, 12)
        for init in (-1, 2):
            ref = SchedRef(v, acc, g, table, Q, policy, init)
            ctx = S.Sushi(-1)
            ctx.sushi_sched_init(v, acc, g, table, Q, policy, init)
            st = Stream(1000 + seed)
            for _ in range(60):
                a_t = float(np.float32(0.55 + 0.4 * st.next_uniform()))
                l_t = float(np.float32(12.0 * st.next_uniform()))
                assert ctx.sushi_sched_step(a_t, l_t) == ref.step(a_t, l_t)
            ctx.close()


def _served_stream(name):
    """(arch, list of served SubnetCfg, Q) for the named-SubNet streams of configurations 1, 2, 3, 5."""
    if name == "cfg1":
        arch = A.tiny_arch()
        return arch, streams.stream_uniform(arch, 8, 1), 4
    if name == "cfg2":
        arch = A.resnet_arch()
        return arch, streams.stream_sticky(arch, 1000, 2), 8
    arch = A.mbv3_arch()
    pool = streams.subnet_pool(arch, 32, 3)
    if name == "cfg3":
        return arch, [pool[i] for i, _ in streams.stream_zipf(32, 1000, 3)], 10
    picks = streams.stream_zipf(32, 2000, 5, regime=500, resolutions=[160, 192, 224])
    return arch, [streams.with_resolution(pool[i], r) for i, r in picks], 10


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg5"])
def test_cache_choices_match_the_oracle_on_the_configured_streams(name):
    arch, cfgs, Q = _served_stream(name)
    distinct = {c.key(): c for c in cfgs}
    boxes = [E.subnet_box(arch, c) for c in list(distinct.values())[:40]]
    budget = 2 * 1024 * 1024 if arch.family != A.FAMILY_TINY else 16 * 1024
    cands = streams.candidate_subgraphs(boxes, budget, 2, 40)
    gvecs = [[v for (k, c, r) in b for v in (k, c)] for b in cands]
    assert len(gvecs) >= 2
    n = len(gvecs[0])
    dummy_v, dummy_acc = [[0] * n], [0.0]
    table = [[1.0] * (len(gvecs) + 1)]
    ref = SchedRef(dummy_v, dummy_acc, gvecs, table, Q, STRICT_LATENCY)
    ctx = S.Sushi(-1)
    ctx.sushi_sched_init(dummy_v, dummy_acc, gvecs, table, Q, S.STRICT_LATENCY)
    changes = 0
    for cfg in cfgs:
        vec_lib = [v for (k, c, r) in S.sushi_subnet_layers(arch, cfg) for v in (k, c)]
        vec_ref = E.encode_vector(arch, cfg)
        assert vec_lib == vec_ref
        a, b = ctx.sushi_sched_record(vec_lib), ref.record(vec_ref)
        assert a == b
        changes += a >= 0
    assert changes == len(cfgs) // Q
    ctx.close()


def test_latency_target_stream_matches_the_oracle():
    """Configuration 4's policy: latency targets drawn from 5 levels, STRICT_LATENCY, synthetic
    accuracies increasing with SubNet size, synthetic table."""
    arch = A.resnet_arch()
    pool = streams.subnet_pool(arch, 16, 4)
    boxes = [E.subnet_box(arch, c) for c in pool]
    sizes = [E.weight_count(b) for b in boxes]
    order = np.argsort(sizes)
    acc = [0.0] * 16
    for rank, i in enumerate(order):
        acc[i] = float(np.float32(0.70 + 0.01 * rank))
    cands = streams.candidate_subgraphs(boxes, 64 * 1024 * 1024, 2, 40)
    gvecs = [[v for (k, c, r) in b for v in (k, c)] for b in cands]
    vecs = [E.encode_vector(arch, c) for c in pool]
    table = [[float(np.float32(1e-6 * 2 * (sizes[i] - E.weight_count(E.intersect(boxes[i], g)) + 0.1 * sizes[i])))
              for g in cands] + [float(np.float32(1e-6 * 2 * 1.1 * sizes[i]))] for i in range(16)]
    lo, hi = min(r[-1] for r in table), max(r[-1] for r in table)
    levels = [float(np.float32(lo + (hi - lo) * k / 4)) for k in range(5)]
    ref = SchedRef(vecs, acc, gvecs, table, 8, STRICT_LATENCY)
    ctx = S.Sushi(-1)
    ctx.sushi_sched_init(vecs, acc, gvecs, table, 8, S.STRICT_LATENCY)
    served = set()
    for lv in streams.stream_levels(5, 2000, 4):
        got = ctx.sushi_sched_step(0.0, levels[lv])
        assert got == ref.step(0.0, levels[lv])
        served.add(got[0])
    assert len(served) >= 3
    ctx.close()


# ---------------------------------------------------------------- team-kernel tilings (host side of exec mode 3)

LDS_SCRATCH = 32 * 1024      # bytes of LDS scratch a unit variant may use
TILED_SHAPES = {(2, 1), (2, 2), (3, 1), (3, 2), (3, 4), (4, 1), (4, 2), (4, 4), (6, 1), (6, 2)}
RESIDENT_SHAPES = {(2, 1), (2, 2), (4, 1), (4, 2), (6, 1)}
SPLIT_SHAPES = {(2, 4), (1, 4), (2, 2), (1, 2), (4, 1), (2, 1), (1, 1)}
DW_ITEMS = 5


def _ceil(a, b):
    return -(-a // b)


def _check_team_op(op, team):
    """What the kernels assume of a tiling, restated from their unit layouts."""
    kind, wk, ft, pt = op["kind"], op["wk"], op["ft"], op["pt"]
    M = op["B"] * op["P"] * op["Q"]
    ptiles, ftiles = _ceil(M, 16), _ceil(op["K"], 16)
    nsteps = op["R"] * op["R"] * _ceil(op["C"], 32)
    assert 0 <= op["lds_bytes"] <= LDS_SCRATCH, op
    if kind == 6:                                             # a squeeze-excite block as one op
        # pooling partials [64 channel groups][8 pixel lanes * 8 + 8] floats, then the averages, the hidden vector, the gate
        assert op["C"] % 8 == 0 and op["C"] <= 1024 and op["K"] % 8 == 0 and op["K"] <= 256, op
        assert op["lds_bytes"] == (64 * 72 + 1024 + 256 + 1024) * 4, op
        return
    if kind == 7:
        assert op["lds_bytes"] == 0, op
        return
    if kind in (0, 4) and op["C"] % 8 == 0:                   # dense conv / FC on the matrix cores
        assert op["R"] * op["R"] <= 32 and nsteps + 1 <= 256, op
        if wk == 0:
            assert (ft, pt) in TILED_SHAPES and ptiles >= 8, op
            ks = 1 if pt >= 4 else 2
            pad = _ceil(nsteps, 3 * ks) * 3 * ks
            assert op["lds_bytes"] == 2 * ks * ft * 1024 + ft * 128 + (pad + 3 * ks) * 16, op
            assert op["n_p"] == _ceil(ptiles, 8 * pt) and op["n_units"] == _ceil(ftiles, ft) * op["n_p"], op
        elif wk == -3:
            assert (ft, pt) in RESIDENT_SHAPES and ptiles >= 8, op
            assert op["lds_bytes"] == nsteps * ft * 1024 + ft * 128 + _ceil(nsteps, 4) * 4 * 16, op
            assert op["n_p"] == _ceil(ptiles, 8 * pt) and op["n_units"] == _ceil(ftiles, ft) * op["n_p"], op
        else:
            assert wk in (1, 2, 4, 8) and (ft, pt) in SPLIT_SHAPES, op
            assert ft * pt <= 4 or wk in (1, 8), op
            assert pt <= ptiles or (pt == 4 and ptiles == 3), op
            if ptiles <= 4:
                assert ft <= 2, op                            # only such units can read resident slabs
            assert op["n_p"] == _ceil(ptiles, pt) and op["n_units"] == _ceil(ftiles, ft) * op["n_p"], op
    elif kind == 0:                                           # the stem (3 input channels)
        assert wk == -1 and op["R"] * op["R"] * op["C"] <= 64 and op["K"] <= 64, op
        rows_in = (pt - 1) * op["stride"] + op["R"]
        assert op["lds_bytes"] == rows_in * op["W"] * op["C"] * 2, op
        assert op["n_units"] == op["B"] * _ceil(op["P"], pt), op
    elif kind == 1:                                           # depthwise
        assert wk in (-2, -4) and op["R"] in (3, 5, 7) and op["stride"] in (1, 2) and op["K"] % 8 == 0, op
        if wk == -2:
            assert ft in (1, 2, 4) and 1 <= pt <= op["P"], op
            need = (_ceil(op["Q"], DW_ITEMS) * DW_ITEMS - 1) * op["stride"] + op["R"]
            wp = max(need, op["W"] + op["R"] - 1)
            rows_in = (pt - 1) * op["stride"] + op["R"]
            assert op["lds_bytes"] == op["R"] * op["R"] * ft * 32 + rows_in * wp * ft * 16, op
            assert op["n_units"] == op["B"] * _ceil(op["K"] // 8, ft) * _ceil(op["P"], pt), op


@pytest.mark.parametrize("mk", [A.small_resnet_arch, A.small_mbv3_arch, A.resnet_arch, A.mbv3_arch])
@pytest.mark.parametrize("team", [2, 4, 8, 16, 32])
def test_team_tilings_fit_the_kernels(mk, team):
    """Every op of sampled SubNets, at batch 1 and 16, gets a unit variant the kernels implement, unit
    counts that cover all tiles, and an LDS footprint (restated here from the kernels' layouts)
    within the 32 KiB scratch."""
    arch = mk()
    st = Stream(23)
    res = max(arch.res_choices)
    cfgs = [A.min_cfg(arch, min(arch.res_choices)), A.max_cfg(arch, res)] + [streams.uniform_cfg(arch, st) for _ in range(6)]
    seen = set()
    for batch in (1, 16):
        for cfg in cfgs:
            ops = S.sushi_team_plan(arch, cfg, batch, team)
            assert len(ops) >= 5
            for op in ops:
                _check_team_op(op, team)
                seen.add((op["kind"], op["wk"]))
    assert any(k in (0, 4) and w > 0 for k, w in seen)        # few-pixel layers use split units
    if mk in (A.small_mbv3_arch, A.mbv3_arch):                # every squeeze-excite block is one op plus three skipped slots
        kinds = [op["kind"] for op in S.sushi_team_plan(arch, cfgs[1], 1, team)]
        assert 6 in kinds and 5 not in kinds
        for i, k in enumerate(kinds):
            if k == 6:
                assert kinds[i + 1:i + 4] == [7, 7, 7]
        assert kinds.count(7) == 3 * kinds.count(6)
    if mk in (A.resnet_arch, A.mbv3_arch):
        assert (0, 0) in seen                                 # many-pixel layers use tiled units


def test_team_plan_rejects_bad_arguments():
    arch = A.small_resnet_arch()
    cfg = A.max_cfg(arch, max(arch.res_choices))
    for batch, team in ((0, 8), (1, 0), (1, 33)):
        with pytest.raises(S.SushiError):
            S.sushi_team_plan(arch, cfg, batch, team)


def test_frozen_latency_table_decisions_match_the_oracle():
    """Configuration 4 as the benchmark runs it: the latency table measured on the GPU and frozen to a file,
    synthetic accuracies that grow with SubNet size, five latency targets between the fastest and the slowest
    SubNet, Algorithm 1 with strict latency.  The library and the oracle scheduler read the same file and must
    take the same decisions (SubNet served, cache chosen, and when) on the whole 2000-query stream."""
    from paper_2306_17266_amd import sushiabs
    from workloads import configs
    wl = configs.build("resnet_bs16_levels")
    arch, pool = wl["arch"], wl["pool"]
    boxes = [S.sushi_subnet_layers(arch, c) for c in pool]
    cands = streams.candidate_subgraphs(boxes, wl["budget"], 2, 40)
    frozen = sushiabs.load_table(sushiabs.table_path("resnet_bs16_levels", wl["budget"], 1), len(pool), len(cands))
    assert frozen is not None, "the frozen table does not fit the serving pool and candidate set"
    table = frozen["table"]
    assert table.dtype == np.float32 and (table > 0).all()
    sizes = [streams.box_bytes(b, 2) for b in boxes]
    acc = [0.0] * len(pool)
    for rank, i in enumerate(sorted(range(len(pool)), key=lambda i: sizes[i])):
        acc[i] = float(np.float32(0.70 + 0.01 * rank))
    levels = sushiabs.latency_levels(table, wl["n_levels"])
    vecs = [E.encode_vector(arch, c) for c in pool]
    gvecs = [[v for (k, c, r) in b for v in (k, c)] for b in cands]
    ref = SchedRef(vecs, acc, gvecs, [[float(v) for v in row] for row in table], wl["Q"], STRICT_LATENCY)
    ctx = S.Sushi(-1)
    ctx.sushi_sched_init(vecs, acc, gvecs, table, wl["Q"], S.STRICT_LATENCY)
    served, changes = set(), 0
    for lv in wl["levels"]:
        got = ctx.sushi_sched_step(0.0, levels[lv])
        assert got == ref.step(0.0, levels[lv])
        served.add(got[0])
        changes += got[1] >= 0
    assert len(served) >= 3 and changes == len(wl["levels"]) // wl["Q"]
    ctx.close()


@pytest.mark.parametrize("mk", [A.small_resnet_arch, A.mbv3_arch, A.resnet_arch])
def test_subgraph_overlap_matches_the_oracle(mk):
    """Bytes inside SN ∩ G and the hit ratio of Appendix A.4 from the library's host-only helper against the
    oracle's intersect / weight_count / hit_ratio, for SubNets against shrunken SubGraphs and the empty one."""
    arch = mk()
    st = Stream(29)
    res = max(arch.res_choices)
    cfgs = [A.min_cfg(arch, res), A.max_cfg(arch, res)] + [streams.uniform_cfg(arch, st, res) for _ in range(6)]
    boxes = [E.subnet_box(arch, c) for c in cfgs]
    graphs = [streams.shrink_box(b, 1 << 20, 2) for b in boxes[:4]] + [boxes[1], [(0, 0, 0)] * len(boxes[0])]
    for cfg, sn in zip(cfgs, boxes):
        for g in graphs:
            total, common, hit = S.sushi_subgraph_overlap(sn, g, 2)
            assert total == 2 * E.weight_count(sn)
            assert common == 2 * E.weight_count(E.intersect(sn, g))
            want = E.hit_ratio(E.encode_vector(arch, cfg), [v for (k, c, r) in g for v in (k if k else 0, c if k else 0)])
            assert abs(hit - want) < 1e-12
    assert S.sushi_subgraph_overlap(boxes[0], boxes[1], 2)[2] == 1.0      # G ⊇ SN


# ---------------------------------------------------------------- weight packer (host side of sushi_load_supernet)

def _bf16_bits(a):
    """float32 -> bf16 bit patterns, round to nearest even (written here, not taken from the generators)."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return (((b + 0x7FFF + ((b >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)


@pytest.mark.parametrize("mk", [A.tiny_arch, A.small_resnet_arch, A.small_mbv3_arch])
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_packer_round_trip_and_slices_are_prefixes(mk, dtype):
    """Unpacking the packed image by the layout the header states gives back every weight bit for bit (bf16: rounded
    to nearest even); everything else in the image is zero; a SubNet's slice (K', C') of a dense layer is, per tap and
    channel group, the first K' * 8 elements of that group's run; a centred r x r crop of a depthwise layer is its
    first r * r taps."""
    arch = mk()
    table = S.sushi_describe_supernet(arch)
    tensors = T.make_weights([(s, k) for _, s, k in table], 77, False)       # (not pre-rounded: the packer rounds)
    img, layers = S.sushi_pack_supernet(arch, T.flatten(tensors), S.BF16 if dtype == "bf16" else S.FP32)
    conv = lambda a: _bf16_bits(a) if dtype == "bf16" else np.ascontiguousarray(a, dtype=np.float32)
    wts = [(n, t) for (n, _, k), t in zip(table, tensors) if k in (T.KIND_CONV, T.KIND_DWCONV, T.KIND_FC)]
    assert len(wts) == len(layers)
    covered = np.zeros(img.size, dtype=bool)
    st = Stream(5)
    for (name, w), L in zip(wts, layers):
        K, Cc, R, Kpad, CG, off = L["K"], L["C"], L["R"], L["Kpad"], L["CG"], L["offset"]
        assert Kpad % 16 == 0 and Kpad >= K and Kpad - K < 16, name
        w4 = w.reshape(K, Cc, R, R) if w.ndim != 2 else w.reshape(K, Cc, 1, 1)
        want = conv(w4)
        if L["depthwise"]:
            assert Cc == 1 and CG == 0, name
            block = img[off:off + R * R * Kpad].reshape(R * R, Kpad)
            covered[off:off + R * R * Kpad] = True
            assert not block[:, K:].any(), name
            for r in (3, 5, 7):
                if r > R:
                    break
                o = (R - r) // 2
                crop = want[:, 0, o:o + r, o:o + r].reshape(K, r * r)
                got = block[:r * r, :K].T                                 # [filter][first r*r taps]
                # the same values, tap for tap, in whatever order the ring layout lists them
                np.testing.assert_array_equal(np.sort(got, axis=1), np.sort(crop, axis=1), err_msg="%s crop %d" % (name, r))
            # and the full kernel tap by tap: every packed tap row is one (dr, ds) plane of the tensor, each used once
            planes = {want[:, 0, r, s].tobytes(): (r, s) for r in range(R) for s in range(R)}
            seen = {planes[block[t, :K].tobytes()] for t in range(R * R)}
            assert len(planes) == R * R and len(seen) == R * R, name
        else:
            assert CG == _ceil(Cc, 8), name
            n = R * R * CG * Kpad * 8
            block = img[off:off + n].reshape(R * R, CG, Kpad, 8)
            covered[off:off + n] = True
            full = np.zeros((R * R, CG * 8, Kpad), dtype=img.dtype)          # [tap][channel][filter]
            full[:, :Cc, :K] = want.reshape(K, Cc, R * R).transpose(2, 1, 0)
            np.testing.assert_array_equal(block, full.reshape(R * R, CG, 8, Kpad).transpose(0, 1, 3, 2), err_msg=name)
            # a slice as the kernels address it: per (tap, group) one run of K' * 8 elements from the group's start
            for _ in range(3):
                k1 = 1 + st.randint(K)
                c1 = 8 * (1 + st.randint(max(1, Cc // 8))) if Cc >= 8 else Cc
                c1 = min(c1, Cc)
                flat = img[off:off + n]
                for tap in range(R * R):
                    for g in range(_ceil(c1, 8)):
                        start = ((tap * CG + g) * Kpad) * 8
                        run = flat[start:start + k1 * 8].reshape(k1, 8)
                        ch = min(8, Cc - g * 8)
                        np.testing.assert_array_equal(run[:, :ch], want.reshape(K, Cc, R * R)[:k1, g * 8:g * 8 + ch, tap])
    assert not img[~covered].any()                                          # gaps between layers
