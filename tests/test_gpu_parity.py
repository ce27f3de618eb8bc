"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, same seeded inputs.

Tolerances (relative L2 on the logits of one query): 1e-4 in float32 mode, 1e-2 in bf16 mode.
bf16 mode: both sides use the same bf16-rounded weights and inputs; the oracle computes in
float32/double, the GPU stores bf16 activations and accumulates in float32.
"""
import numpy as np
import pytest
import torch

from oracle import subnet_eval as E
from tests.common import make_problem, oracle_logits, rel_l2
from workloads import arch as A
from workloads import streams, tensors as T
from workloads.rng import Stream

pytestmark = pytest.mark.gpu

TOL = {False: 1e-4, True: 1e-2}


def _ctx(arch, seed, bf16):
    import paper_2306_17266_amd as S
    blob, wts = make_problem(arch, seed, bf16)
    ctx = S.Sushi(0)
    ctx.sushi_load_supernet(arch, blob, S.BF16 if bf16 else S.FP32)
    return ctx, wts


def _run(ctx, cfg, x_np, bf16, n_classes):
    x = torch.from_numpy(x_np).cuda()
    if bf16:
        x = x.to(torch.bfloat16)
    logits = torch.full((x_np.shape[0], n_classes), float("nan"), device="cuda", dtype=torch.float32)
    ctx.sushi_infer(cfg, x.contiguous(), logits)
    torch.cuda.synchronize()
    return logits.cpu().numpy()


def _check_stream(arch, cfgs, bf16, seed, batch=1):
    ctx, wts = _ctx(arch, seed, bf16)
    worst = 0.0
    for t, cfg in enumerate(cfgs):
        x = T.make_input(seed, t, batch, cfg.resolution, arch.in_channels, bf16)
        print("query", t, "cfg", cfg.key(), flush=True)
        got = _run(ctx, cfg, x, bf16, arch.n_classes)
        want = oracle_logits(arch, wts, cfg, x)
        assert np.isfinite(got).all()
        err = rel_l2(got, want)
        worst = max(worst, err)
        assert err <= TOL[bf16], (t, err, cfg)
    ctx.close()
    return worst


def test_config1_tiny_stream_fp32():
    """Configuration 1: Tiny SuperNet, 8 uniformly random SubNets, float32, cache = leading 16
    channels of every layer; every query checked."""
    import paper_2306_17266_amd as S
    arch = A.tiny_arch()
    ctx, wts = _ctx(arch, 1, False)
    box = [(16, 3, 3), (16, 16, 3), (16, 16, 3), (16, 16, 3), (0, 0, 0)]
    ctx.sushi_set_subgraph_cache(box, 16 * 1024 * 1024)
    cfgs = streams.stream_uniform(arch, 8, 1)
    for t, cfg in enumerate(cfgs):
        x = T.make_input(1, t, 1, 32)
        got = _run(ctx, cfg, x, False, 10)
        want = oracle_logits(arch, wts, cfg, x)
        assert rel_l2(got, want) <= 1e-4, (t, cfg)
        st = ctx.sushi_get_stats()
        sn = E.subnet_box(arch, cfg)
        assert st["last_weight_bytes"] == 4 * E.weight_count(sn)
        assert st["last_in_subgraph_bytes"] == 4 * E.weight_count(E.intersect(sn, box))
        assert abs(st["last_hit_ratio"] - E.hit_ratio(E.encode_vector(arch, cfg),
                                                      [v for (k, c, r) in box for v in (k, c)])) < 1e-12
    assert ctx.sushi_get_stats()["queries"] == 8
    ctx.close()


@pytest.mark.parametrize("bf16", [False, True])
def test_tiny_all_depths_and_batches(bf16):
    arch = A.tiny_arch()
    st = Stream(3)
    cfgs = [A.min_cfg(arch), A.max_cfg(arch)] + [streams.uniform_cfg(arch, st) for _ in range(6)]
    for batch in (1, 3):
        _check_stream(arch, cfgs, bf16, 11, batch)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("fam", ["resnet", "mbv3"])
def test_small_supernets(fam, bf16):
    """Shrunken bottleneck / inverted-residual SuperNets: many SubNets, two resolutions, ragged
    batch; spans several tiles and ragged tails in every kernel."""
    arch = A.small_resnet_arch() if fam == "resnet" else A.small_mbv3_arch()
    st = Stream(17)
    for res, batch in ((64, 1), (96, 3)):
        cfgs = [A.min_cfg(arch, res), A.max_cfg(arch, res)] + [streams.uniform_cfg(arch, st, res) for _ in range(5)]
        worst = _check_stream(arch, cfgs, bf16, 23, batch)
        print(fam, bf16, res, batch, "worst rel err", worst)


@pytest.mark.parametrize("fam", ["resnet", "mbv3"])
def test_full_size_bf16_batch1(fam):
    """The benchmarked shapes: full-size SuperNets, bf16, batch 1, smallest / largest / random SubNets."""
    arch = A.resnet_arch() if fam == "resnet" else A.mbv3_arch()
    st = Stream(29)
    res = 224
    cfgs = [A.min_cfg(arch, res), A.max_cfg(arch, res)] + [streams.uniform_cfg(arch, st, res) for _ in range(3)]
    worst = _check_stream(arch, cfgs, True, 31, 1)
    print(fam, "worst rel err", worst)


def test_mbv3_resolutions_bf16():
    arch = A.mbv3_arch()
    st = Stream(37)
    cfgs = [streams.uniform_cfg(arch, st, r) for r in (160, 192, 224)]
    _check_stream(arch, cfgs, True, 41, 1)


def test_resnet_full_size_batch16_sampled():
    """Configuration 4's shape (batch 16): the smallest SubNet and one random SubNet, all 16 images."""
    arch = A.resnet_arch()
    st = Stream(43)
    cfgs = [A.min_cfg(arch, 224), streams.uniform_cfg(arch, st, 224)]
    _check_stream(arch, cfgs, True, 47, 16)


@pytest.mark.parametrize("fam", ["tiny", "resnet", "mbv3"])
def test_patch_conv_kernel_on_every_layer_it_covers(fam):
    """The large-batch dense conv kernel (input patch in LDS) forced onto every 1x1 / 3x3 layer it supports,
    whatever the pixel count: ragged tiles (pixel counts that are no multiple of 128, tiles that cross rows and
    images), filter counts that are no multiple of 32, both strides, residuals, with and without activation.
    Checked against the oracle, and the same queries with the kernel switched off stay within tolerance too."""
    import paper_2306_17266_amd as S
    arch = {"tiny": A.tiny_arch, "resnet": A.small_resnet_arch, "mbv3": A.small_mbv3_arch}[fam]()
    ctx, wts = _ctx(arch, 67, True)
    st = Stream(71)
    for res, batch in ((64, 1), (64, 5), (96, 3)) if fam != "tiny" else ((32, 1), (32, 7)):
        cfgs = [A.min_cfg(arch, res), A.max_cfg(arch, res)] + [streams.uniform_cfg(arch, st, res) for _ in range(3)]
        for t, cfg in enumerate(cfgs):
            x = T.make_input(67, t, batch, cfg.resolution, arch.in_channels, True)
            want = oracle_logits(arch, wts, cfg, x)
            for min_pixels in (1, 0):
                ctx.sushi_set_option(S.OPT_PATCH_CONV_MIN_PIXELS, min_pixels)
                print(fam, "res", res, "batch", batch, "query", t, "patch kernel from", min_pixels, "pixels", flush=True)
                got = _run(ctx, cfg, x, True, arch.n_classes)
                assert np.isfinite(got).all()
                assert rel_l2(got, want) <= 1e-2, (fam, res, batch, t, min_pixels, rel_l2(got, want))
    ctx.sushi_set_option(S.OPT_KERNEL_TIMING, 1)
    ctx.sushi_set_option(S.OPT_PATCH_CONV_MIN_PIXELS, 1)
    r0 = arch.res_choices[0]
    _run(ctx, A.max_cfg(arch, r0), T.make_input(67, 0, 2, r0, arch.in_channels, True), True, arch.n_classes)
    used = {k["name"]: k["launches"] for k in ctx.sushi_get_kernel_stats()}
    assert used["conv_patch_kernel"] > 0, used
    ctx.close()


def test_logits_do_not_depend_on_the_cache_state():
    """SGS is exact: identical logits with nothing cached, with a SubGraph cached, and across a
    cache change in mid-stream."""
    arch = A.small_resnet_arch()
    ctx, wts = _ctx(arch, 5, True)
    st = Stream(53)
    cfgs = [streams.uniform_cfg(arch, st, 64) for _ in range(6)]
    xs = [T.make_input(5, t, 2, 64, 3, True) for t in range(6)]
    base = [_run(ctx, c, x, True, arch.n_classes) for c, x in zip(cfgs, xs)]
    boxes = [E.subnet_box(arch, A.min_cfg(arch, 64)), E.subnet_box(arch, cfgs[2])]
    ctx.sushi_set_subgraph_cache(boxes[0], 1 << 30)
    for t in range(6):
        if t == 3:
            ctx.sushi_set_subgraph_cache(boxes[1], 1 << 30)
        got = _run(ctx, cfgs[t], xs[t], True, arch.n_classes)
        np.testing.assert_array_equal(got, base[t])
    ctx.sushi_set_subgraph_cache(None, 0)
    np.testing.assert_array_equal(_run(ctx, cfgs[0], xs[0], True, arch.n_classes), base[0])
    ctx.close()


def test_errors_are_reported_not_raised_in_c():
    import paper_2306_17266_amd as S
    arch = A.tiny_arch()
    ctx = S.Sushi(0)
    x = torch.zeros(1, 32, 32, 3, device="cuda")
    y = torch.zeros(1, 10, device="cuda")
    with pytest.raises(S.SushiError) as e:
        ctx.sushi_infer(A.max_cfg(arch), x, y)
    assert e.value.code == -3                                  # before load
    blob, _ = make_problem(arch, 1, False)
    with pytest.raises(S.SushiError) as e:
        ctx.sushi_load_supernet(arch, blob[:-1], S.FP32)
    assert e.value.code == -1
    ctx.sushi_load_supernet(arch, blob, S.FP32)
    bad = A.max_cfg(arch)
    bad.depth = [1]
    with pytest.raises(S.SushiError) as e:
        ctx.sushi_infer(bad, x, y)
    assert e.value.code == -1
    with pytest.raises(S.SushiError) as e:
        ctx.sushi_set_subgraph_cache([(16, 3, 3), (16, 16, 3), (16, 16, 3), (16, 16, 3), (0, 0, 0)], 100)
    assert e.value.code == -4                                  # over budget
    with pytest.raises(S.SushiError) as e:
        ctx.sushi_set_subgraph_cache([(64, 3, 3), (16, 16, 3), (16, 16, 3), (16, 16, 3), (0, 0, 0)], 1 << 30)
    assert e.value.code == -1                                  # outside the SuperNet
    ctx.close()


def test_graph_replay_matches_eager_every_time():
    """Exec mode 1 replays a recorded HIP graph per SubNet.  Several replays, with eager work and
    synchronisations in between, different inputs in the same buffer, all equal to eager results."""
    import paper_2306_17266_amd as S
    arch = A.small_mbv3_arch()
    ctx, wts = _ctx(arch, 7, True)
    st = Stream(61)
    cfgs = [streams.uniform_cfg(arch, st, 64) for _ in range(3)]
    xbuf = torch.empty(2, 64, 64, 3, device="cuda", dtype=torch.bfloat16)
    out = torch.empty(2, arch.n_classes, device="cuda", dtype=torch.float32)
    eager = {}
    for t in range(9):
        x = torch.from_numpy(T.make_input(7, t, 2, 64, 3, True)).cuda().to(torch.bfloat16)
        xbuf.copy_(x)
        ctx.sushi_infer(cfgs[t % 3], xbuf, out)
        torch.cuda.synchronize()
        eager[t] = out.cpu().numpy().copy()
    ctx.sushi_set_option(S.OPT_EXEC_MODE, 1)
    for rep in range(2):
        for t in range(9):
            x = torch.from_numpy(T.make_input(7, t, 2, 64, 3, True)).cuda().to(torch.bfloat16)
            xbuf.copy_(x)
            out.fill_(float("nan"))
            ctx.sushi_infer(cfgs[t % 3], xbuf, out)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(out.cpu().numpy(), eager[t])
            (xbuf.float().sum() + out.sum()).item()          # unrelated eager work between replays
    # a different output buffer forces a re-record
    out2 = torch.empty_like(out)
    xbuf.copy_(torch.from_numpy(T.make_input(7, 4, 2, 64, 3, True)).cuda().to(torch.bfloat16))
    ctx.sushi_infer(cfgs[4 % 3], xbuf, out2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out2.cpu().numpy(), eager[4])
    want = oracle_logits(arch, wts, cfgs[1], T.make_input(7, 4, 2, 64, 3, True))
    assert rel_l2(out2.cpu().numpy(), want) <= 1e-2
    ctx.close()
