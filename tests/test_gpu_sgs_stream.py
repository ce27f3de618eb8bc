"""GPU parity of the configuration the benchmark times: full-size SuperNets in exec mode 3 (the
persistent XCD-team kernel) with the scheduler choosing the cached SubGraph every Q queries, so that
installs land between queries that are still in flight.

Every distinct SubNet of the stream's first queries is compared with the CPU oracle (relative L2 of
the logits <= 1e-2, bf16 mode), and the whole stream must give the same logits, bit for bit, with
SubGraph caching switched off (Section 4.3: keeping the common SubGraph on chip changes where
weights come from, never the result)."""
import numpy as np
import pytest
import torch

from tests.common import make_problem, oracle_logits, rel_l2
from workloads import arch as A
from workloads import configs, streams, tensors as T

pytestmark = pytest.mark.gpu

_oracle_cache = {}


def _want(tag, arch, wts, cfg, seed, t, batch):
    """Oracle logits of (cfg, input t), computed once per test session."""
    key = (tag, cfg.key(), seed, t, batch)
    if key not in _oracle_cache:
        x = T.make_input(seed, t, batch, cfg.resolution, arch.in_channels, True)
        _oracle_cache[key] = oracle_logits(arch, wts, cfg, x)
    return _oracle_cache[key]


def _team_ctx(arch, seed, teams_per_xcd):
    import paper_2306_17266_amd as S
    blob, wts = make_problem(arch, seed, True)
    ctx = S.Sushi(0)
    ctx.sushi_load_supernet(arch, blob, S.BF16)
    ctx.sushi_set_option(S.OPT_EXEC_MODE, 3)
    ctx.sushi_set_option(S.OPT_TEAMS_PER_XCD, teams_per_xcd)
    return ctx, wts


def _drive(ctx, arch, cfgs, xs, n_classes, Q, budget, sgs):
    """The benchmark's step loop: infer, account the served vector, enact a changed cache choice."""
    import paper_2306_17266_amd as S
    distinct = {}
    for c in cfgs:
        distinct.setdefault(c.key(), c)
    box_of = {k: S.sushi_subnet_layers(arch, c) for k, c in distinct.items()}
    vec_of = {k: np.array([v for (kk, cc, r) in b for v in (kk, cc)], dtype=np.int32) for k, b in box_of.items()}
    cands = streams.candidate_subgraphs(list(box_of.values()), budget, 2, 40)
    gvecs = [[v for (k, c, r) in b for v in (k, c)] for b in cands]
    n = len(gvecs[0])
    ctx.sushi_sched_init([[0] * n], [0.0], gvecs, [[1.0] * (len(gvecs) + 1)], Q, S.STRICT_LATENCY)
    ctx.sushi_set_subgraph_cache(None, 0)
    outs = [torch.full((x.shape[0], n_classes), float("nan"), device="cuda") for x in xs]
    cache, installs = -1, 0
    for cfg, x, o in zip(cfgs, xs, outs):
        ctx.sushi_infer(cfg, x, o)
        j = ctx.sushi_sched_record(vec_of[cfg.key()])
        if sgs and j >= 0 and j != cache:
            ctx.sushi_set_subgraph_cache(cands[j], budget)
            cache, installs = j, installs + 1
    ctx.sushi_synchronize()
    return [o.cpu().numpy() for o in outs], installs


@pytest.mark.parametrize("workload,teams", [("resnet_bs1_sticky", 16), ("mbv3_bs1_zipf", 16),
                                            ("resnet_bs1_sticky", 8), ("mbv3_bs1_zipf", 8),
                                            ("resnet_bs1_sticky", 1), ("mbv3_bs1_zipf", 1)])
def test_full_size_stream_with_scheduler_driven_installs(workload, teams):
    wl = configs.build(workload)
    arch, seed, n_q = wl["arch"], 31, 64
    cfgs = wl["cfgs"][:n_q]
    ctx, wts = _team_ctx(arch, seed, teams)
    xs_np = [T.make_input(seed, t, 1, c.resolution, 3, True) for t, c in enumerate(cfgs)]
    xs = [torch.from_numpy(x).cuda().to(torch.bfloat16).contiguous() for x in xs_np]
    torch.cuda.synchronize()
    print(workload, teams, "stream with caching", flush=True)
    on, installs = _drive(ctx, arch, cfgs, xs, arch.n_classes, wl["Q"], wl["budget"], True)
    stats = ctx.sushi_get_stats()
    assert installs >= 2 and stats["cache_installs"] == installs
    assert stats["weight_bytes_lds"] > 0                          # some queries did read resident slabs
    print(workload, teams, "stream without caching", flush=True)
    off, none = _drive(ctx, arch, cfgs, xs, arch.n_classes, wl["Q"], wl["budget"], False)
    assert none == 0
    for t in range(n_q):
        np.testing.assert_array_equal(on[t], off[t], err_msg="query %d" % t)
    seen = set()
    for t, cfg in enumerate(cfgs):
        if cfg.key() in seen:
            continue
        seen.add(cfg.key())
        print(workload, teams, "oracle for query", t, flush=True)
        err = rel_l2(on[t], _want(workload, arch, wts, cfg, seed, t, 1))
        assert err <= 1e-2, (t, err, cfg)
    assert len(seen) >= 5
    ctx.close()


@pytest.mark.parametrize("teams", [1, 8])
def test_full_size_batch16_in_the_team_kernel(teams):
    """Configuration 4's shape in the mode its benchmark runs: batch 16, smallest SubNet and one random
    SubNet of the serving pool, a SubGraph of the 64 MiB budget cached."""
    import paper_2306_17266_amd as S
    wl = configs.build("resnet_bs16_levels")
    arch, seed = wl["arch"], 47
    pool = wl["pool"]
    cfgs = [A.min_cfg(arch, 224), pool[5]]
    ctx, wts = _team_ctx(arch, seed, teams)
    box = streams.shrink_box(S.sushi_subnet_layers(arch, pool[3]), wl["budget"], 2)
    ctx.sushi_set_subgraph_cache(box, wl["budget"])
    xs_np = [T.make_input(seed, t, 16, 224, 3, True) for t in range(len(cfgs))]
    xs = [torch.from_numpy(x).cuda().to(torch.bfloat16).contiguous() for x in xs_np]
    outs = [torch.full((16, arch.n_classes), float("nan"), device="cuda") for _ in cfgs]
    torch.cuda.synchronize()
    for cfg, x, o in zip(cfgs, xs, outs):
        ctx.sushi_infer(cfg, x, o)
    ctx.sushi_synchronize()
    for t, cfg in enumerate(cfgs):
        print("batch 16, teams", teams, "oracle for query", t, flush=True)
        err = rel_l2(outs[t].cpu().numpy(), _want("bs16", arch, wts, cfg, seed, t, 16))
        assert err <= 1e-2, (t, err, cfg)
    ctx.close()


def test_resolution_stream_with_cache_changes():
    """A sample of configuration 5: per-query resolutions 160 / 192 / 224, the cache re-chosen every 10
    queries under the 4 MiB budget, sixteen teams per XCD (the benchmark's default at batch 1)."""
    wl = configs.build("mbv3_bs1_regimes")
    arch, seed, n_q = wl["arch"], 41, 60
    cfgs = wl["cfgs"][:n_q]
    assert {c.resolution for c in cfgs} == {160, 192, 224}
    ctx, wts = _team_ctx(arch, seed, 16)
    xs_np = [T.make_input(seed, t, 1, c.resolution, 3, True) for t, c in enumerate(cfgs)]
    xs = [torch.from_numpy(x).cuda().to(torch.bfloat16).contiguous() for x in xs_np]
    torch.cuda.synchronize()
    on, installs = _drive(ctx, arch, cfgs, xs, arch.n_classes, wl["Q"], wl["budget"], True)
    assert installs >= 2
    off, _ = _drive(ctx, arch, cfgs, xs, arch.n_classes, wl["Q"], wl["budget"], False)
    seen = set()
    for t, cfg in enumerate(cfgs):
        np.testing.assert_array_equal(on[t], off[t], err_msg="query %d" % t)
        if cfg.key() in seen:
            continue
        seen.add(cfg.key())
        print("config 5 sample: oracle for query", t, "resolution", cfg.resolution, flush=True)
        err = rel_l2(on[t], _want("cfg5", arch, wts, cfg, seed, t, 1))
        assert err <= 1e-2, (t, err, cfg)
    ctx.close()


def test_a_larger_supernet_loaded_into_a_used_context():
    """Loading another SuperNet into a context that has served queries in mode 3 re-sizes the per-team
    activation arenas: the shrunken net first, then the full-size one, both checked."""
    import paper_2306_17266_amd as S
    small, big = A.small_resnet_arch(), A.resnet_arch()
    blob_s, wts_s = make_problem(small, 5, True)
    blob_b, wts_b = make_problem(big, 31, True)
    ctx = S.Sushi(0)
    ctx.sushi_set_option(S.OPT_EXEC_MODE, 3)
    ctx.sushi_set_option(S.OPT_TEAMS_PER_XCD, 8)
    for arch, blob, wts, seed, res in ((small, blob_s, wts_s, 5, 64), (big, blob_b, wts_b, 31, 224), (small, blob_s, wts_s, 5, 96)):
        ctx.sushi_load_supernet(arch, blob, S.BF16)
        cfgs = [A.max_cfg(arch, res), A.min_cfg(arch, res)] * 8       # every team of an XCD gets work
        xs_np = [T.make_input(seed, t, 1, res, 3, True) for t in range(len(cfgs))]
        xs = [torch.from_numpy(x).cuda().to(torch.bfloat16).contiguous() for x in xs_np]
        outs = [torch.full((1, arch.n_classes), float("nan"), device="cuda") for _ in cfgs]
        torch.cuda.synchronize()
        for cfg, x, o in zip(cfgs, xs, outs):
            ctx.sushi_infer(cfg, x, o)
        ctx.sushi_synchronize()
        for t in (0, 1, 14, 15):
            print("reload test:", arch.stage_base_out[-1], "query", t, flush=True)
            tag = "reload%d" % arch.stage_base_out[-1]
            if arch is big:
                tag = "resnet_bs1_reload"
            err = rel_l2(outs[t].cpu().numpy(), _want(tag, arch, wts, cfgs[t], seed, t, 1))
            assert err <= 1e-2, (arch.stage_base_out, t, err)
    ctx.close()
