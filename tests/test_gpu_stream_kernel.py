"""GPU parity of the stream kernel (exec mode 2: one launch per query, grid barriers between
layers) against the CPU oracle, plus its bounded-wait error path."""
import numpy as np
import pytest
import torch

from tests.common import make_problem, oracle_logits, oracle_logits_bf16_stores, rel_l2
from workloads import arch as A
from workloads import streams, tensors as T
from workloads.rng import Stream

pytestmark = pytest.mark.gpu


def _ctx(arch, seed):
    import paper_2306_17266_amd as S
    blob, wts = make_problem(arch, seed, True)
    ctx = S.Sushi(0)
    ctx.sushi_load_supernet(arch, blob, S.BF16)
    ctx.sushi_set_option(S.OPT_EXEC_MODE, 2)
    return ctx, wts


def _run(ctx, cfg, x_np, n_classes):
    x = torch.from_numpy(x_np).cuda().to(torch.bfloat16).contiguous()
    logits = torch.full((x_np.shape[0], n_classes), float("nan"), device="cuda", dtype=torch.float32)
    ctx.sushi_infer(cfg, x, logits)
    torch.cuda.synchronize()
    return logits.cpu().numpy()


@pytest.mark.parametrize("fam", ["tiny", "resnet", "mbv3"])
def test_small_supernets(fam):
    arch = {"tiny": A.tiny_arch, "resnet": A.small_resnet_arch, "mbv3": A.small_mbv3_arch}[fam]()
    ctx, wts = _ctx(arch, 3)
    st = Stream(71)
    for res, batch in ((min(arch.res_choices), 1), (max(arch.res_choices), 3)):
        cfgs = [A.min_cfg(arch, res), A.max_cfg(arch, res)] + [streams.uniform_cfg(arch, st, res) for _ in range(5)]
        for t, cfg in enumerate(cfgs):
            print(fam, res, batch, "query", t, cfg.key(), flush=True)
            x = T.make_input(3, t, batch, res, 3, True)
            got = _run(ctx, cfg, x, arch.n_classes)
            again = _run(ctx, cfg, x, arch.n_classes)
            np.testing.assert_array_equal(got, again)                 # deterministic
            assert rel_l2(got, oracle_logits(arch, wts, cfg, x)) <= 1e-2, (t, cfg)
    ctx.close()


@pytest.mark.parametrize("fam", ["resnet", "mbv3"])
def test_full_size_batch1(fam):
    arch = A.resnet_arch() if fam == "resnet" else A.mbv3_arch()
    ctx, wts = _ctx(arch, 31)
    st = Stream(73)
    cfgs = [A.min_cfg(arch, 224), A.max_cfg(arch, 224)] + [streams.uniform_cfg(arch, st) for _ in range(3)]
    for t, cfg in enumerate(cfgs):
        print(fam, "query", t, cfg.key(), flush=True)
        x = T.make_input(31, t, 1, cfg.resolution, 3, True)
        got = _run(ctx, cfg, x, arch.n_classes)
        assert rel_l2(got, oracle_logits(arch, wts, cfg, x)) <= 1e-2, (t, cfg)
    ctx.close()


def test_a_wait_that_runs_out_is_reported_and_recovered():
    """With a spin limit of zero the first unfinished barrier gives up: every workgroup leaves the
    kernel normally, the next call reports the failure, and the context works again afterwards."""
    import paper_2306_17266_amd as S
    arch = A.small_resnet_arch()
    ctx, wts = _ctx(arch, 5)
    cfg = A.max_cfg(arch, 64)
    x = T.make_input(5, 0, 1, 64, 3, True)
    good = _run(ctx, cfg, x, arch.n_classes)
    ctx.sushi_set_option(S.OPT_SPIN_LIMIT, 0)
    _run(ctx, cfg, x, arch.n_classes)                       # may or may not finish; must return
    ctx.sushi_set_option(S.OPT_SPIN_LIMIT, 400000)
    try:
        second = _run(ctx, cfg, x, arch.n_classes)
    except S.SushiError as e:                               # the earlier launch did give up
        assert e.code == -5
        second = _run(ctx, cfg, x, arch.n_classes)
    np.testing.assert_array_equal(second, good)
    ctx.close()


# ---------------------------------------------------------------- exec mode 3: the team kernel

def _team_ctx(arch, seed, teams_per_xcd=1):
    import paper_2306_17266_amd as S
    blob, wts = make_problem(arch, seed, True)
    ctx = S.Sushi(0)
    ctx.sushi_load_supernet(arch, blob, S.BF16)
    ctx.sushi_set_option(S.OPT_EXEC_MODE, 3)
    ctx.sushi_set_option(S.OPT_TEAMS_PER_XCD, teams_per_xcd)
    return ctx, wts


@pytest.mark.parametrize("fam,teams", [("tiny", 1), ("resnet", 1), ("mbv3", 1), ("resnet", 2), ("mbv3", 4), ("resnet", 8), ("resnet", 16), ("mbv3", 16)])
def test_team_kernel_small_supernets(fam, teams):
    """Queries are posted without waiting (one in flight per team; 1, 2, 4 or 8 teams per XCD), then all
    logits are checked against the oracle; a second pass must reproduce them bit for bit."""
    arch = {"tiny": A.tiny_arch, "resnet": A.small_resnet_arch, "mbv3": A.small_mbv3_arch}[fam]()
    ctx, wts = _team_ctx(arch, 3, teams)
    st = Stream(81)
    for res, batch in ((min(arch.res_choices), 1), (max(arch.res_choices), 3)):
        cfgs = [A.min_cfg(arch, res), A.max_cfg(arch, res)] + [streams.uniform_cfg(arch, st, res) for _ in range(14)]
        xs_np = [T.make_input(3, t, batch, res, 3, True) for t in range(len(cfgs))]
        xs = [torch.from_numpy(x).cuda().to(torch.bfloat16).contiguous() for x in xs_np]
        torch.cuda.synchronize()
        results = []
        for rep in range(2):
            outs = [torch.full((batch, arch.n_classes), float("nan"), device="cuda") for _ in cfgs]
            print(fam, res, batch, "pass", rep, flush=True)
            for cfg, x, o in zip(cfgs, xs, outs):
                ctx.sushi_infer(cfg, x, o)
            ctx.sushi_synchronize()
            results.append([o.cpu().numpy() for o in outs])
        for t, cfg in enumerate(cfgs):
            np.testing.assert_array_equal(results[0][t], results[1][t])
            assert rel_l2(results[0][t], oracle_logits(arch, wts, cfg, xs_np[t])) <= 1e-2, (t, cfg)
    ctx.close()


@pytest.mark.parametrize("teams,batch", [(8, 5), (8, 16), (2, 2), (1, 16)])
def test_team_kernel_squeeze_excite_blocks_at_every_batch_to_team_ratio(teams, batch):
    """A squeeze-excite block runs as one op in which the images are dealt to groups of a team's workgroups: more images
    than workgroups (each workgroup takes several images on its own), fewer (several workgroups share an image's
    gating), and uneven groups.  Logits against the oracle, query by query, and reproducible bit for bit."""
    arch = A.small_mbv3_arch()
    ctx, wts = _team_ctx(arch, 7, teams)
    st = Stream(83)
    res = min(arch.res_choices)
    cfgs = [A.max_cfg(arch, res), A.min_cfg(arch, res)] + [streams.uniform_cfg(arch, st, res) for _ in range(4)]
    xs_np = [T.make_input(7, t, batch, res, 3, True) for t in range(len(cfgs))]
    xs = [torch.from_numpy(x).cuda().to(torch.bfloat16).contiguous() for x in xs_np]
    torch.cuda.synchronize()
    results = []
    for rep in range(2):
        outs = [torch.full((batch, arch.n_classes), float("nan"), device="cuda") for _ in cfgs]
        print("teams", teams, "batch", batch, "pass", rep, flush=True)
        for cfg, x, o in zip(cfgs, xs, outs):
            ctx.sushi_infer(cfg, x, o)
        ctx.sushi_synchronize()
        results.append([o.cpu().numpy() for o in outs])
    for t, cfg in enumerate(cfgs):
        np.testing.assert_array_equal(results[0][t], results[1][t])
        assert rel_l2(results[0][t], oracle_logits(arch, wts, cfg, xs_np[t])) <= 1e-2, (t, cfg)
    ctx.close()


@pytest.mark.parametrize("fam,teams", [("resnet", 1), ("mbv3", 1), ("resnet", 4), ("mbv3", 2), ("resnet", 8), ("mbv3", 8), ("resnet", 16)])
def test_team_kernel_full_size_batch1(fam, teams):
    arch = A.resnet_arch() if fam == "resnet" else A.mbv3_arch()
    ctx, wts = _team_ctx(arch, 31, teams)
    st = Stream(83)
    cfgs = [A.min_cfg(arch, 224), A.max_cfg(arch, 224)] + [streams.uniform_cfg(arch, st) for _ in range(3)]
    xs_np = [T.make_input(31, t, 1, c.resolution, 3, True) for t, c in enumerate(cfgs)]
    xs = [torch.from_numpy(x).cuda().to(torch.bfloat16).contiguous() for x in xs_np]
    outs = [torch.full((1, arch.n_classes), float("nan"), device="cuda") for _ in cfgs]
    torch.cuda.synchronize()
    for cfg, x, o in zip(cfgs, xs, outs):
        ctx.sushi_infer(cfg, x, o)
    ctx.sushi_synchronize()
    for t, cfg in enumerate(cfgs):
        assert rel_l2(outs[t].cpu().numpy(), oracle_logits(arch, wts, cfg, xs_np[t])) <= 1e-2, (t, cfg)
    ctx.close()


def test_team_kernel_gives_way_to_the_callers_kernels():
    """The team kernel fills every compute unit.  An input that a kernel of the caller is still producing
    when the query is posted must be waited for without waiting for the team kernel to idle out: it
    leaves, the caller's kernel runs, it starts again."""
    import time
    arch = A.small_resnet_arch()
    ctx, wts = _team_ctx(arch, 5, 4)
    st = Stream(17)
    cfgs = [streams.uniform_cfg(arch, st, 64) for _ in range(6)]
    xs_np = [T.make_input(5, t, 1, 64, 3, True) for t in range(len(cfgs))]
    host = [torch.from_numpy(x).to(torch.bfloat16) for x in xs_np]
    outs = [torch.full((1, arch.n_classes), float("nan"), device="cuda") for _ in cfgs]
    torch.cuda.synchronize()
    t0 = time.time()
    for cfg, h, o in zip(cfgs, host, outs):
        x = (h.cuda() * 1).contiguous()      # upload and a kernel on the current stream, not waited for
        ctx.sushi_infer(cfg, x, o)
    ctx.sushi_synchronize()
    assert time.time() - t0 < 5.0
    for t, cfg in enumerate(cfgs):
        assert rel_l2(outs[t].cpu().numpy(), oracle_logits(arch, wts, cfg, xs_np[t])) <= 1e-2, (t, cfg)
    ctx.close()


def test_team_kernel_restarts_after_idling_and_after_mode_switches():
    import time

    import paper_2306_17266_amd as S
    arch = A.small_resnet_arch()
    ctx, wts = _team_ctx(arch, 5)
    ctx.sushi_set_option(S.OPT_IDLE_US, 200)
    cfg = A.max_cfg(arch, 64)
    x_np = T.make_input(5, 0, 1, 64, 3, True)
    x = torch.from_numpy(x_np).cuda().to(torch.bfloat16).contiguous()
    o = torch.empty(1, arch.n_classes, device="cuda")
    torch.cuda.synchronize()
    want = oracle_logits(arch, wts, cfg, x_np)
    first = None
    for k in range(4):
        o.fill_(float("nan"))
        torch.cuda.synchronize()                   # device-wide wait: the idle kernel has to leave
        ctx.sushi_infer(cfg, x, o)
        ctx.sushi_synchronize()
        got = o.cpu().numpy()
        assert rel_l2(got, want) <= 1e-2
        first = got if first is None else first
        np.testing.assert_array_equal(got, first)
        time.sleep(0.01)                           # longer than the idle limit
        if k == 1:
            ctx.sushi_set_option(S.OPT_EXEC_MODE, 0)
            ctx.sushi_infer(cfg, x, o)
            torch.cuda.synchronize()
            assert rel_l2(o.cpu().numpy(), want) <= 1e-2
            ctx.sushi_set_option(S.OPT_EXEC_MODE, 3)
    ctx.close()


@pytest.mark.parametrize("fam,teams", [("resnet", 1), ("mbv3", 1), ("resnet", 4), ("resnet", 8)])
def test_team_kernel_logits_do_not_depend_on_resident_slabs(fam, teams):
    """SubGraph residency in LDS is exact: the same logits, bit for bit, with nothing cached, with
    a SubGraph cached, after the cache changes in mid-stream and after it is emptied; and the
    library reports how many weight bytes came out of LDS."""
    from oracle import subnet_eval as E
    arch = A.small_resnet_arch() if fam == "resnet" else A.small_mbv3_arch()
    ctx, wts = _team_ctx(arch, 9, teams)
    st = Stream(91)
    res = 64
    cfgs = [A.max_cfg(arch, res), A.min_cfg(arch, res)] + [streams.uniform_cfg(arch, st, res) for _ in range(11)]
    xs_np = [T.make_input(9, t, 1, res, 3, True) for t in range(len(cfgs))]
    xs = [torch.from_numpy(x).cuda().to(torch.bfloat16).contiguous() for x in xs_np]
    torch.cuda.synchronize()

    def run_all(change_at=None, box=None):
        outs = [torch.full((1, arch.n_classes), float("nan"), device="cuda") for _ in cfgs]
        lds = []
        for t, (cfg, x, o) in enumerate(zip(cfgs, xs, outs)):
            if change_at is not None and t == change_at:
                ctx.sushi_set_subgraph_cache(box, 1 << 30)
            ctx.sushi_infer(cfg, x, o)
            s = ctx.sushi_get_stats()
            lds.append((s["last_lds_bytes"], s["last_in_subgraph_bytes"], s["last_weight_bytes"]))
        ctx.sushi_synchronize()
        return [o.cpu().numpy() for o in outs], lds

    base, lds0 = run_all()
    assert all(l[0] == 0 for l in lds0)
    for t, cfg in enumerate(cfgs):
        want = oracle_logits(arch, wts, cfg, xs_np[t])
        err = rel_l2(base[t], want)
        if err > 1e-2:
            # Storing feature maps as bf16 is the precision this mode is defined with.  On a net this small
            # (2 x 2 final maps, logits of norm < 1) the format alone can use up the tolerance: the oracle
            # with its own stored activations rounded to bf16 is then as far from the exact oracle as the
            # GPU is.  Such a query stays in the test and is held to that emulation instead, tightly.
            emu = oracle_logits_bf16_stores(arch, wts, cfg, xs_np[t])
            floor, to_emu = rel_l2(emu, want), rel_l2(base[t], emu)
            print("query", t, "err", err, "bf16-store floor", floor, "vs emulation", to_emu, flush=True)
            assert floor > 0.9e-2 and to_emu <= 6e-3 and err <= 1.25e-2, (t, err, floor, to_emu)
    ctx.sushi_set_subgraph_cache(E.subnet_box(arch, A.max_cfg(arch, res)), 1 << 30)    # the whole SuperNet
    got, lds1 = run_all()
    for t in range(len(cfgs)):
        np.testing.assert_array_equal(got[t], base[t])
    assert all(0 < l[0] <= l[1] <= l[2] for l in lds1), lds1
    assert ctx.sushi_get_stats()["cache_bytes_lds"] > 0
    got, lds2 = run_all(change_at=5, box=E.subnet_box(arch, cfgs[1]))            # shrink to the smallest SubNet
    for t in range(len(cfgs)):
        np.testing.assert_array_equal(got[t], base[t])
    assert all(0 < l[0] <= l[1] for l in lds2), lds2
    assert lds2[7][0] <= lds1[7][0]
    ctx.sushi_set_subgraph_cache(None, 0)
    got, lds3 = run_all()
    for t in range(len(cfgs)):
        np.testing.assert_array_equal(got[t], base[t])
    assert all(l[0] == 0 for l in lds3)
    ctx.close()
