"""Per-op report of one SubNet inside the persistent team kernel (exec mode 3) with every team of the chip busy.

    python -m paper_2306_17266_amd.team_report --workload resnet_bs1_sticky --teams-per-xcd 8 --subnet 0

Every team runs the same SubNet over and over; the team leaders stamp a 100 MHz clock after the barrier of
every op (sushi_team_trace).  The report lists, per op of the plan, the unit variant and tiling the library
chose, the mean duration over all teams, the op's algorithmic bytes, and the fraction of the op's own bound on
the team's share of the chip: max(bytes / (HBM peak / teams), flops / (MFMA peak / teams)).
"""
import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_GBS, MFMA_TFLOPS = 8000.0, 2500.0
KIND = {0: "conv", 1: "dwconv", 2: "maxpool", 3: "gap", 4: "fc", 5: "gate", 6: "se", 7: "(fused)"}


def main():
    import torch

    import paper_2306_17266_amd as S
    from paper_2306_17266_amd.layer_report import op_cost
    from workloads import arch as A
    from workloads import configs
    from workloads import tensors as T
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet_bs1_sticky")
    ap.add_argument("--teams-per-xcd", type=int, default=8, choices=[1, 2, 4, 8, 16])
    ap.add_argument("--subnet", default="0", help="min, max, or an index into the workload's stream / pool")
    ap.add_argument("--rounds", type=int, default=6, help="queries per team")
    args = ap.parse_args()
    wl = configs.build(args.workload)
    arch, batch, teams = wl["arch"], wl["batch"], args.teams_per_xcd
    res = max(arch.res_choices)
    if args.subnet == "max":
        cfg = A.max_cfg(arch, res)
    elif args.subnet == "min":
        cfg = A.min_cfg(arch, res)
    else:
        cfg = (wl["cfgs"] or wl["pool"])[int(args.subnet)]
    table = S.sushi_describe_supernet(arch)
    ctx = S.Sushi(0)
    ctx.sushi_load_supernet(arch, T.flatten(T.make_weights([(s, k) for _, s, k in table], 1, True)), S.BF16)
    ctx.sushi_set_option(S.OPT_EXEC_MODE, 3)
    ctx.sushi_set_option(S.OPT_TEAMS_PER_XCD, teams)
    x = torch.from_numpy(T.make_input(11, 0, batch, cfg.resolution, arch.in_channels, True)).cuda().to(torch.bfloat16)
    y = torch.empty(batch, arch.n_classes, device="cuda", dtype=torch.float32)
    torch.cuda.synchronize()
    n_teams = 8 * teams
    for _ in range(2 * n_teams):
        ctx.sushi_infer(cfg, x, y)
    ctx.sushi_synchronize()
    ctx.sushi_team_trace(1)
    for _ in range(args.rounds * n_teams):
        ctx.sushi_infer(cfg, x, y)
    ctx.sushi_synchronize()
    stamps = ctx.sushi_team_trace(0)
    ctx.close()
    rows = []
    for row in stamps:
        n = int((row > 0).sum())
        if n > 2:
            rows.append(np.diff(row[:n].astype(np.int64)) / 100.0)      # microseconds per op
    ops = S.sushi_team_plan(arch, cfg, batch, 32 // teams)
    n_ops = min(min(len(r) for r in rows), len(ops))
    mean = np.mean([r[:n_ops] for r in rows], axis=0)
    print("# %s, SubNet %s, batch %d, %d teams per XCD (%d workgroups each), %d teams traced, all teams busy" %
          (args.workload, args.subnet, batch, teams, 32 // teams, len(rows)))
    print("# a team's share of the peaks: %.1f GB/s, %.2f TFLOP/s" % (HBM_GBS / n_teams, MFMA_TFLOPS / n_teams))
    print("%3s %-7s %-34s %4s %3s %3s %6s %8s %8s %8s %5s %6s" %
          ("op", "kind", "shape HxWxC->PxQxK rxr/s", "wk", "ft", "pt", "units", "us", "MB", "bound us", "by", "frac"))
    tot_bound = 0.0
    by_kind = {}
    for i in range(n_ops):
        op = ops[i]
        if op["kind"] == 7:      # done by the squeeze-excite op before it
            continue
        if op["kind"] == 6:      # map in and out, both FC layers' weights; flops of the FC layers
            cells, w = op["B"] * op["H"] * op["W"] * op["C"], 2 * op["C"] * op["K"]
            byts, flops = 2.0 * (2 * cells + w), 2.0 * op["B"] * w
        else:
            byts, flops = op_cost(op)
        t_mem, t_mma = byts / (HBM_GBS * 1e3 / n_teams), flops / (MFMA_TFLOPS * 1e6 / n_teams)
        bound = max(t_mem, t_mma)
        tot_bound += bound
        shape = "%dx%dx%d->%dx%dx%d %dx%d/%d" % (op["H"], op["W"], op["C"], op["P"], op["Q"], op["K"], op["R"], op["R"], op["stride"])
        kind = KIND.get(op["kind"], "?")
        if kind == "conv" and op["R"] > 1:
            kind = "conv%dx%d" % (op["R"], op["R"])
        print("%3d %-7s %-34s %4d %3d %3d %6d %8.1f %8.3f %8.2f %5s %6.3f" %
              (i, kind, shape, op["wk"], op["ft"], op["pt"], op["n_units"], mean[i], byts / 1e6, bound,
               "mfma" if t_mma > t_mem else "hbm", bound / mean[i]))
        k = by_kind.setdefault(kind, [0.0, 0.0])
        k[0] += mean[i]; k[1] += bound
    print("# whole query: %.1f us per query inside a team, summed per-op bound %.1f us, fraction %.3f" %
          (mean.sum(), tot_bound, tot_bound / mean.sum()))
    for kind, (us, b) in sorted(by_kind.items()):
        print("# %-8s %8.1f us (%4.1f %% of the query), fraction of its bound %.3f" % (kind, us, 100.0 * us / mean.sum(), b / us))


if __name__ == "__main__":
    main()
