"""Per-layer roofline report of one SubNet in exec mode 0 (one launch per op).

    python -m paper_2306_17266_amd.layer_report --workload resnet_bs16_levels --subnet max --reps 20

The report lists, per op of the SubNet's plan, the median duration over `reps` queries, the algorithmic bytes
and flops the library counts for it (active slice only), the achieved GB/s and TFLOP/s, and the fraction of the
op's own bound max(flops / MFMA peak, bytes / HBM peak).

Durations come from one of two clocks:
  * by default, HIP events the library puts around every launch (SUSHI_OPT_KERNEL_TIMING).  An event pair adds
    several microseconds to a short kernel, so these figures are upper bounds on the kernels' own time;
  * with --from-trace FILE, the kernel trace of a profiler run of this same command:
        rocprofv3 --kernel-trace --output-format csv -d DIR -o lr -- python3 -m paper_2306_17266_amd.layer_report ... --plain
        python3 -m paper_2306_17266_amd.layer_report ... --from-trace DIR/lr_kernel_trace.csv
    (--plain runs the queries without events; the second call needs no GPU: the k-th launch of a query is the
    k-th op of its plan, and the library's kernels are told apart from others by name).
"""
import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_GBS, MFMA_TFLOPS = 8000.0, 2500.0
KIND = {0: "conv", 1: "dwconv", 2: "maxpool", 3: "gap", 4: "fc", 5: "gate"}


def main():
    import torch

    import paper_2306_17266_amd as S
    from workloads import arch as A
    from workloads import configs
    from workloads import tensors as T
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet_bs16_levels")
    ap.add_argument("--subnet", default="max", help="min, max, or an index into the workload's stream / pool")
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--resolution", type=int, default=224)
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--patch-min-pixels", type=int, default=-1,
                    help="SUSHI_OPT_PATCH_CONV_MIN_PIXELS (0 = never use the patch conv kernel; default: the library's)")
    ap.add_argument("--int8", action="store_true", help="the int8 path (ResNet50-shaped and Tiny SuperNets)")
    ap.add_argument("--plain", action="store_true", help="run the queries without events and print nothing (profiler run)")
    ap.add_argument("--from-trace", default="", help="kernel-trace CSV of a --plain run under rocprofv3")
    args = ap.parse_args()
    wl = configs.build(args.workload)
    arch, batch = wl["arch"], args.batch or wl["batch"]
    if args.subnet == "max":
        cfg = A.max_cfg(arch, args.resolution)
    elif args.subnet == "min":
        cfg = A.min_cfg(arch, args.resolution)
    else:
        cfg = (wl["cfgs"] or wl["pool"])[int(args.subnet)]
    if args.from_trace:
        return report_from_trace(args, arch, cfg, batch)
    table = S.sushi_describe_supernet(arch)
    ctx = S.Sushi(0)
    if args.int8:
        from workloads import quant
        tens = T.make_weights([(s, k) for _, s, k in table], 1, False)
        ctx.sushi_load_supernet_int8(arch, *quant.flatten_int8(quant.make_int8_model(table, tens, quant.layer_roles(arch))))
    else:
        ctx.sushi_load_supernet(arch, T.flatten(T.make_weights([(s, k) for _, s, k in table], 1, True)), S.BF16)
    if args.patch_min_pixels >= 0:
        ctx.sushi_set_option(S.OPT_PATCH_CONV_MIN_PIXELS, args.patch_min_pixels)
    if args.int8:
        x = torch.from_numpy(quant.quantize_input(T.make_input(11, 0, batch, cfg.resolution, arch.in_channels, False))).cuda()
    else:
        x = torch.from_numpy(T.make_input(11, 0, batch, cfg.resolution, arch.in_channels, True)).cuda().to(torch.bfloat16)
    y = torch.empty(batch, arch.n_classes, device="cuda", dtype=torch.float32)
    for _ in range(5):
        ctx.sushi_infer(cfg, x, y)
    ctx.sushi_synchronize()
    if args.plain:
        torch.cuda.synchronize()
        for _ in range(args.reps):
            ctx.sushi_infer(cfg, x, y)
        ctx.sushi_synchronize()
        ctx.close()
        return
    ctx.sushi_set_option(S.OPT_KERNEL_TIMING, 1)
    for _ in range(args.reps):
        ctx.sushi_infer(cfg, x, y)
    ctx.sushi_synchronize()
    recs = ctx.sushi_get_launch_records()
    names = [k["name"] for k in ctx.sushi_get_kernel_stats()]
    ctx.sushi_set_option(S.OPT_KERNEL_TIMING, 0)
    ops = S.sushi_team_plan(arch, cfg, batch, 32)
    per_op = {}
    for op_index, kc, ms, byts, flops in recs:
        per_op.setdefault(op_index, []).append((ms, names[kc], byts, flops))
    ctx.close()
    print_report(args, cfg, batch, ops, per_op, "HIP events around every launch")


def op_cost(op, es=2.0):
    """Algorithmic bytes and flops of one op, as the library counts them (active slice, every tensor once)."""
    kind = op["kind"]
    cin = float(op["B"] * op["H"] * op["W"] * op["C"])
    taps = float(op["R"] * op["R"])
    if kind in (0, 1, 4):
        out = float(op["B"] * op["P"] * op["Q"] * op["K"])
        wts = op["K"] * taps if kind == 1 else op["K"] * op["C"] * taps
        byts = (cin + wts + (out if op["res"] else 0.0)) * es + out * (4.0 if op["out_f32"] else es) + 8.0 * op["K"]
        flops = 2.0 * out * (taps if kind == 1 else op["C"] * taps)
        return byts, flops
    out = cin if kind == 5 else float(op["B"] * op["P"] * op["Q"] * op["C"])
    return (cin + out) * es + (4.0 * op["B"] * op["C"] if kind == 5 else 0.0), (9.0 * out if kind == 2 else cin)


def report_from_trace(args, arch, cfg, batch):
    import csv

    import paper_2306_17266_amd as S
    ops = S.sushi_team_plan(arch, cfg, batch, 32)
    mine = ("conv_i8_kernel", "conv_i8_direct_kernel", "maxpool_i8_kernel", "gap_i8_kernel", "fc_i8_kernel",
            "conv_direct_kernel", "conv_mfma_kernel", "conv_mfma_splitk_kernel", "conv_patch_kernel", "dwconv_kernel",
            "dwconv_rows_kernel", "maxpool_kernel", "gap_kernel", "gate_kernel")
    rows = []
    for r in csv.DictReader(open(args.from_trace)):
        name = r["Kernel_Name"]
        short = next((m for m in mine if "sushi::" + m in name or name.startswith(m) or ("::" + m + "<") in name or (" " + m + "<") in name), None)
        if short is None:
            continue
        rows.append((int(r["Start_Timestamp"]), (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) * 1e-6, short))
    rows.sort()
    n_ops = len(ops)
    assert len(rows) % n_ops == 0 and len(rows) >= n_ops * args.reps, (len(rows), n_ops)
    rows = rows[-n_ops * args.reps:]                                  # the timed queries come last
    per_op = {}
    for k, (_, ms, short) in enumerate(rows):
        i = k % n_ops
        byts, flops = op_cost(ops[i], 1.0 if args.int8 else 2.0)
        per_op.setdefault(i, []).append((ms, short, byts, flops))
    print_report(args, cfg, batch, ops, per_op, "rocprofv3 kernel trace")


def print_report(args, cfg, batch, ops, per_op, clock):
    names = None
    print("# %s, SubNet %s, batch %d, resolution %d, exec mode 0, median of %d launches per op; durations: %s" %
          (args.workload, args.subnet, batch, cfg.resolution, args.reps, clock))
    mfma_peak = 5000.0 if getattr(args, "int8", False) else MFMA_TFLOPS
    print("# peaks: HBM %.0f GB/s, dense %s MFMA %.0f T%sOP/s; bound = max(flops / peak, bytes / peak)" %
          (HBM_GBS, "int8" if mfma_peak > MFMA_TFLOPS else "bf16", mfma_peak, "" if mfma_peak > MFMA_TFLOPS else "FL"))
    print("%3s %-7s %-26s %-24s %9s %9s %9s %9s %8s %5s %6s" %
          ("op", "kind", "shape BxHxWxC->PxQxK rxr/s", "kernel", "us", "MB", "GFLOP", "GB/s", "TFLOP/s", "bound", "frac"))
    tot_us = tot_bound = 0.0
    by_kind = {}
    for i in sorted(per_op):
        ms = float(np.median([r[0] for r in per_op[i]]))
        _, kname, byts, flops = per_op[i][0]
        op = ops[i]
        us = ms * 1e3
        t_mem, t_mma = byts / (HBM_GBS * 1e3), flops / (mfma_peak * 1e6)      # microseconds
        bound_us = max(t_mem, t_mma)
        which = "mfma" if t_mma > t_mem else "hbm"
        shape = "%dx%dx%dx%d->%dx%dx%d %dx%d/%d" % (op["B"], op["H"], op["W"], op["C"], op["P"], op["Q"], op["K"],
                                                   op["R"], op["R"], op["stride"])
        print("%3d %-7s %-26s %-24s %9.2f %9.3f %9.3f %9.1f %8.1f %5s %6.3f" %
              (i, KIND.get(op["kind"], "?"), shape, kname, us, byts / 1e6, flops / 1e9, byts / us / 1e3,
               flops / us / 1e6, which, bound_us / us))
        tot_us += us
        tot_bound += bound_us
        k = by_kind.setdefault((KIND.get(op["kind"], "?"), which), [0.0, 0.0, 0.0, 0.0])
        k[0] += us; k[1] += byts; k[2] += flops; k[3] += bound_us
    print("# whole query: %.1f us in kernels, summed per-op bound %.1f us, fraction %.3f" % (tot_us, tot_bound, tot_bound / tot_us))
    for (kind, which), (us, byts, flops, b) in sorted(by_kind.items()):
        print("# %-7s %-4s-bound ops: %9.1f us, %8.1f GB/s, %8.1f TFLOP/s, fraction of their bound %.3f" %
              (kind, which, us, byts / us / 1e3, flops / us / 1e6, b / us))


if __name__ == "__main__":
    main()
