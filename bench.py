"""Benchmark of the SubNet-stream hot path on one MI355X.

One step = one query: the scheduler's cache bookkeeping (sushi_sched_record, and
sushi_set_subgraph_cache when the cached SubGraph changes) plus sushi_infer of the query's SubNet
on one input batch that already sits in HBM.  The default workload is the ResNet50-shaped
SuperNet at batch 1 with the sticky 1000-query stream (next SubNet repeats with p = 0.8).

Prints ONE JSON line: queries/s over the timed steps, plus
  roofline      the kernel with the largest summed time, measured with HIP events on the stream it
                runs on: for the persistent team kernel (default) and the stream kernel inside the
                timed region itself, for the per-layer modes in a second, identical pass;
  cpu_baseline  the CPU oracle timed on a bounded sample of the same stream.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def kernel_sources_digest():
    """SHA-256 over the library's sources: a stored counter reading only describes the kernels it
    was taken with."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2306_17266_amd", "csrc", "*"))):
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()


def stored_traffic(workload, mode, teams_per_xcd, sgs, Q):
    """HBM-side bytes per query (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size) from
    profiles/team_kernel_traffic.txt, or None when that reading was taken for another configuration
    or before the kernels last changed."""
    path = os.path.join(ROOT, "profiles", "team_kernel_traffic.txt")
    if not os.path.exists(path):
        return None
    kv = dict(line.strip().split("=", 1) for line in open(path) if "=" in line and not line.startswith("#"))
    want = {"workload": workload, "exec_mode": str(mode), "teams_per_xcd": str(teams_per_xcd), "sgs": sgs, "Q": str(Q)}
    if any(kv.get(k) != v for k, v in want.items()) or kv.get("sources_sha256") != kernel_sources_digest():
        return None
    return float(kv["fetch_bytes_per_query"]) + float(kv["write_bytes_per_query"])


def build_workload(name):
    from workloads import arch as A
    from workloads import streams
    if name == "resnet_bs1_sticky":
        arch = A.resnet_arch()
        return dict(arch=arch, batch=1, cfgs=streams.stream_sticky(arch, 1000, 2, 0.8, 224), Q=8,
                    budget=16 << 20, desc="ResNet50-shaped SuperNet, bf16, batch 1, 224x224, 1000-query stream, "
                    "next SubNet repeats with p=0.8 else uniform, cache re-chosen every 8 queries, budget 16 MiB")
    if name == "mbv3_bs1_zipf":
        arch = A.mbv3_arch()
        pool = streams.subnet_pool(arch, 32, 3, 224)
        cfgs = [pool[i] for i, _ in streams.stream_zipf(32, 1000, 3, 1.2)]
        return dict(arch=arch, batch=1, cfgs=cfgs, Q=10, budget=4 << 20,
                    desc="MobileNetV3-shaped SuperNet, bf16, batch 1, 224x224, 1000-query stream, Zipf(1.2) over a "
                    "pool of 32 SubNets, cache re-chosen every 10 queries, budget 4 MiB")
    if name == "resnet_bs16_levels":
        arch = A.resnet_arch()
        pool = streams.subnet_pool(arch, 16, 4, 224)
        lv = streams.stream_levels(5, 2000, 4)
        # without a measured latency table the level picks a SubNet of the pool by size rank
        return dict(arch=arch, batch=16, cfgs=None, pool=pool, levels=lv, Q=8, budget=64 << 20,
                    desc="ResNet50-shaped SuperNet, bf16, batch 16, 224x224, 2000-query stream, SubNet picked by "
                    "a latency target drawn from 5 levels (table = weight bytes not cached), budget 64 MiB")
    raise SystemExit("unknown workload %r" % name)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="resnet_bs1_sticky")
    ap.add_argument("--exec-mode", type=int, default=3,
                    help="0 = launch per layer, 1 = HIP graph replay, 2 = stream kernel, 3 = persistent XCD-team kernel")
    ap.add_argument("--teams-per-xcd", type=int, default=8, choices=[1, 2, 4, 8],
                    help="mode 3: teams per XCD (2 = twice as many queries in flight, each on half the workgroups)")
    ap.add_argument("--sgs", choices=["sched", "fixed", "off"], default="sched",
                    help="sched = the scheduler re-chooses the cached SubGraph every Q queries; fixed = the smallest "
                         "SubNet of the stream, shrunk to the budget, is cached once and kept (the state-unaware "
                         "baseline of the paper's scheduler ablation); off = nothing is cached")
    ap.add_argument("--Q", type=int, default=0, help="queries between cache re-choices (default: the workload's)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="run one 256 MiB device-to-device copy first (reference dispatch for byte counters)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: the library runs on ONE GPU; --gpus %d is not supported (with more GPUs each "
                         "would hold a replica of the SuperNet and serve its own share of the queries)" % args.gpus)

    import numpy as np
    import torch

    import paper_2306_17266_amd as S
    from workloads import tensors as T

    wl = build_workload(args.workload)
    arch, batch, Q, budget = wl["arch"], wl["batch"], args.Q or wl["Q"], wl["budget"]
    table = S.sushi_describe_supernet(arch)
    tensors = T.make_weights([(s, k) for _, s, k in table], 1, True)
    ctx = S.Sushi(0)
    ctx.sushi_load_supernet(arch, T.flatten(tensors), S.BF16)

    # the stream, each SubNet's vector/box (library's encoder) and the candidate SubGraphs
    from workloads import streams
    if wl["cfgs"] is None:
        pool = wl["pool"]
        boxes = [S.sushi_subnet_layers(arch, c) for c in pool]
        order = sorted(range(len(pool)), key=lambda i: streams.box_bytes(boxes[i], 2))
        pick = [order[(lv * (len(pool) - 1)) // 4] for lv in range(5)]
        cfgs = [pool[pick[lv]] for lv in wl["levels"]]
    else:
        cfgs = wl["cfgs"]
    distinct = {}
    for c in cfgs:
        distinct.setdefault(c.key(), c)
    box_of = {k: S.sushi_subnet_layers(arch, c) for k, c in distinct.items()}
    vec_of = {k: np.array([v for (kk, cc, r) in b for v in (kk, cc)], dtype=np.int32) for k, b in box_of.items()}
    cands = streams.candidate_subgraphs(list(box_of.values()), budget, 2, 40)
    gvecs = [[v for (k, c, r) in b for v in (k, c)] for b in cands]
    n = len(gvecs[0])
    ctx.sushi_sched_init([[0] * n], [0.0], gvecs, [[1.0] * (len(gvecs) + 1)], Q, S.STRICT_LATENCY)

    n_inputs, n_outputs = 8, 64
    res = cfgs[0].resolution
    xs = [torch.from_numpy(T.make_input(11, t, batch, res, arch.in_channels, True)).cuda().to(torch.bfloat16)
          for t in range(n_inputs)]
    outs = [torch.empty(batch, arch.n_classes, device="cuda", dtype=torch.float32) for _ in range(n_outputs)]
    torch.cuda.synchronize()
    state = {"cache": -1, "t": 0}

    def step():
        t = state["t"]
        cfg = cfgs[t % len(cfgs)]
        ctx.sushi_infer(cfg, xs[t % n_inputs], outs[t % n_outputs])
        j = ctx.sushi_sched_record(vec_of[cfg.key()])
        if args.sgs == "sched" and j >= 0 and j != state["cache"]:
            ctx.sushi_set_subgraph_cache(cands[j], budget)
            state["cache"] = j
        state["t"] = t + 1

    if args.calibration_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    mode = args.exec_mode
    ctx.sushi_set_option(S.OPT_EXEC_MODE, mode)
    ctx.sushi_set_option(S.OPT_TEAMS_PER_XCD, args.teams_per_xcd)
    if args.sgs == "fixed":
        smallest = min(box_of.values(), key=lambda b: streams.box_bytes(b, 2))
        ctx.sushi_set_subgraph_cache(streams.shrink_box(smallest, budget, 2), budget)
    for _ in range(args.warmup):
        step()
    ctx.sushi_synchronize()
    t_start = state["t"]
    # The timed region.  Modes 2 and 3 are timed with their HIP events in place (one pair per query
    # launch / one pair around the persistent kernel); modes 0 and 1 are timed bare and measured per
    # kernel in a second pass below.
    live_events = mode in (2, 3) and not args.no_roofline
    if mode == 3:
        ctx.sushi_quiesce()          # the timed region gets a kernel launch of its own
    if live_events:
        ctx.sushi_set_option(S.OPT_KERNEL_TIMING, 1)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    ctx.sushi_synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    stats = ctx.sushi_get_stats()
    ks = None
    if live_events:
        ks = [k for k in ctx.sushi_get_kernel_stats() if k["launches"]]
        ctx.sushi_set_option(S.OPT_KERNEL_TIMING, 0)

    # p50 latency of a lone query: post, wait, repeat (same steps as the timed region)
    lat = []
    state["t"] = t_start
    for _ in range(min(args.steps, 200)):
        a = time.perf_counter()
        step()
        ctx.sushi_synchronize()
        lat.append(time.perf_counter() - a)
    p50_ms = float(np.median(lat) * 1e3)

    roofline = None
    if not args.no_roofline:
        if ks is None:
            # identical pass, one launch per layer, HIP events around every launch
            ctx.sushi_set_option(S.OPT_EXEC_MODE, 0)
            state["t"] = t_start
            for _ in range(20):
                step()
            ctx.sushi_synchronize()
            state["t"] = t_start
            ctx.sushi_set_option(S.OPT_KERNEL_TIMING, 1)
            for _ in range(args.steps):
                step()
            ctx.sushi_synchronize()
            ks = [k for k in ctx.sushi_get_kernel_stats() if k["launches"]]
            ctx.sushi_set_option(S.OPT_KERNEL_TIMING, 0)
            ctx.sushi_set_option(S.OPT_EXEC_MODE, mode)
        dom = max(ks, key=lambda k: k["total_ms"])
        sec = dom["total_ms"] * 1e-3
        ai = dom["flops"] / dom["bytes"]
        if ai >= MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
            achieved, peak, unit, bound = dom["flops"] / sec / 1e12, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s", "mfma"
        else:
            achieved, peak, unit, bound = dom["bytes"] / sec / 1e9, HBM_PEAK_GBS, "GB/s", "hbm"
        # measured bytes per launch of the dominant kernel: known only for the team kernel, whose one
        # launch serves all timed queries
        traffic = None
        if mode == 3 and dom["launches"] == 1:
            per_query = stored_traffic(args.workload, mode, args.teams_per_xcd, args.sgs, Q)
            if per_query is not None:
                traffic = per_query * args.steps
        roofline = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
                    "traffic": traffic, "kernel": dom["name"], "launches": dom["launches"],
                    "avg_launch_us": dom["total_ms"] * 1e3 / dom["launches"],
                    "alg_bytes_per_launch": dom["bytes"] / dom["launches"],
                    "alg_flops_per_launch": dom["flops"] / dom["launches"],
                    "arithmetic_intensity": ai,
                    "share_of_kernel_time": dom["total_ms"] / sum(k["total_ms"] for k in ks),
                    "all_kernels": {k["name"]: {"launches": k["launches"], "avg_us": k["total_ms"] * 1e3 / k["launches"],
                                                "GBps": k["bytes"] / (k["total_ms"] * 1e-3) / 1e9,
                                                "TFLOPps": k["flops"] / (k["total_ms"] * 1e-3) / 1e12} for k in ks}}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import subnet_eval as E
        wts = E.name_weights(arch, tensors)
        n_sample = 16 if batch == 1 else 2
        sample = [cfgs[(t_start + i * 7) % len(cfgs)] for i in range(n_sample)]
        x0 = np.ascontiguousarray(T.make_input(11, 0, batch, res, arch.in_channels, True).transpose(0, 3, 1, 2))
        E.forward(arch, wts, sample[0], x0)
        c0 = time.perf_counter()
        for cfg in sample:
            E.forward(arch, wts, cfg, x0)
        c1 = time.perf_counter()
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = {"value": n_sample / (c1 - c0), "unit": "queries/s", "cores": cores, "kind": "oracle",
               "sample": "%d queries of the same stream (every 7th from the first timed step), batch %d, "
                         "%.1f s of CPU work" % (n_sample, batch, c1 - c0)}

    out = {"metric": "SubNet queries/sec (batch %d)" % batch, "value": args.steps / elapsed, "unit": "queries/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": args.workload, "description": wl["desc"], "exec_mode": args.exec_mode, "teams_per_xcd": args.teams_per_xcd, "sgs": args.sgs, "Q": Q,
                      "distinct_subnets": len(distinct), "candidate_subgraphs": len(cands)},
           "p50_latency_ms": p50_ms,
           "weight_bytes_per_query": stats["weight_bytes_total"] / max(1, stats["queries"]),
           "weight_bytes_per_query_in_cached_subgraph": stats["weight_bytes_resident"] / max(1, stats["queries"]),
           "weight_bytes_per_query_from_lds": stats["weight_bytes_lds"] / max(1, stats["queries"]),
           "mean_hit_ratio": stats["sum_hit_ratio"] / max(1, stats["queries"]),
           "cache_installs": stats["cache_installs"],
           "roofline": roofline, "cpu_baseline": cpu}
    print(json.dumps(out))
    ctx.close()


if __name__ == "__main__":
    main()
