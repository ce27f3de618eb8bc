"""Benchmark of the SubNet-stream hot path on one MI355X.

One step = one block of `queries_per_step` consecutive queries of the workload's stream (200 at
batch 1, 100 at batch 16), so that `--steps 20 --warmup 5` times 4000 queries of steady state after
1000 warm-up queries.  A query is: the scheduler's part (sushi_sched_step when the stream gives
latency targets, else sushi_sched_record of the named SubNet; sushi_set_subgraph_cache when the
cached SubGraph changes) plus sushi_infer on one input batch that already sits in HBM.  The timed
region starts with the persistent kernel stopped and ends when it has stopped again, so it holds
exactly one launch of it.

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
MFMA_INT8_PEAK_TOPS = 5000.0


def kernel_sources_digest():
    """SHA-256 over the library's sources: a stored counter reading only describes the kernels it
    was taken with."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2306_17266_amd", "csrc", "*"))):
        if not os.path.isfile(path):
            continue
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


def main():
    from workloads import configs
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20, help="timed blocks of queries")
    ap.add_argument("--warmup", type=int, default=5, help="untimed blocks of queries before them")
    ap.add_argument("--queries-per-step", type=int, default=0, help="default: 200 at batch 1, 100 at batch 16")
    ap.add_argument("--workload", default="resnet_bs1_sticky", choices=[n for n in configs.NAMES if n != "tiny_uniform"])
    ap.add_argument("--budget-mib", type=int, default=0, help="SubGraph cache budget (default: the workload's)")
    ap.add_argument("--dtype", choices=["bf16", "int8"], default="bf16",
                    help="int8: the paper's own precision (ResNet50-shaped workloads, exec mode 0 only)")
    ap.add_argument("--exec-mode", type=int, default=-1,
                    help="0 = launch per layer, 1 = HIP graph replay, 2 = stream kernel, 3 = persistent XCD-team kernel "
                         "(default: 3 for bf16, 0 for int8)")
    ap.add_argument("--teams-per-xcd", type=int, default=0, choices=[0, 1, 2, 4, 8, 16],
                    help="mode 3: teams per XCD (default 16 at batch 1, 1 at batch 16)")
    ap.add_argument("--sgs", choices=["sched", "fixed", "off"], default="sched",
                    help="sched = the scheduler re-chooses the cached SubGraph every Q queries; fixed = the smallest "
                         "SubNet of the stream, shrunk to the budget, is cached once and kept (the state-unaware "
                         "baseline of the paper's scheduler ablation); off = nothing is cached")
    ap.add_argument("--Q", type=int, default=0, help="queries between cache re-choices (default: the workload's)")
    ap.add_argument("--cold-sweep", action="store_true",
                    help="modes 0-2: stream a 512 MiB scratch buffer through the caches before every query (a device "
                         "whose caches are lost between queries)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="run one 256 MiB device-to-device copy first (reference dispatch for byte counters)")
    ap.add_argument("--table-out", default="", help="directory that receives a latency table measured in this run (to freeze it)")
    ap.add_argument("--measure-table", action="store_true",
                    help="latency-target stream: measure the latency table in this run even if a frozen one is shipped")
    ap.add_argument("--table-runs", type=int, default=3, help="runs per table entry when it is measured")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--no-latency", action="store_true", help="skip the lone-query latency passes")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: the library runs on ONE GPU; --gpus %d is not supported (with more GPUs each "
                         "would hold a replica of the SuperNet and serve its own share of the queries)" % args.gpus)

    import numpy as np
    import torch

    import paper_2306_17266_amd as S
    from paper_2306_17266_amd import sushiabs
    from workloads import streams
    from workloads import tensors as T

    wl = configs.build(args.workload, args.budget_mib or None)
    arch, batch, Q, budget = wl["arch"], wl["batch"], args.Q or wl["Q"], wl["budget"]
    qps = args.queries_per_step or (200 if batch == 1 else 100)
    teams = args.teams_per_xcd or (16 if batch == 1 else 1)
    table = S.sushi_describe_supernet(arch)
    int8 = args.dtype == "int8"
    es = 1 if int8 else 2                       # bytes per weight
    if args.exec_mode < 0:
        args.exec_mode = 0 if int8 else 3
    if int8 and args.exec_mode != 0:
        raise SystemExit("bench.py: the int8 path runs in exec mode 0 only")
    tensors = T.make_weights([(s, k) for _, s, k in table], 1, not int8)
    ctx = S.Sushi(0)
    qmodel = None
    if int8:
        from workloads import quant
        qmodel = quant.make_int8_model(table, tensors, quant.layer_roles(arch))
        ctx.sushi_load_supernet_int8(arch, *quant.flatten_int8(qmodel))
    else:
        ctx.sushi_load_supernet(arch, T.flatten(tensors), S.BF16)
    mode = args.exec_mode
    ctx.sushi_set_option(S.OPT_EXEC_MODE, mode)
    ctx.sushi_set_option(S.OPT_TEAMS_PER_XCD, teams)
    if args.cold_sweep:
        ctx.sushi_set_option(S.OPT_COLD_SWEEP_MIB, 512)

    # the serving SubNets, each one's vector/box (library's encoder) and the candidate SubGraphs
    by_target = wl["cfgs"] is None
    serving = wl["pool"] if by_target else wl["cfgs"]
    distinct = {}
    for c in serving:
        distinct.setdefault(c.key(), c)
    box_of = {k: S.sushi_subnet_layers(arch, c) for k, c in distinct.items()}
    vec_of = {k: np.array([v for (kk, cc, r) in b for v in (kk, cc)], dtype=np.int32) for k, b in box_of.items()}
    cands = streams.candidate_subgraphs(list(box_of.values()), budget, es, 40)
    gvecs = [[v for (k, c, r) in b for v in (k, c)] for b in cands]
    n = len(gvecs[0])

    res_list = sorted({c.resolution for c in serving})
    n_inputs, n_outputs = 8, 64
    if int8:
        xs = {r: [torch.from_numpy(quant.quantize_input(T.make_input(11, t, batch, r, arch.in_channels, False))).cuda()
                  for t in range(n_inputs)] for r in res_list}
    else:
        xs = {r: [torch.from_numpy(T.make_input(11, t, batch, r, arch.in_channels, True)).cuda().to(torch.bfloat16)
                  for t in range(n_inputs)] for r in res_list}
    outs = [torch.empty(batch, arch.n_classes, device="cuda", dtype=torch.float32) for _ in range(n_outputs)]
    torch.cuda.synchronize()

    levels = None
    table_info = None
    if by_target:
        # Algorithm 1 in the loop: the latency table L[SubNet][cached SubGraph] measured on this GPU (frozen
        # to a file when one is shipped for this workload), synthetic accuracies that grow with SubNet size
        pool = wl["pool"]
        sizes = [streams.box_bytes(box_of[c.key()], es) for c in pool]
        acc = [0.0] * len(pool)
        for rank, i in enumerate(sorted(range(len(pool)), key=lambda i: sizes[i])):
            acc[i] = float(np.float32(0.70 + 0.01 * rank))
        tpath = sushiabs.table_path(args.workload, budget, teams)
        frozen = sushiabs.load_table(tpath, len(pool), len(cands)) if mode == 3 and not args.measure_table else None
        if frozen is not None:
            lat, table_info = frozen["table"], "frozen: " + os.path.relpath(tpath, ROOT)
        else:
            lat = sushiabs.measure_table(ctx, pool, cands, budget, xs[res_list[0]][0], outs[0], runs=args.table_runs)
            table_info = "measured in this run (median of %d runs per entry)" % args.table_runs
            if args.table_out and os.path.isdir(args.table_out):
                sushiabs.save_table(os.path.join(args.table_out, os.path.basename(tpath)), lat, args.workload, budget, args.table_runs,
                                    "exec mode %d, %d teams per XCD, batch %d" % (mode, teams, batch))
        levels = sushiabs.latency_levels(lat, wl["n_levels"])
        ctx.sushi_sched_init([vec_of[c.key()] for c in pool], acc, gvecs, lat, Q, S.STRICT_LATENCY)
    else:
        ctx.sushi_sched_init([[0] * n], [0.0], gvecs, [[1.0] * (len(gvecs) + 1)], Q, S.STRICT_LATENCY)

    state = {"cache": -1, "t": 0}
    served = {}
    # everything a query passes to the library, marshalled once (the loop below is the host's share of a query)
    import ctypes
    m_of = {k: (ctx.marshal_cfg(c), ctx.marshal_vec(vec_of[k]), c.resolution) for k, c in distinct.items()}
    m_serving = [m_of[c.key()] for c in serving]
    m_cands = [ctx.marshal_subgraph(b) for b in cands]
    x_ptrs = {r: [ctypes.c_void_p(x.data_ptr()) for x in xs[r]] for r in res_list}
    out_ptrs = [ctypes.c_void_p(o.data_ptr()) for o in outs]
    n_serving = len(m_serving)
    use_sched = args.sgs == "sched"

    def one_query():
        t = state["t"]
        if by_target:
            i, j = ctx.sushi_sched_step(0.0, levels[wl["levels"][t % len(wl["levels"])]])
            served[i] = served.get(i, 0) + 1
            ctx.infer_marshalled(m_serving[i][0], x_ptrs[m_serving[i][2]][t % n_inputs], batch, out_ptrs[t % n_outputs])
        else:
            cs, vec, r = m_serving[t % n_serving]
            ctx.infer_marshalled(cs, x_ptrs[r][t % n_inputs], batch, out_ptrs[t % n_outputs])
            j = ctx.sched_record_marshalled(vec)
        if use_sched and j >= 0 and j != state["cache"]:
            ctx.set_subgraph_cache_marshalled(m_cands[j], budget)
            state["cache"] = j
        state["t"] = t + 1

    def step():
        for _ in range(qps):
            one_query()

    if args.calibration_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ctx.sushi_set_subgraph_cache(None, 0)
    if args.sgs == "fixed":
        smallest = min(box_of.values(), key=lambda b: streams.box_bytes(b, es))
        ctx.sushi_set_subgraph_cache(streams.shrink_box(smallest, budget, es), budget)
    for _ in range(args.warmup):
        step()
    ctx.sushi_quiesce()          # the timed region gets a kernel launch of its own (mode 3)
    t_start = state["t"]
    # The timed region.  Modes 2 and 3 are timed with their HIP events in place (one pair per query
    # launch / one pair around the persistent kernel); modes 0 and 1 are timed bare and measured per
    # kernel in a second pass below.
    live_events = mode in (2, 3) and not args.no_roofline
    if live_events:
        ctx.sushi_set_option(S.OPT_KERNEL_TIMING, 1)
    stats0 = ctx.sushi_get_stats()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    ctx.sushi_quiesce()          # all queries done and the persistent kernel gone: its launch lies inside [t0, t1]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    n_queries = args.steps * qps
    stats = ctx.sushi_get_stats()
    dstat = {k: stats[k] - stats0[k] for k in stats if isinstance(stats[k], int) or k == "sum_hit_ratio"}
    ks = None
    if live_events:
        ks = [k for k in ctx.sushi_get_kernel_stats() if k["launches"]]
        ctx.sushi_set_option(S.OPT_KERNEL_TIMING, 0)

    # p50 latency of a lone query: post, wait, repeat (same queries as the timed region); then the same
    # through one launch per layer (mode 0), the shortest path for a query that has the GPU to itself
    p50_ms = p50_mode0_ms = None
    if not args.no_latency:
        def lone_pass(count):
            lat = []
            state["t"] = t_start
            for _ in range(count):
                a = time.perf_counter()
                one_query()
                ctx.sushi_synchronize()
                lat.append(time.perf_counter() - a)
            return float(np.median(lat) * 1e3)
        p50_ms = lone_pass(200 if batch == 1 else 50)
        if mode != 0 and not args.cold_sweep:
            ctx.sushi_set_option(S.OPT_EXEC_MODE, 0)
            lone_pass(10)
            p50_mode0_ms = lone_pass(200 if batch == 1 else 50)
            ctx.sushi_set_option(S.OPT_EXEC_MODE, mode)

    roofline = None
    if not args.no_roofline:
        if ks is None:
            # identical pass, one launch per layer, HIP events around every launch
            ctx.sushi_set_option(S.OPT_EXEC_MODE, 0)
            state["t"] = t_start
            for _ in range(20):
                one_query()
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
        mfma_peak = MFMA_INT8_PEAK_TOPS if int8 else MFMA_BF16_PEAK_TFLOPS
        if ai >= mfma_peak * 1e12 / (HBM_PEAK_GBS * 1e9):
            achieved, peak, unit, bound = dom["flops"] / sec / 1e12, mfma_peak, "TOP/s" if int8 else "TFLOP/s", "mfma"
        else:
            achieved, peak, unit, bound = dom["bytes"] / sec / 1e9, HBM_PEAK_GBS, "GB/s", "hbm"
        # measured bytes per launch of the dominant kernel: a STORED counter reading (two rocprofv3 --pmc runs
        # of this command), valid only for the configuration and the sources it was taken with
        traffic = None
        if mode == 3 and dom["launches"] == 1:
            per_query = stored_traffic(args.workload, mode, teams, args.sgs, Q)
            if per_query is not None:
                traffic = per_query * n_queries
        roofline = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
                    "traffic": traffic,
                    "traffic_source": "stored reading, profiles/team_kernel_traffic.txt" if traffic is not None else None,
                    "kernel": dom["name"], "launches": dom["launches"],
                    "avg_launch_us": dom["total_ms"] * 1e3 / dom["launches"],
                    "kernel_ms_per_step": dom["total_ms"] / args.steps,
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
        n_sample = 64 if batch == 1 else 4
        sample = [serving[(t_start + i * 7) % len(serving)] for i in range(n_sample)]
        if int8:
            from oracle import int8_eval as QE
            qm = QE.name_model(qmodel)
            x_of = {r: np.ascontiguousarray(quant.quantize_input(T.make_input(11, 0, batch, r, arch.in_channels, False)).transpose(0, 3, 1, 2))
                    for r in res_list}

            def ref_forward(cfg):
                return QE.forward_int8(arch, qm, cfg, x_of[cfg.resolution])
        else:
            wts = E.name_weights(arch, tensors)
            x_of = {r: np.ascontiguousarray(T.make_input(11, 0, batch, r, arch.in_channels, True).transpose(0, 3, 1, 2))
                    for r in res_list}

            def ref_forward(cfg):
                return E.forward(arch, wts, cfg, x_of[cfg.resolution])
        ref_forward(sample[0])
        c0 = time.perf_counter()
        done = 0
        for cfg in sample:
            ref_forward(cfg)
            done += 1
            if time.perf_counter() - c0 > 25.0:
                break
        c1 = time.perf_counter()
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = {"value": done / (c1 - c0), "unit": "queries/s", "cores": cores, "kind": "oracle",
               "sample": "%d queries of the same stream (every 7th from the first timed query), batch %d, "
                         "%.1f s of CPU work" % (done, batch, c1 - c0)}

    nq = max(1, dstat["queries"])
    out = {"metric": "SubNet queries/sec (batch %d)" % batch, "value": n_queries / elapsed, "unit": "queries/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "i8" if int8 else "bf16", "data": "synthetic",
           "config": {"workload": args.workload, "description": wl["desc"], "queries_per_step": qps,
                      "timed_queries": n_queries, "warmup_queries": args.warmup * qps, "exec_mode": mode,
                      "teams_per_xcd": teams, "sgs": args.sgs, "Q": Q, "budget_bytes": budget,
                      "cold_sweep": bool(args.cold_sweep),
                      "distinct_subnets": len(distinct), "candidate_subgraphs": len(cands),
                      "latency_table": table_info,
                      "subnets_served": len(served) if by_target else len({c.key() for c in serving})},
           "p50_latency_ms": p50_ms, "p50_latency_ms_mode0": p50_mode0_ms,
           "weight_bytes_per_query": dstat["weight_bytes_total"] / nq,
           "weight_bytes_per_query_inside_cached_subgraph": dstat["weight_bytes_in_subgraph"] / nq,
           "weight_bytes_per_query_from_lds": dstat["weight_bytes_lds"] / nq,
           "mean_hit_ratio": dstat["sum_hit_ratio"] / nq,
           "cache_installs": dstat["cache_installs"],
           "residency_changes": dstat["residency_changes"],
           "install_bytes_per_team_lds": dstat["install_bytes_lds"],
           "roofline": roofline, "cpu_baseline": cpu}
    print(json.dumps(out))
    ctx.close()


if __name__ == "__main__":
    main()
