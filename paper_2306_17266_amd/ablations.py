"""Scheduler ablations on the synthetic streams (the counterparts of the paper's Appendix A.1 - A.4), host only:

    python -m paper_2306_17266_amd.ablations [--workload resnet_bs1_sticky] [--budget-mib 16]

For a stream that names its SubNets, the library's scheduler (Algorithm 1, every-Q cache choice) runs over the
whole stream for every window length Q and every table width M (number of candidate SubGraphs, the first M of
the candidate set); the report gives, per (Q, M): the mean hit ratio of Appendix A.4 between the served
SubNet and the SubGraph cached at that moment, the share of the stream's weight bytes that lie inside the
cached SubGraph, the number of cache changes per 1000 queries, and the scheduler's time per query
(sushi_sched_record through the C ABI: the "lookup time" of Appendix A.3).  "fixed" rows cache the stream's
smallest SubNet, shrunk to the budget, once (the state-unaware baseline of Section 5.4); no GPU is used.
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def run_stream(S, B, boxes_m, vecs_m, cands, Q, cfg_keys):
    """(mean hit ratio, bytes inside G / bytes, cache changes, seconds in the scheduler)."""
    ctx = S.Sushi(-1)
    gvecs = [[v for (k, c, r) in b for v in (k, c)] for b in cands]
    n = len(gvecs[0])
    ctx.sushi_sched_init([[0] * n], [0.0], gvecs, [[1.0] * (len(gvecs) + 1)], Q, S.STRICT_LATENCY)
    m_cands = [B.marshal_box(b) for b in cands]
    cache, changes, hit_sum, tot, com, t_sched = -1, 0, 0.0, 0, 0, 0.0
    overlap = {}
    for key in cfg_keys:
        if cache >= 0:
            o = overlap.get((key, cache))
            if o is None:
                o = overlap[(key, cache)] = S.sushi_subgraph_overlap(boxes_m[key], m_cands[cache])
            tot, com, hit_sum = tot + o[0], com + o[1], hit_sum + o[2]
        else:
            o = overlap.get((key, -1))
            if o is None:
                o = overlap[(key, -1)] = S.sushi_subgraph_overlap(boxes_m[key], boxes_m[key])
            tot += o[0]
        a = time.perf_counter()
        j = ctx.sched_record_marshalled(vecs_m[key])
        t_sched += time.perf_counter() - a
        if j >= 0 and j != cache:
            cache, changes = j, changes + 1
    ctx.close()
    return hit_sum / len(cfg_keys), com / max(1, tot), changes, t_sched


def main():
    import paper_2306_17266_amd as S
    from paper_2306_17266_amd import binding as B
    from workloads import configs, streams
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet_bs1_sticky", choices=["resnet_bs1_sticky", "mbv3_bs1_zipf", "mbv3_bs1_regimes"])
    ap.add_argument("--budget-mib", type=int, default=0)
    ap.add_argument("--Q", default="1,2,4,8,16,32,64")
    ap.add_argument("--M", default="5,10,20,40")
    args = ap.parse_args()
    wl = configs.build(args.workload, args.budget_mib or None)
    arch, cfgs, budget = wl["arch"], wl["cfgs"], wl["budget"]
    distinct = {}
    for c in cfgs:
        distinct.setdefault(c.key(), c)
    box_of = {k: S.sushi_subnet_layers(arch, c) for k, c in distinct.items()}
    boxes_m = {k: B.marshal_box(b) for k, b in box_of.items()}
    helper = S.Sushi(-1)
    vecs_m = {k: helper.marshal_vec([v for (kk, cc, r) in b for v in (kk, cc)]) for k, b in box_of.items()}
    keys = [c.key() for c in cfgs]
    all_cands = streams.candidate_subgraphs(list(box_of.values()), budget, 2, 500)
    print("# %s: %d queries, %d distinct SubNets, budget %d MiB, %d candidate SubGraphs in all" %
          (args.workload, len(cfgs), len(distinct), budget >> 20, len(all_cands)))
    print("%-6s %4s %4s %10s %12s %14s %12s" % ("cache", "Q", "M", "hit ratio", "bytes in G", "changes/1000", "sched us/q"))
    smallest = min(box_of.values(), key=lambda b: streams.box_bytes(b, 2))
    fixed = streams.shrink_box(smallest, budget, 2)
    hit = tot = com = 0
    m_fixed = B.marshal_box(fixed)
    for k in keys:
        o = S.sushi_subgraph_overlap(boxes_m[k], m_fixed)
        tot, com, hit = tot + o[0], com + o[1], hit + o[2]
    print("%-6s %4s %4s %10.4f %12.4f %14.1f %12s" % ("fixed", "-", "1", hit / len(keys), com / tot, 0.0, "-"))
    for M in [int(v) for v in args.M.split(",")]:
        cands = all_cands[:M]
        for Q in [int(v) for v in args.Q.split(",")]:
            h, share, changes, t = run_stream(S, B, boxes_m, vecs_m, cands, Q, keys)
            print("%-6s %4d %4d %10.4f %12.4f %14.1f %12.2f" %
                  ("sched", Q, len(cands), h, share, changes * 1000.0 / len(keys), t / len(keys) * 1e6))
    helper.close()


if __name__ == "__main__":
    main()
