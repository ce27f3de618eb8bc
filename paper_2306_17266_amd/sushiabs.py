"""SushiAbs for MI355X: the latency table the scheduler decides from (paper Section 3.2; Appendix
A.2 / A.3 on how wide it is and what a lookup costs).

L[i][j] is the latency of serving SubNet i while SubGraph j is cached; the extra last column is
"nothing cached".  Two generators:

  measure_table   runs every (SubNet, SubGraph) pair on the GPU through the library (lone query:
                  post, wait; median of `runs`) - the counterpart of the paper's table measured on
                  its accelerator;
  model_table     an analytic stand-in (the counterpart of the analytic model of Section 5.1): per
                  op max(flops / peak, bytes not cached / bandwidth) plus a fixed cost per op, from
                  the library's own per-query plan (sushi_team_plan) - needs no GPU.

Both only marshal calls into the library and do arithmetic on its answers; tables are frozen as
JSON so that the library's scheduler and any reference scheduler decide from identical numbers.
"""
import json
import os
import time

import numpy as np

from . import binding as B

HERE = os.path.dirname(os.path.abspath(__file__))
TABLE_DIR = os.path.join(HERE, "tables")


def table_path(workload, budget_bytes, teams_per_xcd):
    """Where the frozen table of a workload lives: measured in exec mode 3 with that many teams per XCD."""
    return os.path.join(TABLE_DIR, "%s_%dMiB_%dteams_mi355x.json" % (workload, budget_bytes >> 20, teams_per_xcd))


def save_table(path, table, workload, budget_bytes, runs, note=""):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    tab = np.asarray(table, dtype=np.float32)
    with open(path, "w") as f:
        json.dump({"workload": workload, "budget_bytes": int(budget_bytes), "runs": runs, "unit": "ms",
                   "n_subnets": int(tab.shape[0]), "n_subgraphs": int(tab.shape[1] - 1), "note": note,
                   "table": [[float(v) for v in row] for row in tab]}, f, indent=0)


def load_table(path, n_subnets, n_subgraphs):
    """The frozen table as a dict with 'table' = float32 array [n_subnets][n_subgraphs + 1], or None
    when there is no file or it was made for another pool / candidate set."""
    if not os.path.exists(path):
        return None
    d = json.load(open(path))
    tab = np.asarray(d["table"], dtype=np.float32)
    if tab.shape != (n_subnets, n_subgraphs + 1):
        return None
    d["table"] = tab
    return d


def measure_table(ctx, subnets, subgraphs, budget_bytes, x, logits, runs=5):
    """Lone-query latency in ms of every SubNet under every cached SubGraph, in the context's current
    execution mode.  x / logits: device tensors of the workload's batch size (contents irrelevant)."""
    n, m = len(subnets), len(subgraphs)
    tab = np.zeros((n, m + 1), dtype=np.float32)
    for j in range(m + 1):
        ctx.sushi_set_subgraph_cache(subgraphs[j] if j < m else None, budget_bytes)
        for i, cfg in enumerate(subnets):
            ctx.sushi_infer(cfg, x, logits)           # plan built, slabs installed, kernel running
            ctx.sushi_synchronize()
            lat = []
            for _ in range(runs):
                a = time.perf_counter()
                ctx.sushi_infer(cfg, x, logits)
                ctx.sushi_synchronize()
                lat.append(time.perf_counter() - a)
            tab[i, j] = np.float32(np.median(lat) * 1e3)
    ctx.sushi_set_subgraph_cache(None, 0)
    return tab


def model_table(arch, subnets, subgraphs, batch, team_wgs, peak_tflops=2500.0, bw_gbs=8000.0, share=1.0 / 64,
                op_floor_us=4.5):
    """Analytic table in ms.  A query runs on `share` of the chip (a team), so it sees that share of the
    peak rates; every op pays `op_floor_us` (team barrier, descriptor and first loads).  Weight bytes of a
    conv / FC op that lie inside the cached SubGraph's box are not counted."""
    m = len(subgraphs)
    tab = np.zeros((len(subnets), m + 1), dtype=np.float32)
    for i, cfg in enumerate(subnets):
        ops = B.sushi_team_plan(arch, cfg, batch, team_wgs)
        for j in range(m + 1):
            g = subgraphs[j] if j < m else None
            t_us = 0.0
            for op in ops:
                kind = op["kind"]
                cin = op["B"] * op["H"] * op["W"] * op["C"]
                cout = op["B"] * op["P"] * op["Q"] * (op["K"] if kind in (0, 1, 4) else op["C"])
                taps = op["R"] * op["R"]
                if kind in (0, 4):
                    wts, flops = op["K"] * op["C"] * taps, 2.0 * cout * op["C"] * taps
                    if g is not None and op["layer"] >= 0:
                        gk, gc, gr = g[op["layer"]]
                        wts -= min(op["K"], gk) * min(op["C"], gc) * min(op["R"], gr) ** 2
                elif kind == 1:
                    wts, flops = op["K"] * taps, 2.0 * cout * taps
                else:
                    wts, flops = 0, float(cin)
                byts = 2.0 * (cin + cout + wts)
                t_us += op_floor_us + max(flops / (peak_tflops * 1e6 * share), byts / (bw_gbs * 1e3 * share))
            tab[i, j] = np.float32(t_us * 1e-3)
    return tab


def latency_levels(table, n_levels):
    """n_levels latency targets evenly spaced between the fastest and the slowest SubNet of the table's
    'nothing cached' column (float32, as the scheduler compares them)."""
    col = np.asarray(table, dtype=np.float32)[:, -1]
    lo, hi = float(col.min()), float(col.max())
    return [float(np.float32(lo + (hi - lo) * k / (n_levels - 1))) for k in range(n_levels)]
