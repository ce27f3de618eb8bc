"""Seeded query streams and SubGraph candidate sets for the five configurations.

A stream is a list of SubnetCfg (one per query) or, for the latency-target
stream, a list of level indices.  The SubGraph candidate generator works on
per-layer (K, C, r) triples that the caller computes with its own encoder; it
only shrinks those boxes until they fit a byte budget.
"""
from .arch import FAMILY_TINY, SubnetCfg, max_cfg, min_cfg
from .rng import Stream, derive


def uniform_cfg(arch, st, resolution=None):
    """One SubNet drawn uniformly over every elastic choice."""
    nd = len(arch.depth_drop_choices)
    if arch.family == FAMILY_TINY:
        depth = [arch.n_stages - arch.depth_drop_choices[st.randint(nd)]]
    else:
        depth = [m - arch.depth_drop_choices[st.randint(nd)] for m in arch.stage_max_depth]
    width = [st.randint(len(arch.width_choices)) for _ in range(arch.n_stages + 1)]
    nb = arch.n_block_slots
    expand = [st.randint(len(arch.expand_choices)) for _ in range(nb)]
    kernel = [st.randint(len(arch.kernel_choices)) for _ in range(nb)]
    if resolution is None:
        resolution = arch.res_choices[st.randint(len(arch.res_choices))] \
            if len(arch.res_choices) > 1 else arch.res_choices[0]
    return SubnetCfg(resolution, depth, width, expand, kernel)


def stream_uniform(arch, n, seed, resolution=None):
    """Config 1: n queries, each SubNet uniform."""
    st = Stream(derive(seed, 1))
    return [uniform_cfg(arch, st, resolution) for _ in range(n)]


def stream_sticky(arch, n, seed, p_repeat=0.8, resolution=None):
    """Config 2: the next SubNet repeats the previous one with probability p_repeat, else uniform."""
    st = Stream(derive(seed, 2))
    out = [uniform_cfg(arch, st, resolution)]
    for _ in range(n - 1):
        if st.next_uniform() < p_repeat:
            out.append(out[-1])
        else:
            out.append(uniform_cfg(arch, st, resolution))
    return out


def subnet_pool(arch, n_pool, seed, resolution=None):
    """n_pool seeded SubNets including the smallest and the largest."""
    st = Stream(derive(seed, 3))
    res = resolution or max(arch.res_choices)
    pool = [min_cfg(arch, res), max_cfg(arch, res)]
    while len(pool) < n_pool:
        pool.append(uniform_cfg(arch, st, res))
    return pool


def _zipf_cdf(n, s):
    w = [(r + 1) ** (-s) for r in range(n)]
    tot = sum(w)
    acc, cdf = 0.0, []
    for x in w:
        acc += x / tot
        cdf.append(acc)
    return cdf


def stream_zipf(n_pool, n, seed, s=1.2, regime=None, resolutions=None):
    """Configs 3 and 5: indices into a pool; P(rank r) ~ r^-s under a seeded rank permutation,
    re-drawn every `regime` queries if given.  Returns (pool_index, resolution_or_None) pairs."""
    st = Stream(derive(seed, 4))
    cdf = _zipf_cdf(n_pool, s)
    perm = st.permutation(n_pool)
    out = []
    for t in range(n):
        if regime and t > 0 and t % regime == 0:
            perm = st.permutation(n_pool)
        u = st.next_uniform()
        r = 0
        while r < n_pool - 1 and u >= cdf[r]:
            r += 1
        res = resolutions[st.randint(len(resolutions))] if resolutions else None
        out.append((perm[r], res))
    return out


def stream_levels(n_levels, n, seed):
    """Config 4: a latency-target level per query, uniform over n_levels."""
    st = Stream(derive(seed, 5))
    return [st.randint(n_levels) for _ in range(n)]


def with_resolution(cfg, res):
    return SubnetCfg(res, list(cfg.depth), list(cfg.width_idx), list(cfg.expand_idx), list(cfg.kernel_idx))


def box_bytes(box, bytes_per_weight):
    """box: list of (K, C, r) per layer."""
    return sum(k * c * r * r for (k, c, r) in box) * bytes_per_weight


def shrink_box(box, budget_bytes, bytes_per_weight, grid=8):
    """Scale every layer's K and C (not r) by the largest f = m/64 for which the box fits the
    budget; counts are rounded down to the channel grid, floor one grid step, and a C of 1
    (depthwise) or below the grid (the 3-channel input) is kept."""
    def scaled(v, m):
        if v <= grid:
            return v
        return max(grid, (v * m // 64) // grid * grid)
    for m in range(64, 0, -1):
        cand = [(scaled(k, m) if k else 0, scaled(c, m) if k else 0, r if k else 0) for (k, c, r) in box]
        if box_bytes(cand, bytes_per_weight) <= budget_bytes:
            return cand
    return [(0, 0, 0) for _ in box]


def candidate_subgraphs(boxes, budget_bytes, bytes_per_weight, max_candidates):
    """SubGraph set S: each given SubNet box shrunk to the budget, duplicates removed, in order."""
    seen, out = set(), []
    for b in boxes:
        g = tuple(shrink_box(b, budget_bytes, bytes_per_weight))
        if g not in seen:
            seen.add(g)
            out.append(list(g))
        if len(out) >= max_candidates:
            break
    return out
