"""Reference SushiSched — TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Follows the paper's scheduling algorithm (Algorithm 1 and Section 3.3) step by step:

  per query   policy STRICT_ACCURACY: among SubNets with accuracy >= A_t serve the one with the
              smallest table latency under the current cache state;
              policy STRICT_LATENCY:  among SubNets whose table latency under the current cache
              state is <= L_t serve the most accurate one;
  every Q     keep the vectors of the last Q served SubNets; after every Q-th query cache the
  queries     candidate SubGraph whose vector is nearest to their average.

Readings where the text leaves a choice (all mirrored by the GPU library's host code):
  * distance = squared Euclidean, evaluated exactly in integers as sum_k (Q*g[k] - sum_window v[k])^2,
    which orders candidates exactly as the distance to the mean does;
  * ties (argmin / argmax) go to the lowest index;
  * empty feasible set: STRICT_ACCURACY serves the most accurate SubNet, STRICT_LATENCY the one
    with the smallest table latency;
  * the table has one extra last column for "nothing cached", used while the cache state is empty
    (Algorithm 1 starts from an empty cache state).
"""

STRICT_ACCURACY = 0
STRICT_LATENCY = 1


class SchedRef:
    def __init__(self, subnet_vecs, accuracy, subgraph_vecs, table, Q, policy, initial_cache=-1):
        """subnet_vecs: N integer vectors; subgraph_vecs: M integer vectors of the same length;
        table: N rows of M+1 latencies (column M = nothing cached); initial_cache: -1 = empty."""
        self.v = [list(map(int, x)) for x in subnet_vecs]
        self.acc = [float(a) for a in accuracy]
        self.g = [list(map(int, x)) for x in subgraph_vecs]
        self.L = [[float(x) for x in row] for row in table]
        self.N, self.M = len(self.v), len(self.g)
        assert all(len(r) == self.M + 1 for r in self.L)
        self.Q, self.policy = int(Q), policy
        self.cache = int(initial_cache)
        self.window = []
        self.t = 0

    def _col(self):
        return self.M if self.cache < 0 else self.cache

    def select(self, a_t, l_t):
        """SubNet index for a query with accuracy target a_t and latency target l_t."""
        col = self._col()
        if self.policy == STRICT_ACCURACY:
            feas = [i for i in range(self.N) if self.acc[i] >= a_t]
            if not feas:
                return max(range(self.N), key=lambda i: (self.acc[i], -i))
            return min(feas, key=lambda i: (self.L[i][col], i))
        feas = [i for i in range(self.N) if self.L[i][col] <= l_t]
        if not feas:
            return min(range(self.N), key=lambda i: (self.L[i][col], i))
        return max(feas, key=lambda i: (self.acc[i], -i))

    def record(self, vec):
        """Account one served SubNet vector; returns the new cache index if the cache is re-chosen
        on this query (after every Q-th), else -1."""
        self.window.append(list(map(int, vec)))
        if len(self.window) > self.Q:
            self.window.pop(0)
        self.t += 1
        if self.t % self.Q != 0 or self.M == 0:
            return -1
        sums = [sum(col) for col in zip(*self.window)]
        n = len(self.window)
        best, best_d = -1, None
        for j in range(self.M):
            d = sum((n * gk - sk) ** 2 for gk, sk in zip(self.g[j], sums))
            if best_d is None or d < best_d:
                best, best_d = j, d
        self.cache = best
        return best

    def step(self, a_t, l_t):
        """One query: (served SubNet index, new cache index or -1)."""
        i = self.select(a_t, l_t)
        return i, self.record(self.v[i])
