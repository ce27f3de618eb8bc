"""Pins for the reference scheduler (oracle/sched_ref.py) against Algorithm 1 and Section 3.3.

The paper gives no worked scheduling example; the one below is worked by hand in the comments.
"""
import numpy as np

from oracle.sched_ref import STRICT_ACCURACY, STRICT_LATENCY, SchedRef
from workloads.rng import Stream

# Three SubNets (two layers -> vectors [K1,C1,K2,C2]) and two candidate SubGraphs.
V = [[8, 3, 8, 8], [16, 3, 16, 16], [32, 3, 32, 32]]
ACC = [0.70, 0.75, 0.80]
G = [[8, 3, 8, 8], [16, 3, 32, 16]]
#            G0    G1   nothing cached
TABLE = [[1.0, 1.5, 2.0],      # SubNet 0
         [3.0, 2.2, 4.0],      # SubNet 1
         [6.0, 4.5, 7.0]]      # SubNet 2


def test_hand_worked_strict_latency():
    s = SchedRef(V, ACC, G, TABLE, Q=2, policy=STRICT_LATENCY)
    # t=0, cache empty -> column 2 = [2,4,7]; L_t=4.5 -> feasible {0,1} -> most accurate = 1
    assert s.step(0.0, 4.5) == (1, -1)
    # t=1, still column 2; L_t=7 -> feasible {0,1,2} -> 2.  Second query: window = V1, V2,
    # sums = [48,6,48,48], n=2.  d(G0) = (16-48)^2+0+(16-48)^2+(16-48)^2 = 3072;
    # d(G1) = (32-48)^2+0+(64-48)^2+(32-48)^2 = 768 -> cache G1
    assert s.step(0.0, 7.0) == (2, 1)
    # t=2, column 1 = [1.5,2.2,4.5]; L_t=4.5 now admits SubNet 2 (it did not with nothing cached)
    assert s.step(0.0, 4.5) == (2, -1)
    # t=3: L_t=1.0 admits nobody -> smallest latency = SubNet 0.  Window = V2, V0: sums = [40,6,40,40]
    # d(G0) = 3*(16-40)^2 = 1728; d(G1) = (32-40)^2 + (64-40)^2 + (32-40)^2 = 704 -> G1 again
    assert s.step(0.0, 1.0) == (0, 1)
    # t=4,5: two small queries: window = V0, V0 -> sums [16,6,16,16]; d(G0) = 0 -> cache G0
    assert s.step(0.0, 1.6) == (0, -1)
    assert s.step(0.0, 1.6) == (0, 0)
    assert s.cache == 0


def test_hand_worked_strict_accuracy():
    s = SchedRef(V, ACC, G, TABLE, Q=3, policy=STRICT_ACCURACY, initial_cache=0)
    # column 0 = [1,3,6]; A_t = 0.72 -> feasible {1,2} -> min latency = 1
    assert s.step(0.72, 0.0) == (1, -1)
    # A_t = 0.70 -> feasible all -> SubNet 0
    assert s.step(0.70, 0.0) == (0, -1)
    # A_t = 0.9 -> nobody -> most accurate = 2; third query -> re-choose:
    # sums = V1+V0+V2 = [56,9,56,56], n=3: d(G0) = 3*(24-56)^2 = 3072,
    # d(G1) = (48-56)^2 + (96-56)^2 + (48-56)^2 = 1728 -> G1
    assert s.step(0.90, 0.0) == (2, 1)


def _random_problem(seed, n=6, m=5, length=8):
    st = Stream(seed)
    v = [[8 * (1 + st.randint(8)) for _ in range(length)] for _ in range(n)]
    g = [[8 * (1 + st.randint(8)) for _ in range(length)] for _ in range(m)]
    acc = sorted(0.6 + 0.3 * st.next_uniform() for _ in range(n))
    table = [[1.0 + 9.0 * st.next_uniform() for _ in range(m + 1)] for _ in range(n)]
    return v, acc, g, table


def test_hard_constraint_holds_when_feasible():
    """Section 3.3: under strict accuracy the served accuracy >= A_t, under strict latency the
    table latency under the current cache <= L_t, whenever some SubNet qualifies."""
    for seed in range(5):
        v, acc, g, table = _random_problem(seed)
        st = Stream(100 + seed)
        for policy in (STRICT_ACCURACY, STRICT_LATENCY):
            s = SchedRef(v, acc, g, table, Q=3, policy=policy)
            for _ in range(40):
                a_t, l_t = 0.55 + 0.4 * st.next_uniform(), 12.0 * st.next_uniform()
                col = s.M if s.cache < 0 else s.cache
                i, _ = s.step(a_t, l_t)
                if policy == STRICT_ACCURACY and any(a >= a_t for a in acc):
                    assert acc[i] >= a_t
                    assert all(table[i][col] <= table[k][col] for k in range(len(v)) if acc[k] >= a_t)
                if policy == STRICT_LATENCY and any(table[k][col] <= l_t for k in range(len(v))):
                    assert table[i][col] <= l_t
                    assert all(acc[i] >= acc[k] for k in range(len(v)) if table[k][col] <= l_t)


def test_q1_with_subnets_as_candidates_follows_last_served():
    v, acc, _, table = _random_problem(3, n=5, m=5)
    table = [row[:6] for row in table]
    s = SchedRef(v, acc, v, table, Q=1, policy=STRICT_LATENCY)
    st = Stream(7)
    for _ in range(20):
        i = st.randint(5)
        new = s.record(v[i])
        assert v[new] == v[i]          # distance 0 to itself (lowest index among duplicates)


def test_constant_stream_settles_on_nearest_candidate():
    v, acc, g, table = _random_problem(4)
    s = SchedRef(v, acc, g, table, Q=4, policy=STRICT_LATENCY)
    want = int(np.argmin([sum((a - b) ** 2 for a, b in zip(gj, v[2])) for gj in g]))
    seen = [s.record(v[2]) for _ in range(16)]
    assert seen == [-1, -1, -1, want] * 4


def test_distance_is_distance_to_the_mean():
    """The integer form sum (n*g - sum v)^2 orders candidates like ||g - mean(v)||."""
    v, acc, g, table = _random_problem(5, n=6, m=7)
    s = SchedRef(v, acc, g, table, Q=3, policy=STRICT_LATENCY)
    st = Stream(11)
    for t in range(30):
        i = st.randint(6)
        new = s.record(v[i])
        if new >= 0:
            mean = np.mean(np.array(s.window, dtype=np.float64), axis=0)
            d = [np.sum((np.array(gj) - mean) ** 2) for gj in g]
            assert abs(d[new] - min(d)) < 1e-9


def test_window_is_the_last_q_and_ties_take_lowest_index():
    g = [[8, 8], [8, 8], [24, 24]]
    v = [[8, 8], [24, 24]]
    s = SchedRef(v, [0.1, 0.2], g, [[1, 1, 1, 1], [2, 2, 2, 2]], Q=2, policy=STRICT_LATENCY)
    assert [s.record(v[0]), s.record(v[0])] == [-1, 0]      # tie between G0 and G1 -> 0
    assert [s.record(v[1]), s.record(v[1])] == [-1, 2]      # old entries left the window
    # argmax tie on accuracy -> lowest index
    s2 = SchedRef(v, [0.5, 0.5], g, [[1, 1, 1, 1], [1, 1, 1, 1]], Q=2, policy=STRICT_LATENCY)
    assert s2.select(0.0, 5.0) == 0
    s3 = SchedRef(v, [0.5, 0.5], g, [[1, 1, 1, 1], [1, 1, 1, 1]], Q=2, policy=STRICT_ACCURACY)
    assert s3.select(0.4, 0.0) == 0


def test_permuting_candidates_permutes_decisions():
    v, acc, g, table = _random_problem(6, n=5, m=6)
    perm = [3, 0, 5, 1, 4, 2]
    g2 = [g[p] for p in perm]
    table2 = [[row[p] for p in perm] + [row[6]] for row in table]
    a = SchedRef(v, acc, g, table, Q=2, policy=STRICT_LATENCY)
    b = SchedRef(v, acc, g2, table2, Q=2, policy=STRICT_LATENCY)
    st = Stream(21)
    for _ in range(30):
        l_t = 1.0 + 10.0 * st.next_uniform()
        ia, ca = a.step(0.0, l_t)
        ib, cb = b.step(0.0, l_t)
        assert ia == ib
        assert (ca == -1 and cb == -1) or perm[cb] == ca
