"""A model of the team kernel's mailbox protocol, checked over EVERY interleaving of host and team leader.

The host posts queries into a ring of POST_RING slots per team and publishes residency tables in a ring of
table generations; the team leader (a GPU thread) polls the `posted` counter, reads the post, reads the table
the post names if it differs from the one its team holds, runs the query and writes `done`.  Nothing but two
counters orders the two sides, so the protocol is only right if

  * a mailbox slot is rewritten only after `done` has passed the post that sat in it, and
  * a table generation is rewritten only after `done` has passed the last post that names it.

The model below restates both sides word by word (one step = one access to a shared word, in program order;
the release fence on the host and the leader's wait for the counter's value before it asks for the post make
that the right granularity) and explores all interleavings exhaustively for small rings.  Every word the
leader reads must belong to the post / table it expects.  Two planted mistakes (a ring guard that is off by
one, a generation reused without the wait) must each be caught, which shows that the exploration can see the
failures it is meant to exclude.
"""
import pytest


def explore(n_posts, ring, gens, table_changes, ring_guard_slack=0, wait_for_generation=True):
    """Depth-first search over all interleavings.  Returns None if every run ends with all posts served and
    no inconsistent read, else a string naming the first violation found.

    Shared words: posted, done, per slot (a, b, seq, tab, tab_seq), per generation (t1, t2).
    table_changes: posts (1-based) before which the host publishes a new table."""
    # host program, as a list of micro-steps per post
    host_prog = []
    for k in range(1, n_posts + 1):
        if k in table_changes:
            host_prog += [("gen_wait",), ("gen_w1",), ("gen_w2",), ("gen_commit",)]
        host_prog += [("ring_wait", k), ("w_a", k), ("w_b", k), ("w_tab", k), ("w_seq", k), ("publish", k)]
    init = dict(posted=0, done=0,
                slots=tuple((0, 0, 0, -1, 0) for _ in range(ring)),       # a, b, seq, table slot, table seq
                tables=tuple((0, 0) for _ in range(gens)),                # two words, both = the table's number
                # host-private
                hpc=0, gen_cur=0, table_seq=1, last_ref=tuple(0 for _ in range(gens)), cur_valid=False,
                # leader-private
                dpc="poll", my_seq=0, held=0, got=None, tslot=-1, tseq=0, t1=0)
    seen = set()
    stack = [init]

    def freeze(s):
        return tuple(sorted((k, v) for k, v in s.items()))

    while stack:
        s = stack.pop()
        key = freeze(s)
        if key in seen:
            continue
        seen.add(key)
        moves = []
        # ---- host step
        if s["hpc"] < len(host_prog):
            op = host_prog[s["hpc"]]
            h = dict(s)
            h["hpc"] += 1
            kind = op[0]
            ok = True
            if kind == "gen_wait":
                nxt = (s["gen_cur"] + 1) % gens
                if wait_for_generation and s["done"] < s["last_ref"][nxt]:
                    ok = False                                           # blocked: the step is not enabled
            elif kind == "gen_w1":
                nxt = (s["gen_cur"] + 1) % gens
                t = list(s["tables"]); t[nxt] = (s["table_seq"] + 1, t[nxt][1]); h["tables"] = tuple(t)
            elif kind == "gen_w2":
                nxt = (s["gen_cur"] + 1) % gens
                t = list(s["tables"]); t[nxt] = (t[nxt][0], s["table_seq"] + 1); h["tables"] = tuple(t)
            elif kind == "gen_commit":
                h["gen_cur"] = (s["gen_cur"] + 1) % gens
                h["table_seq"] = s["table_seq"] + 1
                h["cur_valid"] = True
            elif kind == "ring_wait":
                if s["posted"] - s["done"] >= ring + ring_guard_slack:
                    ok = False
            elif kind in ("w_a", "w_b", "w_tab", "w_seq"):
                k = op[1]
                sl = list(s["slots"]); a, b, q, ts, tq = sl[k % ring]
                if kind == "w_a":
                    a = k
                elif kind == "w_b":
                    b = k
                elif kind == "w_tab":
                    ts, tq = (s["gen_cur"] if s["cur_valid"] else -1), s["table_seq"]
                    lr = list(s["last_ref"]); lr[s["gen_cur"]] = k; h["last_ref"] = tuple(lr)
                else:
                    q = k
                sl[k % ring] = (a, b, q, ts, tq); h["slots"] = tuple(sl)
            elif kind == "publish":
                h["posted"] = op[1]
            if ok:
                moves.append(h)
        # ---- leader step
        d = dict(s)
        pc = s["dpc"]
        if pc == "poll":
            if s["posted"] > s["my_seq"]:
                d["dpc"] = "r_a"
                moves.append(d)
            elif s["hpc"] >= len(host_prog) and s["done"] == n_posts:
                pass                                                     # finished
            elif s["hpc"] < len(host_prog):
                pass                                                     # polling again changes nothing: not a move
        else:
            want = s["my_seq"] + 1
            slot = s["slots"][want % ring]
            if pc == "r_a":
                if slot[0] != want:
                    return "post %d: first payload word read as %d" % (want, slot[0])
                d["dpc"] = "r_b"
            elif pc == "r_b":
                if slot[1] != want:
                    return "post %d: second payload word read as %d" % (want, slot[1])
                d["dpc"] = "r_seq"
            elif pc == "r_seq":
                if slot[2] != want:
                    return "post %d: sequence word read as %d" % (want, slot[2])
                d["dpc"] = "r_tab"
            elif pc == "r_tab":
                d["tslot"], d["tseq"] = slot[3], slot[4]
                d["dpc"] = "t1" if (slot[4] != s["held"] and slot[3] >= 0) else "finish"
                if slot[3] < 0:
                    d["held"] = slot[4]
            elif pc == "t1":
                d["t1"] = s["tables"][s["tslot"]][0]
                d["dpc"] = "t2"
            elif pc == "t2":
                t2 = s["tables"][s["tslot"]][1]
                if s["t1"] != s["tseq"] or t2 != s["tseq"]:
                    return "post %d names table %d, read words (%d, %d)" % (want, s["tseq"], s["t1"], t2)
                d["held"] = s["tseq"]
                d["dpc"] = "finish"
            elif pc == "finish":
                d["done"] = want
                d["my_seq"] = want
                d["dpc"] = "poll"
            moves.append(d)
        if not moves:
            if not (s["hpc"] >= len(host_prog) and s["done"] == n_posts):
                return "deadlock at host step %d, leader %s, posted %d, done %d" % (s["hpc"], pc, s["posted"], s["done"])
        stack.extend(moves)
    return None


@pytest.mark.parametrize("ring,gens", [(1, 2), (2, 2), (3, 2), (2, 3)])
def test_every_interleaving_reads_consistent_posts_and_tables(ring, gens):
    assert explore(6, ring, gens, table_changes={2, 3, 4, 6}) is None
    assert explore(5, ring, gens, table_changes=set()) is None
    assert explore(5, ring, gens, table_changes={1, 2, 3, 4, 5}) is None


def test_a_ring_guard_off_by_one_is_caught():
    bad = explore(5, 2, 2, table_changes={2}, ring_guard_slack=1)
    assert bad is not None and "read as" in bad


def test_a_generation_reused_without_the_wait_is_caught():
    bad = explore(6, 3, 2, table_changes={2, 3, 4}, wait_for_generation=False)
    assert bad is not None and "names table" in bad
