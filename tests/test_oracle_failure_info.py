"""Pins of the oracle's first and second failure-information scheme (section
"Failure information": the list of failed processes, and its length).

The expected lists are not taken from the oracle's bookkeeping: they are written
out from the scheme's definition ("each process appends the ids of all processes
it can not receive a value from") with the tree, groups and send rounds of
oracle.structure (pinned on their own in test_oracle_pins.py):

  - the root selects the lowest-numbered child whose subtree reports no failure,
    i.e. in which every listed process is still alive when it sends its tree
    message;
  - nobody in that subtree misses a tree message, so its list holds exactly the
    processes q outside it that did not send their up-correction message to their
    group mate p inside it: q failed before the operation, or before the round
    t = (pos(p) - pos(q)) mod groupsize in which that message is due.
"""
import itertools

import numpy as np
import pytest

NO_RANK = 0xFFFFFFFF


def _expected(oracle, P, f, root, fail_rank, fail_round):
    """(selected subtree, set of ids in its list) from the definition; None if the root fails."""
    s = oracle.structure(P, f, root)
    F = {int(q): int(r) for q, r in zip(fail_rank, fail_round) if q != NO_RANK}
    if root in F and not (F[root] != 0 and F[root] > f + s["D"]):
        return None                      # the root does not live through the f + D rounds
    subtree, group, gpos, gsize, send = s["subtree"], s["group"], s["gpos"], s["gsize"], s["send_round"]

    def sends_tree_message(q):
        return F[q] != 0 and F[q] > send[q]

    for k in range(1, f + 2):
        if all(sends_tree_message(q) for q in F if subtree[q] == k):
            break
    else:
        return (None, None)
    ids = set()
    for q, rq in F.items():
        if subtree[q] == k or group[q] < 0:
            continue
        for p in range(P):
            if group[p] == group[q] and subtree[p] == k:
                t = (int(gpos[p]) - int(gpos[q])) % int(gsize[q])
                if rq == 0 or t >= rq:
                    ids.add(q)
    return k, ids


def _expected_children(oracle, P, f, root, fail_rank, fail_round):
    """What the root holds from each child at the end, from the definition: a list of
    (state, set of ids), state 0 = no message, 1 = message without the failed bit, 2 = with it.
    A process's observations reach the root's child iff it and all its ancestors send their tree
    messages; such a process lists the group mates that did not send to it and its children that
    sent nothing."""
    s = oracle.structure(P, f, root)
    F = {int(q): int(r) for q, r in zip(fail_rank, fail_round) if q != NO_RANK}
    subtree, group, gpos, gsize, send, parent = (s[k] for k in ("subtree", "group", "gpos", "gsize", "send_round",
                                                                "parent"))

    def sends(q):
        return q not in F or (F[q] != 0 and F[q] > send[q])

    kids = {}
    for p in range(P):
        if parent[p] >= 0:
            kids.setdefault(int(parent[p]), []).append(p)
    out = []
    for top in sorted(kids[root], key=lambda c: subtree[c]):
        k = subtree[top]
        if not sends(top):
            out.append((0, set()))
            continue
        ids, flagged = set(), False
        stack = [top]
        while stack:                                   # the processes connected to the top
            p = stack.pop()
            if group[p] >= 0:
                for q in F:
                    if q != p and group[q] == group[p]:
                        t = (int(gpos[p]) - int(gpos[q])) % int(gsize[p])
                        if F[q] == 0 or t >= F[q]:
                            ids.add(q)
            for c in kids.get(p, []):
                if sends(c):
                    stack.append(c)
                else:
                    ids.add(c)
                    flagged = True
        assert all(subtree[q] == k for q in [top])
        out.append((2 if flagged else 1, ids))
    return out


def _check_children(oracle, b, i, P, f, root, fr, fo):
    want = _expected_children(oracle, P, f, root, fr, fo)
    got = b["info_child"][i]
    assert len(got) == f + 1
    for c, ((state, count, ids), (wstate, wids)) in enumerate(zip(got, want)):
        assert state == wstate, (i, c, got, want)
        assert set(ids) == wids and len(ids) == len(wids) == count, (i, c, got, want)
    # the selected message is the first one without the failed bit
    first = next(c for c, g in enumerate(got) if g[0] == 1)
    assert b["info_ids"][i] == got[first][2] and b["info_count"][i] == got[first][1]


def test_worked_example_list(oracle):
    """Seven processes, f = 1, process 1 failed (second tree figure of the paper): process 2 is the
    one that would exchange values with process 1 and gets nothing from it, so its list is [1];
    the root can only select process 2's message."""
    x = np.arange(7, dtype=np.int64).reshape(1, 7, 1)
    r = oracle.reduce_info_batch(7, 1, x, oracle.I64, oracle.SUM, 1, fail_rank=[[1]], fail_round=[[0]])
    assert r["status"][0] == oracle.ST_OK and int(r["result"][0, 0]) == 20
    assert r["info_ids"][0] == [1] and r["info_count"][0] == 1
    # without failures the list is empty
    r = oracle.reduce_info_batch(7, 1, x, oracle.I64, oracle.SUM, 1, fail_rank=[[NO_RANK]], fail_round=[[0]])
    assert r["info_ids"][0] == [] and r["info_count"][0] == 0


@pytest.mark.parametrize("P,f", [(4, 1), (7, 1), (8, 1), (5, 2), (9, 2), (10, 2), (11, 2), (6, 3), (12, 3), (13, 3)])
def test_every_failure_set_before_the_operation(oracle, P, f):
    """All subsets of size <= f, every root for the small P: list = definition, length = counter,
    value and status as without the bookkeeping."""
    rng = np.random.default_rng(100 + P + f)
    x = rng.integers(-2**40, 2**40, size=(P, 2), dtype=np.int64)
    sets = [c for k in range(f + 1) for c in itertools.combinations(range(P), k)]
    roots = range(P) if P <= 9 else (0, 1, P - 1, f + 1)
    for root in roots:
        S = len(sets)
        fr = np.full((S, max(f, 1)), NO_RANK, np.uint32)
        for i, c in enumerate(sets):
            fr[i, :len(c)] = c
        fo = np.zeros_like(fr)
        rt = np.full(S, root, np.uint32)
        a = oracle.reduce_batch(P, f, x, oracle.I64, oracle.SUM, S, root=rt, fail_rank=fr, fail_round=fo)
        b = oracle.reduce_info_batch(P, f, x, oracle.I64, oracle.SUM, S, root=rt, fail_rank=fr, fail_round=fo)
        assert np.array_equal(a["result"], b["result"]) and np.array_equal(a["status"], b["status"])
        assert np.array_equal(a["msgs"], b["msgs"])
        for i, c in enumerate(sets):
            want = _expected(oracle, P, f, root, fr[i], fo[i])
            if want is None:
                assert b["status"][i] == oracle.ST_ROOT_FAILED and b["info_ids"][i] == []
                continue
            k, ids = want
            assert b["status"][i] == oracle.ST_OK and k is not None
            got = b["info_ids"][i]
            assert set(got) == ids and len(got) == len(ids), (root, c, got, ids)
            assert b["info_count"][i] == len(got)
            _check_children(oracle, b, i, P, f, root, fr[i], fo[i])


@pytest.mark.parametrize("P,f", [(7, 1), (9, 2), (10, 2), (13, 3), (64, 2), (100, 6), (257, 7), (1000, 4)])
def test_failures_during_the_operation(oracle, P, f):
    """Random failure sets with failures during the operation: concatenated lists are disjoint (the
    paper's remark), so length = counter and no id repeats; the list is the one the definition gives."""
    from paper_2602_22445_amd import workloads as w
    S = 600 if P <= 100 else 150
    D = oracle.structure(P, f, 0)["D"]
    fr, fo = w.random_failure_sets(900 + P, S, P, f, inop_permille=700, rounds_per_attempt=f + D + 1)
    root = w.random_roots(900 + P, S, P)
    x = w.payload_int(900 + P, S, P, 1, "i64", 40)
    a = oracle.reduce_batch(P, f, x, oracle.I64, oracle.SUM, S, root=root, fail_rank=fr, fail_round=fo)
    b = oracle.reduce_info_batch(P, f, x, oracle.I64, oracle.SUM, S, root=root, fail_rank=fr, fail_round=fo)
    assert np.array_equal(a["result"], b["result"]) and np.array_equal(a["status"], b["status"])
    seen_nonempty = 0
    for i in range(S):
        got = b["info_ids"][i]
        assert len(got) == len(set(got)) == b["info_count"][i]
        if b["status"][i] != oracle.ST_OK:
            assert got == []
            continue
        want = _expected(oracle, P, f, int(root[i]), fr[i], fo[i])
        assert want is not None and want[0] is not None
        assert set(got) == want[1], (i, fr[i], fo[i], got, want)
        _check_children(oracle, b, i, P, f, int(root[i]), fr[i], fo[i])
        seen_nonempty += bool(got)
    assert seen_nonempty > S // 10


def test_allreduce_reports_the_reduce_that_counted(oracle):
    """Allreduce with dead leading root candidates: the information is that of the attempt that
    succeeded, i.e. of a reduce to the first live candidate."""
    from paper_2602_22445_amd import workloads as w
    P, f, S = 50, 3, 300
    D = oracle.structure(P, f, 0)["D"]
    fr, fo = w.random_failure_sets(77, S, P, f, inop_permille=0, rounds_per_attempt=2 * (f + D), protected=f + 1)
    fr[:40, 0], fo[:40, 0] = 0, 0
    fr[:15, 1], fo[:15, 1] = 1, 0
    for i in range(40):                      # no duplicates in the edited rows
        for k in range(1 if i >= 15 else 2, fr.shape[1]):
            if fr[i, k] in (0, 1):
                fr[i, k] = NO_RANK
    x = w.payload_int(77, S, P, 2, "i64", 40)
    b = oracle.allreduce_info_batch(P, f, x, oracle.I64, oracle.SUM, S, fail_rank=fr, fail_round=fo)
    a = oracle.allreduce_batch(P, f, x, oracle.I64, oracle.SUM, S, fail_rank=fr, fail_round=fo)
    assert np.array_equal(a["result"], b["result"]) and np.array_equal(a["attempts"], b["attempts"])
    assert np.all(b["status"] == oracle.ST_OK)
    for i in range(S):
        root = int(b["attempts"][i]) - 1
        want = _expected(oracle, P, f, root, fr[i], fo[i])
        assert set(b["info_ids"][i]) == want[1] and b["info_count"][i] == len(want[1])
    assert b["attempts"][:15].min() == 3 and b["attempts"][15:40].min() == 2
