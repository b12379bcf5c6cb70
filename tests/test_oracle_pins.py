"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests retypes the oracle's own formulae: they use the paper's
worked example, its closed forms, its theorems as invariants, and brute force
against the plain definition of a valid result (oracle.definition).
"""
import itertools
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

PF_SMALL = [(3, 1), (4, 1), (5, 1), (7, 1), (8, 1), (9, 1), (4, 2), (5, 2), (6, 2), (9, 2), (10, 2),
            (11, 2), (5, 3), (6, 3), (9, 3), (12, 3), (13, 3), (2, 0), (3, 0), (5, 0), (6, 4), (11, 4)]


def _parse_golden():
    d = {}
    with open(os.path.join(GOLDEN, "worked_example_n7_f1.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *rest = line.split()
            d[key] = rest
    return d


# --------------------------------------------------------------------------
# the paper's worked example (section "Reduce / Algorithm", second tree figure)


def test_worked_example_values(oracle):
    g = _parse_golden()
    n, f = int(g["n"][0]), int(g["f"][0])
    failed = [int(x) for x in g["failed"]]
    x = np.arange(n, dtype=np.int64).reshape(n, 1)
    r = oracle.reduce(n, f, x, oracle.I64, oracle.SUM, fail_rank=failed, fail_round=[0] * len(failed), trace=True)
    assert r["status"] == oracle.ST_OK
    assert int(r["result"][0]) == int(g["result"][0])
    for item in g["after_up_correction"]:
        p, v = map(int, item.split(":"))
        assert int(r["v_after_uc"][p, 0]) == v, f"process {p} after up-correction"
    senders = set()
    for item in g["tree_message"]:
        p, v = map(int, item.split(":"))
        senders.add(p)
        assert r["tree_sent"][p] == 1
        assert int(r["tree_msg"][p, 0]) == v, f"tree message of process {p}"
        assert r["tree_flag"][p] == 0
    # "Process 1 does not send any messages"; exactly the listed processes send
    assert set(np.nonzero(r["tree_sent"])[0].tolist()) == senders


def test_worked_example_structure(oracle):
    g = _parse_golden()
    n, f = int(g["n"][0]), int(g["f"][0])
    s = oracle.structure(n, f, 0)
    for item in g["tree_children"]:
        p, kids = item.split(":")
        kids = sorted(int(k) for k in kids.split(","))
        got = sorted(np.nonzero(s["parent"] == int(p))[0].tolist())
        assert got == kids
    groups = [sorted(int(m) for m in grp.split(",")) for grp in g["groups"]]
    for grp in groups:
        ids = {int(s["group"][m]) for m in grp}
        assert len(ids) == 1 and -1 not in ids
        assert sorted(np.nonzero(s["group"] == ids.pop())[0].tolist()) == grp
    assert s["group"][0] == -1          # the root is in no group: n-1 = 6 divisible by f+1 = 2


def test_plain_tree_control_loses_a_subtree(oracle):
    """Without up-correction the failed process cuts off its subtree (first tree
    figure of the paper: the children of process 1 do not get to contribute).
    In the numbering of the second figure these are processes 3 and 5."""
    x = np.arange(7, dtype=np.int64).reshape(7, 1)
    r = oracle.reduce(7, 1, x, oracle.I64, oracle.SUM, fail_rank=[1], fail_round=[0], disable_uc=True)
    # the only complete-looking message comes from process 2: 2 + 4 + 6, plus the root's 0
    assert r["msgs"][0] == 0
    assert int(r["result"][0]) == 0 + 2 + 4 + 6
    assert int(r["result"][0]) != 20


def test_in_operation_failure_is_all_or_nothing_example(oracle):
    """Process 3 of the worked example's tree fails during the operation."""
    x = np.arange(7, dtype=np.int64).reshape(7, 1)
    total = 21
    # fails before sending anything: as if failed beforehand
    r = oracle.reduce(7, 1, x, oracle.I64, oracle.SUM, fail_rank=[3], fail_round=[1])
    assert r["status"] == 0 and int(r["result"][0]) == total - 3
    # completes the up-correction send (round 1) but not its tree send (round 2):
    # subtree 1 reports a failure, subtree 2 holds 3's value via process 4
    r = oracle.reduce(7, 1, x, oracle.I64, oracle.SUM, fail_rank=[3], fail_round=[2], trace=True)
    assert r["status"] == 0 and int(r["result"][0]) == total
    assert r["tree_flag"][1] == 1 and r["tree_flag"][2] == 0
    # fails after its last send: not visible at all
    r = oracle.reduce(7, 1, x, oracle.I64, oracle.SUM, fail_rank=[3], fail_round=[3])
    assert r["status"] == 0 and int(r["result"][0]) == total


# --------------------------------------------------------------------------
# structure: the definition of the I(f)-tree and the group / subtree rules


@pytest.mark.parametrize("P,f", PF_SMALL + [(64, 2), (100, 6), (1024, 3), (257, 7)])
def test_structure_rules(oracle, P, f):
    for root in sorted({0, 1, P - 1, P // 2}):
        s = oracle.structure(P, f, root)
        # relabelling: swap the numbers of the root and of process 0
        virt = np.arange(P)
        virt[root], virt[0] = 0, root
        if root == 0:
            virt[0] = 0
        parent = s["parent"]
        assert parent[root] == -1 and (parent >= 0).sum() == P - 1
        # I(f)-tree, item 1: the root has f+1 children
        kids_of_root = np.nonzero(parent == root)[0]
        assert len(kids_of_root) == f + 1
        # item 2: sizes of the subtrees of the root differ by at most one
        sizes = [(s["subtree"] == k).sum() for k in range(1, f + 2)]
        assert max(sizes) - min(sizes) <= 1 and sum(sizes) == P - 1
        for p in range(P):
            v = virt[p]
            if v == 0:
                continue
            # "the process numbered a is in the k-th subtree, because (a-1) mod (f+1) = k-1"
            assert s["subtree"][p] == (v - 1) % (f + 1) + 1
            # the k-th subtree is the one spanned by the process numbered k
            q = p
            while parent[q] != root:
                q = parent[q]
            assert virt[q] == s["subtree"][p]
            # a child is in its parent's subtree
            if parent[p] != root:
                assert s["subtree"][parent[p]] == s["subtree"][p]
            # group number floor((p-1)/(f+1))
            assert s["group"][p] == (v - 1) // (f + 1)
        # the root joins the last group iff that group has fewer than f+1 members
        last = (P - 2) // (f + 1)
        n_last = sum(1 for p in range(P) if virt[p] != 0 and (virt[p] - 1) // (f + 1) == last)
        if n_last < f + 1:
            assert s["group"][root] == last and s["gsize"][root] == n_last + 1
        else:
            assert s["group"][root] == -1
        # members of one group sit in pairwise different subtrees (root aside)
        for gid in range(last + 1):
            mem = [p for p in range(P) if s["group"][p] == gid and p != root]
            assert len({int(s["subtree"][p]) for p in mem}) == len(mem)
        # every non-root process has at most two children; send rounds follow the heights
        for p in range(P):
            if p != root:
                assert (parent == p).sum() <= 2
                kids = np.nonzero(parent == p)[0]
                h = 0 if len(kids) == 0 else 1 + max(int(s["height"][k]) for k in kids)
                assert s["height"][p] == h
                assert s["send_round"][p] == f + 1 + h
                for k in kids:
                    assert s["send_round"][k] < s["send_round"][p]
        assert s["D"] == 1 + max(int(s["height"][k]) for k in kids_of_root)


@pytest.mark.parametrize("P,f,D", [(7, 1, 2), (8, 1, 3), (64, 2, 5), (1024, 3, 9), (16384, 4, 12)])
def test_round_counts_of_the_benchmark_configurations(oracle, P, f, D):
    """Tree heights of this repository's round model (a definition of the
    repository, not a number of the paper; listed in the baseline table)."""
    assert oracle.structure(P, f, 0)["D"] == D


# --------------------------------------------------------------------------
# values: no failures, failures before the operation (brute force)


def _payload(rng, P, elems, dtype, oracle):
    if dtype == oracle.I64:
        return rng.integers(-2**62, 2**62, size=(P, elems), dtype=np.int64)
    if dtype == oracle.U32:
        return rng.integers(0, 2**32, size=(P, elems), dtype=np.uint32)
    return rng.standard_normal((P, elems))


@pytest.mark.parametrize("P,f", PF_SMALL + [(64, 2), (257, 7), (1000, 3)])
def test_no_failures_gives_full_reduction(oracle, P, f):
    rng = np.random.default_rng(P * 100 + f)
    for dtype, op in [(oracle.I64, oracle.SUM), (oracle.U32, oracle.SUM), (oracle.U32, oracle.BOR),
                      (oracle.I64, oracle.BOR), (oracle.F64, oracle.SUM)]:
        x = _payload(rng, P, 3, dtype, oracle)
        for root in {0, P - 1}:
            r = oracle.reduce(P, f, x, dtype, op, root=root)
            assert r["status"] == oracle.ST_OK
            want = oracle.survivor_reduce(x, dtype, op)
            if dtype == oracle.F64:
                assert np.all(np.abs(r["result"] - want) <= 1e-12 * np.abs(x).sum(axis=0))
            else:
                assert np.array_equal(r["result"], want)


@pytest.mark.parametrize("P,f", [pf for pf in PF_SMALL if pf[0] <= 13 and pf[1] <= 3])
def test_bruteforce_every_preoperational_failure_set(oracle, P, f):
    """<= f failures before the operation: the result is the reduction over the
    processes that did not fail; a failed root makes the operation a no-op."""
    rng = np.random.default_rng(7 * P + f)
    x = _payload(rng, P, 2, oracle.I64, oracle)
    xu = _payload(rng, P, 2, oracle.U32, oracle)
    for root in sorted({0, P - 1, 1}):
        for k in range(f + 1):
            for F in itertools.combinations(range(P), k):
                r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, root=root, fail_rank=F, fail_round=[0] * k)
                if root in F:
                    assert r["status"] == oracle.ST_ROOT_FAILED
                    continue
                assert r["status"] == oracle.ST_OK, (P, f, root, F)
                assert np.array_equal(r["result"], oracle.survivor_reduce(x, oracle.I64, oracle.SUM, F)), (P, f, root, F)
                r = oracle.reduce(P, f, xu, oracle.U32, oracle.BOR, root=root, fail_rank=F, fail_round=[0] * k)
                assert np.array_equal(r["result"], oracle.survivor_reduce(xu, oracle.U32, oracle.BOR, F))


def test_f0_is_a_plain_tree_reduce(oracle):
    """f = 0: groups of one process, no up-correction message; n-1 tree messages."""
    for P in (2, 3, 5, 16, 33):
        x = np.arange(1, P + 1, dtype=np.int64).reshape(P, 1)
        r = oracle.reduce(P, 0, x, oracle.I64, oracle.SUM)
        assert int(r["result"][0]) == P * (P + 1) // 2
        assert r["msgs"][0] == 0 and r["msgs"][1] == P - 1


def test_fp64_sum_is_within_the_stated_tolerance(oracle):
    rng = np.random.default_rng(5)
    P, f = 500, 4
    x = rng.standard_normal((P, 8)) * np.exp(rng.uniform(-20, 20, size=(P, 8)))
    F = [3, 77, 250, 499]
    r = oracle.reduce(P, f, x, oracle.F64, oracle.SUM, fail_rank=F, fail_round=[0] * 4)
    assert oracle.is_valid_result(r["result"], x, oracle.F64, oracle.SUM, F, [])
    assert not oracle.is_valid_result(r["result"], x, oracle.F64, oracle.SUM, F[:3], [])


# --------------------------------------------------------------------------
# message counts (theorem on the number of messages)


def _uc_ff(n, f):
    a = (n - 1) % (f + 1) + 1
    return f * (f + 1) * ((n - 1) // (f + 1)) + a * (a - 1)


@pytest.mark.parametrize("P,f", PF_SMALL + [(64, 2), (1024, 3), (16384, 4), (1000, 8)])
def test_message_counts_failure_free(oracle, P, f):
    x = np.ones((P, 1), dtype=np.int64)
    r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM)
    assert r["msgs"][0] == _uc_ff(P, f)
    assert r["msgs"][1] == P - 1


def test_message_counts_printed_in_the_baseline_table(oracle):
    # closed form evaluated at the benchmark configurations
    assert [_uc_ff(8, 1), _uc_ff(64, 2), _uc_ff(1024, 3), _uc_ff(16384, 4), _uc_ff(1 << 20, 8)] == \
        [8, 126, 3072, 65532, 8388588]


@pytest.mark.parametrize("P,f", [(7, 1), (8, 1), (9, 2), (10, 2), (11, 2), (13, 3), (12, 3)])
def test_message_counts_with_failures(oracle, P, f):
    """Failed processes send fewer messages, nobody sends more: a process failed
    before the operation drops exactly its own sends (g-1 in a group of g, one
    tree message if it is not the root)."""
    x = np.ones((P, 1), dtype=np.int64)
    s = oracle.structure(P, f, 0)
    for k in range(1, f + 1):
        for F in itertools.combinations(range(P), k):
            r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=F, fail_round=[0] * k)
            drop_uc = sum(int(s["gsize"][p]) - 1 for p in F if s["group"][p] >= 0)
            drop_tree = sum(1 for p in F if p != 0)
            assert r["msgs"][0] == _uc_ff(P, f) - drop_uc
            assert r["msgs"][1] == P - 1 - drop_tree


def test_message_counts_in_operation(oracle):
    """A process failing in round r keeps exactly its sends of rounds < r."""
    P, f = 11, 2
    x = np.ones((P, 1), dtype=np.int64)
    s = oracle.structure(P, f, 0)
    R = f + s["D"]
    for p in range(1, P):
        for rnd in range(1, R + 2):
            r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=[p], fail_round=[rnd])
            g = int(s["gsize"][p])
            uc_done = min(rnd - 1, g - 1)
            tree_done = 1 if int(s["send_round"][p]) < rnd else 0
            assert r["msgs"][0] == _uc_ff(P, f) - (g - 1) + uc_done
            assert r["msgs"][1] == P - 1 - 1 + tree_done


# --------------------------------------------------------------------------
# multiplicities: one-hot payload makes double or partial inclusion visible


def _onehot(P):
    return np.eye(P, dtype=np.int64)


@pytest.mark.parametrize("P,f", [(4, 1), (7, 1), (8, 1), (5, 2), (9, 2), (10, 2), (11, 2), (6, 3), (9, 3)])
def test_all_or_nothing_every_failure_time(oracle, P, f):
    """Every set of <= f failed processes, every failure time: never-failed
    processes are included exactly once, processes failed beforehand not at all,
    processes failed during the operation zero times or once."""
    x = _onehot(P)
    R = f + oracle.structure(P, f, 0)["D"]
    times = list(range(0, R + 1))
    for k in range(f + 1):
        for F in itertools.combinations(range(1, P), k):       # root alive
            for T in itertools.product(times, repeat=k):
                r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=F, fail_round=T)
                assert r["status"] == oracle.ST_OK, (F, T)     # a failure-free subtree always exists
                mult = r["result"]
                for p in range(P):
                    if p not in F:
                        assert mult[p] == 1, (F, T, p)
                    elif T[F.index(p)] == 0:
                        assert mult[p] == 0, (F, T, p)
                    else:
                        assert mult[p] in (0, 1), (F, T, p)


@pytest.mark.parametrize("P,f", [(7, 1), (8, 1), (9, 2), (10, 2), (11, 2), (13, 3), (12, 3), (30, 4)])
def test_replication_theorem(oracle, P, f):
    """After up-correction and the tree phase, every subtree of the root that
    reports no failure holds every never-failed value outside the root's group
    exactly once; the root's group is held (once) iff the subtree has a member
    of it."""
    x = _onehot(P)
    s = oracle.structure(P, f, 0)
    rng = np.random.default_rng(P + f)
    sets = [()]
    for k in range(1, f + 1):
        combos = list(itertools.combinations(range(1, P), k))
        rng.shuffle(combos)
        sets += combos[:60]
    root_group = int(s["group"][0])
    for F in sets:
        r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=F, fail_round=[0] * len(F), trace=True)
        clean = 0
        for k in range(1, f + 2):
            if not r["tree_sent"][k] or r["tree_flag"][k]:
                # a subtree with a failed member must not claim "no failure"
                continue
            clean += 1
            assert not any(s["subtree"][p] == k for p in F)
            has_root_group_member = any(s["group"][p] == root_group and s["subtree"][p] == k
                                        for p in range(1, P)) if root_group >= 0 else False
            for p in range(P):
                in_root_group = (p == 0) or (root_group >= 0 and s["group"][p] == root_group)
                want = 0 if p in F else 1
                if in_root_group and not has_root_group_member:
                    want = 0
                assert r["tree_msg"][k][p] == want, (F, k, p)
        assert clean >= f + 1 - len(F)
        # subtrees with a failed member never claim "no failure"
        for k in range(1, f + 2):
            if any(s["subtree"][p] == k for p in F):
                assert (not r["tree_sent"][k]) or r["tree_flag"][k]


def test_more_than_f_failures_can_leave_no_clean_subtree(oracle):
    """The bound f is tight: f+1 failures, one per subtree, and the root has no
    failure-free subtree to select."""
    for P, f in [(7, 1), (10, 2), (13, 3)]:
        x = _onehot(P)
        F = list(range(1, f + 2))
        r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=F, fail_round=[0] * len(F))
        assert r["status"] == oracle.ST_NO_CLEAN_SUBTREE


def test_bad_failure_sets(oracle):
    x = np.ones((8, 1), dtype=np.int64)
    assert oracle.reduce(8, 1, x, oracle.I64, oracle.SUM, fail_rank=[8], fail_round=[0])["status"] == oracle.ST_BAD_FAILURE_SET
    assert oracle.reduce(8, 2, x, oracle.I64, oracle.SUM, fail_rank=[3, 3], fail_round=[0, 0])["status"] == oracle.ST_BAD_FAILURE_SET
    assert oracle.allreduce(8, 1, x, oracle.I64, oracle.SUM, fail_rank=[1], fail_round=[2])["status"] == oracle.ST_BAD_FAILURE_SET
    with pytest.raises(ValueError):
        oracle.reduce(2, 1, x[:2], oracle.I64, oracle.SUM)      # needs P >= f + 2
