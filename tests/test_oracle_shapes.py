"""Pins of the CPU oracle for the other tree shapes inside a subtree of the root (the
definition of the I(f)-tree fixes only the root's f+1 children and the sizes of their
subtrees) and for the latency bookkeeping (detected failures, message steps).

What the paper fixes does not depend on the shape: the I(f) rules, the values under
failures before the operation, all-or-nothing under failures during it, the replication
theorem, the message counts.  The shapes themselves are pinned by their textbook
properties (children per process, heights), the bookkeeping by closed forms on perfect
trees and by who must notice a failed process."""
import itertools

import numpy as np
import pytest

SHAPES = [2, 3, 4, 8, 1]            # k children per process (2 = the default), 1 = binomial
PF = [(5, 1), (7, 1), (8, 1), (10, 1), (15, 1), (9, 2), (10, 2), (14, 2), (13, 3), (12, 3), (6, 4), (23, 4), (4, 0), (9, 0)]


def _subtree_members(s, P, k):
    return [p for p in range(1, P) if s["subtree"][p] == k]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("P,f", PF)
def test_if_tree_rules_hold_for_every_shape(oracle, P, f, shape):
    """Definition of the I(f)-tree: the root has f+1 children and their subtrees differ in size by at most one;
    proof of the replication theorem: process a is in subtree k iff (a-1) mod (f+1) = k-1; the groups do not
    depend on the shape."""
    s = oracle.structure(P, f, 0, shape)
    s2 = oracle.structure(P, f, 0, 2)
    kids0 = [p for p in range(1, P) if s["parent"][p] == 0]
    assert kids0 == list(range(1, f + 2))
    sizes = [len(_subtree_members(s, P, k)) for k in range(1, f + 2)]
    assert max(sizes) - min(sizes) <= 1 and sum(sizes) == P - 1
    for a in range(1, P):
        assert s["subtree"][a] == (a - 1) % (f + 1) + 1
        assert s["subtree"][s["parent"][a]] in (0, s["subtree"][a])        # parents stay inside the subtree
    for key in ("group", "gpos", "gsize", "subtree"):
        assert np.array_equal(s[key], s2[key])
    # heights and depths are those of the parent links
    for a in range(1, P):
        assert s["depth"][a] == s["depth"][s["parent"][a]] + 1
    for p in range(P):
        ch = [a for a in range(1, P) if s["parent"][a] == p]
        assert s["height"][p] == (1 + max(s["height"][a] for a in ch) if ch else 0)
    assert s["D"] == s["height"][0]


@pytest.mark.parametrize("P,f", [(16, 0), (41, 1), (100, 2), (64, 3)])
def test_shapes_are_the_textbook_ones(oracle, P, f):
    for k in (2, 3, 4, 8):
        s = oracle.structure(P, f, 0, k)
        for sub in range(1, f + 2):
            mem = _subtree_members(s, P, sub)              # in the order they joined
            m = len(mem)
            nk = [sum(1 for a in mem if s["parent"][a] == p) for p in mem]
            # filled breadth-first: the j-th process has children k*j+1 .. k*j+k of the joining order
            for j, p in enumerate(mem):
                want = [mem[c] for c in range(k * j + 1, k * j + k + 1) if c < m]
                assert [a for a in mem if s["parent"][a] == p] == want
            assert max(nk) <= k
            # height of a k-ary tree filled breadth-first: the fewest levels that hold m processes
            h, cap = 0, 1
            while cap < m:
                h += 1
                cap += k ** h
            assert s["height"][mem[0]] == h
    s = oracle.structure(P, f, 0, oracle.BINOMIAL)
    for sub in range(1, f + 2):
        mem = _subtree_members(s, P, sub)
        m = len(mem)
        for j, p in enumerate(mem):
            if j:           # joined as number j: child of number j without its highest bit
                assert s["parent"][p] == mem[j - (1 << (j.bit_length() - 1))]
        # the first process of a binomial tree of m processes has ceil(log2 m) children (numbers 1, 2, 4, ..), and a
        # process stands as many levels below it as its number has one bits
        assert sum(1 for a in mem if s["parent"][a] == mem[0]) == (m - 1).bit_length()
        assert s["height"][mem[0]] == max(bin(j).count("1") for j in range(m))
        for p in mem:
            assert s["depth"][p] == 1 + bin(mem.index(p)).count("1")


@pytest.mark.parametrize("shape", [3, 4, 1])
@pytest.mark.parametrize("P,f", [(5, 1), (8, 1), (9, 2), (11, 2), (13, 3), (10, 1), (14, 2)])
def test_bruteforce_every_preoperational_failure_set(oracle, P, f, shape):
    """<= f failures before the operation: the result is the reduction over the processes that did not fail,
    whatever the shape; a failed root makes the reduce a no-op; failed processes send fewer messages, nobody
    sends more (message-count theorem: the counts do not depend on the shape either)."""
    rng = np.random.default_rng(100 * P + 10 * f + shape)
    x = rng.integers(-1000, 1000, size=(P, 2)).astype(np.int64)
    ff = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, shape=shape)
    a = (P - 1) % (f + 1) + 1
    assert ff["msgs"][0] == f * (f + 1) * ((P - 1) // (f + 1)) + a * (a - 1) and ff["msgs"][1] == P - 1
    s = oracle.structure(P, f, 0, shape)
    for k in range(f + 1):
        for F in itertools.combinations(range(P), k):
            r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=list(F), fail_round=[0] * k, shape=shape)
            if 0 in F:
                assert r["status"] == oracle.ST_ROOT_FAILED
                continue
            assert r["status"] == oracle.ST_OK
            assert np.array_equal(r["result"], oracle.survivor_reduce(x, oracle.I64, oracle.SUM, list(F)))
            drop_uc = sum(int(s["gsize"][p]) - 1 for p in F if s["group"][p] >= 0)
            assert r["msgs"][0] == ff["msgs"][0] - drop_uc and r["msgs"][1] == P - 1 - len(F)


@pytest.mark.parametrize("shape", [3, 1])
@pytest.mark.parametrize("P,f", [(8, 1), (9, 2), (11, 2), (12, 3)])
def test_all_or_nothing_every_failure_time(oracle, P, f, shape):
    """Every set of <= f failed processes, every failure time (one-hot inputs): never-failed processes count
    exactly once, processes failed beforehand not at all, processes failed during the operation not or once."""
    x = np.eye(P, dtype=np.int64)
    R = f + oracle.structure(P, f, 0, shape)["D"]
    rng = np.random.default_rng(P * 7 + f + shape)
    for k in range(1, f + 1):
        for F in itertools.combinations(range(1, P), k):
            times = list(itertools.product(range(R + 2), repeat=k))
            if len(times) > 40:
                times = [times[i] for i in rng.choice(len(times), 40, replace=False)]
            for T in times:
                r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=list(F), fail_round=list(T), shape=shape)
                assert r["status"] == oracle.ST_OK
                mult = r["result"]
                for p in range(P):
                    if p not in F:
                        assert mult[p] == 1, (F, T, p)
                    elif T[F.index(p)] == 0:
                        assert mult[p] == 0, (F, T, p)
                    else:
                        assert mult[p] in (0, 1), (F, T, p)


@pytest.mark.parametrize("shape", [3, 4, 1])
@pytest.mark.parametrize("P,f", [(7, 1), (9, 2), (13, 3), (30, 4), (16, 1)])
def test_replication_theorem(oracle, P, f, shape):
    """Every subtree of the root that reports no failure holds every never-failed value outside the root's group
    exactly once; the root's group is held (once) iff the subtree has a member of it."""
    x = np.eye(P, dtype=np.int64)
    s = oracle.structure(P, f, 0, shape)
    rng = np.random.default_rng(P + f + shape)
    for _ in range(30):
        k = int(rng.integers(0, f + 1))
        F = sorted(rng.choice(np.arange(1, P), size=k, replace=False).tolist())
        r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=F, fail_round=[0] * k, trace=True, shape=shape)
        root_group = s["group"][0]
        for child in range(1, f + 2):
            if not r["tree_sent"][child] or r["tree_flag"][child]:
                continue
            mult = r["tree_msg"][child]
            has_root_mate = any(s["group"][p] == root_group and s["subtree"][p] == child for p in range(1, P)) \
                if root_group >= 0 else False
            for p in range(1, P):
                in_root_group = root_group >= 0 and s["group"][p] == root_group
                want = 0 if p in F else 1
                if in_root_group and not has_root_mate:
                    want = 0
                assert mult[p] == want, (shape, F, child, p)
            assert mult[0] == (1 if has_root_mate else 0)


@pytest.mark.parametrize("shape", [3, 1])
@pytest.mark.parametrize("P,f", [(7, 1), (9, 2), (10, 2)])
def test_allreduce_bruteforce(oracle, P, f, shape):
    """Every failure set of size <= f, failures before the operation and (for ranks that are no root candidates)
    at every time: all never-failed processes hold the one value, attempts = 1 + leading failed candidates."""
    rng = np.random.default_rng(P + 3 * f + shape)
    x = rng.integers(-500, 500, size=(P, 1)).astype(np.int64)
    Ratt = 2 * (f + oracle.structure(P, f, 0, shape)["D"])
    for k in range(f + 1):
        for F in itertools.combinations(range(P), k):
            times = [(0,) * k]
            late = [i for i, p in enumerate(F) if p > f]
            for _ in range(6):
                t = [0] * k
                for i in late:
                    t[i] = int(rng.integers(0, 2 * Ratt + 2))
                times.append(tuple(t))
            for T in times:
                o = oracle.allreduce_batch(P, f, x[None], oracle.I64, oracle.SUM, 1, fail_rank=[list(F) or [oracle.NO_RANK]],
                                           fail_round=[list(T) or [0]], want_has=True, want_out=True, shape=shape)
                assert o["status"][0] == oracle.ST_OK
                lead = 0
                while lead in F:
                    lead += 1
                assert o["attempts"][0] == lead + 1
                never = [p for p in range(P) if p not in F]
                assert all(o["has"][0][p] for p in never)
                assert all(np.array_equal(o["out"][0][p], o["result"][0]) for p in never)
                pre = [p for i, p in enumerate(F) if T[i] == 0]
                inop = [p for i, p in enumerate(F) if T[i] != 0]
                assert oracle.is_valid_result(o["result"][0], x, oracle.I64, oracle.SUM, pre, inop)


# --------------------------------------------------------------------------
# latency bookkeeping


def test_message_steps_of_perfect_trees(oracle):
    """One port per process.  Perfect subtrees (every level full): a process of a k-ary tree receives k tree
    messages in the round of its children and sends k broadcast messages in its own; the root has f+1 children;
    in a binomial tree of 2^b processes the reduce brings one message per process and round, while the broadcast
    of this library (every holder forwards to ALL its children in one round) makes the first process send b at
    once.  Up-correction and broadcast correction: one message per process and round, f rounds."""
    for f, h, k in [(1, 3, 2), (2, 4, 2), (1, 3, 3), (3, 2, 4), (0, 3, 2), (2, 2, 8)]:
        m = (k ** h - 1) // (k - 1)                 # processes of a perfect k-ary tree with h levels
        P = (f + 1) * m + 1
        st = oracle.latency_steps(P, f, k)
        assert st == dict(uc=f, tree=k * (h - 1) + (f + 1), bcast_tree=(f + 1) + k * (h - 1), bcast_corr=f), (f, h, k)
        assert oracle.structure(P, f, 0, k)["D"] == h
    for f, b in [(1, 3), (2, 4), (0, 5)]:
        P = (f + 1) * (1 << b) + 1
        st = oracle.latency_steps(P, f, oracle.BINOMIAL)
        # reduce: rounds 1..b bring one message each to a process, the last one f+1 to the root;
        # broadcast: the root sends f+1, then the first process of a subtree b at once, its children b-1, ...
        assert st["tree"] == b + (f + 1) and st["uc"] == f and st["bcast_corr"] == f
        assert st["bcast_tree"] == (f + 1) + sum(range(1, b + 1))
        assert oracle.structure(P, f, 0, oracle.BINOMIAL)["D"] == b + 1


@pytest.mark.parametrize("shape", [2, 3, 1])
def test_who_is_detected(oracle, shape):
    """A failed process is detected when a process that is alive waits in vain for one of its messages.
    All groups full (P - 1 divisible by f + 1), f >= 1: every process that failed beforehand has a living group
    mate, which misses its up-correction message.  A process that fails after its last message is not noticed;
    nobody waits for a message of the root during a reduce, but its children do in the broadcast."""
    P, f = 16, 2
    x = np.ones((P, 1), dtype=np.int64)
    D = oracle.structure(P, f, 0, shape)["D"]
    assert oracle.reduce(P, f, x, oracle.I64, oracle.SUM, shape=shape)["detected"] == 0
    for k in range(1, f + 1):
        for F in itertools.combinations(range(1, P), k):
            r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=list(F), fail_round=[0] * k, shape=shape)
            assert r["detected"] == (1 << k) - 1, F
    # fails after the reduce's last round: never missed
    r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=[5], fail_round=[f + D + 1], shape=shape)
    assert r["detected"] == 0 and r["status"] == oracle.ST_OK
    # a leaf that fails in the round of its tree message (after the up-correction): only its parent notices
    s = oracle.structure(P, f, 0, shape)
    leaf = max(p for p in range(1, P) if s["height"][p] == 0)
    r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=[leaf], fail_round=[f + 1], shape=shape)
    assert r["detected"] == 1
    r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=[leaf, int(s["parent"][leaf])], fail_round=[f + 1, f + 1],
                      shape=shape)
    assert r["detected"] == 2          # the parent is missed by ITS parent; nobody alive waits for the leaf's tree message
    # the root: not missed in a reduce (it is in no group here), missed by its children in the broadcast
    r = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=[0], fail_round=[0], shape=shape)
    assert r["detected"] == 0 and r["status"] == oracle.ST_ROOT_FAILED
    o = oracle.allreduce_batch(P, f, x[None], oracle.I64, oracle.SUM, 1, fail_rank=[[0, oracle.NO_RANK]], fail_round=[[0, 0]],
                               shape=shape, want_detected=True)
    assert o["detected"][0] == 1 and o["attempts"][0] == 2
    # detected is a subset of the listed slots, whatever happens
    rng = np.random.default_rng(shape)
    for _ in range(200):
        k = int(rng.integers(0, f + 1))
        F = rng.choice(np.arange(f + 1, P), size=k, replace=False).tolist() + [oracle.NO_RANK] * (f - k)
        T = rng.integers(0, 4 * (f + D) + 2, size=f).tolist()
        o = oracle.allreduce_batch(P, f, x[None], oracle.I64, oracle.SUM, 1, fail_rank=[F], fail_round=[T], shape=shape,
                                   want_detected=True)
        assert int(o["detected"][0]) >> k == 0
