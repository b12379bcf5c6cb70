"""Pins of the oracle's allreduce (reduce to a root, broadcast from it, retry
with the next root while the root had failed) against the allreduce semantics
of the paper: every non-failed value is included, a failed value is included at
every non-failed process or at none, a failed root is detected consistently and
the next root is tried, and f failures cost at most the (f+1)-fold messages."""
import itertools

import numpy as np
import pytest


def _uc_ff(n, f):
    a = (n - 1) % (f + 1) + 1
    return f * (f + 1) * ((n - 1) // (f + 1)) + a * (a - 1)


def _check_one(oracle, P, f, F, T, R_attempt, x):
    r = oracle.allreduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=F, fail_round=T)
    assert r["status"] == oracle.ST_OK, (F, T, r["status"])
    lead = 0
    while lead in F:
        lead += 1
    assert r["attempts"] == lead + 1, (F, T)
    assert r["rounds"] == (lead + 1) * R_attempt
    mult = r["result"]
    for p in range(P):
        if p not in F:
            assert mult[p] == 1, (F, T, p)
            # every non-failed process holds the one result
            assert r["has"][p] == 1, (F, T, p)
            assert np.array_equal(r["out"][p], mult), (F, T, p)
        elif T[F.index(p)] == 0:
            assert mult[p] == 0 and r["has"][p] == 0
        else:
            assert mult[p] in (0, 1)
            if r["has"][p]:
                assert np.array_equal(r["out"][p], mult)
    ff = _uc_ff(P, f) + (P - 1) + (P - 1) + _uc_ff(P, f)
    assert int(r["msgs"].sum()) <= (f + 1) * ff
    return r


@pytest.mark.parametrize("P,f", [(4, 1), (7, 1), (8, 1), (5, 2), (9, 2), (10, 2), (3, 0), (6, 0)])
def test_allreduce_bruteforce_all_failure_sets_and_times(oracle, P, f):
    x = np.eye(P, dtype=np.int64)
    R_attempt = 2 * (f + oracle.structure(P, f, 0)["D"])
    for k in range(f + 1):
        for F in itertools.combinations(range(P), k):
            lead = 0
            while lead in F:
                lead += 1
            horizon = (lead + 1) * R_attempt
            choices = [[0] if p <= f else list(range(0, horizon + 1)) for p in F]
            for T in itertools.product(*choices):
                _check_one(oracle, P, f, F, T, R_attempt, x)


@pytest.mark.parametrize("P,f", [(8, 3), (12, 3), (14, 4), (23, 4)])
def test_allreduce_sampled_failure_sets_and_times(oracle, P, f):
    x = np.eye(P, dtype=np.int64)
    R_attempt = 2 * (f + oracle.structure(P, f, 0)["D"])
    rng = np.random.default_rng(P * 10 + f)
    for _ in range(3000):
        k = int(rng.integers(0, f + 1))
        # bias towards the root candidates so that retries happen
        pool = np.concatenate([np.arange(P), np.arange(min(f + 1, P))])
        F = []
        while len(F) < k:
            c = int(rng.choice(pool))
            if c not in F:
                F.append(c)
        F = tuple(F)
        lead = 0
        while lead in F:
            lead += 1
        horizon = (lead + 1) * R_attempt
        T = tuple(0 if (p <= f or rng.random() < 0.3) else int(rng.integers(1, horizon + 1)) for p in F)
        _check_one(oracle, P, f, F, T, R_attempt, x)


def test_allreduce_root_alive_costs_reduce_plus_broadcast(oracle):
    """Root alive, no failure: exactly the messages of one reduce and one
    broadcast.  (The tree broadcast sends one message per non-root process; the
    correction rounds mirror the up-correction exchange.)"""
    for P, f in [(7, 1), (8, 1), (64, 2), (1024, 3), (100, 5)]:
        x = np.ones((P, 2), dtype=np.int64)
        red = oracle.reduce(P, f, x, oracle.I64, oracle.SUM)
        r = oracle.allreduce(P, f, x, oracle.I64, oracle.SUM)
        assert r["attempts"] == 1
        assert r["msgs"][0] == red["msgs"][0] and r["msgs"][1] == red["msgs"][1]
        assert r["msgs"][2] == P - 1
        assert r["msgs"][3] == _uc_ff(P, f)
        assert np.all(r["has"] == 1) and np.all(r["out"] == P)


def test_allreduce_failed_roots_multiply_the_messages(oracle):
    """Roots 0..f-1 failed beforehand: f+1 attempts, and the failed attempts send
    the reduce messages again (to a root that never answers), nothing else."""
    P, f = 23, 3
    x = np.ones((P, 1), dtype=np.int64)
    F = list(range(f))
    r = oracle.allreduce(P, f, x, oracle.I64, oracle.SUM, fail_rank=F, fail_round=[0] * f)
    assert r["status"] == oracle.ST_OK and r["attempts"] == f + 1
    assert int(r["result"][0]) == P - f
    one = oracle.reduce(P, f, x, oracle.I64, oracle.SUM, root=f, fail_rank=F, fail_round=[0] * f)
    assert r["msgs"][2] + r["msgs"][3] <= (P - 1) + _uc_ff(P, f)
    assert r["msgs"][0] + r["msgs"][1] <= (f + 1) * int(one["msgs"].sum() + f * (f + 1))
    assert np.all(r["has"][f:] == 1) and np.all(r["has"][:f] == 0)


@pytest.mark.parametrize("op_name", ["sum", "bor"])
def test_config_allreduce_p64_f2_exhaustive(oracle, op_name):
    """Allreduce, P=64, f=2, uint32, every failure set of size 0..2 failed
    beforehand (2081 scenarios): every surviving process holds the reduction
    over the survivors."""
    from paper_2602_22445_amd import workloads as w
    P, f, E = 64, 2, 8
    op = oracle.SUM if op_name == "sum" else oracle.BOR
    fr, fo = w.exhaustive_failure_sets(P, f)
    S = fr.shape[0]
    assert S == 2081
    x = w.payload_int(2, S, P, E, "u32", 32)
    r = oracle.allreduce_batch(P, f, x, oracle.U32, op, S, fail_rank=fr, fail_round=fo, want_out=True)
    assert np.all(r["status"] == oracle.ST_OK)
    for s in range(S):
        F = [int(q) for q in fr[s] if q != w.NO_RANK]
        want = oracle.survivor_reduce(x[s], oracle.U32, op, F)
        assert np.array_equal(r["result"][s], want)
        alive = np.ones(P, bool)
        alive[F] = False
        assert np.all(r["has"][s][alive] == 1) and np.all(r["has"][s][~alive] == 0)
        assert np.all(r["out"][s][alive] == want)
        lead = 0
        while lead in F:
            lead += 1
        assert r["attempts"][s] == lead + 1


def test_config_reduce_p8_f1_exhaustive(oracle):
    """Reduce, P=8, f=1, root 0, wrapping int64 sum, 4 values per process; the 9
    failure sets of size 0..1, each with 32 payload seeds (288 runs)."""
    from paper_2602_22445_amd import workloads as w
    P, f, E = 8, 1, 4
    fr9, fo9 = w.exhaustive_failure_sets(P, f)
    assert fr9.shape[0] == 9
    fr = np.repeat(fr9, 32, axis=0)
    fo = np.repeat(fo9, 32, axis=0)
    S = fr.shape[0]
    x = w.payload_int(1, S, P, E, "i64", 32)
    assert x.min() >= -2**31 and x.max() < 2**31
    r = oracle.reduce_batch(P, f, x, oracle.I64, oracle.SUM, S, fail_rank=fr, fail_round=fo)
    for s in range(S):
        F = [int(q) for q in fr[s] if q != w.NO_RANK]
        if 0 in F:
            assert r["status"][s] == oracle.ST_ROOT_FAILED
        else:
            assert r["status"][s] == oracle.ST_OK
            assert np.array_equal(r["result"][s], oracle.survivor_reduce(x[s], oracle.I64, oracle.SUM, F))


def test_batch_equals_single_calls(oracle):
    from paper_2602_22445_amd import workloads as w
    P, f, E, S = 200, 3, 5, 40
    R_attempt = 2 * (f + oracle.structure(P, f, 0)["D"])
    fr, fo = w.random_failure_sets(11, S, P, f, inop_permille=600, rounds_per_attempt=R_attempt, protected=f + 1)
    x = w.payload_normal(11, S, P, E, threads=1)
    b = oracle.allreduce_batch(P, f, x, oracle.F64, oracle.SUM, S, fail_rank=fr, fail_round=fo, want_out=True)
    for s in range(S):
        r = oracle.allreduce(P, f, x[s], oracle.F64, oracle.SUM, fail_rank=fr[s], fail_round=fo[s])
        assert r["status"] == b["status"][s] and r["attempts"] == b["attempts"][s]
        assert np.array_equal(r["result"], b["result"][s])
        assert np.array_equal(r["has"], b["has"][s]) and np.array_equal(r["out"], b["out"][s])
        assert np.array_equal(r["msgs"], b["msgs"][s])
        pre = [int(q) for q, t in zip(fr[s], fo[s]) if q != w.NO_RANK and t == 0]
        inop = [int(q) for q, t in zip(fr[s], fo[s]) if q != w.NO_RANK and t != 0]
        assert oracle.is_valid_result(r["result"], x[s], oracle.F64, oracle.SUM, pre, inop)
