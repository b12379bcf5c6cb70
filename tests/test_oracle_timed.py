"""Pins of the event-driven times of the reduce in the CPU oracle (every process has a
clock of its own: sends take t_msg, a receive from a process that has stopped ends by
time-outs; section "Related work", last paragraph, and section "Up-Correction", last
paragraph).

The C oracle stamps the times onto its round loop.  It is pinned here by a worked
example done by hand, by closed forms of the failure-free run, by invariants (scaling,
monotony), and by ``oracle/event_sim.py``: a discrete-event simulation with blocking
receives, a time-out queue and a monitor that knows the moment a process stopped, which
runs the processes in the order of TIME and shares nothing with the round loop but the
tree.  That the event-driven execution computes the round model's values, statuses and
message counts is checked on the way."""
import itertools

import numpy as np
import pytest

from oracle import event_sim

SHAPES = [2, 3, 1]


def _event(oracle, P, f, x, fail, m, tau, root=0, shape=2):
    st = oracle.structure(P, f, root, shape)
    return event_sim.run_reduce(st, [int(v) for v in x[:, 0]], lambda a, b: (a + b) & (2**64 - 1), fail, m, tau, root=root, f=f)


def _timed(oracle, P, f, x, fails, m, tau, roots=None, shape=2):
    """fails: one {rank: round} per scenario."""
    S = len(fails)
    nf = max(1, max(len(d) for d in fails))
    fr = np.full((S, nf), oracle.NO_RANK, np.uint32)
    fo = np.zeros((S, nf), np.uint32)
    for i, d in enumerate(fails):
        for q, (p, r) in enumerate(sorted(d.items())):
            fr[i, q], fo[i, q] = p, r
    return oracle.reduce_timed_batch(P, f, x, oracle.I64, oracle.SUM, S, m, tau,
                                     root=roots, fail_rank=fr, fail_round=fo, shape=shape, threads=2), fr, fo


def _same(oracle, P, f, x, fails, m, tau, roots=None, shape=2):
    got, fr, fo = _timed(oracle, P, f, x, fails, m, tau, roots, shape)
    plain = oracle.reduce_batch(P, f, x, oracle.I64, oracle.SUM, len(fails), root=roots, fail_rank=fr, fail_round=fo, shape=shape)
    # the timed mode does not disturb the round model ...
    assert np.array_equal(got["result"], plain["result"]) and np.array_equal(got["status"], plain["status"])
    assert np.array_equal(got["msgs"], plain["msgs"])
    names = {oracle.ST_OK: "ok", oracle.ST_ROOT_FAILED: "root_failed", oracle.ST_NO_CLEAN_SUBTREE: "no_clean"}
    for i, d in enumerate(fails):
        root = 0 if roots is None else int(roots[i])
        e = _event(oracle, P, f, x, d, m, tau, root, shape)
        tag = (P, f, shape, root, d, m, tau)
        # ... and the event-driven execution computes what the round model computes
        assert e["status"] == names[int(got["status"][i])], tag
        if e["status"] == "ok":
            assert e["result"] == int(got["result"][i, 0]) & (2**64 - 1), tag
        assert (e["msgs_uc"], e["msgs_tree"]) == tuple(int(v) for v in got["msgs"][i]), tag
        want_done = oracle.NEVER if e["t_done"] is None else e["t_done"]
        assert int(got["t_done"][i]) == want_done, tag
        want = [oracle.NEVER if t is None else t for t in e["t_proc"]]
        assert [int(v) for v in got["t_proc"][i]] == want, tag


def _payload(P, seed=1):
    rng = np.random.default_rng(seed)
    return rng.integers(0, 2**40, size=(P, 1), dtype=np.int64)


@pytest.mark.parametrize("m,tau", [(1, 1), (1, 2), (1, 5), (3, 1), (3, 4), (2, 7), (10, 3)])
def test_worked_example_by_hand(oracle, m, tau):
    """n = 7, f = 1 (the paper's second tree figure: 1 -> {3, 5}, 2 -> {4, 6}; groups {1,2}, {3,4}, {5,6}), process 1
    failed beforehand.  By hand: 3..6 exchange (m) and send (2m).  Process 2 sends to 1 (m), gives up on 1 at
    m + tau, has the messages of 4 and 6 at 2m, sends: max(m + tau, 2m) + m.  The root gives up on child 1 at tau
    and takes child 2: max(tau, max(m + tau, 2m) + m) = max(2m + tau, 3m)."""
    P, f = 7, 1
    x = np.arange(P, dtype=np.int64).reshape(P, 1)
    got, _, _ = _timed(oracle, P, f, x, [{1: 0}], m, tau)
    assert int(got["result"][0, 0]) == 20 and got["status"][0] == oracle.ST_OK
    assert int(got["t_done"][0]) == max(2 * m + tau, 3 * m)
    never = oracle.NEVER
    assert [int(v) for v in got["t_proc"][0]] == [max(2 * m + tau, 3 * m), never, max(m + tau, 2 * m) + m, 2 * m, 2 * m, 2 * m, 2 * m]
    # failure-free: every process is done at the end of its send round
    got, _, _ = _timed(oracle, P, f, x, [{}], m, tau)
    assert int(got["t_done"][0]) == 3 * m
    assert [int(v) for v in got["t_proc"][0]] == [3 * m, 3 * m, 3 * m, 2 * m, 2 * m, 2 * m, 2 * m]


@pytest.mark.parametrize("shape", [2, 3, 4, 8, 1])
@pytest.mark.parametrize("P,f", [(7, 1), (9, 1), (13, 2), (10, 2), (41, 3), (64, 2), (101, 4), (100, 4), (33, 0), (257, 7), (1000, 8)])
def test_failure_free_times(oracle, P, f, shape):
    """Nobody fails, nobody waits beyond an arrival: a process whose group is complete is done at t_msg x (its send
    round of the round model), by induction over the tree; a short last group (fewer exchange rounds) can only be
    earlier, and by less than one round at the root."""
    m, tau = 3, 50
    x = _payload(P)
    st = oracle.structure(P, f, 0, shape)
    got, _, _ = _timed(oracle, P, f, x, [{}], m, tau, shape=shape)
    D = int(st["D"])
    full = (P - 1) % (f + 1) == 0 or P % (f + 1) == 0             # the last group is complete (without / with the root)
    t = [int(v) for v in got["t_proc"][0]]
    assert (f + D - 1) * m <= int(got["t_done"][0]) <= (f + D) * m
    assert t[0] == int(got["t_done"][0])
    for p in range(1, P):
        assert t[p] <= m * int(st["send_round"][p])
        if full:
            assert t[p] == m * int(st["send_round"][p]), p
    if full:
        assert int(got["t_done"][0]) == (f + D) * m


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("P,f", [(5, 1), (6, 1), (7, 1), (8, 1), (7, 2), (9, 2), (4, 0), (6, 0)])
def test_event_simulation_every_failure_set_and_time(oracle, P, f, shape):
    """Every failure set of at most f processes (root and others), every failure time, two pairs of (t_msg, t_timeout):
    the discrete-event simulation and the stamped round loop agree on every process's time, and on values, statuses
    and message counts."""
    x = _payload(P, 3)
    D = int(oracle.structure(P, f, 0, shape)["D"])
    rounds = range(0, f + D + 2)
    fails = [{}]
    for k in range(1, f + 1):
        for procs in itertools.combinations(range(P), k):
            for rr in itertools.product(rounds, repeat=k):
                fails.append(dict(zip(procs, rr)))
    if len(fails) > 1500:
        fails = fails[:: len(fails) // 1500 + 1]
    for m, tau in [(1, 1), (2, 5)]:
        _same(oracle, P, f, x, fails, m, tau, shape=shape)


@pytest.mark.parametrize("shape", [2, 3, 4, 1])
@pytest.mark.parametrize("P,f", [(23, 2), (40, 3), (31, 4), (64, 1), (50, 5), (29, 3)])
def test_event_simulation_random(oracle, P, f, shape):
    """Larger trees, random roots, failures before and during the operation, time constants with and without ties
    (a time-out that ends at the very moment a message arrives or a process stops)."""
    rng = np.random.default_rng(100 * P + 10 * f + shape)
    x = _payload(P, 5)
    D = int(oracle.structure(P, f, 0, shape)["D"])
    for m, tau in [(1, 1), (1, 3), (4, 2), (3, 7)]:
        fails, roots = [], []
        for _ in range(40):
            k = int(rng.integers(0, f + 1))
            procs = rng.choice(P, size=k, replace=False)
            d = {}
            for p in procs:
                d[int(p)] = 0 if rng.random() < 0.4 else int(rng.integers(1, f + D + 2))
            fails.append(d)
            roots.append(int(rng.integers(0, P)))
        _same(oracle, P, f, x, fails, m, tau, roots=np.array(roots, np.uint32), shape=shape)


@pytest.mark.parametrize("P,f,shape", [(100, 3, 2), (77, 4, 3), (64, 2, 1)])
def test_scaling_and_monotony(oracle, P, f, shape):
    """Times are made of t_msg and t_timeout only: scaling both scales every time; a longer time-out never makes
    anybody earlier as long as it stays a multiple (the moments of the monitor's answers are then a subset)."""
    rng = np.random.default_rng(7)
    x = _payload(P, 9)
    D = int(oracle.structure(P, f, 0, shape)["D"])
    fails = []
    for _ in range(60):
        k = int(rng.integers(0, f + 1))
        fails.append({int(p): (0 if rng.random() < 0.5 else int(rng.integers(1, f + D + 1))) for p in rng.choice(P, size=k, replace=False)})
    a, _, _ = _timed(oracle, P, f, x, fails, 2, 3, shape=shape)
    b, _, _ = _timed(oracle, P, f, x, fails, 14, 21, shape=shape)
    fin = a["t_proc"] != oracle.NEVER
    assert np.array_equal(fin, b["t_proc"] != oracle.NEVER)
    assert np.array_equal(a["t_proc"][fin] * 7, b["t_proc"][fin])
    c, _, _ = _timed(oracle, P, f, x, fails, 2, 6, shape=shape)
    assert np.all(c["t_proc"][fin] >= a["t_proc"][fin])
    ok = a["status"] != oracle.ST_ROOT_FAILED
    assert np.all(c["t_done"][ok] >= a["t_done"][ok])
    # a failed process costs somebody a time-out: with one listed process that has failed beforehand and is not the
    # root, the root is done no earlier than without it less one round, and no later than that plus the time-outs
    # on the longest chain (one per level and one in the exchange)
    free, _, _ = _timed(oracle, P, f, x, [{}], 2, 3, shape=shape)
    for p in (1, 2, P // 2, P - 1):
        one, _, _ = _timed(oracle, P, f, x, [{p: 0}], 2, 3, shape=shape)
        assert one["status"][0] == oracle.ST_OK
        assert int(one["t_done"][0]) <= int(free["t_done"][0]) + 3 * (D + 2)


def test_a_late_stop_costs_more_than_one_time_out(oracle):
    """The monitor confirms a failure only once the process has stopped: process 3 (n = 7, f = 1) stops after its
    exchange, which it ends late because its mate 4 has failed (m + tau); its parent 1 starts waiting for it at m and
    asks the monitor at m + tau (3 stops at that very moment: not yet confirmed) and at m + 2 tau (confirmed)."""
    P, f, m, tau = 7, 1, 2, 5
    x = np.arange(P, dtype=np.int64).reshape(P, 1)
    got, _, _ = _timed(oracle, P, f, x, [{4: 0, 3: 2}], m, tau)      # two failures, f = 1: outside the guarantee, fine for times
    t = [int(v) for v in got["t_proc"][0]]
    # process 1: exchange with 2 done at m; waits for 3: m + 2 tau; has 5's message (2m) by then; sends
    assert t[1] == m + 2 * tau + m
    e = _event(oracle, P, f, x, {4: 0, 3: 2}, m, tau)
    assert e["t_proc"][1] == t[1]
