"""Parity with the CPU oracle for the other shapes of the tree inside a subtree of the
root (the definition of the I(f)-tree leaves it free): k children per process, filled
breadth-first, and the binomial tree.  Reduce with a root per scenario and allreduce,
failures before and during the operation; every output bit-exact, as for the default
shape.  The shapes decide the number of rounds, so the failure times of the recipes use
each plan's own rounds."""
import numpy as np
import pytest
import torch

from _cmp import compare_allreduce, compare_reduce

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ft():
    from paper_2602_22445_amd import binding
    binding.lib()                       # raises if the library is not built: no fallback
    assert torch.cuda.is_available()
    return binding


@pytest.fixture(scope="module")
def w():
    from paper_2602_22445_amd import workloads
    return workloads


CASES = [  # P, f, E, dtype, op, S
    (7, 1, 1, 0, 0, 40), (8, 1, 4, 0, 0, 64), (64, 2, 8, 1, 1, 96), (100, 6, 5, 2, 0, 64), (257, 7, 2, 0, 1, 64),
    (1000, 8, 1, 0, 0, 48), (1024, 3, 16, 0, 0, 64), (1500, 4, 8, 2, 0, 64), (4099, 5, 3, 2, 0, 32),
    (3000, 12, 2, 0, 0, 24), (17, 15, 1, 0, 0, 32), (20000, 2, 4, 1, 0, 12), (2, 0, 1, 0, 0, 4), (33, 0, 3, 2, 0, 16),
]
SHAPES = [3, 4, 8, 1]


def _payload(w, seed, S, P, E, dtype):
    if dtype == 0:
        return w.payload_int(seed, S, P, E, "i64", 41)
    if dtype == 1:
        return w.payload_int(seed, S, P, E, "u32", 32)
    return w.payload_normal(seed, S, P, E, threads=4)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("P,f,E,dtype,op,S", CASES)
def test_other_tree_shapes(ft, oracle, w, P, f, E, dtype, op, S, shape):
    seed = 9000 + P + 31 * f + E + 7 * shape
    plan = ft.Plan(P, f, E, dtype, op, shape=shape)
    D = oracle.structure(P, f, 0, shape)["D"]
    assert plan.info.D == D and plan.info.rounds_attempt == 2 * (f + D)
    Rred, Ratt = f + D, 2 * (f + D)
    x = _payload(w, seed, S, P, E, dtype)

    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=Rred + 1)
    root = w.random_roots(seed, S, P)
    root[: S // 4] = 0
    if f >= 1:
        fr[1], fo[1] = w.NO_RANK, 0
        fr[1, 0], fo[1, 0] = root[1], 0                  # a failed root
        fr[2], fo[2] = w.NO_RANK, 0
        fr[2, 0], fo[2, 0] = (P - 1 if root[2] != P - 1 else P - 2), 1
    compare_reduce(ft, oracle, plan, x, fr, fo, root=root, shape=shape)

    fr, fo = w.random_failure_sets(seed + 1, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1)
    if f >= 1:
        fr[0], fo[0] = w.NO_RANK, 0
        fr[0, 0], fo[0, 0] = 0, 0                        # a second attempt
        fr[3], fo[3] = w.NO_RANK, 0
        fr[3, 0], fo[3, 0] = min(f + 1, P - 1), Ratt // 2 + 1      # fails during the broadcast
    if f >= 2:
        fr[1], fo[1] = w.NO_RANK, 0
        fr[1, :2], fo[1, :2] = [1, 0], [0, 0]            # a third attempt
    compare_allreduce(ft, oracle, plan, x, fr, fo, shape=shape)


@pytest.mark.parametrize("shape", [2, 3, 8, 1])
@pytest.mark.parametrize("P,f", [(7, 1), (8, 1), (16, 2), (64, 2), (100, 6), (257, 7), (1000, 8), (1024, 3), (4099, 5), (17, 15),
                                 (5000, 4), (33, 0)])
def test_detected_processes(ft, oracle, w, P, f, shape):
    """ftred_detect (which listed processes some living process waits for in vain, worked out from the failure
    lists) against the oracle, which marks them while it simulates: reduce with a root per scenario and allreduce
    with its retries, failures at any time."""
    from _cmp import to_dev
    S, seed = 200, 12000 + P + 17 * f + shape
    plan = ft.Plan(P, f, 1, ft.I64, ft.SUM, shape=shape)
    Rred, Ratt = plan.info.rounds_reduce, plan.info.rounds_attempt
    x = np.ones((P, 1), dtype=np.int64)                   # one payload for all scenarios: values do not matter here

    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=700, rounds_per_attempt=Rred + 2)
    root = w.random_roots(seed, S, P)
    root[: S // 4] = 0
    if f >= 1:
        fr[1, 0], fo[1, 0] = root[1], 0
        fr[2, 0], fo[2, 0] = root[2], Rred                # the root fails in the last round
    o = oracle.reduce_batch(P, f, x, 0, 0, S, root=root, fail_rank=fr, fail_round=fo, shape=shape, want_detected=True)
    got = ft.detect(plan, 0, S, to_dev(fr), to_dev(fo), root=to_dev(root.astype(np.uint32))).cpu().numpy()
    bad = np.nonzero(got != o["detected"])[0]
    assert bad.size == 0, (bad[:5], got[bad[:5]], o["detected"][bad[:5]], fr[bad[:5]], fo[bad[:5]], root[bad[:5]])

    fr, fo = w.random_failure_sets(seed + 1, S, P, f, inop_permille=700, rounds_per_attempt=Ratt, protected=f + 1)
    if f >= 1:
        fr[0], fo[0] = w.NO_RANK, 0
        fr[0, 0], fo[0, 0] = 0, 0
    if f >= 2:
        fr[1], fo[1] = w.NO_RANK, 0
        fr[1, :2], fo[1, :2] = [1, 0], [0, 0]
        fr[2], fo[2] = w.NO_RANK, 0
        fr[2, :2], fo[2, :2] = [0, 2], [0, 3]             # a root candidate failing during the operation: not valid
    o = oracle.allreduce_batch(P, f, x, 0, 0, S, fail_rank=fr, fail_round=fo, shape=shape, want_has=False, want_detected=True)
    got = ft.detect(plan, 1, S, to_dev(fr), to_dev(fo)).cpu().numpy()
    bad = np.nonzero(got != o["detected"])[0]
    assert bad.size == 0, (bad[:5], got[bad[:5]], o["detected"][bad[:5]], fr[bad[:5]], fo[bad[:5]])
    # the reading as a number: message steps of the plan times the attempts, plus a time-out per detected process
    lat = ft.latency(plan, 1, o["attempts"], got, t_message=1.0, t_timeout=10.0)
    i = plan.info
    per = i.steps_uc + i.steps_tree + i.steps_bcast_tree + i.steps_bcast_corr
    ok = o["status"] == 0
    assert np.all(lat[ok] >= per) and lat[ok].max() <= per * (f + 1) + 10.0 * f


def test_the_default_shape_by_its_number_is_the_default(ft, oracle, w):
    """Shape 2 asked for explicitly is the default path (register / LDS-tile kernels), not the plain kernels."""
    a, b = ft.Plan(5000, 2, 4, ft.I64, ft.SUM).info, ft.Plan(5000, 2, 4, ft.I64, ft.SUM, shape=2).info
    assert (a.D, a.tiers, a.deep_kernel, a.fused) == (b.D, b.tiers, b.deep_kernel, b.fused) and a.tiers > 0
    assert ft.Plan(5000, 2, 4, ft.I64, ft.SUM, shape=3).info.tiers == 0


def test_failure_lists_are_not_carried_by_other_shapes(ft, w):
    plan = ft.Plan(100, 2, 1, ft.I64, ft.SUM, shape=3)
    x = torch.zeros((4, 100, 1), dtype=torch.int64, device="cuda")
    fr = torch.from_numpy(np.full((4, 2), w.NO_RANK, dtype=np.uint32)).cuda()
    fo = torch.zeros((4, 2), dtype=torch.int32, device="cuda").view(torch.uint32)
    with pytest.raises(ft.FtredError) as e:
        ft.run_reduce_info(plan, 4, x, fr, fo)
    assert e.value.code == ft.EUNSUPPORTED
