"""Parity of ftred_reduce_times with the CPU oracle's event-driven times of the reduce:
the moment the root delivers and the moment every process has done its part, for every
tree shape, roots per scenario, failures before and during the operation, several time
constants (with ties between time-outs, arrivals and the moments processes stop); bit
for bit (integer times).  The oracle's times are pinned on the CPU by a discrete-event
simulation (tests/test_oracle_timed.py)."""
import numpy as np
import pytest
import torch

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


def _compare(ft, oracle, P, f, shape, fr, fo, root, m, tau, threads=16):
    S = fr.shape[0]
    plan = ft.Plan(P, f, 1, ft.I64, ft.SUM, shape=shape)
    frd, fod = torch.from_numpy(fr).cuda(), torch.from_numpy(fo).cuda()
    rd = None if root is None else torch.from_numpy(root.astype(np.uint32)).cuda()
    t_done, t_proc = ft.reduce_times(plan, S, frd, fod, m, tau, root=rd)
    torch.cuda.synchronize()
    x = np.zeros((P, 1), np.int64)
    want = oracle.reduce_timed_batch(P, f, x, oracle.I64, oracle.SUM, S, m, tau, root=root, fail_rank=fr, fail_round=fo,
                                     shape=shape, threads=threads)
    got_done, got_proc = t_done.cpu().numpy(), t_proc.cpu().numpy()
    bad = np.nonzero(got_done != want["t_done"])[0]
    assert bad.size == 0, (P, f, shape, m, tau, int(bad[0]), int(got_done[bad[0]]), int(want["t_done"][bad[0]]), fr[bad[0]], fo[bad[0]])
    neq = np.argwhere(got_proc != want["t_proc"])
    assert neq.size == 0, (P, f, shape, m, tau, neq[0], int(got_proc[tuple(neq[0])]), int(want["t_proc"][tuple(neq[0])]),
                           fr[neq[0][0]], fo[neq[0][0]], None if root is None else int(root[neq[0][0]]))
    return want


CASES = [  # P, f, S
    (7, 1, 40), (8, 1, 64), (9, 2, 64), (64, 2, 96), (100, 6, 64), (257, 7, 64), (1000, 8, 48), (1024, 3, 64), (1500, 4, 64),
    (4099, 5, 32), (3000, 12, 24), (17, 15, 32), (20000, 2, 12), (2, 0, 4), (33, 0, 16), (6, 4, 16), (16385, 4, 24),
]


@pytest.mark.parametrize("shape", [2, 3, 4, 8, 1])
@pytest.mark.parametrize("P,f,S", CASES)
def test_times_against_the_oracle(ft, oracle, w, P, f, S, shape):
    seed = 52000 + P + 31 * f + 7 * shape
    D = int(oracle.structure(P, f, 0, shape)["D"])
    Rred = f + D
    for k, (m, tau) in enumerate([(1, 1), (3, 7), (4, 2), (1000, 1)]):
        fr, fo = w.random_failure_sets(seed + k, S, P, f, inop_permille=600, rounds_per_attempt=Rred + 1)
        root = w.random_roots(seed + k, S, P)
        root[: S // 4] = 0
        fr[0], fo[0] = w.NO_RANK, 0                      # nobody fails
        if f >= 1:
            fr[1], fo[1] = w.NO_RANK, 0
            fr[1, 0], fo[1, 0] = root[1], 0              # a failed root
            fr[2], fo[2] = w.NO_RANK, 0
            fr[2, 0], fo[2, 0] = (P - 1 if root[2] != P - 1 else P - 2), 1
            fr[3], fo[3] = w.NO_RANK, 0
            fr[3, 0], fo[3, 0] = root[3], 2              # a root that stops during its exchange (or later)
        want = _compare(ft, oracle, P, f, shape, fr, fo, root if k != 2 else None, m, tau)
        if k == 0:
            # failure-free: the root is done within one round of t_msg x (f + D)
            assert (f + D - 1) * m <= int(want["t_done"][0]) <= (f + D) * m


def test_failure_sets_outside_the_semantics(ft, oracle):
    """A rank beyond P, a rank twice, a root beyond P: every time is "never", nothing is read or written out of
    bounds (the library checks the set before it follows any rank)."""
    P, f, S = 100, 3, 4
    plan = ft.Plan(P, f, 1, ft.I64, ft.SUM)
    fr = np.full((S, f), ft.NO_RANK, np.uint32)
    fo = np.zeros((S, f), np.uint32)
    fr[0, 0] = P + 5
    fr[1, :2] = [7, 7]
    root = np.array([0, 3, P + 1, 9], np.uint32)
    t_done, t_proc = ft.reduce_times(plan, S, torch.from_numpy(fr).cuda(), torch.from_numpy(fo).cuda(), 2, 5,
                                     root=torch.from_numpy(root).cuda(),
                                     t_proc=torch.from_numpy(np.full((S, P), 12345, np.uint64)).cuda())
    torch.cuda.synchronize()
    d, p = t_done.cpu().numpy(), t_proc.cpu().numpy()
    assert np.all(d[:3] == ft.NEVER) and np.all(p[:2] == ft.NEVER)
    # the root beyond P has no entry of its own: every entry of the scenario is one of a process below P
    assert np.all(p[2] == ft.NEVER)
    x = np.zeros((P, 1), np.int64)
    want = oracle.reduce_timed_batch(P, f, x, oracle.I64, oracle.SUM, 1, 2, 5, root=root[3:], fail_rank=fr[3:], fail_round=fo[3:])
    assert d[3] == want["t_done"][0] and np.array_equal(p[3], want["t_proc"][0])
    with pytest.raises(ft.FtredError):
        ft.reduce_times(plan, S, torch.from_numpy(fr).cuda(), torch.from_numpy(fo).cuda(), 0, 5)


@pytest.mark.parametrize("P,f,S,shape", [(16384, 4, 96, 2), (16384, 4, 32, 1), (1 << 20, 8, 4, 2), (1 << 18, 8, 6, 8)])
def test_times_at_full_size(ft, oracle, w, P, f, S, shape):
    """The shapes of the large workloads (the oracle stamps a million processes in a few seconds)."""
    D = int(oracle.structure(P, f, 0, shape)["D"])
    fr, fo = w.random_failure_sets(777 + P, S, P, f, inop_permille=500, rounds_per_attempt=f + D + 1)
    root = w.random_roots(778 + P, S, P)
    fr[0], fo[0] = w.NO_RANK, 0
    _compare(ft, oracle, P, f, shape, fr, fo, root, 5, 13)
