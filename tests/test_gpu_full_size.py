"""The three large workloads at their full sizes, in the launch configuration the
benchmark times (default plan flags, the whole batch in one call): the HIP library
runs every scenario; the CPU oracle runs a sample of them, and every compared
output of the sample must agree as in the small parity tests.  Properties that
hold at any size are checked over the whole batch: the library's own validation
pass finds no invalid scenario, statuses are OK, attempts are 1 + the number of
leading root candidates listed as failed.

Inputs: the failure sets of the whole batch and the payload of the sampled
scenarios come from the seeded host generators; the payload of the whole batch
comes from the host generator (floating point) or from the library's device
generator, which implements the same counter-based generator and is compared
with the host's on the sample."""
import numpy as np
import pytest
import torch

from _cmp import assert_values, to_dev, unpack_bitmap

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


def _sample(S, n, extra=()):
    idx = sorted(set(np.linspace(0, S - 1, n).astype(np.int64).tolist()) | {int(e) for e in extra})
    return np.array(idx, dtype=np.int64)


def _expected_attempts(fr, fo, f):
    """1 + number of leading root candidates 0, 1, .. listed as failed before the operation."""
    S = fr.shape[0]
    att = np.ones(S, dtype=np.int64)
    for r in range(f + 1):
        dead = ((fr == r) & (fo == 0)).any(axis=1)
        att += (dead & (att == r + 1)).astype(np.int64)
    return att


def test_reduce_p1024_f3_65536_scenarios(ft, oracle, w):
    """Reduce, P = 1024, f = 3, 16 x int64 in [-2^40, 2^40), a root per scenario, failure sets of
    size 0..3 before the operation."""
    P, f, E, S, seed = 1024, 3, 16, 65536, 3
    plan = ft.Plan(P, f, E, ft.I64, ft.SUM)
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=0, rounds_per_attempt=plan.info.rounds_reduce + 1)
    root = w.random_roots(seed, S, P)
    xd = ft.gen_payload_int(plan, seed, S, 41)
    frd, fod, rd = to_dev(fr), to_dev(fo), to_dev(root.astype(np.uint32))
    g = ft.run_reduce(plan, S, xd, frd, fod, root=rd)
    v = ft.validate(plan, 0, S, xd, frd, fod, g["result"], g["status"], root=rd, msgs=g["msgs"])
    torch.cuda.synchronize()
    assert v["n_invalid"] == 0

    idx = _sample(S, 768)
    x = np.concatenate([w.payload_int(seed, 1, P, E, "i64", 41, scen0=int(s)) for s in idx])
    sel = torch.from_numpy(idx).cuda()
    assert np.array_equal(xd[sel].cpu().numpy(), x), "device generator differs from the host generator"
    o = oracle.reduce_batch(P, f, x, 0, 0, len(idx), root=root[idx], fail_rank=fr[idx], fail_round=fo[idx])
    st = g["status"].cpu().numpy()[idx]
    assert np.array_equal(st, o["status"])
    assert np.array_equal(g["result"][sel].cpu().numpy(), o["result"])
    assert np.array_equal(g["msgs"].cpu().numpy()[idx], o["msgs"])
    # the root is listed in some scenarios of a batch this large
    st_all = g["status"].cpu().numpy()
    root_listed = (fr == root[:, None]).any(axis=1)
    assert root_listed.any() and np.array_equal(st_all != 0, root_listed)


def test_allreduce_p16384_f4_4096_scenarios_f64(ft, oracle, w):
    """Allreduce, P = 16384, f = 4, 8 x fp64 N(0,1), k ~ U(0..4) failures, half of them during the
    operation at a uniform round."""
    P, f, E, S, seed = 16384, 4, 8, 4096, 4
    plan = ft.Plan(P, f, E, ft.F64, ft.SUM)
    Ratt = plan.info.rounds_attempt
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1)
    # a batch this size lists a root candidate only now and then: make sure of some retries
    fr[100], fo[100] = w.NO_RANK, 0
    fr[100, 0], fo[100, 0] = 0, 0
    fr[200], fo[200] = w.NO_RANK, 0
    fr[200, :3], fo[200, :3] = [1, 0, 9000], [0, 0, Ratt + 3]
    fr[300], fo[300] = [3, 2, 1, 0], [0, 0, 0, 0]
    xd = torch.empty((S, P, E), dtype=torch.float64, device="cuda")
    step = 256
    host = np.empty((step, P, E), dtype=np.float64)
    idx = _sample(S, 40, extra=(100, 200, 300))
    keep = {}
    for s0 in range(0, S, step):
        w.payload_normal(seed, step, P, E, scen0=s0, threads=16, out=host)
        xd[s0:s0 + step].copy_(torch.from_numpy(host))
        for s in idx:
            if s0 <= s < s0 + step:
                keep[int(s)] = host[s - s0].copy()
    x = np.stack([keep[int(s)] for s in idx])
    frd, fod = to_dev(fr), to_dev(fo)
    g = ft.run_allreduce(plan, S, xd, frd, fod)
    v = ft.validate(plan, 1, S, xd, frd, fod, g["result"], g["status"], has_bitmap=g["has_bitmap"],
                    per_process_out=g["per_process_out"], attempts=g["attempts"], msgs=g["msgs"])
    torch.cuda.synchronize()
    assert v["n_invalid"] == 0
    assert np.all(g["status"].cpu().numpy() == 0)
    att = g["attempts"].cpu().numpy().astype(np.int64)
    assert np.array_equal(att, _expected_attempts(fr, fo, f))
    assert att[100] == 2 and att[200] == 3 and att[300] == 5

    sel = torch.from_numpy(idx).cuda()
    o = oracle.allreduce_batch(P, f, x, 2, 0, len(idx), fail_rank=fr[idx], fail_round=fo[idx], want_has=True,
                               want_out=True)
    assert np.array_equal(g["status"].cpu().numpy()[idx], o["status"])
    assert np.array_equal(att[idx], o["attempts"])
    assert_values(g["result"][sel].cpu().numpy(), o["result"], 2, x, "result")
    assert np.array_equal(g["msgs"].cpu().numpy()[idx], o["msgs"])
    assert np.array_equal(unpack_bitmap(g["has_bitmap"].cpu().numpy()[idx], P), o["has"])
    assert np.array_equal(g["per_process_out"][sel].cpu().numpy(), o["out"])


def test_allreduce_p2e20_f8_1024_scenarios(ft, oracle, w):
    """Allreduce, P = 2^20, f = 8, one int64 in [-2^31, 2^31) per process, failure sets of size 0..8,
    a quarter of the failures during the operation."""
    P, f, E, S, seed = 1 << 20, 8, 1, 1024, 5
    plan = ft.Plan(P, f, E, ft.I64, ft.SUM)
    Ratt = plan.info.rounds_attempt
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=250, rounds_per_attempt=Ratt, protected=f + 1)
    fr[10], fo[10] = w.NO_RANK, 0
    fr[10, :2], fo[10, :2] = [0, 1], [0, 0]
    fr[20], fo[20] = w.NO_RANK, 0
    fr[20, :4], fo[20, :4] = [0, P - 1, 9, 12345], [0, 5, 2 * Ratt - 1, Ratt + 1]
    xd = ft.gen_payload_int(plan, seed, S, 32)
    frd, fod = to_dev(fr), to_dev(fo)
    g = ft.run_allreduce(plan, S, xd, frd, fod)
    v = ft.validate(plan, 1, S, xd, frd, fod, g["result"], g["status"], has_bitmap=g["has_bitmap"],
                    per_process_out=g["per_process_out"], attempts=g["attempts"], msgs=g["msgs"])
    torch.cuda.synchronize()
    assert v["n_invalid"] == 0
    assert np.all(g["status"].cpu().numpy() == 0)
    att = g["attempts"].cpu().numpy().astype(np.int64)
    assert np.array_equal(att, _expected_attempts(fr, fo, f))
    assert att[10] == 3 and att[20] == 2

    idx = _sample(S, 6, extra=(10, 20))
    x = np.concatenate([w.payload_int(seed, 1, P, E, "i64", 32, scen0=int(s)) for s in idx])
    sel = torch.from_numpy(idx).cuda()
    assert np.array_equal(xd[sel].cpu().numpy(), x), "device generator differs from the host generator"
    o = oracle.allreduce_batch(P, f, x, 0, 0, len(idx), fail_rank=fr[idx], fail_round=fo[idx], want_has=True,
                               want_out=True)
    assert np.array_equal(g["status"].cpu().numpy()[idx], o["status"])
    assert np.array_equal(att[idx], o["attempts"])
    assert np.array_equal(g["result"][sel].cpu().numpy(), o["result"])
    assert np.array_equal(g["msgs"].cpu().numpy()[idx], o["msgs"])
    assert np.array_equal(unpack_bitmap(g["has_bitmap"].cpu().numpy()[idx], P), o["has"])
    assert np.array_equal(g["per_process_out"][sel].cpu().numpy(), o["out"])


def test_allreduce_p2e20_f1_u32_deep_binary_groups(ft, oracle, w):
    """A tree of 19 levels with groups of two (P = 2^20, f = 1, one uint32 per process): the narrowest rows
    (8 bytes) through the eight-lanes-per-subtree kernel and two LDS-tile tiers of seven levels each; every
    scenario against the oracle."""
    from _cmp import compare_allreduce
    P, f, E, S, seed = 1 << 20, 1, 1, 6, 55
    plan = ft.Plan(P, f, E, ft.U32, ft.SUM)
    assert plan.info.deep_kernel == 2 and plan.info.tiers == 3
    Ratt = plan.info.rounds_attempt
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1)
    fr[0], fo[0] = w.NO_RANK, 0
    fr[1, 0], fo[1, 0] = 0, 0                        # a second attempt
    fr[2, 0], fo[2, 0] = P - 1, 0
    fr[3, 0], fo[3, 0] = 2, 0                        # the top of a subtree of the second root
    x = w.payload_int(seed, S, P, E, "u32", 32)
    compare_allreduce(ft, oracle, plan, x, fr, fo)
