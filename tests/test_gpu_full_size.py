"""The three large workloads at their full sizes, in the launch configuration the
benchmark times (default plan flags, the whole batch in one call): the HIP library
runs every scenario, and so does the CPU oracle, slice by slice so that host
memory stays bounded; EVERY scenario's status, result, message counters, attempts,
holder bitmap and receive buffers must agree as in the small parity tests.  As a
second check the library's own validation pass must find no invalid scenario.

Inputs: failure sets and roots of the whole batch come from the seeded host
generators.  The integer payloads the GPU works on are written by the library's
device generator; each slice is generated again on the host for the oracle
(scen0 = first scenario of the slice) and the two must be identical.  The
floating-point payload is generated on the host and uploaded."""
from concurrent.futures import ThreadPoolExecutor

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


def _expected_attempts(fr, fo, f):
    """1 + number of leading root candidates 0, 1, .. listed as failed before the operation."""
    S = fr.shape[0]
    att = np.ones(S, dtype=np.int64)
    for r in range(f + 1):
        dead = ((fr == r) & (fo == 0)).any(axis=1)
        att += (dead & (att == r + 1)).astype(np.int64)
    return att


def _host_payload_int(w, seed, s0, n, P, E, dtype, bits, threads=16):
    """payload_int for scenarios s0 .. s0+n-1, a few scenarios per task."""
    out = np.empty((n, P, E), dtype=np.int64 if dtype == "i64" else np.uint32)
    step = max(1, min(64, n // threads))

    def one(a):
        out[a:a + step] = w.payload_int(seed, min(step, n - a), P, E, dtype, bits, scen0=s0 + a)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(one, range(0, n, step)))
    return out


def test_reduce_p1024_f3_65536_scenarios(ft, oracle, w):
    """Reduce, P = 1024, f = 3, 16 x int64 in [-2^40, 2^40), a root per scenario, failure sets of
    size 0..3 before the operation: all 65536 scenarios against the oracle."""
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
    st, res, msgs = g["status"].cpu().numpy(), g["result"].cpu().numpy(), g["msgs"].cpu().numpy()

    step, done = 8192, 0
    for s0 in range(0, S, step):
        x = _host_payload_int(w, seed, s0, step, P, E, "i64", 41)
        assert np.array_equal(xd[s0:s0 + step].cpu().numpy(), x), "device generator differs from the host generator"
        o = oracle.reduce_batch(P, f, x, 0, 0, step, root=root[s0:s0 + step], fail_rank=fr[s0:s0 + step],
                                fail_round=fo[s0:s0 + step])
        assert np.array_equal(st[s0:s0 + step], o["status"]), s0
        assert np.array_equal(res[s0:s0 + step], o["result"]), s0
        assert np.array_equal(msgs[s0:s0 + step], o["msgs"]), s0
        done += step
    assert done == S
    # the root is listed in some scenarios of a batch this large
    root_listed = (fr == root[:, None]).any(axis=1)
    assert root_listed.any() and np.array_equal(st != 0, root_listed)


def _compare_allreduce_slice(oracle, plan, g, x, fr, fo, s0, n, att):
    """Scenarios s0 .. s0+n-1 of the batch result g against the oracle on payload x[n][P][E]."""
    P, f = plan.P, plan.f
    o = oracle.allreduce_batch(P, f, x, plan.dtype, plan.op, n, fail_rank=fr[s0:s0 + n], fail_round=fo[s0:s0 + n],
                               want_has=True, want_out=True)
    assert np.array_equal(g["status"][s0:s0 + n].cpu().numpy(), o["status"]), s0
    assert np.array_equal(att[s0:s0 + n], o["attempts"]), s0
    assert_values(g["result"][s0:s0 + n].cpu().numpy(), o["result"], plan.dtype, x, "result of slice %d" % s0)
    assert np.array_equal(g["msgs"][s0:s0 + n].cpu().numpy(), o["msgs"]), s0
    assert np.array_equal(unpack_bitmap(g["has_bitmap"][s0:s0 + n].cpu().numpy(), P), o["has"]), s0
    assert np.array_equal(g["per_process_out"][s0:s0 + n].cpu().numpy(), o["out"]), s0


def test_allreduce_p16384_f4_4096_scenarios_f64(ft, oracle, w):
    """Allreduce, P = 16384, f = 4, 8 x fp64 N(0,1), k ~ U(0..4) failures, half of them during the
    operation at a uniform round: all 4096 scenarios against the oracle."""
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
    for s0 in range(0, S, step):
        w.payload_normal(seed, step, P, E, scen0=s0, threads=16, out=host)
        xd[s0:s0 + step].copy_(torch.from_numpy(host))
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

    done = 0
    for s0 in range(0, S, step):
        w.payload_normal(seed, step, P, E, scen0=s0, threads=16, out=host)     # the oracle's input: from the host generator
        _compare_allreduce_slice(oracle, plan, g, host, fr, fo, s0, step, att)
        done += step
    assert done == S


class _P2e20:
    """The P = 2^20 batch, run once on the GPU; the oracle takes it a quarter at a time."""
    P, f, E, S, seed = 1 << 20, 8, 1, 1024, 5
    g = None


@pytest.fixture(scope="module")
def p2e20(ft, w):
    c = _P2e20
    plan = ft.Plan(c.P, c.f, c.E, ft.I64, ft.SUM)
    Ratt = plan.info.rounds_attempt
    fr, fo = w.random_failure_sets(c.seed, c.S, c.P, c.f, inop_permille=250, rounds_per_attempt=Ratt, protected=c.f + 1)
    fr[10], fo[10] = w.NO_RANK, 0
    fr[10, :2], fo[10, :2] = [0, 1], [0, 0]
    fr[20], fo[20] = w.NO_RANK, 0
    fr[20, :4], fo[20, :4] = [0, c.P - 1, 9, 12345], [0, 5, 2 * Ratt - 1, Ratt + 1]
    xd = ft.gen_payload_int(plan, c.seed, c.S, 32)
    frd, fod = to_dev(fr), to_dev(fo)
    g = ft.run_allreduce(plan, c.S, xd, frd, fod)
    v = ft.validate(plan, 1, c.S, xd, frd, fod, g["result"], g["status"], has_bitmap=g["has_bitmap"],
                    per_process_out=g["per_process_out"], attempts=g["attempts"], msgs=g["msgs"])
    torch.cuda.synchronize()
    yield dict(plan=plan, fr=fr, fo=fo, xd=xd, g=g, n_invalid=v["n_invalid"])
    del xd, g
    torch.cuda.empty_cache()


def test_allreduce_p2e20_f8_1024_scenarios_whole_batch_properties(p2e20):
    """Allreduce, P = 2^20, f = 8, one int64 in [-2^31, 2^31) per process, failure sets of size 0..8,
    a quarter of the failures during the operation: what holds for the batch as a whole."""
    c, g, fr, fo = _P2e20, p2e20["g"], p2e20["fr"], p2e20["fo"]
    assert p2e20["n_invalid"] == 0
    assert np.all(g["status"].cpu().numpy() == 0)
    att = g["attempts"].cpu().numpy().astype(np.int64)
    assert np.array_equal(att, _expected_attempts(fr, fo, c.f))
    assert att[10] == 3 and att[20] == 2


@pytest.mark.parametrize("quarter", [0, 1, 2, 3])
def test_allreduce_p2e20_f8_1024_scenarios_against_the_oracle(p2e20, oracle, w, quarter):
    """The same batch, every scenario against the oracle (256 scenarios per test, 32 per call of the oracle)."""
    c, plan, g, fr, fo = _P2e20, p2e20["plan"], p2e20["g"], p2e20["fr"], p2e20["fo"]
    att = g["attempts"].cpu().numpy().astype(np.int64)
    step, per = 32, c.S // 4
    done = 0
    for s0 in range(quarter * per, (quarter + 1) * per, step):
        x = _host_payload_int(w, c.seed, s0, step, c.P, c.E, "i64", 32)
        assert np.array_equal(p2e20["xd"][s0:s0 + step].cpu().numpy(), x), "device generator differs from the host generator"
        _compare_allreduce_slice(oracle, plan, g, x, fr, fo, s0, step, att)
        done += step
    assert done == per


def test_allreduce_p2e20_f4_deep_tree_in_parts(ft, oracle, w):
    """A tree too deep for one workgroup per scenario (P = 2^20, f = 4, 8 x fp64: 8192 subtrees of the deepest tier):
    the fused kernel folds it in parts below the rows of one depth, one LDS-tile launch takes it from there; every
    scenario against the oracle, failures aimed at the seams (tops of parts, the rows just above them, the last
    rows)."""
    from _cmp import compare_allreduce
    P, f, E, S, seed = 1 << 20, 4, 8, 6, 77
    plan = ft.Plan(P, f, E, ft.F64, ft.SUM)
    assert plan.info.deep_kernel == 1 and plan.info.fused == 1 and plan.info.tiers == 2
    Ratt = plan.info.rounds_attempt
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1)
    fr[0], fo[0] = w.NO_RANK, 0
    fr[1], fo[1] = w.NO_RANK, 0
    fr[1, 0], fo[1, 0] = 0, 0                        # a second attempt
    W = f + 1
    # rows 63 .. 126 are the 64 rows of depth 6 (tops of the parts at this size), 31 .. 62 the level above
    fr[2], fo[2] = [1 + 63 * W, 1 + 64 * W + 1, 1 + 126 * W + 4, 1 + 31 * W + 2], [0, 3, 0, 9]
    fr[3], fo[3] = [P - 1, P - 2, 1 + 62 * W, 1 + 127 * W + 3], [0, 5, 20, 0]
    x = w.payload_normal(seed, S, P, E, threads=8)
    compare_allreduce(ft, oracle, plan, x, fr, fo)


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
