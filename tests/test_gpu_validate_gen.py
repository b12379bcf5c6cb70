"""GPU tests of the validation kernels (against the plain definition of a valid
result in oracle.definition) and of the device generators (bit for bit against
the host generators of the workloads module)."""
import numpy as np
import pytest
import torch

from _cmp import to_dev, unpack_bitmap

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ft():
    from paper_2602_22445_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


@pytest.fixture(scope="module")
def w():
    from paper_2602_22445_amd import workloads
    return workloads


def _payload(w, seed, S, P, E, dtype):
    if dtype == 0:
        return w.payload_int(seed, S, P, E, "i64", 41)
    if dtype == 1:
        return w.payload_int(seed, S, P, E, "u32", 32)
    return w.payload_normal(seed, S, P, E, threads=4)


# ---------------------------------------------------------------------------
# device generators == host generators


@pytest.mark.parametrize("P,f,permille,protected", [(16384, 4, 500, 5), (64, 2, 0, 0), (1 << 20, 8, 250, 9),
                                                    (9, 7, 600, 8), (1024, 3, 0, 0), (50, 0, 0, 0)])
def test_device_failure_generator_matches_host(ft, w, P, f, permille, protected):
    S, seed, scen0, rpa = 3000, 12345678901234, 17, 2 * (f + 13)
    plan = ft.Plan(P, f, 1, ft.I64, ft.SUM)
    fr_d, fo_d, root_d = ft.gen_failures(plan, seed, S, scen0=scen0, inop_permille=permille, rounds_per_attempt=rpa,
                                         protected=protected, want_root=True)
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=permille, rounds_per_attempt=rpa,
                                   protected=protected, scen0=scen0)
    root = w.random_roots(seed, S, P, scen0=scen0)
    assert np.array_equal(fr_d.cpu().numpy(), fr)
    assert np.array_equal(fo_d.cpu().numpy(), fo)
    assert np.array_equal(root_d.cpu().numpy(), root)
    if f > 0:
        k = (fr != w.NO_RANK).sum(axis=1)
        assert k.min() == 0 and k.max() == f        # all sizes 0..f occur


@pytest.mark.parametrize("P,E,dtype,bits", [(8, 4, 0, 32), (1024, 16, 0, 41), (64, 8, 1, 32), (1001, 3, 1, 17),
                                            (77, 1, 0, 64), (16384, 1, 0, 32)])
def test_device_payload_generator_matches_host(ft, w, P, E, dtype, bits):
    S, seed, scen0 = 5, 3, 1000
    plan = ft.Plan(P, 1, E, dtype, ft.SUM)
    xd = ft.gen_payload_int(plan, seed, S, bits, scen0=scen0)
    x = w.payload_int(seed, S, P, E, "i64" if dtype == 0 else "u32", bits, scen0=scen0)
    assert np.array_equal(xd.cpu().numpy(), x)


# ---------------------------------------------------------------------------
# validation kernels


def _run_and_validate(ft, plan, kind, S, xd, frd, fod, root=None):
    if kind == 1:
        g = ft.run_allreduce(plan, S, xd, frd, fod)
        v = ft.validate(plan, 1, S, xd, frd, fod, g["result"], g["status"], has_bitmap=g["has_bitmap"],
                        per_process_out=g["per_process_out"], attempts=g["attempts"], msgs=g["msgs"])
    else:
        g = ft.run_reduce(plan, S, xd, frd, fod, root=root)
        v = ft.validate(plan, 0, S, xd, frd, fod, g["result"], g["status"], root=root, msgs=g["msgs"])
    return g, v


CASES = [(10, 2, 2, 0, 0, 200), (64, 2, 8, 1, 1, 300), (64, 2, 8, 1, 0, 300), (1000, 8, 1, 0, 0, 100),
         (1500, 4, 8, 2, 0, 128), (4099, 5, 3, 2, 0, 64), (3000, 12, 2, 0, 1, 40), (2000, 1, 300, 2, 0, 6)]


@pytest.mark.parametrize("P,f,E,dtype,op,S", CASES)
@pytest.mark.parametrize("kind", [0, 1])
def test_validation_accepts_the_library_results_and_the_definition_agrees(ft, oracle, w, P, f, E, dtype, op, S, kind):
    seed = 3000 + P + f
    plan = ft.Plan(P, f, E, dtype, op)
    rpa = plan.info.rounds_attempt if kind == 1 else plan.info.rounds_reduce
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=600, rounds_per_attempt=rpa,
                                   protected=f + 1 if kind == 1 else 0)
    root = None
    if kind == 0:
        root = w.random_roots(seed, S, P)
        fr[1], fo[1] = w.NO_RANK, 0
        fr[1, 0] = root[1]                          # a failed root
    else:
        fr[1], fo[1] = w.NO_RANK, 0
        fr[1, 0] = 0                                # a retry
    fr[2, 0] = P + 3                                # a bad failure set
    x = _payload(w, seed, S, P, E, dtype)
    xd, frd, fod = to_dev(x), to_dev(fr), to_dev(fo)
    rd = None if root is None else to_dev(root)
    g, v = _run_and_validate(ft, plan, kind, S, xd, frd, fod, rd)
    verdict = v["verdict"].cpu().numpy()
    assert v["n_invalid"] == 0 and np.all(verdict == 0), np.nonzero(verdict)[0][:10]
    st = g["status"].cpu().numpy()
    assert st[2] == ft.ST_BAD_FAILURE_SET
    assert st[1] == (ft.ST_ROOT_FAILED if kind == 0 else ft.ST_OK)
    # the plain definition accepts the same results
    res = g["result"].cpu().numpy()
    for s in range(0, S, max(1, S // 40)):
        if st[s] != ft.ST_OK:
            continue
        pre = [int(q) for q, t in zip(fr[s], fo[s]) if q != w.NO_RANK and t == 0]
        inop = [int(q) for q, t in zip(fr[s], fo[s]) if q != w.NO_RANK and t != 0]
        assert oracle.is_valid_result(res[s], x[s], dtype, op, pre, inop), s


def test_validation_rejects_wrong_values_holders_statuses_and_counters(ft, oracle, w):
    P, f, E, S = 2000, 4, 8, 64
    plan = ft.Plan(P, f, E, ft.F64, ft.SUM)
    fr, fo = w.random_failure_sets(8, S, P, f, inop_permille=500, rounds_per_attempt=plan.info.rounds_attempt,
                                   protected=f + 1)
    for s in range(10, 20):                          # make sure these have a failure before the operation
        fr[s], fo[s] = w.NO_RANK, 0
        fr[s, 0] = 100 + s
    x = w.payload_normal(8, S, P, E)
    xd, frd, fod = to_dev(x), to_dev(fr), to_dev(fo)
    g = ft.run_allreduce(plan, S, xd, frd, fod)
    torch.cuda.synchronize()

    def verdicts(**over):
        a = dict(result=g["result"], status=g["status"], has_bitmap=g["has_bitmap"],
                 per_process_out=g["per_process_out"], attempts=g["attempts"], msgs=g["msgs"])
        a.update(over)
        v = ft.validate(plan, 1, S, xd, frd, fod, a["result"], a["status"], has_bitmap=a["has_bitmap"],
                        per_process_out=a["per_process_out"], attempts=a["attempts"], msgs=a["msgs"])
        return v["verdict"].cpu().numpy(), v["n_invalid"]

    v0, n0 = verdicts()
    assert n0 == 0

    # a value off by 1e-6 relative; a value that includes a process failed beforehand
    res = g["result"].clone()
    res[3, 2] *= 1.0 + 1e-6
    res[12] += xd[12, 112]                           # rank 112 failed before the operation in scenario 12
    v, n = verdicts(result=res)
    assert n == 2 and (v[3] & ft.BAD_VALUE) and (v[12] & ft.BAD_VALUE)
    assert np.all(v[[s for s in range(S) if s not in (3, 12)]] == 0)
    # ... which the plain definition rejects as well
    assert not oracle.is_valid_result(res[12].cpu().numpy(), x[12], 2, 0, [112], [])
    assert not oracle.is_valid_result(res[3].cpu().numpy(), x[3], 2, 0,
                                      [int(q) for q, t in zip(fr[3], fo[3]) if q != w.NO_RANK and t == 0],
                                      [int(q) for q, t in zip(fr[3], fo[3]) if q != w.NO_RANK and t != 0])

    # a survivor that does not hold the value; a receive buffer with another value
    bm = g["has_bitmap"].clone()
    bm_np = bm.cpu().numpy()
    bm_np[5, 1500 // 32] &= ~np.uint32(1 << (1500 % 32))
    assert 1500 not in fr[5]
    v, n = verdicts(has_bitmap=to_dev(bm_np))
    assert n == 1 and (v[5] & ft.BAD_HOLDER)
    out = g["per_process_out"].clone()
    out[7, 1999, 7] += 1.0
    v, n = verdicts(per_process_out=out)
    assert n == 1 and (v[7] & ft.BAD_HOLDER)

    # a wrong status, wrong attempts, message counters above the failure-free count
    stt = g["status"].cpu().numpy().copy()
    stt[9] = ft.ST_ROOT_FAILED
    v, n = verdicts(status=to_dev(stt))
    assert n == 1 and (v[9] & ft.BAD_STATUS)
    att = g["attempts"].cpu().numpy().copy()
    att[11] += 1
    v, n = verdicts(attempts=to_dev(att))
    assert n == 1 and (v[11] & ft.BAD_STATUS)
    ms = g["msgs"].cpu().numpy().copy()
    ms[13, 0] += 1
    ms[14, 3] = plan.info.msgs_bcast_corr_ff + 1
    v, n = verdicts(msgs=to_dev(ms))
    assert n == 2 and (v[13] & ft.BAD_COUNT) and (v[14] & ft.BAD_COUNT)


def test_validation_of_in_operation_choices(ft, oracle, w):
    """An in-operation failure leaves two valid results; validation accepts both
    and rejects a mix (the failed value included in some elements only)."""
    P, f, E, S = 300, 2, 4, 3
    plan = ft.Plan(P, f, E, ft.I64, ft.SUM)
    fr = np.full((S, f), w.NO_RANK, dtype=np.uint32)
    fo = np.zeros((S, f), dtype=np.uint32)
    fr[:, 0], fo[:, 0] = 200, 3
    fr[:, 1], fo[:, 1] = 50, 0
    x = w.payload_int(21, S, P, E, "i64", 30)
    with_q = np.stack([oracle.survivor_reduce(x[s], 0, 0, [50]) for s in range(S)])
    without_q = np.stack([oracle.survivor_reduce(x[s], 0, 0, [50, 200]) for s in range(S)])
    mixed = with_q.copy()
    mixed[:, 0] = without_q[:, 0]
    res = np.stack([with_q[0], without_q[1], mixed[2]])
    xd, frd, fod = to_dev(x), to_dev(fr), to_dev(fo)
    status = torch.zeros(S, dtype=torch.uint32, device="cuda")
    v = ft.validate(plan, 0, S, xd, frd, fod, to_dev(res), status)
    assert v["verdict"].cpu().numpy().tolist() == [0, 0, ft.BAD_VALUE]
