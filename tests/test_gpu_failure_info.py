"""Parity of the failure-information outputs of ftred_run_reduce_info and
ftred_run_allreduce_info (first and second scheme of section "Failure
information") with the oracle: the length and the set of ids of the list carried
by the message the root selected, and what the root holds from each of its
children (no message / message without / with the failed bit, and its list).
The order inside a list is the library's own (slots of the failure list), so lists
are compared as sets; values, statuses and counters must equal those of the plain
entry points."""
import numpy as np
import pytest
import torch

from _cmp import to_dev

pytestmark = pytest.mark.gpu

NO_RANK = 0xFFFFFFFF


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


def _check_info(g, o, fr, f):
    S = fr.shape[0]
    count = g["info_count"].cpu().numpy()
    ids = g["info_ids"].cpu().numpy()
    child = g["info_child"].cpu().numpy()
    assert np.array_equal(count, o["info_count"]), np.nonzero(count != o["info_count"])[0][:10]
    for s in range(S):
        got = [int(q) for q in ids[s] if q != NO_RANK]
        assert len(got) == count[s] and set(got) == set(o["info_ids"][s]), (s, got, o["info_ids"][s])
        # padding only behind the ids
        assert np.all(ids[s][len(got):] == NO_RANK)
        for k in range(f + 1):
            state, cnt, want = o["info_child"][s][k]
            word = int(child[s, k])
            assert word >> 16 == state, (s, k, hex(word), o["info_child"][s])
            have = {int(fr[s, q]) for q in range(fr.shape[1]) if (word >> q) & 1}
            assert have == set(want) and len(have) == cnt, (s, k, hex(word), o["info_child"][s])


CASES = [
    # P, f, E, dtype, S, inop_permille
    (7, 1, 1, 0, 64, 500), (9, 2, 3, 1, 64, 700), (13, 3, 2, 0, 96, 600), (64, 2, 8, 1, 128, 500),
    (100, 6, 5, 2, 128, 600), (257, 7, 2, 0, 128, 600), (1000, 8, 1, 0, 96, 500), (1024, 3, 16, 0, 128, 400),
    (1500, 4, 8, 2, 128, 500), (4099, 5, 3, 2, 48, 500), (20000, 2, 4, 1, 24, 500), (33333, 4, 8, 2, 12, 500),
    (3000, 12, 2, 0, 32, 500),
    # one value per process (eight lanes per subtree in the deepest tier)
    (5003, 4, 1, 2, 48, 500), (2500, 3, 1, 0, 48, 500),
]


def _payload(w, seed, S, P, E, dtype):
    if dtype == 0:
        return w.payload_int(seed, S, P, E, "i64", 41)
    if dtype == 1:
        return w.payload_int(seed, S, P, E, "u32", 32)
    return w.payload_normal(seed, S, P, E, threads=4)


@pytest.mark.parametrize("P,f,E,dtype,S,permille", CASES)
def test_reduce_info(ft, oracle, w, P, f, E, dtype, S, permille):
    seed = 5000 + P + 31 * f + E
    D = oracle.structure(P, f, 0)["D"]
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=permille, rounds_per_attempt=f + D + 1)
    root = w.random_roots(seed, S, P)
    root[: S // 4] = 0
    x = _payload(w, seed, S, P, E, dtype)
    plan = ft.Plan(P, f, E, dtype, 0)
    xd, frd, fod, rd = to_dev(x), to_dev(fr), to_dev(fo), to_dev(root.astype(np.uint32))
    g = ft.run_reduce_info(plan, S, xd, frd, fod, root=rd)
    plain = ft.run_reduce(plan, S, xd, frd, fod, root=rd)
    torch.cuda.synchronize()
    for k in ("result", "status", "msgs"):
        assert torch.equal(g[k].view(torch.uint8), plain[k].view(torch.uint8)), k
    o = oracle.reduce_info_batch(P, f, x, dtype, 0, S, root=root, fail_rank=fr, fail_round=fo)
    assert np.array_equal(g["status"].cpu().numpy(), o["status"])
    assert np.array_equal(g["result"].cpu().numpy(), o["result"])
    _check_info(g, o, fr, f)


@pytest.mark.parametrize("P,f,E,dtype,S,permille", [c for c in CASES if c[0] >= 9])
def test_allreduce_info(ft, oracle, w, P, f, E, dtype, S, permille):
    seed = 6000 + P + 31 * f + E
    D = oracle.structure(P, f, 0)["D"]
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=permille, rounds_per_attempt=2 * (f + D),
                                   protected=f + 1)
    # retries: leading root candidates failed beforehand
    fr[3], fo[3] = NO_RANK, 0
    fr[3, 0] = 0
    fr[4], fo[4] = NO_RANK, 0
    for k in range(min(f, 2)):
        fr[4, k] = k
    x = _payload(w, seed, S, P, E, dtype)
    plan = ft.Plan(P, f, E, dtype, 0)
    xd, frd, fod = to_dev(x), to_dev(fr), to_dev(fo)
    g = ft.run_allreduce_info(plan, S, xd, frd, fod)
    plain = ft.run_allreduce(plan, S, xd, frd, fod)
    torch.cuda.synchronize()
    for k in ("result", "status", "attempts", "msgs", "has_bitmap", "per_process_out"):
        assert torch.equal(g[k].view(torch.uint8), plain[k].view(torch.uint8)), k
    o = oracle.allreduce_info_batch(P, f, x, dtype, 0, S, fail_rank=fr, fail_round=fo)
    assert np.array_equal(g["status"].cpu().numpy(), o["status"])
    assert np.array_equal(g["attempts"].cpu().numpy(), o["attempts"])
    assert np.array_equal(g["result"].cpu().numpy(), o["result"])
    _check_info(g, o, fr, f)
    assert o["attempts"][3] >= 2 and o["attempts"][4] == min(f, 2) + 1


def test_info_headline_shape_sample(ft, oracle, w):
    """P = 16384, f = 4, 8 x fp64: the register kernel runs most subtrees, the listed ones go through
    the tile kernel with the lists; 256 scenarios against the oracle."""
    P, f, E, S, seed = 16384, 4, 8, 256, 44
    plan = ft.Plan(P, f, E, ft.F64, ft.SUM)
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=plan.info.rounds_attempt,
                                   protected=f + 1)
    x = w.payload_normal(seed, S, P, E, threads=8)
    g = ft.run_allreduce_info(plan, S, to_dev(x), to_dev(fr), to_dev(fo))
    torch.cuda.synchronize()
    o = oracle.allreduce_info_batch(P, f, x, 2, 0, S, fail_rank=fr, fail_round=fo)
    assert np.array_equal(g["result"].cpu().numpy(), o["result"])
    _check_info(g, o, fr, f)


def test_info_needs_an_output(ft, w):
    plan = ft.Plan(64, 2, 1, ft.I64, ft.SUM)
    S = 2
    x = to_dev(w.payload_int(1, S, 64, 1, "i64", 20))
    fr = to_dev(np.full((S, 2), NO_RANK, np.uint32))
    fo = to_dev(np.zeros((S, 2), np.uint32))
    res = torch.empty((S, 1), dtype=torch.int64, device="cuda")
    st = torch.empty(S, dtype=torch.uint32, device="cuda")
    ws = plan.workspace(S)
    rc = ft.lib().ftred_run_reduce_info(plan.handle, S, None, x.data_ptr(), 64, fr.data_ptr(), fo.data_ptr(),
                                        res.data_ptr(), st.data_ptr(), None, None, None, None, ws.data_ptr(),
                                        ws.numel(), None)
    assert rc == ft.EINVAL and b"info_count" in ft.lib().ftred_last_error()
