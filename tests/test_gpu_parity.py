"""Parity of the HIP library (through the C-ABI) with the CPU oracle, element by
element, on the same seeded inputs.  Integer results, statuses, attempts, message
counters, holder bitmaps and receive buffers must be bit-exact; FTRED_F64 results
must lie within 1e-12 * sum|x| of the oracle's (they are in fact bit-identical,
because both sides fold in the same order, and that is asserted too)."""
import numpy as np
import pytest
import torch

from _cmp import compare_allreduce, compare_reduce, to_dev, unpack_bitmap

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


def _payload(w, seed, S, P, E, dtype):
    if dtype == 0:
        return w.payload_int(seed, S, P, E, "i64", 41)
    if dtype == 1:
        return w.payload_int(seed, S, P, E, "u32", 32)
    return w.payload_normal(seed, S, P, E, threads=4)


def _rounds(oracle, P, f):
    D = oracle.structure(P, f, 0)["D"]
    return f + D, 2 * (f + D)


# ---------------------------------------------------------------------------
# a1: device index arithmetic


@pytest.mark.parametrize("P,f,root", [(7, 1, 0), (8, 1, 5), (64, 2, 0), (1000, 8, 999), (1024, 3, 77), (4099, 15, 1)])
def test_device_index_arithmetic(ft, oracle, P, f, root):
    plan = ft.Plan(P, f, 1, ft.I64, ft.SUM)
    d = {k: v.cpu().numpy() for k, v in ft.structure(plan, root).items()}
    s = oracle.structure(P, f, root)
    par = np.where(s["parent"] < 0, ft.NO_RANK, s["parent"]).astype(np.uint32)
    assert np.array_equal(d["parent"], par)
    assert np.array_equal(d["subtree"], s["subtree"])
    assert np.array_equal(d["depth"], s["depth"])
    assert np.array_equal(d["send_round"], s["send_round"])
    assert np.array_equal(d["group_pos"], s["gpos"])
    assert np.array_equal(d["group_size"], s["gsize"])
    grp = np.where(s["group"] < 0, ft.NO_RANK, s["group"]).astype(np.uint32)
    assert np.array_equal(d["group_id"], grp)


# ---------------------------------------------------------------------------
# configuration 1: reduce, P=8, f=1, int64 sum, exhaustive failure sets x 32 payload seeds


def test_config1_reduce_p8_f1_exhaustive(ft, oracle, w):
    P, f, E = 8, 1, 4
    fr9, fo9 = w.exhaustive_failure_sets(P, f)
    fr, fo = np.repeat(fr9, 32, axis=0), np.repeat(fo9, 32, axis=0)
    S = fr.shape[0]
    assert S == 288
    x = w.payload_int(1, S, P, E, "i64", 32)
    plan = ft.Plan(P, f, E, ft.I64, ft.SUM)
    g, o = compare_reduce(ft, oracle, plan, x, fr, fo)
    st = g["status"].cpu().numpy()
    assert (st == ft.ST_ROOT_FAILED).sum() == 32 and (st == ft.ST_OK).sum() == 256
    # the definition: the reduction over the processes that did not fail
    res = g["result"].cpu().numpy()
    for s in range(S):
        F = [int(q) for q in fr[s] if q != w.NO_RANK]
        if 0 not in F:
            assert np.array_equal(res[s], oracle.survivor_reduce(x[s], 0, 0, F))


# ---------------------------------------------------------------------------
# configuration 2: allreduce, P=64, f=2, uint32 sum and or, exhaustive failure sets


@pytest.mark.parametrize("op", [0, 1])
def test_config2_allreduce_p64_f2_exhaustive(ft, oracle, w, op):
    P, f, E = 64, 2, 8
    fr, fo = w.exhaustive_failure_sets(P, f)
    S = fr.shape[0]
    assert S == 2081
    x = w.payload_int(2, S, P, E, "u32", 32)
    plan = ft.Plan(P, f, E, ft.U32, op)
    g, o = compare_allreduce(ft, oracle, plan, x, fr, fo)
    res = g["result"].cpu().numpy()
    out = g["per_process_out"].cpu().numpy()
    for s in range(0, S, 7):
        F = [int(q) for q in fr[s] if q != w.NO_RANK]
        want = oracle.survivor_reduce(x[s], 1, op, F)
        assert np.array_equal(res[s], want)
        alive = np.ones(P, bool)
        alive[F] = False
        assert np.all(out[s][alive] == want) and np.all(out[s][~alive] == 0)


# ---------------------------------------------------------------------------
# sweeps over shapes, types, roots, failure times (several tiles, ragged tails)

REDUCE_CASES = [
    # P, f, E, dtype, op, S, inop_permille
    (2, 0, 1, 0, 0, 5, 0), (3, 1, 1, 0, 0, 40, 500), (5, 3, 2, 1, 1, 40, 500), (7, 1, 1, 0, 0, 64, 500),
    (8, 1, 4, 0, 0, 64, 500), (9, 2, 3, 1, 0, 64, 700), (17, 15, 1, 0, 0, 64, 500), (64, 2, 8, 1, 1, 128, 500),
    (100, 6, 5, 2, 0, 128, 600), (257, 7, 2, 0, 1, 128, 600), (1000, 8, 1, 0, 0, 96, 500),
    (1024, 3, 16, 0, 0, 256, 400), (1500, 4, 8, 2, 0, 128, 500), (4099, 5, 3, 2, 0, 48, 500),
    (5000, 0, 2, 0, 0, 16, 0), (20000, 2, 4, 1, 0, 24, 500), (33333, 4, 8, 2, 0, 12, 500),
    (3000, 12, 2, 0, 0, 32, 500), (1 << 16, 8, 1, 0, 0, 6, 500), (3000, 12, 40, 2, 0, 12, 500),
    # the register kernel of the deepest tier: two passes over the value indices, bitwise or, every group width
    (3000, 1, 80, 1, 0, 24, 500), (2000, 2, 4, 1, 1, 64, 500), (700, 1, 3, 0, 1, 64, 500), (9000, 3, 5, 2, 0, 24, 500),
    (5000, 8, 3, 0, 0, 24, 500),
    # one value per process: eight lanes per subtree, every group width; fewer than eight subtrees in the tier
    (700, 1, 1, 2, 0, 64, 500), (1000, 2, 1, 1, 1, 64, 500), (2500, 3, 1, 0, 1, 48, 500), (5003, 4, 1, 2, 0, 48, 500),
    (81, 1, 1, 0, 0, 64, 500), (200, 1, 1, 1, 0, 64, 500),
]


@pytest.mark.parametrize("P,f,E,dtype,op,S,permille", REDUCE_CASES)
def test_reduce_sweep(ft, oracle, w, P, f, E, dtype, op, S, permille):
    seed = 1000 + P + 31 * f + E
    Rred, _ = _rounds(oracle, P, f)
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=permille, rounds_per_attempt=Rred + 1)
    root = w.random_roots(seed, S, P)
    root[: S // 4] = 0
    if S > 8 and f >= 1:
        # aim some failures at the root, its children and its group
        fr[5], fo[5] = w.NO_RANK, 0
        fr[5, 0], fo[5, 0] = root[5], 0
        fr[6], fo[6] = w.NO_RANK, 0
        fr[6, 0], fo[6, 0] = (root[6] + 1) % P, 1
        fr[7], fo[7] = w.NO_RANK, 0
        fr[7, 0], fo[7, 0] = P - 1 if root[7] != P - 1 else P - 2, 2
    x = _payload(w, seed, S, P, E, dtype)
    plan = ft.Plan(P, f, E, dtype, op)
    compare_reduce(ft, oracle, plan, x, fr, fo, root=root)


ALLREDUCE_CASES = [
    (2, 0, 1, 0, 0, 4, 0), (3, 1, 1, 0, 0, 40, 500), (6, 4, 2, 1, 1, 64, 500), (7, 1, 1, 0, 0, 64, 500),
    (9, 2, 3, 1, 0, 64, 700), (17, 15, 1, 0, 0, 64, 500), (64, 2, 8, 1, 1, 128, 500), (100, 6, 5, 2, 0, 128, 600),
    (257, 7, 2, 0, 1, 128, 600), (1000, 8, 1, 0, 0, 96, 250), (1024, 3, 16, 0, 0, 128, 400),
    (1500, 4, 8, 2, 0, 128, 500), (4099, 5, 3, 2, 0, 48, 500), (20000, 2, 4, 1, 0, 24, 500),
    (33333, 4, 8, 2, 0, 12, 500), (3000, 12, 2, 0, 0, 32, 500), (1 << 16, 8, 1, 0, 0, 6, 250), (3000, 12, 40, 2, 0, 12, 500),
    (3000, 1, 80, 1, 0, 24, 500), (2000, 2, 4, 1, 1, 64, 500), (700, 1, 3, 0, 1, 64, 500), (9000, 3, 5, 2, 0, 24, 500),
    # one 4-byte value per process: four receive buffers per store; and a P that rules that path out
    (1004, 2, 1, 1, 0, 64, 500), (1003, 2, 1, 1, 1, 64, 500),
    (5000, 8, 3, 0, 0, 24, 500),
    # a whole scenario in one workgroup whose top rows take more LDS than a launch gets without asking (64 KiB)
    (16384, 7, 8, 2, 0, 6, 500),
    # one value per process: eight lanes per subtree, every group width; fewer than eight subtrees in the tier
    (700, 1, 1, 2, 0, 64, 500), (2500, 3, 1, 0, 1, 48, 500), (5003, 4, 1, 2, 0, 48, 500),
    (81, 1, 1, 0, 0, 64, 500), (200, 1, 1, 1, 0, 64, 500),
]


def test_the_sweeps_reach_both_kernels_of_the_deepest_tier(ft):
    """Plans of the sweep cases: the register kernels for deep trees (eight lanes per subtree when a process holds
    one value, one lane otherwise; groups of more than 9 with the listed subtrees on the LDS-tile list kernel, as
    long as a subtree fits its tile), LDS tiles otherwise; one case walks the value indices in two passes (more
    than 64 of them)."""
    kinds = {(P, f, E, dt): ft.Plan(P, f, E, dt, op).info.deep_kernel for P, f, E, dt, op, _, _ in ALLREDUCE_CASES}
    assert kinds[(3000, 1, 80, 1)] == 1 and kinds[(2000, 2, 4, 1)] == 1 and kinds[(9000, 3, 5, 2)] == 1
    assert kinds[(1000, 8, 1, 0)] == 2 and kinds[(33333, 4, 8, 2)] == 1 and kinds[(1 << 16, 8, 1, 0)] == 2
    assert kinds[(81, 1, 1, 0)] == 2 and kinds[(200, 1, 1, 1)] == 2 and kinds[(5000, 8, 3, 0)] == 1
    assert kinds[(4099, 5, 3, 2)] == 1 and kinds[(3000, 12, 2, 0)] == 1 and kinds[(64, 2, 8, 1)] == 0
    assert kinds[(3000, 12, 40, 2)] == 0
    assert {f + 1 for (P, f, E, dt), k in kinds.items() if k == 1} >= {2, 3, 4, 5, 9}
    assert {f + 1 for (P, f, E, dt), k in kinds.items() if k == 2} >= {2, 3, 4, 5, 9}


@pytest.mark.parametrize("P,f,E,dtype,op,S,permille", ALLREDUCE_CASES)
def test_allreduce_sweep(ft, oracle, w, P, f, E, dtype, op, S, permille):
    seed = 2000 + P + 31 * f + E
    _, Ratt = _rounds(oracle, P, f)
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=permille, rounds_per_attempt=Ratt, protected=f + 1)
    if f >= 1 and S > 8:
        # force retries: leading root candidates failed beforehand
        fr[3, 0], fo[3, 0] = 0, 0
        for k in range(min(f, 3)):
            fr[4, k], fo[4, k] = k, 0
        # dedupe the rows just edited
        for s in (3, 4):
            seen = set()
            for k in range(fr.shape[1]):
                if fr[s, k] != w.NO_RANK and int(fr[s, k]) in seen:
                    fr[s, k], fo[s, k] = w.NO_RANK, 0
                seen.add(int(fr[s, k]))
        # re-time the in-operation failures of retry scenarios over all their attempts
    x = _payload(w, seed, S, P, E, dtype)
    plan = ft.Plan(P, f, E, dtype, op)
    g, o = compare_allreduce(ft, oracle, plan, x, fr, fo)
    assert np.all(o["status"] == 0)
    if f >= 1 and S > 8:
        assert o["attempts"][3] >= 2 and o["attempts"][4] == min(f, 3) + 1


def test_allreduce_every_failure_time_small(ft, oracle, w):
    """P=10, f=2: every pair of non-candidate ranks from a sample, every pair of failure times."""
    P, f, E = 10, 2, 2
    _, Ratt = _rounds(oracle, P, f)
    rows_r, rows_t = [], []
    for a_, b_ in [(3, 4), (3, 7), (5, 9), (4, 8), (6, 9), (0, 5), (1, 9), (0, 1)]:
        ta = [0] if a_ <= f else range(0, 2 * Ratt + 1)
        tb = [0] if b_ <= f else range(0, 2 * Ratt + 1)
        for x_ in ta:
            for y_ in tb:
                rows_r.append([a_, b_])
                rows_t.append([x_, y_])
    fr = np.array(rows_r, dtype=np.uint32)
    fo = np.array(rows_t, dtype=np.uint32)
    S = fr.shape[0]
    x = w.payload_int(5, S, P, E, "i64", 20)
    plan = ft.Plan(P, f, E, ft.I64, ft.SUM)
    compare_allreduce(ft, oracle, plan, x, fr, fo)


def test_bad_failure_sets_get_a_status_and_zero_outputs(ft, oracle, w):
    P, f, E, S = 50, 3, 2, 6
    fr = np.full((S, f), w.NO_RANK, dtype=np.uint32)
    fo = np.zeros((S, f), dtype=np.uint32)
    fr[1, 0] = 50                       # rank >= P
    fr[2, 0] = fr[2, 2] = 7             # listed twice
    fr[3, 1], fo[3, 1] = 2, 4           # a root candidate failing during the operation (allreduce only)
    fr[4, 0] = 9
    x = w.payload_int(6, S, P, E, "i64", 30)
    plan = ft.Plan(P, f, E, ft.I64, ft.SUM)
    g, o = compare_allreduce(ft, oracle, plan, x, fr, fo)
    assert g["status"].cpu().numpy().tolist() == [0, 3, 3, 3, 0, 0]
    g, o = compare_reduce(ft, oracle, plan, x, fr, fo)
    assert g["status"].cpu().numpy().tolist() == [0, 3, 3, 0, 0, 0]


@pytest.mark.parametrize("flags,min_tiers", [(0, 2), (0x1000 | 8, 3), (0x1000, 2), (0x100 | 0x1000 | 16, 2)])
def test_shared_payload_unaligned_pointer_and_tree_kernel_variants(ft, oracle, w, flags, min_tiers):
    """stride 0 (one payload for all scenarios), a payload pointer that is only
    8-byte aligned (element-wise staging), and the variants of the tree kernels:
    wavefront-per-subtree deepest tier (default), LDS-tile deepest tier (flag
    0x1000) with a small LDS budget (more tiers) and one tile per workgroup."""
    P, f, E, S = 3000, 3, 16, 32
    Rred, Ratt = _rounds(oracle, P, f)
    fr, fo = w.random_failure_sets(77, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1)
    fr[2, 0], fo[2, 0] = 0, 0               # a retry
    x1 = w.payload_normal(77, 1, P, E, threads=1)[0]
    plan = ft.Plan(P, f, E, ft.F64, ft.SUM, flags)
    assert plan.info.tiers >= min_tiers
    buf = torch.empty(P * E + 1, dtype=torch.float64, device="cuda")
    xd = buf[1:].view(P, E)
    xd.copy_(torch.from_numpy(x1))
    assert xd.data_ptr() % 16 == 8
    g = ft.run_allreduce(plan, S, xd, to_dev(fr), to_dev(fo))
    o = oracle.allreduce_batch(P, f, x1, ft.F64, ft.SUM, S, fail_rank=fr, fail_round=fo, want_out=True)
    assert np.array_equal(g["status"].cpu().numpy(), o["status"])
    assert np.array_equal(g["attempts"].cpu().numpy(), o["attempts"]) and o["attempts"][2] == 2
    assert np.array_equal(g["result"].cpu().numpy(), o["result"])
    assert np.array_equal(g["msgs"].cpu().numpy(), o["msgs"])
    assert np.array_equal(unpack_bitmap(g["has_bitmap"].cpu().numpy(), P), o["has"])
    assert np.array_equal(g["per_process_out"].cpu().numpy(), o["out"])


@pytest.mark.parametrize("P,f,E,dtype", [(9000, 8, 1, 0), (9000, 4, 1, 2), (9000, 3, 5, 2), (20000, 2, 4, 1)])
@pytest.mark.parametrize("flags", [0x2000, 0x4000, 0x6000, 0xE000])
def test_groups_of_subtrees_per_wavefront(ft, oracle, w, P, f, E, dtype, flags):
    """Plan flags bits 13..15: a wavefront of the register kernels walks through 1, 2, 4 or (clamped) all groups
    of sibling subtrees of a scenario; one value per process (eight lanes per subtree, top rows staged in LDS)
    and wider payloads (one lane per subtree); reduce with a root per scenario."""
    S, seed = 24, 4000 + P + f + E
    Rred, _ = _rounds(oracle, P, f)
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=Rred + 1)
    fr[:4] = w.NO_RANK                                  # some scenarios without failures
    root = w.random_roots(seed, S, P)
    root[:2] = 0
    x = _payload(w, seed, S, P, E, dtype)
    plan = ft.Plan(P, f, E, dtype, 0, flags)
    assert plan.info.deep_kernel == (2 if E == 1 else 1)
    compare_reduce(ft, oracle, plan, x, fr, fo, root=root)


@pytest.mark.parametrize("P,f,E,dtype,op,S,permille", [c for c in ALLREDUCE_CASES if c[0] >= 64])
def test_allreduce_sweep_lds_tile_kernel(ft, oracle, w, P, f, E, dtype, op, S, permille):
    """The same sweep with the LDS-tile kernel as the deepest tier (flag 0x1000)."""
    seed = 2000 + P + 31 * f + E
    _, Ratt = _rounds(oracle, P, f)
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=permille, rounds_per_attempt=Ratt, protected=f + 1)
    x = _payload(w, seed, S, P, E, dtype)
    plan = ft.Plan(P, f, E, dtype, op, 0x1000)
    compare_allreduce(ft, oracle, plan, x, fr, fo)


def _fused_cases(ft, cases):
    return [c for c in cases if ft.Plan(c[0], c[1], c[2], c[3], c[4]).info.fused]


def test_sweeps_without_the_fused_kernel(ft, oracle, w):
    """The sweep cases whose default plan folds a whole scenario in one workgroup, with that switched off
    (flag 0x10000): the register kernel of the deepest tier and the LDS-tile kernels above it in launches of
    their own, allreduce and reduce with a root per scenario."""
    cases = _fused_cases(ft, ALLREDUCE_CASES)
    assert len(cases) >= 8
    for P, f, E, dtype, op, S, permille in cases:
        seed = 2000 + P + 31 * f + E
        Rred, Ratt = _rounds(oracle, P, f)
        plan = ft.Plan(P, f, E, dtype, op, 0x10000)
        assert plan.info.fused == 0 and plan.info.deep_kernel == 1
        x = _payload(w, seed, S, P, E, dtype)
        fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=permille, rounds_per_attempt=Ratt, protected=f + 1)
        compare_allreduce(ft, oracle, plan, x, fr, fo)
        fr, fo = w.random_failure_sets(seed + 1, S, P, f, inop_permille=permille, rounds_per_attempt=Rred + 1)
        compare_reduce(ft, oracle, plan, x, fr, fo, root=w.random_roots(seed, S, P))


@pytest.mark.parametrize("P,f,E,dtype,op,S", [(1024, 3, 4096, 2, 0, 6), (300, 1, 8192, 0, 0, 4), (64, 2, 3000, 1, 1, 8),
                                              (5000, 4, 1000, 2, 0, 3)])
def test_large_payloads(ft, oracle, w, P, f, E, dtype, op, S):
    """Kilobytes per process (the bandwidth regime): a row no longer fits the LDS tiles.  Where the tree is deep
    enough one workgroup folds a whole scenario, block of value indices by block (no tiers of LDS tiles at all);
    else the plan runs the tree phase on the plain per-depth kernels.  The validation holds up to 8192 values per
    process in LDS."""
    seed = 31000 + P + E
    plan = ft.Plan(P, f, E, dtype, op)
    assert plan.info.shape == 2
    assert (plan.info.tiers, plan.info.fused) == ((0, 0) if P == 64 else (1, 1))
    Rred, Ratt = plan.info.rounds_reduce, plan.info.rounds_attempt
    x = _payload(w, seed, S, P, E, dtype)
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=Rred + 1)
    root = w.random_roots(seed, S, P)
    g, _ = compare_reduce(ft, oracle, plan, x, fr, fo, root=root)
    xd, frd, fod, rd = to_dev(x), to_dev(fr), to_dev(fo), to_dev(root.astype(np.uint32))
    v = ft.validate(plan, 0, S, xd, frd, fod, g["result"], g["status"], root=rd, msgs=g["msgs"])
    assert v["n_invalid"] == 0
    fr, fo = w.random_failure_sets(seed + 1, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1)
    fr[0], fo[0] = w.NO_RANK, 0
    fr[0, 0], fo[0, 0] = 0, 0                            # a second attempt
    g, _ = compare_allreduce(ft, oracle, plan, x, fr, fo)
    frd, fod = to_dev(fr), to_dev(fo)
    v = ft.validate(plan, 1, S, xd, frd, fod, g["result"], g["status"], has_bitmap=g["has_bitmap"],
                    per_process_out=g["per_process_out"], attempts=g["attempts"], msgs=g["msgs"])
    assert v["n_invalid"] == 0
    # and a wrong value is still found among that many
    bad = g["result"].cpu().numpy().copy()
    bad[S - 1, E - 1] = bad[S - 1, E - 1] + 1 if op == 0 else ~bad[S - 1, E - 1]
    v = ft.validate(plan, 1, S, xd, frd, fod, to_dev(bad), g["status"], attempts=g["attempts"])
    assert v["n_invalid"] == 1 and v["verdict"].cpu().numpy()[S - 1] & ft.BAD_VALUE


@pytest.mark.parametrize("P,f,E,dtype", [(5000, 2, 4, 0), (16384, 4, 8, 2), (64, 2, 8, 1), (3000, 3, 48, 2), (1 << 16, 8, 1, 0)])
def test_many_failed_roots(ft, oracle, w, P, f, E, dtype):
    """More attempts with a failed root than ride along in the launches of the tree phase (64): the first 64 are
    simulated as extra scenarios, the messages of the others are counted from the failure lists; every counter
    must equal the oracle's, which simulates them all."""
    S, seed = 150, 41000 + P
    plan = ft.Plan(P, f, E, dtype, ft.SUM)
    Ratt = plan.info.rounds_attempt
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=600, rounds_per_attempt=Ratt, protected=f + 1)
    for s in range(0, S, 3):                             # root 0 failed: a second attempt
        if 0 not in fr[s].tolist():
            fr[s, 0], fo[s, 0] = 0, 0
    for s in range(0, S, 6):                             # roots 0 and 1 failed: a third one
        fr[s, :2], fo[s, :2] = [0, 1], [0, 0]
    x = _payload(w, seed, S, P, E, dtype)
    g, o = compare_allreduce(ft, oracle, plan, x, fr, fo, check_out=P <= 20000)
    assert int((o["attempts"].astype(np.int64) - 1).sum()) > 64


@pytest.mark.parametrize("P,f,E,dtype,op", [(3000, 3, 48, 2, 0), (16384, 4, 32, 2, 0), (2500, 1, 100, 0, 1), (40000, 2, 24, 1, 0)])
def test_medium_payloads_take_the_register_kernels(ft, oracle, w, P, f, E, dtype, op):
    """A few hundred bytes per process: a subtree of the register tier no longer fits the LDS tile of the kernel
    that runs the listed subtrees when the lists of failed processes are asked for, so such runs take a second
    plan on LDS tiles throughout; the plain runs keep the register kernels."""
    S, seed = 12, 43000 + P + E
    plan = ft.Plan(P, f, E, dtype, op)
    assert plan.info.deep_kernel == 1
    Rred, Ratt = plan.info.rounds_reduce, plan.info.rounds_attempt
    x = _payload(w, seed, S, P, E, dtype)
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=Rred + 1)
    root = w.random_roots(seed, S, P)
    g, o = compare_reduce(ft, oracle, plan, x, fr, fo, root=root)
    gi = ft.run_reduce_info(plan, S, to_dev(x), to_dev(fr), to_dev(fo), root=to_dev(root.astype(np.uint32)))
    for k in ("result", "status", "msgs"):
        assert np.array_equal(gi[k].cpu().numpy(), g[k].cpu().numpy()), k
    oi = oracle.reduce_info_batch(P, f, x, dtype, op, S, root=root, fail_rank=fr, fail_round=fo)
    assert np.array_equal(gi["info_count"].cpu().numpy(), oi["info_count"])
    fr, fo = w.random_failure_sets(seed + 1, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1)
    fr[0], fo[0] = w.NO_RANK, 0
    fr[0, 0], fo[0, 0] = 0, 0
    compare_allreduce(ft, oracle, plan, x, fr, fo)


def test_two_streams_with_their_own_workspaces_do_not_disturb_each_other(ft, oracle, w):
    """Two plans run side by side on two streams (default priority), each with its own workspace and output
    buffers, several calls each: the library keeps no device state of its own between or across calls."""
    shapes = [(3000, 3, 5, 2, 0), (2500, 8, 1, 0, 0)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    S = 48
    jobs = []
    for (P, f, E, dtype, op), st in zip(shapes, streams):
        seed = 8800 + P
        _, Ratt = _rounds(oracle, P, f)
        fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1)
        fr[1, 0], fo[1, 0] = 0, 0
        x = _payload(w, seed, S, P, E, dtype)
        plan = ft.Plan(P, f, E, dtype, op)
        jobs.append(dict(plan=plan, x=x, fr=fr, fo=fo, st=st, xd=to_dev(x), frd=to_dev(fr), fod=to_dev(fo),
                         ws=plan.workspace(S), bufs=None))
    torch.cuda.synchronize()
    for _ in range(3):
        for j in jobs:
            with torch.cuda.stream(j["st"]):
                j["bufs"] = ft.run_allreduce(j["plan"], S, j["xd"], j["frd"], j["fod"], workspace=j["ws"],
                                             buffers=j["bufs"], stream=j["st"])
    torch.cuda.synchronize()
    for j in jobs:
        plan, g = j["plan"], j["bufs"]
        o = oracle.allreduce_batch(plan.P, plan.f, j["x"], plan.dtype, plan.op, S, fail_rank=j["fr"],
                                   fail_round=j["fo"], want_has=True, want_out=True)
        assert np.array_equal(g["status"].cpu().numpy(), o["status"])
        assert np.array_equal(g["attempts"].cpu().numpy(), o["attempts"])
        assert np.array_equal(g["result"].cpu().numpy(), o["result"])
        assert np.array_equal(g["msgs"].cpu().numpy(), o["msgs"])
        assert np.array_equal(unpack_bitmap(g["has_bitmap"].cpu().numpy(), plan.P), o["has"])
        assert np.array_equal(g["per_process_out"].cpu().numpy(), o["out"])


def test_runs_are_deterministic(ft, oracle, w):
    P, f, E, S = 4099, 4, 8, 64
    _, Ratt = _rounds(oracle, P, f)
    fr, fo = w.random_failure_sets(9, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1)
    x = to_dev(w.payload_normal(9, S, P, E))
    plan = ft.Plan(P, f, E, ft.F64, ft.SUM)
    a = ft.run_allreduce(plan, S, x, to_dev(fr), to_dev(fo))
    b = ft.run_allreduce(plan, S, x, to_dev(fr), to_dev(fo))
    torch.cuda.synchronize()
    for k in ("result", "per_process_out", "has_bitmap", "status", "attempts", "msgs"):
        assert torch.equal(a[k].view(torch.uint8), b[k].view(torch.uint8)), k


def test_argument_errors(ft, w):
    P, f, E, S = 100, 2, 4, 8
    plan = ft.Plan(P, f, E, ft.I64, ft.SUM)
    x = to_dev(w.payload_int(1, S, P, E, "i64", 20))
    fr, fo = w.random_failure_sets(1, S, P, f)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(ft.FtredError) as ei:
        ft.run_reduce(plan, S, x, to_dev(fr), to_dev(fo), workspace=small)
    assert ei.value.code == ft.EINVAL and "workspace" in str(ei.value)
    with pytest.raises(ft.FtredError):
        ft.run_allreduce(plan, S, x, to_dev(fr), to_dev(fo), workspace=small)
