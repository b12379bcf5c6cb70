"""Parity with the CPU oracle on shapes at the edges of the tree layout: the number
of rows M (up-correction groups) just below, at and just above powers of two (the
deepest level empty but for one row, full, one row short), the last group full,
one member short or holding a single process, for every group width of the
register kernels of the deepest tier (f + 1 = 2 .. 16; from 10 on the subtrees with
listed processes run on the LDS-tile list kernel), with one and with several values
per process.  Reduce with a root per scenario and allreduce,
failures before and during the operation, some aimed at the last rows."""
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


def _shapes():
    out = []
    widths = [2, 3, 4, 5, 9, 6, 7, 8, 11, 10, 13, 16, 12]
    rows = [31, 32, 33, 47, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1023, 1024, 1025]
    k = 0
    for M in rows:
        for W in widths:
            k += 1
            if (k * 7 + M) % 3 != 0:                # a third of the combinations
                continue
            short = (0, 1, W - 1)[k % 3]            # processes missing from the last group
            P = W * M - short + 1
            E = (1, 1, 2, 3, 8)[(k // 3) % 5]
            dtype = (0, 1, 2)[(k // 2) % 3]
            op = 1 if dtype != 2 and k % 4 == 0 else 0
            out.append((P, W - 1, E, dtype, op))
    return out


SHAPES = _shapes()


def test_the_shapes_cover_all_kernels(ft):
    kinds, fused = {}, {0: set(), 1: set()}
    for P, f, E, dtype, op in SHAPES:
        info = ft.Plan(P, f, E, dtype, op).info
        kinds.setdefault(info.deep_kernel, set()).add(f + 1)
        if info.deep_kernel == 1:
            fused[info.fused].add(f + 1)
    every = {2, 3, 4, 5, 6, 7, 8, 9}
    wide = {10, 11, 12, 13, 16}
    assert kinds[1] >= every | wide and kinds[2] >= every | wide
    assert fused[1] >= every and not (fused[1] & wide)            # the whole scenario in one workgroup
    assert len(SHAPES) >= 40


@pytest.mark.parametrize("P,f,E,dtype,op", SHAPES)
def test_edge_shape(ft, oracle, w, P, f, E, dtype, op):
    S, seed = 10, 7000 + P + 13 * f + E
    D = oracle.structure(P, f, 0)["D"]
    Rred, Ratt = f + D, 2 * (f + D)
    if dtype == 0:
        x = w.payload_int(seed, S, P, E, "i64", 41)
    elif dtype == 1:
        x = w.payload_int(seed, S, P, E, "u32", 32)
    else:
        x = w.payload_normal(seed, S, P, E, threads=2)
    plan = ft.Plan(P, f, E, dtype, op)

    # reduce: a root per scenario; failures aimed at the last processes and the root's neighbours
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=Rred + 1)
    root = w.random_roots(seed, S, P)
    root[0], root[1] = 0, P - 1
    fr[0], fo[0] = w.NO_RANK, 0                      # no failure at all
    fr[2], fo[2] = w.NO_RANK, 0
    fr[2, 0], fo[2, 0] = (P - 1 if root[2] != P - 1 else P - 2), 0          # the last process
    fr[3], fo[3] = w.NO_RANK, 0
    fr[3, 0], fo[3, 0] = (P - 2 if root[3] != P - 2 else P - 3), 1          # in the last or last-but-one group
    compare_reduce(ft, oracle, plan, x, fr, fo, root=root)

    # allreduce: candidates 0..f may fail beforehand only
    fr, fo = w.random_failure_sets(seed + 1, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1)
    fr[0], fo[0] = w.NO_RANK, 0
    fr[1], fo[1] = w.NO_RANK, 0
    fr[1, 0], fo[1, 0] = 0, 0                        # a second attempt
    fr[2], fo[2] = w.NO_RANK, 0
    fr[2, 0], fo[2, 0] = P - 1, 0
    compare_allreduce(ft, oracle, plan, x, fr, fo)
