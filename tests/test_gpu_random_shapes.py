"""Seeded random shapes (processes, failure bound, values per process, type,
operator, plan flags): the HIP library against the CPU oracle, reduce with a root
per scenario and allreduce, failures before and during the operation.  The sweeps
elsewhere pick their shapes by hand; this one is there for the shapes nobody
thought of."""
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


def _cases(n, seed0):
    rng = np.random.default_rng(seed0)
    out = []
    for _ in range(n):
        f = int(rng.choice([0, 1, 1, 2, 2, 3, 3, 4, 4, 5, 7, 8, 8, 12, 15]))
        P = int(rng.integers(f + 2, 12000)) if rng.random() < 0.8 else int(rng.integers(f + 2, 60))
        E = int(rng.choice([1, 1, 1, 2, 3, 5, 8, 8, 16, 33, 70]))
        dtype = int(rng.integers(0, 3))
        op = int(rng.integers(0, 2)) if dtype != 2 else 0
        S = int(rng.integers(4, 16))
        seed = int(rng.integers(1, 1 << 30))
        flags = int(rng.choice([0, 0, 0, 0x4000, 0x6000, 0x1000, 0x200]))
        out.append((P, f, E, dtype, op, S, seed, flags))
    return out


CASES = _cases(48, 20260222)


@pytest.mark.parametrize("P,f,E,dtype,op,S,seed,flags", CASES)
def test_random_shape(ft, oracle, w, P, f, E, dtype, op, S, seed, flags):
    plan = ft.Plan(P, f, E, dtype, op, flags)
    D = oracle.structure(P, f, 0)["D"]
    if dtype == 0:
        x = w.payload_int(seed, S, P, E, "i64", 41)
    elif dtype == 1:
        x = w.payload_int(seed, S, P, E, "u32", 32)
    else:
        x = w.payload_normal(seed, S, P, E, threads=2)
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=f + D + 1)
    root = w.random_roots(seed, S, P)
    root[0] = 0
    compare_reduce(ft, oracle, plan, x, fr, fo, root=root)
    fr, fo = w.random_failure_sets(seed + 1, S, P, f, inop_permille=500, rounds_per_attempt=2 * (f + D),
                                   protected=f + 1)
    if f >= 1:
        fr[1, 0], fo[1, 0] = 0, 0                    # a second attempt
    compare_allreduce(ft, oracle, plan, x, fr, fo)
