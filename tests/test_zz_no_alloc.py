"""ftred_run_allreduce_noalloc (the entry point for callers that cannot allocate device
memory: its workspace is a fixed array inside the library) against ftred_run_allreduce on
the same inputs: every output must be bit-identical.  Two calls in a row share the array,
the second with a smaller input, so what the first call left behind must not matter."""
import numpy as np
import pytest
import torch

from _cmp import to_dev

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


def _buffers(ft, plan, S):
    # filled with a pattern: whatever the call does not write would show up in the comparison
    npdt = {ft.I64: np.int64, ft.U32: np.uint32, ft.F64: np.float64}[plan.dtype]
    return dict(result=to_dev(np.full((S, plan.elems), 77, dtype=npdt)),
                has_bitmap=to_dev(np.full((S, (plan.P + 31) // 32), 0x5A5A5A5A, dtype=np.uint32)),
                per_process_out=to_dev(np.full((S, plan.P, plan.elems), 77, dtype=npdt)),
                status=to_dev(np.full(S, 9, dtype=np.uint32)),
                attempts=to_dev(np.full(S, 9, dtype=np.uint32)),
                msgs=to_dev(np.full((S, 4), 9, dtype=np.uint64)))


def _case(ft, w, P, f, E, dtype, S, seed):
    plan = ft.Plan(P, f, E, dtype, ft.SUM)
    assert plan.workspace_bytes(S) <= ft.NOALLOC_WORKSPACE_BYTES
    Ratt = plan.info.rounds_attempt
    fr, fo = w.random_failure_sets(seed, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1)
    fr[0], fo[0] = w.NO_RANK, 0
    fr[0, 0], fo[0, 0] = 0, 0                          # a scenario that needs a second root
    if dtype == ft.F64:
        x = w.payload_normal(seed, S, P, E, threads=1)
    else:
        x = w.payload_int(seed, S, P, E, "i64", 32)
    return plan, to_dev(x), to_dev(fr), to_dev(fo)


def _same(a, b):
    for k in ("result", "has_bitmap", "per_process_out", "status", "attempts", "msgs"):
        ga, gb = a[k].cpu().numpy(), b[k].cpu().numpy()
        assert np.array_equal(ga.view(np.uint8), gb.view(np.uint8)), k


def test_noalloc_equals_run_allreduce_twice_in_a_row(ft, w):
    # first call: a deep tree (register kernels, two tiers above them), 8 x fp64
    plan1, x1, fr1, fo1 = _case(ft, w, 16384, 4, 8, ft.F64, 96, 21)
    # second call: smaller in every respect (fewer scenarios, fewer processes, one tier)
    plan2, x2, fr2, fo2 = _case(ft, w, 200, 2, 3, ft.I64, 17, 22)
    want1 = ft.run_allreduce(plan1, 96, x1, fr1, fo1)
    want2 = ft.run_allreduce(plan2, 17, x2, fr2, fo2)
    torch.cuda.synchronize()
    got1 = ft.run_allreduce_noalloc(plan1, 96, x1, fr1, fo1, _buffers(ft, plan1, 96))
    got2 = ft.run_allreduce_noalloc(plan2, 17, x2, fr2, fo2, _buffers(ft, plan2, 17))
    torch.cuda.synchronize()
    _same(got1, want1)
    _same(got2, want2)
    assert want1["attempts"].cpu().numpy()[0] == 2 and want2["attempts"].cpu().numpy()[0] == 2
    # and once more the larger one, after the smaller one has used the array
    got3 = ft.run_allreduce_noalloc(plan1, 96, x1, fr1, fo1, _buffers(ft, plan1, 96))
    torch.cuda.synchronize()
    _same(got3, want1)


def test_noalloc_on_the_other_deep_paths(ft, w):
    """One value per process (eight lanes per subtree, three more levels folded by the same wavefront) and a tree
    that one workgroup folds in parts: the same array, one call after the other."""
    plan1, x1, fr1, fo1 = _case(ft, w, 65536, 8, 1, ft.I64, 8, 24)
    plan2, x2, fr2, fo2 = _case(ft, w, 40000, 4, 8, ft.F64, 3, 25)
    assert plan1.info.deep_kernel == 2 and plan2.info.fused == 1 and plan2.info.tiers == 2
    want1 = ft.run_allreduce(plan1, 8, x1, fr1, fo1)
    want2 = ft.run_allreduce(plan2, 3, x2, fr2, fo2)
    torch.cuda.synchronize()
    got1 = ft.run_allreduce_noalloc(plan1, 8, x1, fr1, fo1, _buffers(ft, plan1, 8))
    got2 = ft.run_allreduce_noalloc(plan2, 3, x2, fr2, fo2, _buffers(ft, plan2, 3))
    torch.cuda.synchronize()
    _same(got1, want1)
    _same(got2, want2)


def test_noalloc_rejects_what_does_not_fit(ft, w):
    plan, x, fr, fo = _case(ft, w, 16384, 4, 8, ft.F64, 4, 23)
    S = 4096
    assert plan.workspace_bytes(S) > ft.NOALLOC_WORKSPACE_BYTES
    bufs = _buffers(ft, plan, 4)
    # the size check comes before anything is read or enqueued: the small tensors are never touched
    rc = ft.lib().ftred_run_allreduce_noalloc(plan.handle, S, x.data_ptr(), plan.P * plan.elems, fr.data_ptr(),
                                              fo.data_ptr(), bufs["result"].data_ptr(), None, None,
                                              bufs["status"].data_ptr(), bufs["attempts"].data_ptr(), None, None)
    assert rc == ft.EUNSUPPORTED
    assert "workspace" in ft.lib().ftred_last_error().decode()
    torch.cuda.synchronize()
    assert bufs["status"].cpu().numpy()[0] == 9                 # untouched
