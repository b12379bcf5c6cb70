"""The allreduce and its validation captured into one HIP graph and replayed: the library
enqueues kernels only (no memset, no copy, no allocation, no synchronisation when the
caller brings workspace and outputs), so a step can be captured once and replayed with new
inputs in the same buffers.  Every replay is compared with the eager result on the same
inputs, with eager work and synchronisations between the replays."""
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


KEYS = ("result", "status", "attempts", "msgs", "has_bitmap", "per_process_out")


@pytest.mark.parametrize("P,f,E,dtype,S", [(64, 2, 8, 0, 512), (16384, 4, 8, 2, 96), (1 << 16, 8, 1, 0, 8), (3000, 12, 2, 0, 32),
                                           (40000, 4, 8, 2, 12)])
def test_replays_equal_eager_runs(ft, oracle, w, P, f, E, dtype, S):
    plan = ft.Plan(P, f, E, dtype, ft.SUM)
    Ratt = plan.info.rounds_attempt
    x = w.payload_int(5, S, P, E, "i64", 41) if dtype == 0 else w.payload_normal(5, S, P, E, threads=4)
    xd = to_dev(x)
    sets = [w.random_failure_sets(600 + k, S, P, f, inop_permille=500, rounds_per_attempt=Ratt, protected=f + 1) for k in range(4)]
    frd, fod = to_dev(sets[0][0]), to_dev(sets[0][1])
    ws = plan.workspace(S)
    verdict = torch.empty(S, dtype=torch.uint32, device="cuda")
    bufs = ft.run_allreduce(plan, S, xd, frd, fod, workspace=ws)          # allocates the outputs once
    torch.cuda.synchronize()

    def step():
        b = ft.run_allreduce(plan, S, xd, frd, fod, workspace=ws, buffers=bufs)
        ft.validate(plan, 1, S, xd, frd, fod, b["result"], b["status"], has_bitmap=b["has_bitmap"],
                    per_process_out=b["per_process_out"], attempts=b["attempts"], msgs=b["msgs"], workspace=ws,
                    count=False, verdict=verdict)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for k in (1, 2, 3, 0, 2):
        fr, fo = sets[k]
        frd.copy_(torch.from_numpy(fr))
        fod.copy_(torch.from_numpy(fo))
        for t in bufs.values():                          # stale outputs must not pass for fresh ones
            t.view(torch.uint8).fill_(0xA5)
        graph.replay()
        torch.cuda.synchronize()
        got = {key: bufs[key].clone() for key in KEYS}
        got_verdict = verdict.clone()
        # the same inputs through the eager path, into buffers of its own
        eager = ft.run_allreduce(plan, S, xd, frd, fod, workspace=plan.workspace(S))
        torch.cuda.synchronize()
        for key in KEYS:
            assert torch.equal(got[key].view(torch.uint8), eager[key].view(torch.uint8)), (k, key)
        assert int((got_verdict != 0).sum()) == 0
    # and the last replay against the oracle
    o = oracle.allreduce_batch(P, f, x, dtype, oracle.SUM, S, fail_rank=sets[2][0], fail_round=sets[2][1], want_has=False)
    assert np.array_equal(got["result"].cpu().numpy(), o["result"]) and np.array_equal(got["msgs"].cpu().numpy(), o["msgs"])
