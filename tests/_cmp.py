"""Helpers of the GPU parity tests: run the oracle and the HIP library on the same
seeded inputs and compare element by element."""
import numpy as np
import torch

NP_DTYPE = {0: np.int64, 1: np.uint32, 2: np.float64}


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def unpack_bitmap(bm, P):
    """[S][ceil(P/32)] uint32 -> [S][P] uint8 (bit p%32 of word p/32)."""
    b = np.ascontiguousarray(bm).view(np.uint8)
    bits = np.unpackbits(b, axis=1, bitorder="little")
    return bits[:, :P]


def f64_tol(x):
    """Tolerance of the floating-point contract: 1e-12 * sum_p |x_p| per scenario and element."""
    x = np.asarray(x)
    if x.ndim == 2:
        return 1e-12 * np.abs(x).sum(axis=0)[None, :]
    return 1e-12 * np.abs(x).sum(axis=1)


def assert_values(got, want, dtype, x, what, exact_fp=True):
    if dtype == 2:
        assert np.all(np.abs(got - want) <= f64_tol(x)), what + ": outside 1e-12 * sum|x|"
        if exact_fp:
            # both sides fold in the same order, so the sums agree to the last bit
            assert np.array_equal(got, want), what + ": not bit-identical"
    else:
        assert np.array_equal(got, want), what


def compare_reduce(ft, oracle, plan, x, fr, fo, root=None, threads=0, exact_fp=True, shape=2):
    S = fr.shape[0]
    xd = to_dev(x)
    rd = None if root is None else to_dev(root.astype(np.uint32))
    g = ft.run_reduce(plan, S, xd, to_dev(fr), to_dev(fo), root=rd)
    torch.cuda.synchronize()
    o = oracle.reduce_batch(plan.P, plan.f, x, plan.dtype, plan.op, S, root=root, fail_rank=fr, fail_round=fo,
                            threads=threads, shape=shape)
    st = g["status"].cpu().numpy()
    assert np.array_equal(st, o["status"]), "status: %s" % np.nonzero(st != o["status"])[0][:10]
    assert_values(g["result"].cpu().numpy(), o["result"], plan.dtype, x, "result", exact_fp)
    assert np.array_equal(g["msgs"].cpu().numpy(), o["msgs"]), "message counters"
    return g, o


def compare_allreduce(ft, oracle, plan, x, fr, fo, threads=0, exact_fp=True, check_out=True, shape=2):
    S = fr.shape[0]
    xd = to_dev(x)
    g = ft.run_allreduce(plan, S, xd, to_dev(fr), to_dev(fo))
    torch.cuda.synchronize()
    o = oracle.allreduce_batch(plan.P, plan.f, x, plan.dtype, plan.op, S, fail_rank=fr, fail_round=fo,
                               threads=threads, want_has=True, want_out=check_out, shape=shape)
    st = g["status"].cpu().numpy()
    assert np.array_equal(st, o["status"]), "status: %s" % np.nonzero(st != o["status"])[0][:10]
    assert np.array_equal(g["attempts"].cpu().numpy(), o["attempts"]), "attempts"
    assert_values(g["result"].cpu().numpy(), o["result"], plan.dtype, x, "result", exact_fp)
    gm, om = g["msgs"].cpu().numpy(), o["msgs"]
    assert np.array_equal(gm, om), "message counters: %s" % np.nonzero((gm != om).any(axis=1))[0][:10]
    has = unpack_bitmap(g["has_bitmap"].cpu().numpy(), plan.P)
    assert np.array_equal(has, o["has"]), "holders: scenarios %s" % np.nonzero((has != o["has"]).any(axis=1))[0][:10]
    if check_out:
        go = g["per_process_out"].cpu().numpy()
        if plan.dtype == 2 and not exact_fp:
            assert np.all(np.abs(go - o["out"]) <= f64_tol(x)[:, None, :])
        else:
            assert np.array_equal(go, o["out"]), "receive buffers"
    return g, o
