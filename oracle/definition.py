"""The plain definition of a valid reduce / allreduce result.  TEST INFRASTRUCTURE ONLY.

From the paper's introduction and the two "Semantics" sections: with failures
before the operation only, the result is the reduction over the processes that
did not fail; a process that fails during the operation counts either as alive
or as dead, as a whole, never partly.  So a result is valid iff it equals the
reduction over (never-failed processes) plus ONE subset of the processes that
failed during the operation.

Nothing here simulates the protocol: it is numpy / math.fsum over index sets.
"""
from __future__ import annotations

import itertools
import math

import numpy as np

I64, U32, F64 = 0, 1, 2
SUM, BOR = 0, 1


def survivor_reduce(payload, dtype: int, op: int, excluded=()):
    """Reduction of payload[p] over all p not in `excluded`.  payload[P][elems].

    int64/uint32 SUM wraps (two's complement); F64 SUM is the correctly rounded
    exact sum (math.fsum); BOR is bitwise or.
    """
    x = np.asarray(payload)
    P = x.shape[0]
    keep = np.ones(P, dtype=bool)
    for p in excluded:
        keep[int(p)] = False
    xs = x[keep]
    if op == BOR:
        assert dtype != F64
        acc = np.zeros(x.shape[1], dtype=x.dtype)
        for row in xs:
            acc |= row
        return acc
    if dtype == F64:
        return np.array([math.fsum(xs[:, e].tolist()) for e in range(x.shape[1])], dtype=np.float64)
    if dtype == I64:
        with np.errstate(over="ignore"):
            return xs.astype(np.uint64).sum(axis=0, dtype=np.uint64).astype(np.int64)
    with np.errstate(over="ignore"):
        return xs.astype(np.uint32).sum(axis=0, dtype=np.uint32)


def valid_results(payload, dtype: int, op: int, pre_failed, inop_failed):
    """All results the semantics allow: one per subset of `inop_failed` counted as dead."""
    inop = [int(q) for q in inop_failed]
    out = []
    for r in range(len(inop) + 1):
        for dead in itertools.combinations(inop, r):
            out.append((dead, survivor_reduce(payload, dtype, op, list(pre_failed) + list(dead))))
    return out


def is_valid_result(result, payload, dtype: int, op: int, pre_failed, inop_failed, rtol=1e-12):
    """True iff `result` is one of the valid results (exactly for integers; for
    F64 within rtol * sum_p |x_p| per element, the sum taken over all processes
    that are not failed before the operation)."""
    res = np.asarray(result)
    x = np.asarray(payload)
    if dtype == F64:
        keep = np.ones(x.shape[0], dtype=bool)
        for p in pre_failed:
            keep[int(p)] = False
        scale = np.abs(x[keep]).sum(axis=0)
        tol = rtol * scale
    for _dead, cand in valid_results(x, dtype, op, pre_failed, inop_failed):
        if dtype == F64:
            if np.all(np.abs(res - cand) <= tol):
                return True
        elif np.array_equal(res, cand):
            return True
    return False
