"""CPU oracle for the correction-based fault-tolerant reduce / allreduce.

TEST INFRASTRUCTURE ONLY.  This package wraps ``ftred_oracle.c`` (a literal,
slow simulation with per-process message queues) and ``definition.py`` (the
plain definition of a valid result).  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the GPU library never does, and the
two share no code.

numpy in, numpy out; every array is indexed by PHYSICAL rank.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .definition import survivor_reduce, valid_results, is_valid_result  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ftred_oracle.c")
_LIB = os.path.join(_HERE, "libftred_oracle.so")

NO_RANK = 0xFFFFFFFF
I64, U32, F64 = 0, 1, 2
SUM, BOR = 0, 1
ST_OK, ST_ROOT_FAILED, ST_NO_CLEAN_SUBTREE, ST_BAD_FAILURE_SET, ST_INCONSISTENT, ST_NO_LIVE_ROOT = range(6)

_NP_DTYPE = {I64: np.int64, U32: np.uint32, F64: np.float64}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (a second or two).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-ffp-contract=off", _SRC, "-o", _LIB]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _fail_arrays(fail_rank, fail_round):
    fr = np.ascontiguousarray(np.asarray(fail_rank, dtype=np.uint32).reshape(-1))
    fo = np.ascontiguousarray(np.asarray(fail_round, dtype=np.uint32).reshape(-1))
    assert fr.shape == fo.shape
    if fr.size == 0:            # keep the pointers valid
        fr = np.full(1, NO_RANK, dtype=np.uint32)
        fo = np.zeros(1, dtype=np.uint32)
        return fr, fo, 0
    return fr, fo, fr.size


BINARY, BINOMIAL = 2, 1        # tree shapes inside a subtree of the root: k >= 2 = k children per process, 1 = binomial


def structure(P: int, f: int, root: int = 0, shape: int = BINARY) -> dict:
    """Tree and group structure (see ``oracle_structure_shape`` in the C file)."""
    lib = _load()
    out = dict(
        parent=np.zeros(P, np.int64), subtree=np.zeros(P, np.uint32), group=np.zeros(P, np.int64),
        gpos=np.zeros(P, np.uint32), gsize=np.zeros(P, np.uint32), height=np.zeros(P, np.uint32),
        depth=np.zeros(P, np.uint32), send_round=np.zeros(P, np.uint32))
    D = ctypes.c_uint32(0)
    rc = lib.oracle_structure_shape(ctypes.c_uint32(P), ctypes.c_uint32(f), ctypes.c_uint32(root), ctypes.c_int(shape),
                              _p(out["parent"]), _p(out["subtree"]), _p(out["group"]), _p(out["gpos"]),
                              _p(out["gsize"]), _p(out["height"]), _p(out["depth"]),
                              _p(out["send_round"]), ctypes.byref(D))
    if rc != 0:
        raise ValueError("oracle_structure: invalid arguments")
    out["D"] = int(D.value)
    return out


def reduce(P, f, payload, dtype, op, root=0, fail_rank=(), fail_round=(), disable_uc=False, trace=False,
           shape=BINARY):
    """One reduce; payload[P][elems].  Returns a dict (result, status, msgs, rounds, detected, traces)."""
    lib = _load()
    npdt = _NP_DTYPE[dtype]
    x = np.ascontiguousarray(np.asarray(payload, dtype=npdt).reshape(P, -1))
    elems = x.shape[1]
    fr, fo, nfail = _fail_arrays(fail_rank, fail_round)
    result = np.zeros(elems, npdt)
    status = ctypes.c_uint32(0)
    rounds = ctypes.c_uint32(0)
    msgs = np.zeros(2, np.uint64)
    v = np.zeros((P, elems), npdt) if trace else None
    sent = np.zeros(P, np.uint8) if trace else None
    flag = np.zeros(P, np.uint8) if trace else None
    tmsg = np.zeros((P, elems), npdt) if trace else None
    det = ctypes.c_uint32(0)
    rc = lib.oracle_reduce_shape(ctypes.c_uint32(P), ctypes.c_uint32(f), ctypes.c_uint32(elems),
                                 ctypes.c_int(dtype), ctypes.c_int(op), ctypes.c_int(int(disable_uc)), ctypes.c_int(shape),
                                 ctypes.c_uint32(root), _p(x), ctypes.c_uint32(nfail), _p(fr), _p(fo),
                                 _p(result), ctypes.byref(status), _p(msgs), ctypes.byref(rounds), ctypes.byref(det),
                                 _p(v), _p(sent), _p(flag), _p(tmsg))
    if rc != 0:
        raise ValueError("oracle_reduce_shape: invalid arguments")
    return dict(result=result, status=int(status.value), msgs=msgs, rounds=int(rounds.value), detected=int(det.value),
                v_after_uc=v, tree_sent=sent, tree_flag=flag, tree_msg=tmsg)


def allreduce(P, f, payload, dtype, op, fail_rank=(), fail_round=(), want_out=True):
    """One allreduce; payload[P][elems].  Returns a dict."""
    lib = _load()
    npdt = _NP_DTYPE[dtype]
    x = np.ascontiguousarray(np.asarray(payload, dtype=npdt).reshape(P, -1))
    elems = x.shape[1]
    fr, fo, nfail = _fail_arrays(fail_rank, fail_round)
    result = np.zeros(elems, npdt)
    status = ctypes.c_uint32(0)
    attempts = ctypes.c_uint32(0)
    rounds = ctypes.c_uint32(0)
    msgs = np.zeros(4, np.uint64)
    has = np.zeros(P, np.uint8)
    out = np.zeros((P, elems), npdt) if want_out else None
    rc = lib.oracle_allreduce(ctypes.c_uint32(P), ctypes.c_uint32(f), ctypes.c_uint32(elems),
                              ctypes.c_int(dtype), ctypes.c_int(op), _p(x),
                              ctypes.c_uint32(nfail), _p(fr), _p(fo),
                              _p(result), ctypes.byref(status), ctypes.byref(attempts), _p(msgs),
                              ctypes.byref(rounds), _p(has), _p(out))
    if rc != 0:
        raise ValueError("oracle_allreduce: invalid arguments")
    return dict(result=result, status=int(status.value), attempts=int(attempts.value), msgs=msgs,
                rounds=int(rounds.value), has=has, out=out)


def _batch_common(P, payload, dtype, S, fail_rank, fail_round):
    npdt = _NP_DTYPE[dtype]
    x = np.ascontiguousarray(np.asarray(payload, dtype=npdt))
    if x.ndim == 2:                     # one payload shared by all scenarios
        assert x.shape[0] == P
        stride = 0
        elems = x.shape[1]
    else:
        assert x.shape[0] == S and x.shape[1] == P
        elems = x.shape[2]
        stride = P * elems * x.itemsize
    fr = np.ascontiguousarray(np.asarray(fail_rank, dtype=np.uint32).reshape(S, -1))
    fo = np.ascontiguousarray(np.asarray(fail_round, dtype=np.uint32).reshape(S, -1))
    assert fr.shape == fo.shape
    nfail = fr.shape[1]
    if nfail == 0:
        fr = np.full((S, 1), NO_RANK, np.uint32)
        fo = np.zeros((S, 1), np.uint32)
        nfail = 1
    return npdt, x, elems, stride, fr, fo, nfail


def latency_steps(P: int, f: int, shape: int = BINARY) -> dict:
    """Message steps of one failure-free attempt (one port per process): per kind of message the sum over its
    rounds of the messages the busiest process sends or receives in the round."""
    lib = _load()
    st = np.zeros(4, np.uint32)
    if lib.oracle_latency_steps(ctypes.c_uint32(P), ctypes.c_uint32(f), ctypes.c_int(shape), _p(st)) != 0:
        raise ValueError("oracle_latency_steps: invalid arguments")
    return dict(uc=int(st[0]), tree=int(st[1]), bcast_tree=int(st[2]), bcast_corr=int(st[3]))


def reduce_batch(P, f, payload, dtype, op, S, root=None, fail_rank=(), fail_round=(), threads=0, shape=BINARY,
                 want_detected=False):
    """S independent reduces; payload[S][P][elems] or [P][elems] (shared).  shape: the tree inside a subtree of
    the root; want_detected: also `detected`[S], bit q = the process in slot q of the failure list was detected."""
    lib = _load()
    npdt, x, elems, stride, fr, fo, nfail = _batch_common(P, payload, dtype, S, fail_rank, fail_round)
    rt = None if root is None else np.ascontiguousarray(np.asarray(root, dtype=np.uint32).reshape(S))
    result = np.zeros((S, elems), npdt)
    status = np.zeros(S, np.uint32)
    msgs = np.zeros((S, 2), np.uint64)
    det = np.zeros(S, np.uint32) if want_detected else None
    used = lib.oracle_reduce_shape_batch(ctypes.c_uint32(P), ctypes.c_uint32(f), ctypes.c_uint32(elems),
                                         ctypes.c_int(dtype), ctypes.c_int(op), ctypes.c_int(shape), ctypes.c_uint32(S),
                                         _p(rt), _p(x), ctypes.c_uint64(stride), ctypes.c_uint32(nfail), _p(fr), _p(fo),
                                         _p(result), _p(status), _p(msgs), _p(det), ctypes.c_int(threads))
    if used < 0:
        raise ValueError("oracle_reduce_shape_batch: invalid arguments")
    return dict(result=result, status=status, msgs=msgs, threads=used, detected=det)


NEVER = 0xFFFFFFFFFFFFFFFF


def reduce_timed_batch(P, f, payload, dtype, op, S, t_msg, t_timeout, root=None, fail_rank=(), fail_round=(), threads=0,
                       shape=BINARY, want_proc=True):
    """S independent reduces with the event-driven times of every process (``oracle_reduce_timed_batch``):
    reduce_batch's outputs plus t_done[S] and t_proc[S][P] (NEVER = did not get there)."""
    lib = _load()
    npdt, x, elems, stride, fr, fo, nfail = _batch_common(P, payload, dtype, S, fail_rank, fail_round)
    rt = None if root is None else np.ascontiguousarray(np.asarray(root, dtype=np.uint32).reshape(S))
    result = np.zeros((S, elems), npdt)
    status = np.zeros(S, np.uint32)
    msgs = np.zeros((S, 2), np.uint64)
    t_done = np.zeros(S, np.uint64)
    t_proc = np.zeros((S, P), np.uint64) if want_proc else None
    used = lib.oracle_reduce_timed_batch(ctypes.c_uint32(P), ctypes.c_uint32(f), ctypes.c_uint32(elems),
                                         ctypes.c_int(dtype), ctypes.c_int(op), ctypes.c_int(shape), ctypes.c_uint32(S),
                                         _p(rt), _p(x), ctypes.c_uint64(stride), ctypes.c_uint32(nfail), _p(fr), _p(fo),
                                         ctypes.c_uint64(t_msg), ctypes.c_uint64(t_timeout),
                                         _p(result), _p(status), _p(msgs), _p(t_done), _p(t_proc), ctypes.c_int(threads))
    if used < 0:
        raise ValueError("oracle_reduce_timed_batch: invalid arguments")
    return dict(result=result, status=status, msgs=msgs, threads=used, t_done=t_done, t_proc=t_proc)


def allreduce_batch(P, f, payload, dtype, op, S, fail_rank=(), fail_round=(), threads=0,
                    want_has=True, want_out=False, shape=BINARY, want_detected=False):
    """S independent allreduces; payload[S][P][elems] or [P][elems] (shared).  shape, want_detected: as reduce_batch."""
    lib = _load()
    npdt, x, elems, stride, fr, fo, nfail = _batch_common(P, payload, dtype, S, fail_rank, fail_round)
    result = np.zeros((S, elems), npdt)
    status = np.zeros(S, np.uint32)
    attempts = np.zeros(S, np.uint32)
    rounds = np.zeros(S, np.uint32)
    msgs = np.zeros((S, 4), np.uint64)
    has = np.zeros((S, P), np.uint8) if want_has else None
    out = np.zeros((S, P, elems), npdt) if want_out else None
    det = np.zeros(S, np.uint32) if want_detected else None
    used = lib.oracle_allreduce_shape_batch(ctypes.c_uint32(P), ctypes.c_uint32(f), ctypes.c_uint32(elems),
                                            ctypes.c_int(dtype), ctypes.c_int(op), ctypes.c_int(shape), ctypes.c_uint32(S),
                                            _p(x), ctypes.c_uint64(stride), ctypes.c_uint32(nfail), _p(fr), _p(fo),
                                            _p(result), _p(status), _p(attempts), _p(msgs), _p(rounds),
                                            _p(has), _p(out), _p(det), ctypes.c_int(threads))
    if used < 0:
        raise ValueError("oracle_allreduce_shape_batch: invalid arguments")
    return dict(result=result, status=status, attempts=attempts, msgs=msgs, rounds=rounds,
                has=has, out=out, threads=used, detected=det)


def _child_info(child, nfail):
    """[S][f+1][3 + nfail] words -> per scenario a list of (state, counter, ids) per child of the root."""
    out = []
    for rows in child:
        one = []
        for row in rows:
            if row[2] == NO_RANK:
                raise AssertionError("a failure list outgrew the number of listed failures")
            one.append((int(row[0]), int(row[1]), [int(q) for q in row[3:3 + int(row[2])]]))
        out.append(one)
    return out


def _info_lists(info_nids, info_ids):
    """[S][nfail] padded id arrays -> list of python lists (order as appended)."""
    out = []
    for n, ids in zip(info_nids, info_ids):
        if n == NO_RANK:
            raise AssertionError("a failure list outgrew the number of listed failures")
        out.append([int(q) for q in ids[:int(n)]])
    return out


def reduce_info_batch(P, f, payload, dtype, op, S, root=None, fail_rank=(), fail_round=(), threads=0):
    """S independent reduces with the first and second failure-information scheme
    tracked (section "Failure information"): info_count[S] = the counter carried by
    the message the root selected, info_ids = its list of failed processes (one
    python list per scenario, physical ranks in the order appended)."""
    lib = _load()
    npdt, x, elems, stride, fr, fo, nfail = _batch_common(P, payload, dtype, S, fail_rank, fail_round)
    rt = None if root is None else np.ascontiguousarray(np.asarray(root, dtype=np.uint32).reshape(S))
    result = np.zeros((S, elems), npdt)
    status = np.zeros(S, np.uint32)
    msgs = np.zeros((S, 2), np.uint64)
    count = np.zeros(S, np.uint32)
    nids = np.zeros(S, np.uint32)
    ids = np.zeros((S, nfail), np.uint32)
    child = np.zeros((S, f + 1, 3 + nfail), np.uint32)
    used = lib.oracle_reduce_info_batch(ctypes.c_uint32(P), ctypes.c_uint32(f), ctypes.c_uint32(elems),
                                        ctypes.c_int(dtype), ctypes.c_int(op), ctypes.c_uint32(S), _p(rt),
                                        _p(x), ctypes.c_uint64(stride), ctypes.c_uint32(nfail), _p(fr), _p(fo),
                                        _p(result), _p(status), _p(msgs), _p(count), _p(nids), _p(ids),
                                        _p(child), ctypes.c_int(threads))
    if used < 0:
        raise ValueError("oracle_reduce_info_batch: invalid arguments")
    return dict(result=result, status=status, msgs=msgs, info_count=count, info_ids=_info_lists(nids, ids),
                info_child=_child_info(child, nfail), threads=used)


def allreduce_info_batch(P, f, payload, dtype, op, S, fail_rank=(), fail_round=(), threads=0):
    """As reduce_info_batch for the allreduce: the failure information of the
    reduce whose result every survivor holds."""
    lib = _load()
    npdt, x, elems, stride, fr, fo, nfail = _batch_common(P, payload, dtype, S, fail_rank, fail_round)
    result = np.zeros((S, elems), npdt)
    status = np.zeros(S, np.uint32)
    attempts = np.zeros(S, np.uint32)
    msgs = np.zeros((S, 4), np.uint64)
    count = np.zeros(S, np.uint32)
    nids = np.zeros(S, np.uint32)
    ids = np.zeros((S, nfail), np.uint32)
    child = np.zeros((S, f + 1, 3 + nfail), np.uint32)
    used = lib.oracle_allreduce_info_batch(ctypes.c_uint32(P), ctypes.c_uint32(f), ctypes.c_uint32(elems),
                                           ctypes.c_int(dtype), ctypes.c_int(op), ctypes.c_uint32(S),
                                           _p(x), ctypes.c_uint64(stride), ctypes.c_uint32(nfail), _p(fr), _p(fo),
                                           _p(result), _p(status), _p(attempts), _p(msgs), _p(count), _p(nids),
                                           _p(ids), _p(child), ctypes.c_int(threads))
    if used < 0:
        raise ValueError("oracle_allreduce_info_batch: invalid arguments")
    return dict(result=result, status=status, attempts=attempts, msgs=msgs, info_count=count,
                info_ids=_info_lists(nids, ids), info_child=_child_info(child, nfail), threads=used)
