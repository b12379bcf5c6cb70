"""Thin ctypes binding of libftred.so (C-ABI declared in include/ftred.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch is used for device memory (tensors) and the current stream.
There is no CPU fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch  # imported first so that the library binds to the HIP runtime torch loaded

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libftred.so")

OK, EINVAL, ENOMEM, EDEVICE, EUNSUPPORTED = range(5)
I64, U32, F64 = 0, 1, 2
SUM, BOR = 0, 1
SHAPE_BINARY, SHAPE_BINOMIAL = 2, 1
ST_OK, ST_ROOT_FAILED, ST_NO_CLEAN_SUBTREE, ST_BAD_FAILURE_SET = range(4)
BAD_VALUE, BAD_HOLDER, BAD_STATUS, BAD_COUNT = 1, 2, 4, 8
NO_RANK = 0xFFFFFFFF
MAX_F = 15

TORCH_DTYPE = {I64: torch.int64, U32: torch.uint32, F64: torch.float64}
ELEM_SIZE = {I64: 8, U32: 4, F64: 8}


class FtredError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("ftred error %d: %s" % (code, msg))
        self.code = code


class Info(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in
                ("P", "f", "elems", "dtype", "op", "groups_full", "a", "D", "rounds_reduce", "rounds_attempt",
                 "tiers", "deep_kernel")] + \
               [(n, ctypes.c_uint64) for n in
                ("msgs_uc_ff", "msgs_tree_ff", "msgs_bcast_tree_ff", "msgs_bcast_corr_ff")] + \
               [(n, ctypes.c_uint32) for n in ("fused", "shape", "steps_uc", "steps_tree", "steps_bcast_tree",
                                               "steps_bcast_corr", "reserved")]


class Partners(ctypes.Structure):
    _fields_ = [("parent", ctypes.c_uint32), ("n_children", ctypes.c_uint32),
                ("children", ctypes.c_uint32 * 32),
                ("group_size", ctypes.c_uint32), ("group_pos", ctypes.c_uint32),
                ("group", ctypes.c_uint32 * (MAX_F + 1)),
                ("subtree", ctypes.c_uint32), ("depth", ctypes.c_uint32), ("height", ctypes.c_uint32),
                ("send_round", ctypes.c_uint32)]


_lib = None
_vp, _u32, _u64, _int = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int


def lib():
    """The loaded library.  Raises if it is missing: build it with
    `python -m paper_2602_22445_amd.build`."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libftred.so is not built (%s); run `python -m paper_2602_22445_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        # a library built from other sources than those beside it would test or time code that is not there
        from . import build
        try:
            L.ftred_source_hash.restype = ctypes.c_char_p
            have = L.ftred_source_hash().decode()
        except AttributeError:
            have = None
        if have != build.source_hash():
            raise RuntimeError("libftred.so is stale: it was not built from the sources in %s; run "
                               "`python -m paper_2602_22445_amd.build`" % os.path.join(HERE, "csrc"))
        L.ftred_plan.argtypes = [ctypes.POINTER(_vp), _u32, _u32, _u32, _int, _int, _u32]
        L.ftred_plan_info.argtypes = [_vp, ctypes.POINTER(Info)]
        L.ftred_plan_destroy.argtypes = [_vp]
        L.ftred_plan_destroy.restype = None
        L.ftred_last_error.restype = ctypes.c_char_p
        L.ftred_workspace_bytes.argtypes = [_vp, _u32]
        L.ftred_workspace_bytes.restype = _u64
        L.ftred_partners.argtypes = [_vp, _u32, _u32, ctypes.POINTER(Partners)]
        L.ftred_structure.argtypes = [_vp, _u32] + [_vp] * 8
        L.ftred_run_reduce.argtypes = [_vp, _u32, _vp, _vp, _u64, _vp, _vp, _vp, _vp, _vp, _vp, _u64, _vp]
        L.ftred_run_allreduce.argtypes = [_vp, _u32, _vp, _u64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _u64, _vp]
        L.ftred_run_allreduce_noalloc.argtypes = [_vp, _u32, _vp, _u64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
        L.ftred_run_reduce_info.argtypes = [_vp, _u32, _vp, _vp, _u64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _u64,
                                            _vp]
        L.ftred_run_allreduce_info.argtypes = [_vp, _u32, _vp, _u64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                               _vp, _vp, _u64, _vp]
        L.ftred_validate.argtypes = [_vp, _int, _u32, _vp, _vp, _u64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                     ctypes.POINTER(_u64), _vp, _u64, _vp]
        L.ftred_detect.argtypes = [_vp, _int, _u32, _vp, _vp, _vp, _vp, _vp]
        L.ftred_reduce_times.argtypes = [_vp, _u32, _vp, _vp, _vp, ctypes.c_uint64, ctypes.c_uint64, _vp, _vp, _vp]
        L.ftred_gen_failures.argtypes = [_vp, _u64, _u32, _u32, _u32, _u32, _u32, _vp, _vp, _vp, _vp]
        L.ftred_gen_payload_int.argtypes = [_vp, _u64, _u32, _u32, _u32, _vp, _vp]
        L.ftred_timing_begin.argtypes = [_u32]
        L.ftred_timing_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_u64)]
        _lib = L
    return _lib


def _check(rc):
    if rc != OK:
        raise FtredError(rc, lib().ftred_last_error().decode())


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


class Plan:
    """ftred_plan / ftred_plan_info / ftred_plan_destroy."""

    def __init__(self, P, f, elems, dtype, op, flags=0, shape=0):
        """shape: the tree inside a subtree of the root: 0 or 2 = binary (default), k = 3..64 children per
        process, 1 = binomial (flags bits 20..26)."""
        flags |= shape << 20
        self._h = _vp()
        _check(lib().ftred_plan(ctypes.byref(self._h), P, f, elems, dtype, op, flags))
        self.P, self.f, self.elems, self.dtype, self.op = P, f, elems, dtype, op
        self.F = max(f, 1)
        self.info = Info()
        _check(lib().ftred_plan_info(self._h, ctypes.byref(self.info)))

    def __del__(self):
        if getattr(self, "_h", None) is not None and self._h.value and _lib is not None:
            _lib.ftred_plan_destroy(self._h)
            self._h = None

    @property
    def handle(self):
        return self._h

    def workspace_bytes(self, S):
        return int(lib().ftred_workspace_bytes(self._h, S))

    def partners(self, root, rank):
        p = Partners()
        _check(lib().ftred_partners(self._h, root, rank, ctypes.byref(p)))
        return dict(parent=p.parent, children=list(p.children[:p.n_children]), group=list(p.group[:p.group_size]),
                    group_pos=p.group_pos, subtree=p.subtree, depth=p.depth, height=p.height,
                    send_round=p.send_round)

    def workspace(self, S, device="cuda"):
        return torch.empty(self.workspace_bytes(S), dtype=torch.uint8, device=device)


def _payload_stride(plan, payload, S):
    assert payload.is_cuda and payload.is_contiguous() and payload.dtype == TORCH_DTYPE[plan.dtype]
    if payload.dim() == 2:
        assert tuple(payload.shape) == (plan.P, plan.elems)
        return 0
    assert tuple(payload.shape) == (S, plan.P, plan.elems)
    return plan.P * plan.elems


def _fail(plan, S, fail_rank, fail_round):
    for t in (fail_rank, fail_round):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.uint32 and tuple(t.shape) == (S, plan.F)


def structure(plan, root=0, stream=None):
    """ftred_structure: device index arithmetic for every rank."""
    dev = "cuda"
    names = ("parent", "subtree", "group_id", "group_pos", "group_size", "depth", "send_round")
    out = {n: torch.empty(plan.P, dtype=torch.uint32, device=dev) for n in names}
    _check(lib().ftred_structure(plan.handle, root, *[_ptr(out[n]) for n in names], _stream(stream)))
    return out


def run_reduce(plan, S, payload, fail_rank, fail_round, root=None, want_msgs=True, workspace=None, buffers=None,
               stream=None):
    """ftred_run_reduce.  Returns dict(result[S][elems], status[S], msgs[S][2] or None).
    buffers: the dict of an earlier call, to write into the same tensors again."""
    stride = _payload_stride(plan, payload, S)
    _fail(plan, S, fail_rank, fail_round)
    dev = payload.device
    if root is not None:
        assert root.is_cuda and root.dtype == torch.uint32 and tuple(root.shape) == (S,)
    if buffers is not None:
        result, status, msgs = buffers["result"], buffers["status"], buffers["msgs"]
    else:
        result = torch.empty((S, plan.elems), dtype=TORCH_DTYPE[plan.dtype], device=dev)
        status = torch.empty(S, dtype=torch.uint32, device=dev)
        msgs = torch.empty((S, 2), dtype=torch.uint64, device=dev) if want_msgs else None
    ws = workspace if workspace is not None else plan.workspace(S, dev)
    _check(lib().ftred_run_reduce(plan.handle, S, _ptr(root), _ptr(payload), stride, _ptr(fail_rank),
                                  _ptr(fail_round), _ptr(result), _ptr(status), _ptr(msgs), _ptr(ws),
                                  ws.numel(), _stream(stream)))
    return dict(result=result, status=status, msgs=msgs)


def run_allreduce(plan, S, payload, fail_rank, fail_round, want_bitmap=True, want_out=True, want_msgs=True,
                  workspace=None, out=None, buffers=None, stream=None):
    """ftred_run_allreduce.  Returns dict(result, has_bitmap, per_process_out, status, attempts, msgs).
    buffers: the dict of an earlier call, to write into the same tensors again."""
    stride = _payload_stride(plan, payload, S)
    _fail(plan, S, fail_rank, fail_round)
    dev = payload.device
    dt = TORCH_DTYPE[plan.dtype]
    if buffers is not None:
        result, status, attempts = buffers["result"], buffers["status"], buffers["attempts"]
        bitmap, out, msgs = buffers["has_bitmap"], buffers["per_process_out"], buffers["msgs"]
    else:
        result = torch.empty((S, plan.elems), dtype=dt, device=dev)
        status = torch.empty(S, dtype=torch.uint32, device=dev)
        attempts = torch.empty(S, dtype=torch.uint32, device=dev)
        bitmap = torch.empty((S, (plan.P + 31) // 32), dtype=torch.uint32, device=dev) if want_bitmap else None
        if out is None and want_out:
            out = torch.empty((S, plan.P, plan.elems), dtype=dt, device=dev)
        msgs = torch.empty((S, 4), dtype=torch.uint64, device=dev) if want_msgs else None
    ws = workspace if workspace is not None else plan.workspace(S, dev)
    _check(lib().ftred_run_allreduce(plan.handle, S, _ptr(payload), stride, _ptr(fail_rank), _ptr(fail_round),
                                     _ptr(result), _ptr(bitmap), _ptr(out), _ptr(status), _ptr(attempts),
                                     _ptr(msgs), _ptr(ws), ws.numel(), _stream(stream)))
    return dict(result=result, has_bitmap=bitmap, per_process_out=out, status=status, attempts=attempts, msgs=msgs)


NOALLOC_WORKSPACE_BYTES = 32 * 1024 * 1024


def run_allreduce_noalloc(plan, S, payload, fail_rank, fail_round, buffers, stream=None):
    """ftred_run_allreduce_noalloc: the workspace is the library's own fixed array.  `buffers`: the output
    tensors (result, has_bitmap, per_process_out, status, attempts, msgs; the optional ones may be None),
    allocated by the caller beforehand.  Returns `buffers`."""
    stride = _payload_stride(plan, payload, S)
    _fail(plan, S, fail_rank, fail_round)
    _check(lib().ftred_run_allreduce_noalloc(plan.handle, S, _ptr(payload), stride, _ptr(fail_rank), _ptr(fail_round),
                                             _ptr(buffers["result"]), _ptr(buffers["has_bitmap"]),
                                             _ptr(buffers["per_process_out"]), _ptr(buffers["status"]),
                                             _ptr(buffers["attempts"]), _ptr(buffers["msgs"]), _stream(stream)))
    return buffers


def _info_buffers(plan, S, dev):
    return (torch.empty(S, dtype=torch.uint32, device=dev),
            torch.empty((S, plan.F), dtype=torch.uint32, device=dev),
            torch.empty((S, plan.f + 1), dtype=torch.uint32, device=dev))


def run_reduce_info(plan, S, payload, fail_rank, fail_round, root=None, workspace=None, stream=None):
    """ftred_run_reduce_info.  As run_reduce, plus info_count[S], info_ids[S][F], info_child[S][f+1]."""
    stride = _payload_stride(plan, payload, S)
    _fail(plan, S, fail_rank, fail_round)
    dev = payload.device
    if root is not None:
        assert root.is_cuda and root.dtype == torch.uint32 and tuple(root.shape) == (S,)
    result = torch.empty((S, plan.elems), dtype=TORCH_DTYPE[plan.dtype], device=dev)
    status = torch.empty(S, dtype=torch.uint32, device=dev)
    msgs = torch.empty((S, 2), dtype=torch.uint64, device=dev)
    count, ids, child = _info_buffers(plan, S, dev)
    ws = workspace if workspace is not None else plan.workspace(S, dev)
    _check(lib().ftred_run_reduce_info(plan.handle, S, _ptr(root), _ptr(payload), stride, _ptr(fail_rank),
                                       _ptr(fail_round), _ptr(result), _ptr(status), _ptr(msgs), _ptr(count),
                                       _ptr(ids), _ptr(child), _ptr(ws), ws.numel(), _stream(stream)))
    return dict(result=result, status=status, msgs=msgs, info_count=count, info_ids=ids, info_child=child)


def run_allreduce_info(plan, S, payload, fail_rank, fail_round, workspace=None, stream=None):
    """ftred_run_allreduce_info.  As run_allreduce, plus info_count[S], info_ids[S][F], info_child[S][f+1]."""
    stride = _payload_stride(plan, payload, S)
    _fail(plan, S, fail_rank, fail_round)
    dev = payload.device
    dt = TORCH_DTYPE[plan.dtype]
    result = torch.empty((S, plan.elems), dtype=dt, device=dev)
    status = torch.empty(S, dtype=torch.uint32, device=dev)
    attempts = torch.empty(S, dtype=torch.uint32, device=dev)
    bitmap = torch.empty((S, (plan.P + 31) // 32), dtype=torch.uint32, device=dev)
    out = torch.empty((S, plan.P, plan.elems), dtype=dt, device=dev)
    msgs = torch.empty((S, 4), dtype=torch.uint64, device=dev)
    count, ids, child = _info_buffers(plan, S, dev)
    ws = workspace if workspace is not None else plan.workspace(S, dev)
    _check(lib().ftred_run_allreduce_info(plan.handle, S, _ptr(payload), stride, _ptr(fail_rank), _ptr(fail_round),
                                          _ptr(result), _ptr(bitmap), _ptr(out), _ptr(status), _ptr(attempts),
                                          _ptr(msgs), _ptr(count), _ptr(ids), _ptr(child), _ptr(ws), ws.numel(),
                                          _stream(stream)))
    return dict(result=result, has_bitmap=bitmap, per_process_out=out, status=status, attempts=attempts, msgs=msgs,
                info_count=count, info_ids=ids, info_child=child)


def validate(plan, kind, S, payload, fail_rank, fail_round, result, status, root=None, has_bitmap=None,
             per_process_out=None, attempts=None, msgs=None, workspace=None, count=True, verdict=None, stream=None):
    """ftred_validate.  Returns dict(verdict[S], n_invalid or None)."""
    stride = _payload_stride(plan, payload, S)
    _fail(plan, S, fail_rank, fail_round)
    dev = payload.device
    if verdict is None:
        verdict = torch.empty(S, dtype=torch.uint32, device=dev)
    ws = workspace if workspace is not None else plan.workspace(S, dev)
    n = _u64(0)
    _check(lib().ftred_validate(plan.handle, kind, S, _ptr(root), _ptr(payload), stride, _ptr(fail_rank),
                                _ptr(fail_round), _ptr(result), _ptr(has_bitmap), _ptr(per_process_out),
                                _ptr(status), _ptr(attempts), _ptr(msgs), _ptr(verdict),
                                ctypes.byref(n) if count else None, _ptr(ws), ws.numel(), _stream(stream)))
    return dict(verdict=verdict, n_invalid=int(n.value) if count else None)


def detect(plan, kind, S, fail_rank, fail_round, root=None, stream=None):
    """ftred_detect.  Returns detected[S] (bit q = the process in slot q of the failure list was detected)."""
    _fail(plan, S, fail_rank, fail_round)
    det = torch.empty(S, dtype=torch.uint32, device=fail_rank.device)
    _check(lib().ftred_detect(plan.handle, kind, S, _ptr(root), _ptr(fail_rank), _ptr(fail_round), _ptr(det),
                              _stream(stream)))
    return det


NEVER = 0xFFFFFFFFFFFFFFFF


def reduce_times(plan, S, fail_rank, fail_round, t_msg, t_timeout, root=None, t_done=None, t_proc=None, stream=None):
    """ftred_reduce_times.  Returns (t_done[S], t_proc[S][P]) as uint64 tensors (NEVER = did not get there)."""
    _fail(plan, S, fail_rank, fail_round)
    dev = fail_rank.device
    if t_done is None:
        t_done = torch.empty(S, dtype=torch.uint64, device=dev)
    if t_proc is None:
        t_proc = torch.empty((S, plan.P), dtype=torch.uint64, device=dev)
    assert t_proc.is_contiguous() and t_proc.numel() == S * plan.P and t_done.numel() == S
    _check(lib().ftred_reduce_times(plan.handle, S, _ptr(root), _ptr(fail_rank), _ptr(fail_round), int(t_msg),
                                    int(t_timeout), _ptr(t_done), _ptr(t_proc), _stream(stream)))
    return t_done, t_proc


def latency(plan, kind, attempts, detected, t_message=1.0, t_timeout=10.0):
    """The latency reading of ftred_detect for every scenario (numpy in, numpy out): message steps of the plan times
    the attempts, plus a time-out per detected process."""
    import numpy as np
    i = plan.info
    steps = i.steps_uc + i.steps_tree + (i.steps_bcast_tree + i.steps_bcast_corr if kind == 1 else 0)
    ndet = np.array([bin(int(d)).count("1") for d in np.asarray(detected)], dtype=np.int64)
    return t_message * steps * np.asarray(attempts, dtype=np.int64) + t_timeout * ndet


def gen_failures(plan, seed, S, scen0=0, inop_permille=0, rounds_per_attempt=0, protected=0, want_root=False,
                 fail_rank=None, fail_round=None, stream=None):
    """ftred_gen_failures.  Returns (fail_rank[S][F], fail_round[S][F], root[S] or None)."""
    dev = "cuda"
    if fail_rank is None:
        fail_rank = torch.empty((S, plan.F), dtype=torch.uint32, device=dev)
        fail_round = torch.empty((S, plan.F), dtype=torch.uint32, device=dev)
    root = torch.empty(S, dtype=torch.uint32, device=dev) if want_root else None
    _check(lib().ftred_gen_failures(plan.handle, seed, S, scen0, inop_permille, rounds_per_attempt, protected,
                                    _ptr(root), _ptr(fail_rank), _ptr(fail_round), _stream(stream)))
    return fail_rank, fail_round, root


def gen_payload_int(plan, seed, S, bits, scen0=0, out=None, stream=None):
    """ftred_gen_payload_int.  Returns payload[S][P][elems]."""
    if out is None:
        out = torch.empty((S, plan.P, plan.elems), dtype=TORCH_DTYPE[plan.dtype], device="cuda")
    done = 0
    while done < S:                 # the entry point takes at most 65535 scenarios per call
        n = min(S - done, 32768)
        _check(lib().ftred_gen_payload_int(plan.handle, seed, n, scen0 + done, bits, _ptr(out[done:done + n]),
                                           _stream(stream)))
        done += n
    return out


PHASES = ("check", "retry", "tree_deep", "tree_upper", "bcast", "val_partial", "val_final", "gen")


def timing_begin(max_records=65536):
    """ftred_timing_begin."""
    _check(lib().ftred_timing_begin(max_records))


def timing_end():
    """ftred_timing_end.  Returns {phase: (milliseconds, launches)}."""
    ms = (ctypes.c_double * len(PHASES))()
    n = (_u64 * len(PHASES))()
    _check(lib().ftred_timing_end(ms, n))
    return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(PHASES)}
