"""ctypes front end of the measurement aid (``libdl_benchaid.so``): timing loops
around the public ``dl_*`` calls and the runtime copy paths timed beside them.
Used by ``bench.py`` only."""

from __future__ import annotations

import ctypes
import os

from paper_2511_06605_amd import binding

_HERE = os.path.dirname(os.path.abspath(__file__))
AID_PATH = os.path.join(_HERE, "libdl_benchaid.so")

OP_BATCH, OP_BROADCAST, OP_ALLGATHER, OP_ALLTOALL, OP_MEMCPY_ASYNC, OP_MEMCPY_BATCH, OP_SWAP, OP_ALLTOALL_INPLACE, OP_TOKEN_DISPATCH, OP_FANOUT, OP_TOKEN_DISPATCH_DEVICE = range(11)
WAIT_STREAM, WAIT_TRIGGER, WAIT_ARM_AND_TRIGGER, WAIT_SIGNAL = 0, 1, 2, 3


class Request(ctypes.Structure):
    _fields_ = [
        ("op", ctypes.c_int), ("k", ctypes.c_int), ("W", ctypes.c_int), ("pad", ctypes.c_int),
        ("desc", ctypes.POINTER(binding.CopyDesc)), ("n", ctypes.c_size_t),
        ("src", ctypes.c_void_p), ("dsts", ctypes.POINTER(ctypes.c_void_p)), ("bytes", ctypes.c_size_t),
        ("in_", ctypes.POINTER(ctypes.c_void_p)), ("out", ctypes.POINTER(ctypes.c_void_p)),
        ("C", ctypes.POINTER(ctypes.c_size_t)),
        ("tokens", ctypes.POINTER(ctypes.c_uint32)), ("dest", ctypes.POINTER(ctypes.c_uint8)),
    ]


_aid = None


def aid() -> ctypes.CDLL:
    global _aid
    if _aid is None:
        binding.lib()  # the aid links against the library
        if not os.path.exists(AID_PATH):
            raise ImportError(f"{AID_PATH} is missing: run `python bench_aid/build.py`")
        L = ctypes.CDLL(AID_PATH)
        rp, dp = ctypes.POINTER(Request), ctypes.POINTER(ctypes.c_double)
        L.dlb_issue.restype = ctypes.c_int
        L.dlb_issue.argtypes = [rp, ctypes.c_void_p]
        L.dlb_time_host.restype = ctypes.c_int
        L.dlb_time_host.argtypes = [rp, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, dp]
        L.dlb_time_device.restype = ctypes.c_int
        L.dlb_time_device.argtypes = [rp, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, dp]
        L.dlb_time_device_rotating.restype = ctypes.c_int
        L.dlb_time_device_rotating.argtypes = [ctypes.POINTER(rp), ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                               ctypes.c_int, dp]
        L.dlb_time_call.restype = ctypes.c_int
        L.dlb_time_call.argtypes = [rp, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, dp, dp]
        L.dlb_phases.restype = ctypes.c_int
        L.dlb_phases.argtypes = [rp, ctypes.c_int, ctypes.c_int, dp]
        L.dlb_time_token_lowering.restype = ctypes.c_int
        L.dlb_time_token_lowering.argtypes = [rp, ctypes.POINTER(binding.PlanItem), ctypes.c_size_t, ctypes.c_int, dp]
        _aid = L
    return _aid


class Prepared:
    """A request with its marshalled arrays kept alive."""

    def __init__(self, req, keep):
        self.req, self._keep = req, keep


def allgather_request(ins, outs, bytes_per_rank) -> Prepared:
    a, b = binding._ptr_array(list(ins)), binding._ptr_array(list(outs))
    r = Request(op=OP_ALLGATHER, W=len(ins), bytes=int(bytes_per_rank))
    r.in_ = ctypes.cast(a, ctypes.POINTER(ctypes.c_void_p))
    r.out = ctypes.cast(b, ctypes.POINTER(ctypes.c_void_p))
    return Prepared(r, (a, b))


def alltoall_request(ins, outs, C) -> Prepared:
    W = len(ins)
    a, b, c = binding._ptr_array(list(ins)), binding._ptr_array(list(outs)), binding._chunk_array(C, W)
    r = Request(op=OP_ALLTOALL, W=W)
    r.in_ = ctypes.cast(a, ctypes.POINTER(ctypes.c_void_p))
    r.out = ctypes.cast(b, ctypes.POINTER(ctypes.c_void_p))
    r.C = ctypes.cast(c, ctypes.POINTER(ctypes.c_size_t))
    return Prepared(r, (a, b, c))


def broadcast_request(src, dsts, nbytes) -> Prepared:
    d = binding._ptr_array(list(dsts))
    r = Request(op=OP_BROADCAST, k=len(dsts), bytes=int(nbytes), src=binding._addr(src))
    r.dsts = ctypes.cast(d, ctypes.POINTER(ctypes.c_void_p))
    return Prepared(r, (d,))


def copy_list_request(descs, op=OP_BATCH) -> Prepared:
    descs = list(descs)
    d = binding._desc_array(descs)
    r = Request(op=op, n=len(descs))
    r.desc = ctypes.cast(d, ctypes.POINTER(binding.CopyDesc))
    return Prepared(r, (d,))


def alltoall_inplace_request(bufs, chunk_bytes) -> Prepared:
    b = binding._ptr_array(list(bufs))
    r = Request(op=OP_ALLTOALL_INPLACE, W=len(bufs), bytes=int(chunk_bytes))
    r.out = ctypes.cast(b, ctypes.POINTER(ctypes.c_void_p))
    return Prepared(r, (b,))


def token_dispatch_request(ins, outs, tokens, row_bytes, dest) -> Prepared:
    a, b, W, tok, d = binding._dispatch_args(ins, outs, tokens, dest)
    r = Request(op=OP_TOKEN_DISPATCH, W=W, bytes=int(row_bytes))
    r.in_ = ctypes.cast(a, ctypes.POINTER(ctypes.c_void_p))
    r.out = ctypes.cast(b, ctypes.POINTER(ctypes.c_void_p))
    r.tokens = ctypes.cast(tok, ctypes.POINTER(ctypes.c_uint32))
    r.dest = ctypes.cast(d, ctypes.POINTER(ctypes.c_uint8))
    return Prepared(r, (a, b, tok, d))


def token_dispatch_device_request(ins, outs, tokens, row_bytes, mask) -> Prepared:
    """mask: device tensor of (total tokens) x W bytes."""
    ins, outs = list(ins), list(outs)
    W = len(ins)
    a, b = binding._ptr_array(ins), binding._ptr_array(outs)
    tok = (ctypes.c_uint32 * W)(*[int(t) for t in tokens])
    r = Request(op=OP_TOKEN_DISPATCH_DEVICE, W=W, bytes=int(row_bytes))
    r.in_ = ctypes.cast(a, ctypes.POINTER(ctypes.c_void_p))
    r.out = ctypes.cast(b, ctypes.POINTER(ctypes.c_void_p))
    r.tokens = ctypes.cast(tok, ctypes.POINTER(ctypes.c_uint32))
    r.dest = ctypes.cast(ctypes.c_void_p(binding._addr(mask)), ctypes.POINTER(ctypes.c_uint8))
    return Prepared(r, (a, b, tok, mask))


def lowered_token_dispatch(p: Prepared, iters=20):
    """Lower a prepared token dispatch on the host: returns (a fan-out batch request that executes
    the lowered list, microseconds per lowering)."""
    n = binding.lib().dl_plan_token_dispatch(p.req.in_, p.req.out, p.req.W, p.req.tokens, p.req.bytes, p.req.dest,
                                             None, 0)
    if n < 0:
        raise binding.DlError(int(n), "dl_plan_token_dispatch")
    items = (binding.PlanItem * max(n, 1))()
    us = ctypes.c_double(0)
    _rc(aid().dlb_time_token_lowering(ctypes.byref(p.req), items, n, iters, ctypes.byref(us)), "dlb_time_token_lowering")
    r = Request(op=OP_FANOUT, n=n)
    r.desc = ctypes.cast(items, ctypes.POINTER(binding.CopyDesc))
    return Prepared(r, (items, p)), us.value


def _rc(rc, what):
    if rc >= 1000:
        raise RuntimeError(f"{what}: hipError {rc - 1000}")
    if rc:
        raise binding.DlError(rc, what)


def issue(p: Prepared, stream=None) -> None:
    _rc(aid().dlb_issue(ctypes.byref(p.req), binding._stream(stream)), "dlb_issue")


def time_host(p: Prepared, stream=None, wait=WAIT_STREAM, warmup=50, iters=1000):
    """Per-call host-observed latencies in microseconds."""
    out = (ctypes.c_double * iters)()
    _rc(aid().dlb_time_host(ctypes.byref(p.req), binding._stream(stream), wait, warmup, iters, out), "dlb_time_host")
    return list(out)


def time_device(p: Prepared, stream=None, warmup=5, calls=20) -> float:
    """Microseconds per call from HIP events around ``calls`` back-to-back issues."""
    out = ctypes.c_double(0)
    _rc(aid().dlb_time_device(ctypes.byref(p.req), binding._stream(stream), warmup, calls, ctypes.byref(out)),
        "dlb_time_device")
    return out.value


def time_device_rotating(ps, stream=None, warmup_rounds=1, rounds=3) -> float:
    """Microseconds per call from HIP events around ``rounds`` passes over the requests ``ps`` (same shape, buffers
    of their own each), issued back to back: with enough of them every call starts with cold caches."""
    arr = (ctypes.POINTER(Request) * len(ps))(*[ctypes.pointer(p.req) for p in ps])
    out = ctypes.c_double(0)
    _rc(aid().dlb_time_device_rotating(arr, len(ps), binding._stream(stream), warmup_rounds, rounds, ctypes.byref(out)),
        "dlb_time_device_rotating")
    return out.value


def time_call(p: Prepared, stream=None, warmup=20, iters=200):
    """One-shot mode: (host durations of the call itself, call -> stream synchronised), microseconds."""
    a, b = (ctypes.c_double * iters)(), (ctypes.c_double * iters)()
    _rc(aid().dlb_time_call(ctypes.byref(p.req), binding._stream(stream), warmup, iters, a, b), "dlb_time_call")
    return list(a), list(b)


PHASES = ("arming_call", "doorbell_to_seen", "seen_to_first_copy", "copy", "last_copy_to_completion_issued",
          "completion_issued_to_host")


def phases(p: Prepared, warmup=10, iters=100):
    """Prelaunch mode with phase stamps: a list of dicts, microseconds per phase (see PHASES)."""
    out = (ctypes.c_double * (6 * iters))()
    _rc(aid().dlb_phases(ctypes.byref(p.req), warmup, iters, out), "dlb_phases")
    return [dict(zip(PHASES, out[6 * i:6 * i + 6])) for i in range(iters)]
