"""ctypes binding of the C boundary in ``include/dmalatte.h``.

Argument marshalling only: every byte is moved by the HIP kernels behind the
``dl_*`` entry points.  There is no CPU fallback: if the built library is
missing, loading fails with an error.

Device buffers may be given as integer addresses or as objects with a
``data_ptr()`` method (torch tensors); streams as ``None`` (default stream),
integer handles, or objects with a ``cuda_stream`` attribute.
"""

from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# DL_LIBRARY names another build of the same library (the host-sanitizer build of the tests); there is still no
# fallback: whatever it names must exist.
LIB_PATH = os.environ.get("DL_LIBRARY") or os.path.join(_HERE, "libdmalatte.so")

DL_OK = 0
DL_ERR_INVALID = -1
DL_ERR_OVERLAP = -2
DL_ERR_HIP = -3
DL_ERR_TIMEOUT = -4
DL_ERR_STATE = -5
DL_ERR_EXPIRED = -6
DL_ERR_LOST = -7
DL_ERR_CAPACITY = -8
DL_STATIC_MAX_COPIES = 16384
DL_DISPATCH_DEVICE_MAX_TOKENS = 10240
DL_MAX_FANOUT = 64
DL_PLAN_FANOUT = 8
DL_MODE_ONESHOT = 0
DL_MODE_PRELAUNCH = 1
DL_MODE_SIGNAL = 2
DL_MODE_STANDBY = 3
DL_MODE_AUTO = 4
DL_OP_BATCH, DL_OP_BROADCAST, DL_OP_ALLGATHER, DL_OP_ALLTOALL, DL_OP_SWAP, DL_OP_TOKEN_DISPATCH = range(6)
DL_AUTO_STANDBY_TILES = 64
DL_AUTO_SIGNAL_MAX_BYTES = 288 << 20
DL_AUTO_PRELAUNCH_MAX_BYTES = 288 << 20

# every symbol include/dmalatte.h declares
EXPORTS = [
    "dl_init", "dl_shutdown", "dl_set_mode", "dl_get_mode", "dl_set_validate", "dl_strerror",
    "dl_last_hip_error", "dl_batch_copy", "dl_broadcast", "dl_allgather", "dl_alltoall",
    "dl_prelaunch_start", "dl_prelaunch_stop", "dl_last_ticket", "dl_trigger", "dl_wait", "dl_wait_armed",
    "dl_get_config",
    "dl_set_config", "dl_plan_allgather", "dl_plan_alltoall", "dl_plan_broadcast", "dl_plan_batch",
    "dl_plan_first_hazard", "dl_plan_tiles", "dl_batch_swap", "dl_alltoall_inplace", "dl_plan_alltoall_inplace",
    "dl_plan_swap_first_hazard", "dl_batch_fanout", "dl_token_dispatch", "dl_plan_token_dispatch",
    "dl_plan_batch_inferred", "dl_set_trace", "dl_get_trace", "dl_trace_clock",
    "dl_last_device_error", "dl_debug_lose_next_table", "dl_batch_copy_static",
    "dl_plan_mode", "dl_last_mode", "dl_complete", "dl_parse_config", "dl_token_dispatch_device",
]


class DlError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} (status {status}, hip error {last_hip_error()})")


class CopyDesc(ctypes.Structure):
    _fields_ = [("src", ctypes.c_void_p), ("dst", ctypes.c_void_p), ("bytes", ctypes.c_size_t)]


class SwapDesc(ctypes.Structure):
    _fields_ = [("a", ctypes.c_void_p), ("b", ctypes.c_void_p), ("bytes", ctypes.c_size_t)]


class Trace(ctypes.Structure):
    _fields_ = [("doorbell_seen", ctypes.c_uint64), ("copy_begin", ctypes.c_uint64), ("copy_end", ctypes.c_uint64),
                ("completion_issued", ctypes.c_uint64)]


class Config(ctypes.Structure):
    _fields_ = [
        ("tile_bytes", ctypes.c_uint32),
        ("block_threads", ctypes.c_uint32),
        ("nontemporal_min_bytes", ctypes.c_uint64),
        ("armed_blocks", ctypes.c_uint32),
        ("arm_timeout_us", ctypes.c_uint32),
        ("fuse_broadcast", ctypes.c_uint32),
        ("max_blocks", ctypes.c_uint32),
        ("fan_split", ctypes.c_uint32),
        ("infer_broadcast", ctypes.c_uint32),
        ("device_lowering", ctypes.c_uint32),
        ("table_push", ctypes.c_uint32),
        ("write_through_max_bytes", ctypes.c_uint64),
        ("stream_plain_min_bytes", ctypes.c_uint64),
        ("armed_chain_min_bytes", ctypes.c_uint64),
    ]


class PlanItem(ctypes.Structure):
    _fields_ = [
        ("src", ctypes.c_void_p),
        ("bytes", ctypes.c_size_t),
        ("k", ctypes.c_uint32),
        ("reserved", ctypes.c_uint32),
        ("dst", ctypes.c_void_p * DL_PLAN_FANOUT),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2511_06605_amd.build` "
            "(there is no fallback path)")
    try:
        # One HIP runtime per process: PyTorch ships its own, and device memory and streams come
        # from it, so it has to be loaded first for the library to bind to that same runtime.
        import torch  # noqa: F401
    except ImportError:
        pass
    L = ctypes.CDLL(LIB_PATH)
    vp, vpp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)
    szp = ctypes.POINTER(ctypes.c_size_t)
    sig = {
        "dl_init": (ctypes.c_int, [ctypes.c_int]),
        "dl_shutdown": (ctypes.c_int, []),
        "dl_set_mode": (ctypes.c_int, [ctypes.c_int]),
        "dl_get_mode": (ctypes.c_int, []),
        "dl_last_mode": (ctypes.c_int, []),
        "dl_complete": (ctypes.c_int, [vp, ctypes.c_uint64]),
        "dl_plan_mode": (ctypes.c_int, [ctypes.c_int, ctypes.c_size_t, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint64,
                                        ctypes.c_int]),
        "dl_set_validate": (ctypes.c_int, [ctypes.c_int]),
        "dl_strerror": (ctypes.c_char_p, [ctypes.c_int]),
        "dl_last_hip_error": (ctypes.c_int, []),
        "dl_last_device_error": (ctypes.c_int, []),
        "dl_debug_lose_next_table": (ctypes.c_int, [ctypes.c_uint32]),
        "dl_batch_copy": (ctypes.c_int, [ctypes.POINTER(CopyDesc), ctypes.c_size_t, vp]),
        "dl_batch_copy_static": (ctypes.c_int, [ctypes.POINTER(CopyDesc), ctypes.c_size_t, vp]),
        "dl_broadcast": (ctypes.c_int, [vp, vpp, ctypes.c_int, ctypes.c_size_t, vp]),
        "dl_allgather": (ctypes.c_int, [vpp, vpp, ctypes.c_int, ctypes.c_size_t, vp]),
        "dl_alltoall": (ctypes.c_int, [vpp, vpp, ctypes.c_int, szp, vp]),
        "dl_prelaunch_start": (ctypes.c_int, []),
        "dl_prelaunch_stop": (ctypes.c_int, []),
        "dl_last_ticket": (ctypes.c_uint64, []),
        "dl_trigger": (ctypes.c_int, [ctypes.c_uint64]),
        "dl_wait": (ctypes.c_int, [ctypes.c_uint64, ctypes.c_uint64]),
        "dl_wait_armed": (ctypes.c_int, [ctypes.c_uint64, ctypes.c_uint64]),
        "dl_get_config": (ctypes.c_int, [ctypes.POINTER(Config)]),
        "dl_set_config": (ctypes.c_int, [ctypes.POINTER(Config)]),
        "dl_parse_config": (ctypes.c_int, [ctypes.c_char_p, ctypes.POINTER(Config)]),
        "dl_plan_allgather": (ctypes.c_long, [vpp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int,
                                              ctypes.POINTER(PlanItem), ctypes.c_size_t]),
        "dl_plan_alltoall": (ctypes.c_long, [vpp, vpp, ctypes.c_int, szp, ctypes.POINTER(PlanItem), ctypes.c_size_t]),
        "dl_plan_broadcast": (ctypes.c_long, [vp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.POINTER(PlanItem),
                                              ctypes.c_size_t]),
        "dl_plan_batch": (ctypes.c_long, [ctypes.POINTER(CopyDesc), ctypes.c_size_t, ctypes.POINTER(PlanItem),
                                          ctypes.c_size_t]),
        "dl_plan_first_hazard": (ctypes.c_long, [ctypes.POINTER(PlanItem), ctypes.c_size_t]),
        "dl_plan_tiles": (ctypes.c_uint64, [ctypes.POINTER(PlanItem), ctypes.c_size_t, ctypes.c_uint32]),
        "dl_batch_swap": (ctypes.c_int, [ctypes.POINTER(SwapDesc), ctypes.c_size_t, vp]),
        "dl_alltoall_inplace": (ctypes.c_int, [vpp, ctypes.c_int, ctypes.c_size_t, vp]),
        "dl_plan_alltoall_inplace": (ctypes.c_long, [vpp, ctypes.c_int, ctypes.c_size_t, ctypes.POINTER(SwapDesc),
                                                     ctypes.c_size_t]),
        "dl_plan_swap_first_hazard": (ctypes.c_long, [ctypes.POINTER(SwapDesc), ctypes.c_size_t]),
        "dl_set_trace": (ctypes.c_int, [ctypes.c_int]),
        "dl_get_trace": (ctypes.c_int, [ctypes.c_uint64, ctypes.POINTER(Trace)]),
        "dl_trace_clock": (ctypes.c_int, [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]),
        "dl_batch_fanout": (ctypes.c_int, [ctypes.POINTER(PlanItem), ctypes.c_size_t, vp]),
        "dl_token_dispatch": (ctypes.c_int, [vpp, vpp, ctypes.c_int, ctypes.POINTER(ctypes.c_uint32), ctypes.c_size_t,
                                             ctypes.POINTER(ctypes.c_uint8), vp]),
        "dl_token_dispatch_device": (ctypes.c_int, [vpp, vpp, ctypes.c_int, ctypes.POINTER(ctypes.c_uint32), ctypes.c_size_t,
                                                    vp, vp]),
        "dl_plan_token_dispatch": (ctypes.c_long, [vpp, vpp, ctypes.c_int, ctypes.POINTER(ctypes.c_uint32),
                                                   ctypes.c_size_t, ctypes.POINTER(ctypes.c_uint8),
                                                   ctypes.POINTER(PlanItem), ctypes.c_size_t]),
        "dl_plan_batch_inferred": (ctypes.c_long, [ctypes.POINTER(CopyDesc), ctypes.c_size_t, ctypes.POINTER(PlanItem),
                                                   ctypes.c_size_t]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


# ------------------------------------------------------------------ marshalling

def _addr(x) -> int | None:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr()) or None
    return int(x) or None


def _stream(s) -> int | None:
    if s is None:
        return None
    if hasattr(s, "cuda_stream"):
        return int(s.cuda_stream) or None
    return int(s) or None


def _ptr_array(xs):
    return (ctypes.c_void_p * max(len(xs), 1))(*[_addr(x) for x in xs])


def _chunk_array(chunk_bytes, W):
    flat = [int(v) for row in chunk_bytes for v in (row if hasattr(row, "__len__") else [row])]
    if len(flat) != W * W:
        raise ValueError("chunk_bytes must have W*W entries")
    return (ctypes.c_size_t * (W * W))(*flat)


def _desc_array(descs):
    arr = (CopyDesc * max(len(descs), 1))()
    for i, (s, d, n) in enumerate(descs):
        arr[i].src, arr[i].dst, arr[i].bytes = _addr(s), _addr(d), int(n)
    return arr


def _swap_array(descs):
    arr = (SwapDesc * max(len(descs), 1))()
    for i, (a, b, n) in enumerate(descs):
        arr[i].a, arr[i].b, arr[i].bytes = _addr(a), _addr(b), int(n)
    return arr


def _check(status: int, what: str) -> None:
    if status != DL_OK:
        raise DlError(status, what)


# ------------------------------------------------------------------- lifecycle

def strerror(status: int) -> str:
    return lib().dl_strerror(status).decode()


def last_hip_error() -> int:
    return lib().dl_last_hip_error()


def dl_last_device_error() -> int:
    """DL_ERR_LOST if a kernel has given up on its copy table since the last call (clears the report), else DL_OK."""
    return int(lib().dl_last_device_error())


def dl_debug_lose_next_table(tries: int = 4) -> None:
    _check(lib().dl_debug_lose_next_table(int(tries)), "dl_debug_lose_next_table")


def dl_init(device: int = 0) -> None:
    _check(lib().dl_init(device), "dl_init")


def dl_shutdown() -> None:
    _check(lib().dl_shutdown(), "dl_shutdown")


def dl_set_mode(mode: int) -> None:
    _check(lib().dl_set_mode(mode), "dl_set_mode")


def dl_get_mode() -> int:
    return lib().dl_get_mode()


def dl_last_mode() -> int:
    return lib().dl_last_mode()


def dl_complete(stream=None, timeout_ns: int = 5_000_000_000) -> None:
    _check(lib().dl_complete(_stream(stream), timeout_ns), "dl_complete")


def dl_plan_mode(op: int, items: int, max_fanout: int, moved_bytes: int, tiles: int, known_ahead: bool) -> int:
    """The size -> mode table: the dl_mode that suits a lowered list of these dimensions."""
    m = lib().dl_plan_mode(int(op), int(items), int(max_fanout), int(moved_bytes), int(tiles), 1 if known_ahead else 0)
    if m < 0:
        raise DlError(int(m), "dl_plan_mode")
    return int(m)


def dl_set_validate(on: bool) -> None:
    _check(lib().dl_set_validate(1 if on else 0), "dl_set_validate")


def dl_get_config() -> Config:
    c = Config()
    _check(lib().dl_get_config(ctypes.byref(c)), "dl_get_config")
    return c


def dl_parse_config(text: str, cfg: Config | None = None) -> Config:
    """``text`` ("name=value,...") applied to ``cfg`` (or to an all-zero one with arm_timeout_us = 1); host-only."""
    c = cfg or Config(arm_timeout_us=1)
    _check(lib().dl_parse_config(text.encode(), ctypes.byref(c)), "dl_parse_config")
    return c


def dl_set_config(cfg: Config | None = None, **fields) -> None:
    c = cfg or dl_get_config()
    for k, v in fields.items():
        if not hasattr(c, k):
            raise AttributeError(k)
        setattr(c, k, v)
    _check(lib().dl_set_config(ctypes.byref(c)), "dl_set_config")


# ------------------------------------------------------------------ operations

def dl_batch_copy(descs, stream=None) -> None:
    """descs: sequence of (src, dst, bytes)."""
    descs = list(descs)
    _check(lib().dl_batch_copy(_desc_array(descs), len(descs), _stream(stream)), "dl_batch_copy")


def dl_batch_copy_static(descs, stream=None) -> None:
    """descs: sequence of (src, dst, bytes); the variant that allocates nothing."""
    descs = list(descs)
    _check(lib().dl_batch_copy_static(_desc_array(descs), len(descs), _stream(stream)), "dl_batch_copy_static")


def dl_broadcast(src, dsts, nbytes: int, stream=None) -> None:
    dsts = list(dsts)
    _check(lib().dl_broadcast(_addr(src), _ptr_array(dsts), len(dsts), int(nbytes), _stream(stream)), "dl_broadcast")


def dl_allgather(ins, outs, bytes_per_rank: int, stream=None) -> None:
    ins, outs = list(ins), list(outs)
    if len(ins) != len(outs):
        raise ValueError("need as many receive buffers as send buffers")
    _check(lib().dl_allgather(_ptr_array(ins), _ptr_array(outs), len(ins), int(bytes_per_rank), _stream(stream)),
           "dl_allgather")


def dl_alltoall(ins, outs, chunk_bytes, stream=None) -> None:
    ins, outs = list(ins), list(outs)
    W = len(ins)
    if len(outs) != W:
        raise ValueError("need as many receive buffers as send buffers")
    _check(lib().dl_alltoall(_ptr_array(ins), _ptr_array(outs), W, _chunk_array(chunk_bytes, W), _stream(stream)),
           "dl_alltoall")


def dl_batch_swap(descs, stream=None) -> None:
    """descs: sequence of (a, b, bytes)."""
    descs = list(descs)
    _check(lib().dl_batch_swap(_swap_array(descs), len(descs), _stream(stream)), "dl_batch_swap")


def dl_alltoall_inplace(bufs, chunk_bytes: int, stream=None) -> None:
    bufs = list(bufs)
    _check(lib().dl_alltoall_inplace(_ptr_array(bufs), len(bufs), int(chunk_bytes), _stream(stream)),
           "dl_alltoall_inplace")


def _dispatch_args(ins, outs, tokens, dest):
    ins, outs = list(ins), list(outs)
    W = len(ins)
    if len(outs) != W or len(tokens) != W:
        raise ValueError("need W send buffers, W receive buffers and W token counts")
    tok = (ctypes.c_uint32 * W)(*[int(t) for t in tokens])
    total = sum(int(t) for t in tokens)
    flat = bytes(bytearray(int(v) != 0 for row in dest for v in row)) if not hasattr(dest, "tobytes") else \
        (dest != 0).astype("uint8").tobytes()
    if len(flat) != total * W:
        raise ValueError("dest must have one entry per (token, rank)")
    d = (ctypes.c_uint8 * max(len(flat), 1)).from_buffer_copy(flat or b"\0")
    return _ptr_array(ins), _ptr_array(outs), W, tok, d


def dl_batch_fanout(items, stream=None) -> None:
    """items: sequence of dicts {src, bytes, dst: [..]} (as the dl_plan_* functions return)."""
    items = list(items)
    _check(lib().dl_batch_fanout(_items_in(items), len(items), _stream(stream)), "dl_batch_fanout")


def dl_token_dispatch(ins, outs, tokens, row_bytes: int, dest, stream=None) -> None:
    a, b, W, tok, d = _dispatch_args(ins, outs, tokens, dest)
    _check(lib().dl_token_dispatch(a, b, W, tok, int(row_bytes), d, _stream(stream)), "dl_token_dispatch")


def dl_token_dispatch_device(ins, outs, tokens, row_bytes: int, dest_device, stream=None) -> None:
    """dest_device: device buffer of (total tokens) x W bytes, non-zero where a token goes to a rank."""
    ins, outs = list(ins), list(outs)
    W = len(ins)
    if len(outs) != W or len(tokens) != W:
        raise ValueError("need W send buffers, W receive buffers and W token counts")
    tok = (ctypes.c_uint32 * W)(*[int(t) for t in tokens])
    _check(lib().dl_token_dispatch_device(_ptr_array(ins), _ptr_array(outs), W, tok, int(row_bytes), _addr(dest_device),
                                          _stream(stream)), "dl_token_dispatch_device")


# -------------------------------------------------------------------- prelaunch

def dl_prelaunch_start() -> None:
    _check(lib().dl_prelaunch_start(), "dl_prelaunch_start")


def dl_prelaunch_stop() -> None:
    _check(lib().dl_prelaunch_stop(), "dl_prelaunch_stop")


def dl_last_ticket() -> int:
    return int(lib().dl_last_ticket())


def dl_trigger(ticket: int | None = None) -> None:
    t = dl_last_ticket() if ticket is None else ticket
    _check(lib().dl_trigger(t), "dl_trigger")


def dl_wait(ticket: int | None = None, timeout_ns: int = 5_000_000_000) -> None:
    t = dl_last_ticket() if ticket is None else ticket
    _check(lib().dl_wait(t, timeout_ns), "dl_wait")


def dl_wait_armed(ticket: int | None = None, timeout_ns: int = 5_000_000_000) -> None:
    t = dl_last_ticket() if ticket is None else ticket
    _check(lib().dl_wait_armed(t, timeout_ns), "dl_wait_armed")


def dl_set_trace(on: bool) -> None:
    _check(lib().dl_set_trace(1 if on else 0), "dl_set_trace")


def dl_get_trace(ticket: int | None = None) -> dict:
    t = Trace()
    _check(lib().dl_get_trace(dl_last_ticket() if ticket is None else ticket, ctypes.byref(t)), "dl_get_trace")
    return {f[0]: int(getattr(t, f[0])) for f in Trace._fields_}


def dl_trace_clock():
    """(device ticks per microsecond, host CLOCK_MONOTONIC nanoseconds at device tick 0)."""
    a, b = ctypes.c_double(0), ctypes.c_double(0)
    _check(lib().dl_trace_clock(ctypes.byref(a), ctypes.byref(b)), "dl_trace_clock")
    return a.value, b.value


# --------------------------------------------------------------------- lowering

def _items_out(call):
    n = call(None, 0)
    if n < 0:
        raise DlError(int(n), "dl_plan")
    arr = (PlanItem * max(n, 1))()
    m = call(arr, n)
    assert m == n
    return [dict(src=arr[i].src or 0, bytes=arr[i].bytes, k=arr[i].k,
                 dst=[arr[i].dst[j] or 0 for j in range(arr[i].k)]) for i in range(n)]


def dl_plan_allgather(ins, outs, bytes_per_rank: int, fuse_broadcast: bool = True):
    ins, outs = list(ins), list(outs)
    a, b = _ptr_array(ins), _ptr_array(outs)
    return _items_out(lambda arr, cap: lib().dl_plan_allgather(a, b, len(ins), int(bytes_per_rank),
                                                               1 if fuse_broadcast else 0, arr, cap))


def dl_plan_alltoall(ins, outs, chunk_bytes):
    ins, outs = list(ins), list(outs)
    a, b, c = _ptr_array(ins), _ptr_array(outs), _chunk_array(chunk_bytes, len(ins))
    return _items_out(lambda arr, cap: lib().dl_plan_alltoall(a, b, len(ins), c, arr, cap))


def dl_plan_broadcast(src, dsts, nbytes: int):
    dsts = list(dsts)
    d = _ptr_array(dsts)
    return _items_out(lambda arr, cap: lib().dl_plan_broadcast(_addr(src), d, len(dsts), int(nbytes), arr, cap))


def dl_plan_batch(descs):
    descs = list(descs)
    d = _desc_array(descs)
    return _items_out(lambda arr, cap: lib().dl_plan_batch(d, len(descs), arr, cap))


def dl_plan_token_dispatch(ins, outs, tokens, row_bytes: int, dest):
    a, b, W, tok, d = _dispatch_args(ins, outs, tokens, dest)
    return _items_out(lambda arr, cap: lib().dl_plan_token_dispatch(a, b, W, tok, int(row_bytes), d, arr, cap))


def dl_plan_batch_inferred(descs):
    descs = list(descs)
    d = _desc_array(descs)
    return _items_out(lambda arr, cap: lib().dl_plan_batch_inferred(d, len(descs), arr, cap))


def dl_plan_alltoall_inplace(bufs, chunk_bytes: int):
    """The (a, b, bytes) swaps an in-place all-to-all lowers to."""
    bufs = list(bufs)
    p = _ptr_array(bufs)
    n = lib().dl_plan_alltoall_inplace(p, len(bufs), int(chunk_bytes), None, 0)
    if n < 0:
        raise DlError(int(n), "dl_plan_alltoall_inplace")
    arr = (SwapDesc * max(n, 1))()
    assert lib().dl_plan_alltoall_inplace(p, len(bufs), int(chunk_bytes), arr, n) == n
    return [(arr[i].a or 0, arr[i].b or 0, arr[i].bytes) for i in range(n)]


def dl_plan_swap_first_hazard(descs) -> int:
    descs = list(descs)
    return int(lib().dl_plan_swap_first_hazard(_swap_array(descs), len(descs)))


def _items_in(items):
    arr = (PlanItem * max(len(items), 1))()
    for i, it in enumerate(items):
        arr[i].src, arr[i].bytes, arr[i].k = it["src"] or None, it["bytes"], len(it["dst"])
        for j, d in enumerate(it["dst"]):
            arr[i].dst[j] = d or None
    return arr


def dl_plan_first_hazard(items) -> int:
    return int(lib().dl_plan_first_hazard(_items_in(items), len(items)))


def dl_plan_tiles(items, tile_bytes: int) -> int:
    return int(lib().dl_plan_tiles(_items_in(items), len(items), tile_bytes))
