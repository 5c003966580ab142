"""ctypes front end of the CPU checker in ``dl_oracle.c``.

TEST INFRASTRUCTURE: used by the tests, the smoke check and the benchmark's
CPU-baseline leg only.  Nothing here touches the GPU or the HIP library.

All buffers are ``numpy.uint8`` arrays.  The functions marshal pointers and
sizes; every byte is moved by the C code.
"""

from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "dl_oracle.c")
LIB = os.path.join(_HERE, "libdl_oracle.so")


class RefCopy(ctypes.Structure):
    _fields_ = [("src", ctypes.c_void_p), ("dst", ctypes.c_void_p), ("bytes", ctypes.c_size_t)]


class RefSwap(ctypes.Structure):
    _fields_ = [("a", ctypes.c_void_p), ("b", ctypes.c_void_p), ("bytes", ctypes.c_size_t)]


def build(src: str = SRC, out: str = LIB, force: bool = False) -> str:
    """Compile the checker with gcc (plain C, no GPU toolchain)."""
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        subprocess.run(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", src, "-o", out],
                       check=True)
    return out


def load(path: str | None = None) -> ctypes.CDLL:
    lib = ctypes.CDLL(path or build())
    VPP = ctypes.POINTER(ctypes.c_void_p)
    lib.ref_first_hazard.restype = ctypes.c_long
    lib.ref_first_hazard.argtypes = [ctypes.POINTER(RefCopy), ctypes.c_size_t]
    lib.ref_batch_copy.restype = ctypes.c_int
    lib.ref_batch_copy.argtypes = [ctypes.POINTER(RefCopy), ctypes.c_size_t]
    lib.ref_broadcast.restype = ctypes.c_int
    lib.ref_broadcast.argtypes = [ctypes.c_void_p, VPP, ctypes.c_int, ctypes.c_size_t]
    lib.ref_allgather.restype = ctypes.c_int
    lib.ref_allgather.argtypes = [VPP, VPP, ctypes.c_int, ctypes.c_size_t]
    lib.ref_alltoall.restype = ctypes.c_int
    lib.ref_alltoall.argtypes = [VPP, VPP, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    lib.ref_batch_swap.restype = ctypes.c_int
    lib.ref_batch_swap.argtypes = [ctypes.POINTER(RefSwap), ctypes.c_size_t]
    lib.ref_alltoall_inplace.restype = ctypes.c_int
    lib.ref_alltoall_inplace.argtypes = [VPP, ctypes.c_int, ctypes.c_size_t]
    lib.ref_token_dispatch.restype = ctypes.c_int
    lib.ref_token_dispatch.argtypes = [VPP, VPP, ctypes.c_int, ctypes.POINTER(ctypes.c_uint32), ctypes.c_size_t,
                                       ctypes.POINTER(ctypes.c_uint8)]
    return lib


_lib = None


def _get():
    global _lib
    if _lib is None:
        _lib = load()
    return _lib


def _check_buf(a: np.ndarray) -> np.ndarray:
    if a.dtype != np.uint8 or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("buffers must be contiguous uint8 arrays")
    return a


def _ptrs(arrs):
    return (ctypes.c_void_p * len(arrs))(*[a.ctypes.data if a.size else None for a in arrs])


def allgather(ins, lib=None):
    """W send buffers of equal size B -> W receive buffers of W*B bytes."""
    lib = lib or _get()
    ins = [_check_buf(a) for a in ins]
    W = len(ins)
    B = ins[0].size
    if any(a.size != B for a in ins):
        raise ValueError("all-gather needs equal per-rank sizes")
    outs = [np.zeros(W * B, dtype=np.uint8) for _ in range(W)]
    rc = lib.ref_allgather(_ptrs(ins), _ptrs(outs), W, B)
    if rc:
        raise RuntimeError(f"ref_allgather failed: {rc}")
    return outs


def alltoall(ins, C, lib=None):
    """ins[i] has sum_j C[i][j] bytes; returns outs[j] with sum_i C[i][j] bytes."""
    lib = lib or _get()
    ins = [_check_buf(a) for a in ins]
    W = len(ins)
    C = np.ascontiguousarray(np.asarray(C, dtype=np.uint64))
    if C.shape != (W, W):
        raise ValueError("chunk matrix must be W x W")
    for i in range(W):
        if ins[i].size != int(C[i].sum()):
            raise ValueError("send buffer size does not match its row of the chunk matrix")
    outs = [np.zeros(int(C[:, j].sum()), dtype=np.uint8) for j in range(W)]
    Cc = C.astype(np.uintp)
    rc = lib.ref_alltoall(_ptrs(ins), _ptrs(outs), W, Cc.ctypes.data_as(ctypes.POINTER(ctypes.c_size_t)))
    if rc:
        raise RuntimeError(f"ref_alltoall failed: {rc}")
    return outs


def broadcast(src, k, lib=None):
    """k fresh destination buffers, each receiving ``src``."""
    lib = lib or _get()
    src = _check_buf(src)
    dsts = [np.zeros(src.size, dtype=np.uint8) for _ in range(k)]
    rc = lib.ref_broadcast(src.ctypes.data if src.size else None, _ptrs(dsts), k, src.size)
    if rc:
        raise RuntimeError(f"ref_broadcast failed: {rc}")
    return dsts


def _descs(buffers, descs):
    arr = (RefCopy * max(len(descs), 1))()
    for n, (sb, so, db, do, nb) in enumerate(descs):
        sbuf, dbuf = _check_buf(buffers[sb]), _check_buf(buffers[db])
        so, do, nb = int(so), int(do), int(nb)
        if so + nb > sbuf.size or do + nb > dbuf.size:
            raise ValueError("descriptor outside its buffer")
        arr[n].src = sbuf.ctypes.data + so
        arr[n].dst = dbuf.ctypes.data + do
        arr[n].bytes = nb
    return arr


def batch_copy(buffers, descs, lib=None):
    """Run a hazard-free batch in place on ``buffers``.

    descs: iterable of (src_buffer_index, src_offset, dst_buffer_index,
    dst_offset, bytes).  Raises ValueError if the batch has a hazard.
    """
    lib = lib or _get()
    descs = list(descs)
    arr = _descs(buffers, descs)
    rc = lib.ref_batch_copy(arr, len(descs))
    if rc == -2:
        raise ValueError("batch has a data-dependence hazard")
    if rc:
        raise RuntimeError(f"ref_batch_copy failed: {rc}")
    return buffers


def first_hazard(buffers, descs, lib=None) -> int:
    """Index of the first copy whose destination collides, or -1."""
    lib = lib or _get()
    descs = list(descs)
    return int(lib.ref_first_hazard(_descs(buffers, descs), len(descs)))


def batch_swap(buffers, descs, lib=None):
    """Run a batch of swaps in place on ``buffers``.

    descs: iterable of (a_buffer_index, a_offset, b_buffer_index, b_offset,
    bytes).  Raises ValueError if two ranges of the batch overlap.
    """
    lib = lib or _get()
    descs = list(descs)
    arr = (RefSwap * max(len(descs), 1))()
    for n, (ab, ao, bb, bo, nb) in enumerate(descs):
        abuf, bbuf = _check_buf(buffers[ab]), _check_buf(buffers[bb])
        ao, bo, nb = int(ao), int(bo), int(nb)
        if ao + nb > abuf.size or bo + nb > bbuf.size:
            raise ValueError("descriptor outside its buffer")
        arr[n].a = abuf.ctypes.data + ao
        arr[n].b = bbuf.ctypes.data + bo
        arr[n].bytes = nb
    rc = lib.ref_batch_swap(arr, len(descs))
    if rc == -2:
        raise ValueError("two ranges of the batch overlap")
    if rc:
        raise RuntimeError(f"ref_batch_swap failed: {rc}")
    return buffers


def alltoall_inplace(bufs, chunk_bytes, lib=None):
    """In-place all-to-all with equal chunks on copies of ``bufs`` (W buffers
    of W * chunk_bytes bytes); returns the new buffers."""
    lib = lib or _get()
    W, c = len(bufs), int(chunk_bytes)
    outs = [_check_buf(a).copy() for a in bufs]
    if any(a.size != W * c for a in outs):
        raise ValueError("every buffer must hold W chunks")
    rc = lib.ref_alltoall_inplace(_ptrs(outs), W, c)
    if rc:
        raise RuntimeError(f"ref_alltoall_inplace failed: {rc}")
    return outs


def token_dispatch(ins, row_bytes, dest, lib=None):
    """ins[i]: tokens_i rows of ``row_bytes`` bytes.  dest: (total tokens, W)
    array, non-zero where a token goes to a rank.  Returns the W receive
    buffers, rows packed in token order."""
    lib = lib or _get()
    ins = [_check_buf(a) for a in ins]
    W, row_bytes = len(ins), int(row_bytes)
    tokens = np.array([a.size // row_bytes if row_bytes else 0 for a in ins], dtype=np.uint32)
    if any(a.size != int(t) * row_bytes for a, t in zip(ins, tokens)):
        raise ValueError("send buffers must hold whole rows")
    dest = np.ascontiguousarray(np.asarray(dest, dtype=np.uint8))
    if dest.shape != (int(tokens.sum()), W):
        raise ValueError("dest must be (total tokens, W)")
    outs = [np.zeros(int((dest[:, j] != 0).sum()) * row_bytes, dtype=np.uint8) for j in range(W)]
    rc = lib.ref_token_dispatch(_ptrs(ins), _ptrs(outs), W, tokens.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)),
                                row_bytes, dest.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    if rc:
        raise RuntimeError(f"ref_token_dispatch failed: {rc}")
    return outs
