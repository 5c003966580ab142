#!/usr/bin/env python3
"""Benchmark of the MI355X copy collectives.

Workload (one "step"): the all-gather size sweep over W = 8 virtual ranks on one
GPU, per-rank payload 4 KiB ... 64 MiB in powers of two (15 calls), bf16 values
~N(0,1) from a seeded generator, one receive buffer of W x payload per rank.
All buffers are resident in HBM before the timed region starts.

Prints ONE short JSON line (per-size rows and the comparison legs go to
--detail-file).  `value` is algorithmic (read + write) bytes per second
over the timed steps: an all-gather of B bytes per rank reads W*B and writes
W*W*B bytes (each source is read once and written W times).
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

W = 8
KiB, MiB = 1024, 1024 * 1024
RUNTIME_COPY_SIZES = (4 * KiB, 64 * KiB, MiB, 16 * MiB)   # per-rank sizes at which the runtime's own copy calls are timed
HBM_PEAK_GBS = 8000.0


# HBM bytes per launch of the dominant kernel (all-gather, 64 MiB per rank) from hardware counters:
# FETCH_SIZE and WRITE_SIZE of two rocprofv3 --pmc runs, each scaled by the same counter's reading
# for a plain copy of known size.  Valid only for the kernel sources whose digest is given; with
# any other sources the figure is reported as null until the counters are taken again.
KERNEL_SOURCES = ["dl_work.h", "dl_device.h", "dl_exec.hip"]
MEASURED_TRAFFIC = {"sources_sha256": "75a52d98d113b89d66940941dec8f515c05644e8ee7db06877cba48dfc5a87d6", "bytes_per_rank": 64 * MiB, "bytes_per_launch": 4831886239}


def kernel_sources_digest() -> str:
    """Digest of the kernel sources' code: comments and white space do not count."""
    import hashlib
    import re
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2511_06605_amd", "csrc", name), "r") as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)      # block comments
        text = re.sub(r"//[^\n]*", " ", text)                   # line comments (no string in these files holds "//")
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()


def ag_bytes(B: int) -> int:
    return W * B + W * W * B


def pct(xs, q):
    xs = sorted(xs)
    return xs[min(len(xs) - 1, int(q * len(xs)))]


def host_cores() -> int:
    """Cores this process may run on (the scheduler's view, and the box's thread setting if it is narrower)."""
    n = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    try:
        n = min(n, max(1, int(os.environ.get("OMP_NUM_THREADS", n))))
    except ValueError:
        pass
    return max(1, n)


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(sizes, budget_s=6.0):
    """The CPU checker as it stands (plain memcpy, single-threaded source), timed on the host on the whole sweep:
    once from one thread, once from T threads that each call the checker's broadcast on a slice of one source
    (disjoint destinations; the foreign calls run outside the interpreter lock).  One buffer set sized for the
    largest point serves every point (the smaller ones use its front), touched before timing; if the host's
    free memory does not hold it, the largest points are left out and the cap is stated."""
    import ctypes
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np
    from oracle import ref

    ref.build()
    lib = ref.load()
    try:
        avail = os.sysconf("SC_AVPHYS_PAGES") * os.sysconf("SC_PAGE_SIZE")
    except (ValueError, OSError):
        avail = 16 << 30
    sample = [B for B in sizes if (W + W * W) * B <= avail // 3]
    cap_note = "" if len(sample) == len(sizes) else \
        f"; points above {sample[-1] // MiB} MiB per rank left out: {avail / 2**30:.0f} GiB of host memory free"
    big = sample[-1]
    rng = np.random.default_rng(0)
    ins = [rng.integers(0, 256, big, dtype=np.uint8) for _ in range(W)]
    outs = [np.empty(W * big, dtype=np.uint8) for _ in range(W)]   # first touched by the untimed pass below
    pi, po = ref._ptrs(ins), ref._ptrs(outs)
    T = host_cores()

    def one_thread(B):
        assert lib.ref_allgather(pi, po, W, B) == 0

    pool = ThreadPoolExecutor(T)

    def piece(j, B, off, n):
        dsts = (ctypes.c_void_p * W)(*[outs[r].ctypes.data + j * B + off for r in range(W)])
        assert lib.ref_broadcast(ins[j].ctypes.data + off, dsts, W, n) == 0

    def threads(B):
        parts = max(1, min(-(-T // W), B // 4096))      # slices per source: T tasks in all, none under 4 KiB
        cut = -(-B // parts)
        jobs = [pool.submit(piece, j, B, off, min(cut, B - off)) for j in range(W) for off in range(0, B, cut)]
        for f in jobs:
            f.result()

    def leg(fn):
        moved, passes, big_s = 0, 0, []
        t0 = time.perf_counter()
        while True:
            for B in sample:
                t1 = time.perf_counter()
                fn(B)
                if B == big:
                    big_s.append(time.perf_counter() - t1)
                moved += ag_bytes(B)
            passes += 1
            if time.perf_counter() - t0 >= budget_s:
                break
        dt = time.perf_counter() - t0
        return moved / dt / 1e9, ag_bytes(big) / min(big_s) / 1e9, passes, dt

    threads(big)   # untimed: brings every page of the receive buffers in, from all cores at once
    v1, big1, p1, dt1 = leg(one_thread)
    vt, bigt, pt, dtt = leg(threads)
    pool.shutdown()
    # every output must hold the concatenation (the threaded leg ran last)
    for r in (0, W - 1):
        for j in (0, W - 1):
            assert np.array_equal(outs[r][j * big:(j + 1) * big], ins[j]), "CPU baseline result is wrong"
    return {
        "value": vt, "unit": "GB/s", "cores": T, "kind": "oracle",
        "single_thread": v1, "threads": vt,
        f"single_thread_{big // MiB}MiB": big1, f"threads_{big // MiB}MiB": bigt,
        "cpu": cpu_model(), "host_cpus": os.cpu_count(),
        "sample": f"all-gather sweep {sample[0] // KiB} KiB..{big // MiB} MiB per rank (W=8): {p1} passes in {dt1:.1f} s "
                  f"from one thread, {pt} passes in {dtt:.1f} s from {T} threads (each a broadcast of a source slice "
                  f"by the checker){cap_note}",
    }


def runtime_batch_comparison():
    """hipMemcpyBatchAsync on the all-gather's 64 block copies, run by the comparison program that links the
    ROCm installation's HIP runtime (the runtime PyTorch brings along does not export the call)."""
    import subprocess
    from bench_aid import build as aid_build
    exe = aid_build.RUNTIME_BATCH
    if not os.path.exists(exe):
        return {"error": "comparison program not built"}
    try:
        r = subprocess.run([exe] + [str(B) for B in RUNTIME_COPY_SIZES], capture_output=True, text=True, timeout=120)
        return json.loads(r.stdout.strip().splitlines()[-1])
    except Exception as e:   # a comparison leg: report, never fail the benchmark
        return {"error": f"{type(e).__name__}: {e}"}


def short(x):
    """Floats to five significant digits (the printed line is read back whole by the caller's harness)."""
    if isinstance(x, float):
        return float(f"{x:.5g}")
    if isinstance(x, dict):
        return {k: short(v) for k, v in x.items()}
    if isinstance(x, (list, tuple)):
        return [short(v) for v in x]
    return x


def lat_stats(lat):
    return {"p50": pct(lat, .5), "p10": pct(lat, .1), "p90": pct(lat, .9)}


def other_operations(dl, benchaid, inputs, torch, stream, ag_reqs, ag_bufs, ag_sizes, runtime_batch):
    """The other operations of the library and the runtime's own copy paths, timed
    beside the all-gather sweep (context, not part of `value`)."""
    import numpy as np

    res = {}

    def dev(t):
        return torch.from_numpy(t).cuda()

    armed_cases = []   # (row, request, buffers kept alive): timed again in prelaunch and signal mode at the end

    def timed(req, nbytes, small, calls=None):
        us = benchaid.time_device(req, stream, warmup=3, calls=calls or (50 if small else 10))
        row = {"device_us": us, "GBps": nbytes / us / 1e3}
        if small:
            row["oneshot_host_us"] = lat_stats(benchaid.time_host(req, stream, benchaid.WAIT_STREAM, 30, 300))
        return row

    # runtime copy engines / blit path: one hipMemcpyAsync per chunk (W*W calls + one sync), and the batched call
    rows = []
    for B, (d_in, d_out) in zip(ag_sizes, ag_bufs):
        if B not in RUNTIME_COPY_SIZES:
            continue
        descs = [(d_in[j].data_ptr(), d_out[r].data_ptr() + j * B, B) for r in range(W) for j in range(W)]
        row = {"bytes_per_rank": B}
        req = benchaid.copy_list_request(descs, benchaid.OP_MEMCPY_ASYNC)
        row["memcpy_async_per_chunk_host_us"] = lat_stats(benchaid.time_host(req, stream, benchaid.WAIT_STREAM, 5, 50))
        row["memcpy_async_per_chunk_device_us"] = benchaid.time_device(req, stream, warmup=2, calls=5)
        try:
            req = benchaid.copy_list_request(descs, benchaid.OP_MEMCPY_BATCH)
            row["memcpy_batch_host_us"] = lat_stats(benchaid.time_host(req, stream, benchaid.WAIT_STREAM, 5, 50))
        except RuntimeError as e:
            row["memcpy_batch_host_us"] = f"unavailable in the loaded HIP runtime ({e})"
        # the same call and the per-chunk calls under the ROCm installation's runtime, from the comparison program
        if runtime_batch and "rows" in runtime_batch:
            for other in runtime_batch["rows"]:
                if other["bytes_per_rank"] == B:
                    row["rocm_runtime_%s" % runtime_batch["runtime_version"]] = {k: v for k, v in other.items()
                                                                                 if k != "bytes_per_rank"}
        elif runtime_batch:
            row["rocm_runtime"] = runtime_batch
        req = benchaid.copy_list_request(descs, benchaid.OP_BATCH)   # same 64 plain copies through dl_batch_copy
        dl.dl_set_config(infer_broadcast=0)                          # ... kept as 64 copies (each source re-read 8 times)
        row["dl_batch_copy_unfused"] = timed(req, 2 * W * W * B, B <= MiB)
        dl.dl_set_config(infer_broadcast=1)                          # ... merged back into 8 read-once/write-8 copies
        row["dl_batch_copy_inferred_broadcast"] = timed(req, ag_bytes(B), B <= MiB)
        rows.append(row)
    res["allgather_vs_runtime_copies"] = rows

    # all-to-all, uniform per-pair chunk, fp16 ~N(0,1)
    rows = []
    for c in [KiB << i for i in range(13)]:
        C = inputs.uniform_chunks(W, c)
        ins = inputs.alltoall_inputs(C, seed=c.bit_length(), kind="fp16")
        d_in = [dev(a) for a in ins]
        d_out = [torch.empty(W * c, dtype=torch.uint8, device="cuda") for _ in range(W)]
        req = benchaid.alltoall_request(d_in, d_out, C)
        row = {"chunk_bytes": c}
        row.update(timed(req, 2 * W * W * c, c <= 128 * KiB))
        if 64 * KiB <= c:
            # cold: buffer sets of this size rotated so that a pass moves 1 GiB
            sets = max(3, min(48, -(-(1 << 30) // (2 * W * W * c))))
            spare, ring = [], [req]
            for _ in range(sets - 1):
                e_in = [torch.empty(W * c, dtype=torch.uint8, device="cuda").random_(0, 256) for _ in range(W)]
                e_out = [torch.empty(W * c, dtype=torch.uint8, device="cuda") for _ in range(W)]
                spare.append((e_in, e_out))
                ring.append(benchaid.alltoall_request(e_in, e_out, C))
            stream.synchronize()
            us = benchaid.time_device_rotating(ring, stream, 1, 3)
            row["cold"] = {"buffer_sets": sets, "device_us": us, "GBps": 2 * W * W * c / us / 1e3,
                           "frac_of_hbm_peak": 2 * W * W * c / us / 1e3 / HBM_PEAK_GBS}
            del spare, ring
        rows.append(row)
        if c <= 128 * KiB:
            armed_cases.append((row, req, (d_in, d_out)))
    res["alltoall_uniform"] = rows

    # in-place all-to-all (one swap per pair of ranks): every off-diagonal chunk is read once and written once
    rows = []
    for c in [KiB << i for i in range(13)]:
        bufs = inputs.alltoall_inputs(inputs.uniform_chunks(W, c), seed=c.bit_length(), kind="fp16")
        d_buf = [dev(a) for a in bufs]
        req = benchaid.alltoall_inplace_request(d_buf, c)
        row = {"chunk_bytes": c}
        row.update(timed(req, 2 * W * (W - 1) * c, c <= 128 * KiB, calls=(50 if c <= 128 * KiB else 10)))
        rows.append(row)
        if c <= 128 * KiB:
            armed_cases.append((row, req, d_buf))
    res["alltoall_inplace_uniform"] = rows

    # MoE dispatch all-to-all: hidden 7168 bf16, 256 experts over 8 ranks, top-8
    rows = []
    for T in (16, 128, 512):
        C = inputs.moe_dispatch_chunks(W, T, seed=T)
        ins = inputs.alltoall_inputs(C, seed=T + 1, kind="bf16")
        d_in = [dev(a) for a in ins]
        d_out = [torch.empty(int(C[:, j].sum()), dtype=torch.uint8, device="cuda") for j in range(W)]
        req = benchaid.alltoall_request(d_in, d_out, C)
        row = {"tokens_per_rank": T, "total_bytes": int(C.sum()), "zero_chunks": int((C == 0).sum())}
        row.update(timed(req, 2 * int(C.sum()), T <= 16))
        rows.append(row)
    res["alltoall_moe_dispatch"] = rows

    # token-granular MoE dispatch: every token row (14 KiB) is read once and written to the 1..8 ranks that own
    # its top-8 experts; bytes = rows read + rows written
    rows = []
    for T in (16, 128, 512):
        row_bytes = 14336
        dest = inputs.moe_token_destinations(W, T, seed=T)
        ins = inputs.token_rows(W, T, row_bytes, seed=T + 1, kind="bf16")
        d_in = [dev(a) for a in ins]
        d_out = [torch.empty(int(dest[:, j].sum()) * row_bytes, dtype=torch.uint8, device="cuda") for j in range(W)]
        req = benchaid.token_dispatch_request(d_in, d_out, [T] * W, row_bytes, dest)
        nbytes = (W * T + int(dest.sum())) * row_bytes
        row = {"tokens_per_rank": T, "row_bytes": row_bytes, "copies": int(dest.sum()),
               "mean_fanout": float(dest.sum()) / (W * T)}
        # the whole call: from 512 tokens on only the mask goes to the device, which builds the copy list itself
        # (a long warm-up: the GPU idled while the host prepared the inputs, and its first two milliseconds of work
        # after that run slower)
        row["call_to_sync_host_us"] = lat_stats(benchaid.time_host(req, stream, benchaid.WAIT_STREAM, 200, 200))
        row["GBps_call_to_sync"] = nbytes / row["call_to_sync_host_us"]["p50"] / 1e3
        # the same request lowered on the host: the lowering alone, and the whole call with device lowering off
        lowered, row["host_lowering_us"] = benchaid.lowered_token_dispatch(req)
        row["items"] = lowered.req.n
        dl.dl_set_config(device_lowering=0)
        row["host_lowered_call_to_sync_us"] = lat_stats(benchaid.time_host(req, stream, benchaid.WAIT_STREAM, 50, 200))
        dl.dl_set_config(device_lowering=1)
        # the routing mask already in device memory (where a router kernel leaves it): nothing crosses the host link
        d_mask = torch.from_numpy(np.ascontiguousarray(dest)).cuda()
        dreq = benchaid.token_dispatch_device_request(d_in, d_out, [T] * W, row_bytes, d_mask)
        row["mask_in_device_memory_call_to_sync_us"] = lat_stats(benchaid.time_host(dreq, stream, benchaid.WAIT_STREAM, 50, 200))
        row["mask_in_device_memory_device_us"] = benchaid.time_device(dreq, stream, warmup=3, calls=20)
        rows.append(row)
    res["token_dispatch_moe"] = rows

    # tensor-parallel decode all-gather: hidden 8192 bf16
    rows = []
    for tokens in (1, 8, 32, 128, 256):
        B = inputs.tp_decode_bytes_per_rank(tokens)
        ins = inputs.allgather_inputs(W, B, seed=tokens, kind="bf16")
        d_in = [dev(a) for a in ins]
        d_out = [torch.empty(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)]
        req = benchaid.allgather_request(d_in, d_out, B)
        row = {"tokens": tokens, "bytes_per_rank": B}
        row.update(timed(req, ag_bytes(B), True))
        rows.append(row)
        armed_cases.append((row, req, (d_in, d_out)))
    res["allgather_tp_decode"] = rows

    # KV-cache fetch: 256 dispersed blocks per request, pinned host pool -> device pool (over the host link),
    # and the paged device -> device variant; one dl_batch_copy against one hipMemcpyAsync per block
    rows = []
    n_blk = 256
    for blk in (16 * KiB, 64 * KiB, 256 * KiB, MiB, 4 * MiB):
        pairs = inputs.kv_fetch_blocks(n_blk, 320, 320, seed=blk.bit_length())
        host_pool = torch.empty(320 * blk, dtype=torch.uint8, pin_memory=True)
        host_pool.random_(0, 256)
        dev_pool = torch.empty(320 * blk, dtype=torch.uint8, device="cuda")
        dev_src = torch.randint(0, 256, (320 * blk,), dtype=torch.uint8, device="cuda")
        row = {"blocks": n_blk, "block_bytes": blk}
        for name, base in (("host_to_device", host_pool.data_ptr()), ("device_to_device", dev_src.data_ptr())):
            dlist = [(base + int(a) * blk, dev_pool.data_ptr() + int(b) * blk, blk) for a, b in pairs]
            nbytes = n_blk * blk * (1 if name == "host_to_device" else 2)   # host link: bytes delivered; HBM: read + write
            req = benchaid.copy_list_request(dlist, benchaid.OP_BATCH)
            us = benchaid.time_device(req, stream, warmup=2, calls=5)
            sub = {"dl_batch_copy_device_us": us, "dl_batch_copy_GBps": nbytes / us / 1e3,
                   "dl_batch_copy_host_us": lat_stats(benchaid.time_host(req, stream, benchaid.WAIT_STREAM, 3, 20))}
            req = benchaid.copy_list_request(dlist, benchaid.OP_MEMCPY_ASYNC)
            sub["memcpy_async_per_block_host_us"] = lat_stats(benchaid.time_host(req, stream, benchaid.WAIT_STREAM, 2, 10))
            sub["memcpy_async_per_block_GBps"] = nbytes / sub["memcpy_async_per_block_host_us"]["p50"] / 1e3
            row[name] = sub
        rows.append(row)
        del host_pool, dev_pool, dev_src
    res["kv_fetch"] = rows

    # broadcast 2 MiB -> 7 destinations; 64 back-to-back copies of 16 KiB in a 64 MiB arena
    n = 2 * MiB
    src = dev(inputs.payload(np.random.default_rng(7), n, "bf16"))
    dsts = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(7)]
    row = {"bytes": n, "k": 7}
    req = benchaid.broadcast_request(src, dsts, n)
    row.update(timed(req, 8 * n, True))
    armed_cases.append((row, req, (src, dsts)))
    res["broadcast"] = row
    arena_h, descs = inputs.b2b_batch(64, 16 * KiB, 64 * MiB, seed=3)
    arena = dev(arena_h)
    p = arena.data_ptr()
    dlist = [(p + int(a), p + int(b), int(m)) for a, b, m in descs]
    row = {"copies": 64, "copy_bytes": 16 * KiB}
    row.update(timed(benchaid.copy_list_request(dlist, benchaid.OP_BATCH), 2 * 64 * 16 * KiB, True))
    req = benchaid.copy_list_request(dlist, benchaid.OP_MEMCPY_ASYNC)
    row["memcpy_async_per_copy_host_us"] = lat_stats(benchaid.time_host(req, stream, benchaid.WAIT_STREAM, 5, 50))
    armed_cases.append((row, benchaid.copy_list_request(dlist, benchaid.OP_BATCH), arena))
    res["batch_b2b"] = row

    # requests that do not stand on any grid: an all-gather of 16 MiB - 32 bytes per rank (so that every rank's share
    # of a receive buffer begins off the 128-byte lines) with the send and receive buffers moved by a few bytes, and
    # 64 copies of 4 MiB - 32 bytes; GB/s of algorithmic read + write traffic
    rows = []
    n = 16 * MiB - 32
    s_in = [torch.empty(n + 256, dtype=torch.uint8, device="cuda").random_(0, 256) for _ in range(W)]
    s_out = [torch.empty(W * n + 256, dtype=torch.uint8, device="cuda") for _ in range(W)]
    # (fresh buffers, and the device has idled while they were filled: 150 untimed calls, 30 ms, first, or the first rows read 8 % low)
    benchaid.time_device(benchaid.allgather_request(s_in, s_out, n), stream, warmup=150, calls=1)
    for so, do in ((0, 0), (4, 0), (1, 0), (0, 1), (5, 2), (0, 16)):
        req = benchaid.allgather_request([t[so:] for t in s_in], [t[do:] for t in s_out], n)
        row = {"op": "allgather", "bytes_per_rank": n, "send_shift": so, "recv_shift": do}
        row.update(timed(req, (W + W * W) * n, False, calls=20))
        rows.append(row)
    del s_in, s_out
    n = 4 * MiB - 32
    c_in = [torch.empty(n + 256, dtype=torch.uint8, device="cuda").random_(0, 256) for _ in range(64)]
    c_out = [torch.empty(n + 256, dtype=torch.uint8, device="cuda") for _ in range(64)]
    for so, do in ((0, 0), (1, 0), (0, 1), (7, 2)):
        req = benchaid.copy_list_request([(x[so:], y[do:], n) for x, y in zip(c_in, c_out)], benchaid.OP_BATCH)
        row = {"op": "batch_copy", "copies": 64, "copy_bytes": n, "src_shift": so, "dst_shift": do}
        row.update(timed(req, 2 * 64 * n, False, calls=20))
        rows.append(row)
    del c_in, c_out
    res["off_grid"] = rows

    # the latency-bound cases again in prelaunch mode (doorbell -> completion word) and in signal mode
    # (call -> completion word, no stream synchronisation); before the sections below create further streams:
    # a waiting kernel holds the hardware queue of its stream, and more streams than queues would share them
    dl.dl_prelaunch_start()
    for row, req, _keep in armed_cases:
        dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
        row["prelaunch_trigger_to_done_us"] = lat_stats(benchaid.time_host(req, None, benchaid.WAIT_TRIGGER, 30, 300))
        dl.dl_set_mode(dl.DL_MODE_SIGNAL)
        row["signal_call_to_done_us"] = lat_stats(benchaid.time_host(req, None, benchaid.WAIT_SIGNAL, 30, 300))
        # requests short enough for a kernel that already waits (standby mode): decode all-gathers up to 32 tokens,
        # all-to-alls with chunks up to 8 KiB
        if row.get("tokens", 99) <= 32 or row.get("chunk_bytes", 1 << 30) <= 8 * KiB:
            dl.dl_set_mode(dl.DL_MODE_STANDBY)
            row["standby_call_to_done_us"] = lat_stats(benchaid.time_host(req, None, benchaid.WAIT_SIGNAL, 30, 300))
    dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    dl.dl_prelaunch_stop()

    # a decode step's worth of collectives (32 all-gathers of 8 tokens x hidden 8192 bf16, buffers of their own)
    # issued one by one and replayed from a HIP graph captured once; microseconds per step, call -> synchronised
    L, B = 32, inputs.tp_decode_bytes_per_rank(8)
    layers = [([torch.zeros(B, dtype=torch.uint8, device="cuda") for _ in range(W)],
               [torch.empty(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)]) for _ in range(L)]
    ptrs = [([t.data_ptr() for t in i], [t.data_ptr() for t in o]) for i, o in layers]

    def issue_all(st):
        for i, o in ptrs:
            dl.dl_allgather(i, o, B, st)

    def host_us(fn, reps=60):
        lat = []
        for r in range(reps + 10):
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            if r >= 10:
                lat.append((time.perf_counter() - t0) * 1e6)
        return lat_stats(lat)

    side = torch.cuda.Stream()
    side.wait_stream(stream)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        issue_all(torch.cuda.current_stream())
    res["decode_step_32_allgathers"] = {
        "bytes_per_rank": B, "collectives": L,
        "eager_calls_through_the_python_binding_us": host_us(lambda: issue_all(stream)),
        "graph_replay_us": host_us(graph.replay),
    }

    # the price of copying on compute units (the paper's motive for DMA offload, Sec. I): a bf16 GEMM 8192^3 on one
    # stream, all-gathers of 16 MiB per rank back to back on another for as long as the GEMMs run
    B = 16 * MiB
    ag_req, ag_keep = None, None
    for size, bufs in zip(ag_sizes, ag_bufs):
        if size == B:
            ag_req, ag_keep = ag_reqs[B], bufs
    if ag_req is not None:
        n = 8192
        ga = torch.randn(n, n, dtype=torch.bfloat16, device="cuda")
        gb = torch.randn(n, n, dtype=torch.bfloat16, device="cuda")
        gc = torch.empty(n, n, dtype=torch.bfloat16, device="cuda")
        other = torch.cuda.Stream()

        def gemms(k):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(k):
                torch.matmul(ga, gb, out=gc)
            e1.record(stream)
            return e0, e1

        torch.matmul(ga, gb, out=gc)
        torch.cuda.synchronize()
        e0, e1 = gemms(10)
        torch.cuda.synchronize()
        gemm_alone = e0.elapsed_time(e1) * 1e2
        ag_alone = benchaid.time_device(ag_req, other, warmup=2, calls=10)
        e0, e1 = gemms(10)
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s0.record(other)
        issued = 0
        while not e1.query() and issued < 1000:
            benchaid.issue(ag_req, other)
            issued += 1
            if issued % 4 == 0:
                other.synchronize()
        s1.record(other)
        torch.cuda.synchronize()
        res["overlap_with_gemm"] = {
            "gemm": "bf16 8192 x 8192 x 8192 (torch.matmul)", "allgather_bytes_per_rank": B,
            "gemm_alone_us": gemm_alone, "allgather_alone_us": ag_alone,
            "gemm_beside_allgathers_us": e0.elapsed_time(e1) * 1e2,
            "allgather_beside_gemm_us": s0.elapsed_time(s1) * 1e3 / max(issued, 1), "allgathers_issued": issued,
        }

    return res


def pmc_case(args, dl, benchaid, torch, stream) -> int:
    """A few launches of the dominant kernel (all-gather at the largest sweep
    point: dl_exec_rows_kernel<dl_fused_item,...>) and of a plain copy of known
    size (dl_exec_rows_kernel<dl_plain_item,...>: reads 1 GiB, writes 1 GiB) so
    that counter readings of the first can be scaled by those of the second."""
    B = args.max_bytes
    d_in = [torch.randint(0, 256, (B,), dtype=torch.uint8, device="cuda") for _ in range(W)]
    d_out = [torch.empty(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)]
    ag = benchaid.allgather_request(d_in, d_out, B)
    n = 1 << 30
    a = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
    b = torch.empty(n, dtype=torch.uint8, device="cuda")
    cp = benchaid.copy_list_request([(a.data_ptr(), b.data_ptr(), n)], benchaid.OP_BATCH)
    # the calibration copy with ordinary loads and stores, like the kernel that is being calibrated (a plain list
    # of this size would use streaming ones by default)
    dl.dl_set_config(stream_plain_min_bytes=(1 << 64) - 1)
    stream.synchronize()
    for _ in range(args.warmup + args.steps):
        benchaid.issue(ag, stream)
        benchaid.issue(cp, stream)
    stream.synchronize()
    dl.dl_shutdown()
    print(json.dumps({"case": "pmc", "launches_each": args.warmup + args.steps,
                      "allgather": {"bytes_per_rank": B, "algorithmic_read": W * B, "algorithmic_write": W * W * B},
                      "copy": {"read": n, "write": n}}))
    return 0


def token_case(args, dl, benchaid, inputs, torch, stream) -> int:
    """Only the token-granular MoE dispatch (W = 8, 14 KiB rows, top-8 of 256 experts), --steps calls per
    tokens-per-rank point with a synchronisation after each: for kernel traces of the table kernels."""
    row_bytes = 14336
    for T in (16, 128, 512):
        dest = inputs.moe_token_destinations(W, T, seed=T)
        ins = inputs.token_rows(W, T, row_bytes, seed=T + 1, kind="bf16")
        d_in = [torch.from_numpy(a).cuda() for a in ins]
        d_out = [torch.empty(int(dest[:, j].sum()) * row_bytes, dtype=torch.uint8, device="cuda") for j in range(W)]
        req = benchaid.token_dispatch_request(d_in, d_out, [T] * W, row_bytes, dest)
        for _ in range(args.warmup + args.steps):
            benchaid.issue(req, stream)
            stream.synchronize()
    dl.dl_shutdown()
    print(json.dumps({"case": "token_dispatch", "calls_per_point": args.warmup + args.steps}))
    return 0


def alltoall_case(args, dl, benchaid, inputs, torch, stream) -> int:
    """Only the all-to-all sweep (W = 8, uniform chunks 1 KiB .. 4 MiB, fp16) and the MoE dispatch all-to-all
    (tokens per rank 16 / 128 / 512), every point with buffers of its own, --steps passes over all points with
    one synchronisation per pass: for kernel traces."""
    reqs, keep = [], []
    for c in [KiB << i for i in range(13)]:
        C = inputs.uniform_chunks(W, c)
        ins = inputs.alltoall_inputs(C, seed=c.bit_length(), kind="fp16")
        d_in = [torch.from_numpy(a).cuda() for a in ins]
        d_out = [torch.empty(W * c, dtype=torch.uint8, device="cuda") for _ in range(W)]
        reqs.append(benchaid.alltoall_request(d_in, d_out, C))
        keep.append((d_in, d_out))
    for T in (16, 128, 512):
        C = inputs.moe_dispatch_chunks(W, T, seed=T)
        ins = inputs.alltoall_inputs(C, seed=T + 1, kind="bf16")
        d_in = [torch.from_numpy(a).cuda() for a in ins]
        d_out = [torch.empty(int(C[:, j].sum()), dtype=torch.uint8, device="cuda") for j in range(W)]
        reqs.append(benchaid.alltoall_request(d_in, d_out, C))
        keep.append((d_in, d_out))
    for _ in range(args.warmup + args.steps):
        for r in reqs:
            benchaid.issue(r, stream)
        stream.synchronize()
    dl.dl_shutdown()
    print(json.dumps({"case": "alltoall", "passes": args.warmup + args.steps}))
    return 0


def armed_case(args, dl, benchaid, inputs, torch, stream) -> int:
    """The kernels behind the latency figures (Sec. IV-E on compute units): all-gathers of 4 KiB .. 4 MiB per rank,
    each armed, seen resident, triggered and waited for --steps times in prelaunch mode, then issued --steps times in
    signal mode and (where they fit a waiting kernel) in standby mode.  Prints host-observed medians; meant to
    run under a kernel trace."""
    rows = []
    reqs = []
    for B in [4 * KiB << i for i in range(11)]:
        ins = inputs.allgather_inputs(W, B, seed=B.bit_length() - 1, kind="bf16")
        d_in = [torch.from_numpy(a).cuda() for a in ins]
        d_out = [torch.empty(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)]
        reqs.append((B, benchaid.allgather_request(d_in, d_out, B), (d_in, d_out)))
    stream.synchronize()
    dl.dl_prelaunch_start()
    for B, req, _keep in reqs:
        row = {"bytes_per_rank": B}
        dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
        row["prelaunch_trigger_to_done_us"] = pct(benchaid.time_host(req, None, benchaid.WAIT_TRIGGER, args.warmup, args.steps), .5)
        dl.dl_set_mode(dl.DL_MODE_SIGNAL)
        row["signal_call_to_done_us"] = pct(benchaid.time_host(req, None, benchaid.WAIT_SIGNAL, args.warmup, args.steps), .5)
        if W * B <= 64 * 8192:
            dl.dl_set_mode(dl.DL_MODE_STANDBY)
            row["standby_call_to_done_us"] = pct(benchaid.time_host(req, None, benchaid.WAIT_SIGNAL, args.warmup, args.steps), .5)
        rows.append(row)
    dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    dl.dl_prelaunch_stop()
    dl.dl_shutdown()
    print(json.dumps({"case": "armed", "calls_per_point_and_mode": args.warmup + args.steps, "rows": rows}))
    return 0


def off_grid_case(args, dl, benchaid, torch, stream) -> int:
    """Only requests that stand on no grid: all-gathers of 16 MiB - 32 bytes per rank (every rank's share of a receive
    buffer off the 128-byte lines) with send / receive buffers moved by 0, 4, 1 bytes, and 64 copies of 4 MiB - 32
    bytes with the source or the destination moved by one byte; --steps launches each: for kernel traces."""
    n = 16 * MiB - 32
    s_in = [torch.empty(n + 256, dtype=torch.uint8, device="cuda").random_(0, 256) for _ in range(W)]
    s_out = [torch.empty(W * n + 256, dtype=torch.uint8, device="cuda") for _ in range(W)]
    m = 4 * MiB - 32
    c_in = [torch.empty(m + 256, dtype=torch.uint8, device="cuda").random_(0, 256) for _ in range(64)]
    c_out = [torch.empty(m + 256, dtype=torch.uint8, device="cuda") for _ in range(64)]
    reqs = [("allgather send+%d recv+%d" % (so, do),
             benchaid.allgather_request([t[so:] for t in s_in], [t[do:] for t in s_out], n))
            for so, do in ((0, 0), (4, 0), (1, 0), (0, 1), (0, 16))]
    reqs += [("batch_copy src+%d dst+%d" % (so, do),
              benchaid.copy_list_request([(x[so:], y[do:], m) for x, y in zip(c_in, c_out)], benchaid.OP_BATCH))
             for so, do in ((0, 0), (1, 0), (0, 1))]
    rows = []
    benchaid.time_device(reqs[0][1], stream, warmup=150, calls=1)   # 30 ms of work: clocks up, buffers touched
    for name, req in reqs:
        us = benchaid.time_device(req, stream, warmup=max(args.warmup, 20), calls=args.steps)
        rows.append({"request": name, "device_us": us})
    dl.dl_shutdown()
    print(json.dumps({"case": "off_grid", "launches_per_request": max(args.warmup, 20) + args.steps,
                      "allgather_bytes_per_rank": n, "copy_bytes": m, "rows": rows}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--max-bytes", type=int, default=64 * MiB, help="largest per-rank payload of the sweep")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU baseline leg")
    ap.add_argument("--no-detail", action="store_true", help="skip per-size latency and comparison legs")
    ap.add_argument("--detail-file", default=os.path.join(ROOT, "gpurun_out", "bench_detail.json"),
                    help="where the per-size latency and comparison rows go (the printed line stays short)")
    ap.add_argument("--case", choices=["sweep", "pmc", "token_dispatch", "alltoall", "armed", "off_grid"], default="sweep",
                    help="pmc: only --steps launches of the largest all-gather and of a plain 1 GiB copy "
                         "(the calibration kernel), for hardware-counter runs; token_dispatch: only the "
                         "token-granular MoE dispatch, for kernel traces; armed: all-gathers of 4 KiB .. 4 MiB per "
                         "rank armed, triggered and waited for (prelaunch), then in signal and standby mode, for "
                         "kernel traces of the waiting kernels; off_grid: only all-gathers and copies whose buffers and "
                         "lengths stand on no grid, for kernel traces")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU (W virtual ranks share its HBM); --gpus must be 1",
              file=sys.stderr)
        return 2

    # the runtime's batched copy call, timed by a program of its own before this process touches the GPU
    runtime_batch = None
    if args.case == "sweep" and not args.no_detail:
        from bench_aid import build as aid_build
        if not os.path.exists(aid_build.RUNTIME_BATCH):
            try:
                aid_build.build()
            except Exception as e:   # a comparison leg: report, never fail the benchmark
                print(f"bench.py: comparison program did not build: {e}", file=sys.stderr)
        runtime_batch = runtime_batch_comparison()

    import numpy as np
    import torch

    import paper_2511_06605_amd as dl
    from paper_2511_06605_amd import inputs
    from bench_aid import benchaid, build as aid_build
    if not os.path.exists(aid_build.AID_LIB):   # normally built beforehand, with the library
        aid_build.build()

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dl.dl_init(0)
    stream = torch.cuda.current_stream()

    if args.case == "pmc":
        return pmc_case(args, dl, benchaid, torch, stream)
    if args.case == "token_dispatch":
        return token_case(args, dl, benchaid, inputs, torch, stream)
    if args.case == "alltoall":
        return alltoall_case(args, dl, benchaid, inputs, torch, stream)
    if args.case == "armed":
        return armed_case(args, dl, benchaid, inputs, torch, stream)
    if args.case == "off_grid":
        return off_grid_case(args, dl, benchaid, torch, stream)

    sizes = [B for B in (4 * KiB << i for i in range(15)) if B <= args.max_bytes]
    reqs, keep, check = {}, [], None
    for B in sizes:
        ins = inputs.allgather_inputs(W, B, seed=B.bit_length() - 1, kind="bf16")
        d_in = [torch.from_numpy(a).cuda() for a in ins]
        d_out = [torch.empty(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)]
        reqs[B] = benchaid.allgather_request(d_in, d_out, B)
        keep.append((d_in, d_out))
        if B == 64 * KiB or (check is None and B == sizes[-1]):
            check = (ins, d_out)
    stream.synchronize()
    big = sizes[-1]

    def step(ev=None):
        for B in sizes:
            if ev is not None and B == big:
                ev[0].record(stream)
                benchaid.issue(reqs[B], stream)
                ev[1].record(stream)
            else:
                benchaid.issue(reqs[B], stream)

    for _ in range(args.warmup):
        step()
    stream.synchronize()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    stream.synchronize()
    dt = time.perf_counter() - t0

    # result check on one sweep point against the CPU checker
    from oracle import ref
    want = ref.allgather(check[0])
    for r in range(W):
        assert np.array_equal(check[1][r].cpu().numpy(), want[r]), "all-gather result differs from the CPU checker"

    step_bytes = sum(ag_bytes(B) for B in sizes)
    value = step_bytes * args.steps / dt / 1e9
    big_ms = sum(a.elapsed_time(b) for a, b in events) / len(events)
    achieved = ag_bytes(big) / (big_ms * 1e-3) / 1e9
    traffic = None
    if MEASURED_TRAFFIC["bytes_per_rank"] == big and MEASURED_TRAFFIC["sources_sha256"] == kernel_sources_digest():
        traffic = MEASURED_TRAFFIC["bytes_per_launch"]

    out = {
        "metric": "all-gather sweep (W=8, 4 KiB..64 MiB per rank) algorithmic read+write throughput",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"all-gather size sweep, W=8 virtual ranks on one GPU, {sizes[0] // KiB} KiB.."
                               f"{big // MiB} MiB per rank in powers of 2, bf16 ~N(0,1) seeded",
                   "W": W, "calls_per_step": len(sizes), "bytes_per_step": step_bytes, "mode": "oneshot"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "dl_exec_rows_kernel<dl_fused_item, 8, 0, true>",
                     "launch": f"all-gather {big // MiB} MiB/rank: {ag_bytes(big)} B in {big_ms * 1e3:.1f} us "
                               f"(mean of {len(events)} launches, HIP events)"},
    }

    detail = None
    LAT_MAX = 16 * MiB    # host-observed latencies are taken up to this size, past every crossover between the modes

    def lat_iters(B):
        return 1000 if B <= MiB else 300 if B <= 4 * MiB else 100

    if not args.no_detail:
        detail = {"allgather": []}
        for B in sizes:
            row = {"bytes_per_rank": B, "device_us": benchaid.time_device(reqs[B], stream, warmup=3,
                                                                          calls=50 if B <= MiB else 10)}
            row["GBps"] = ag_bytes(B) / row["device_us"] / 1e3
            if B <= LAT_MAX:
                lat = benchaid.time_host(reqs[B], stream, benchaid.WAIT_STREAM, warmup=50, iters=lat_iters(B))
                row["oneshot_host_us"] = lat_stats(lat)
            detail["allgather"].append(row)
        # The same sizes with cold caches: enough buffer sets of each size that one pass over them moves more than
        # the on-die caches hold (256 MiB Infinity Cache, 32 MiB of L2), issued round-robin back to back.
        spare = {}
        for row in detail["allgather"]:
            B = row["bytes_per_rank"]
            if B < 64 * KiB or B > 8 * MiB:
                continue
            sets = max(3, min(64, -(-(1 << 30) // ag_bytes(B))))
            ring = [reqs[B]]
            for q in range(sets - 1):
                d_in = [torch.empty(B, dtype=torch.uint8, device="cuda").random_(0, 256) for _ in range(W)]
                d_out = [torch.empty(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)]
                ring.append(benchaid.allgather_request(d_in, d_out, B))
                spare[(B, q)] = (d_in, d_out)
            stream.synchronize()
            row["cold"] = {"buffer_sets": sets, "device_us": benchaid.time_device_rotating(ring, stream, 1, 3)}
            row["cold"]["GBps"] = ag_bytes(B) / row["cold"]["device_us"] / 1e3
            row["cold"]["frac_of_hbm_peak"] = row["cold"]["GBps"] / HBM_PEAK_GBS
            for q in range(sets - 1):
                del spare[(B, q)]
        # prelaunch mode: the request is armed ahead of time; timed from the doorbell write to the
        # completion word seen on the host, and from the arming call for comparison
        dl.dl_prelaunch_start()
        dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
        for row in detail["allgather"]:
            B = row["bytes_per_rank"]
            if B > LAT_MAX:
                continue
            lat = benchaid.time_host(reqs[B], None, benchaid.WAIT_TRIGGER, warmup=50, iters=lat_iters(B))
            row["prelaunch_trigger_to_done_us"] = lat_stats(lat)
            lat = benchaid.time_host(reqs[B], None, benchaid.WAIT_ARM_AND_TRIGGER, warmup=50, iters=lat_iters(B))
            row["prelaunch_arm_to_done_us"] = lat_stats(lat)
            # signal mode: an ordinary launch whose completion word the host watches instead of synchronising the stream
            dl.dl_set_mode(dl.DL_MODE_SIGNAL)
            lat = benchaid.time_host(reqs[B], None, benchaid.WAIT_SIGNAL, warmup=50, iters=lat_iters(B))
            row["signal_call_to_done_us"] = lat_stats(lat)
            if W * B <= 64 * 8192:
                # standby mode: the request is handed to a kernel that is already waiting (no launch in between)
                dl.dl_set_mode(dl.DL_MODE_STANDBY)
                lat = benchaid.time_host(reqs[B], None, benchaid.WAIT_SIGNAL, warmup=50, iters=1000)
                row["standby_call_to_done_us"] = lat_stats(lat)
            dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
        # The size -> mode table (the form of the paper's Tables II / III), measured: per size the fastest way to
        # run a request that is known ahead (armed and triggered, or one-shot) and one known only when issued
        # (standby where it fits, signal, or one-shot), and the largest size at which each mode still wins.
        table = []
        for row in detail["allgather"]:
            if "oneshot_host_us" not in row:
                continue
            one = row["oneshot_host_us"]["p50"]
            ahead = {"prelaunch": row["prelaunch_trigger_to_done_us"]["p50"], "oneshot": one}
            issue = {"signal": row["signal_call_to_done_us"]["p50"], "oneshot": one}
            if "standby_call_to_done_us" in row:
                issue["standby"] = row["standby_call_to_done_us"]["p50"]
            table.append({"bytes_per_rank": row["bytes_per_rank"], "moved_bytes": ag_bytes(row["bytes_per_rank"]),
                          "known_ahead": min(ahead, key=ahead.get), "known_on_issue": min(issue, key=issue.get),
                          "us": {**ahead, **issue}})
        detail["mode_table_measured"] = {
            "rows": table,
            "largest_moved_bytes_won_by": {
                m: max([r_["moved_bytes"] for r_ in table if r_["known_ahead" if m == "prelaunch" else "known_on_issue"] == m],
                       default=0) for m in ("prelaunch", "standby", "signal")},
            "library_thresholds": {"prelaunch_max_bytes": dl.DL_AUTO_PRELAUNCH_MAX_BYTES,
                                   "signal_max_bytes": dl.DL_AUTO_SIGNAL_MAX_BYTES,
                                   "standby_tiles": dl.DL_AUTO_STANDBY_TILES},
        }
        # phase breakdown (the form of the paper's Fig. 4: one transfer split into control / schedule / copy / sync,
        # 4 KB .. 2 MB), medians in microseconds
        med = lambda xs: pct(xs, .5)
        rows = []
        for row in detail["allgather"]:
            B = row["bytes_per_rank"]
            if B > 2 * MiB:
                continue
            ph = benchaid.phases(reqs[B], warmup=10, iters=100)
            m = {k: med([p[k] for p in ph]) for k in benchaid.PHASES}
            rows.append({"bytes_per_rank": B, "prelaunch": {
                "control_arming_call_off_critical_path": m["arming_call"],
                "schedule_and_sync_over_host_link": m["doorbell_to_seen"] + m["completion_issued_to_host"],
                "schedule_fanout_to_workgroups": m["seen_to_first_copy"],
                "copy": m["copy"],
                "sync_arrival_count": m["last_copy_to_completion_issued"],
                "host_link_split_estimate": {"doorbell_to_seen": m["doorbell_to_seen"],
                                             "completion_issued_to_host": m["completion_issued_to_host"]}}})
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_prelaunch_stop()
        for r_ in rows:
            B = r_["bytes_per_rank"]
            call, total = benchaid.time_call(reqs[B], stream, 20, 200)
            dev_us = next(x["device_us"] for x in detail["allgather"] if x["bytes_per_rank"] == B)
            r_["oneshot"] = {"control_call": med(call), "copy_device": dev_us,
                             "schedule_and_sync_launch_and_stream_sync": med(total) - med(call) - dev_us,
                             "total": med(total)}
        detail["phase_breakdown_allgather"] = rows
        detail.update(other_operations(dl, benchaid, inputs, torch, stream, reqs, keep, sizes, runtime_batch))
        out["mode_crossover_moved_MiB"] = {k: v >> 20 for k, v in
                                           detail["mode_table_measured"]["largest_moved_bytes_won_by"].items()}
        small = detail["allgather"][0]
        out["latency_us_4KiB_allgather"] = {
            "oneshot_call_to_stream_sync_p50": round(small["oneshot_host_us"]["p50"], 2),
            "oneshot_device": round(small["device_us"], 2),
            "prelaunch_trigger_to_done_p50": round(small["prelaunch_trigger_to_done_us"]["p50"], 2),
            "prelaunch_arm_to_done_p50": round(small["prelaunch_arm_to_done_us"]["p50"], 2),
            "signal_call_to_done_p50": round(small["signal_call_to_done_us"]["p50"], 2),
            "standby_call_to_done_p50": round(small["standby_call_to_done_us"]["p50"], 2),
        }
        # fraction of HBM peak per sweep point from 1 MiB per rank, cold caches where measured
        out["alltoall_frac_of_hbm_peak_by_MiB_per_pair"] = {
            str(r_["chunk_bytes"] // MiB): round(r_["cold"]["frac_of_hbm_peak"], 3)
            for r_ in detail["alltoall_uniform"] if r_["chunk_bytes"] >= MiB and "cold" in r_}
        out["frac_of_hbm_peak_by_MiB_per_rank"] = {
            str(r_["bytes_per_rank"] // MiB): round((r_["cold"]["GBps"] if "cold" in r_ else r_["GBps"]) / HBM_PEAK_GBS, 3)
            for r_ in detail["allgather"] if r_["bytes_per_rank"] >= MiB}

    dl.dl_shutdown()
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(sizes)
    if detail is not None:
        # the long part goes to a file: the printed line has to stay short enough to be read back whole
        detail["summary"] = out
        try:
            os.makedirs(os.path.dirname(args.detail_file), exist_ok=True)
            with open(args.detail_file, "w") as f:
                json.dump(detail, f, indent=1)
            out["detail_file"] = os.path.relpath(args.detail_file, ROOT)
        except OSError as e:
            out["detail_file"] = f"not written: {e}"
    print(json.dumps(short(out)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
