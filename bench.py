#!/usr/bin/env python3
"""Benchmark of the MI355X copy collectives.

Workload (one "step"): the all-gather size sweep over W = 8 virtual ranks on one
GPU, per-rank payload 4 KiB ... 64 MiB in powers of two (15 calls), bf16 values
~N(0,1) from a seeded generator, one receive buffer of W x payload per rank.
All buffers are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is algorithmic (read + write) bytes per second
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
HBM_PEAK_GBS = 8000.0


def ag_bytes(B: int) -> int:
    return W * B + W * W * B


def pct(xs, q):
    xs = sorted(xs)
    return xs[min(len(xs) - 1, int(q * len(xs)))]


def cpu_baseline(sizes, budget_s=10.0):
    """The CPU checker as it stands (single thread, plain memcpy), timed on the
    host on the sweep points up to 16 MiB per rank, repeated until the budget
    is used.  Buffers are touched once before timing."""
    import numpy as np
    from oracle import ref

    ref.build()
    lib = ref.load()
    sample = [B for B in sizes if B <= 16 * MiB]
    rng = np.random.default_rng(0)
    cases = []
    for B in sample:
        ins = [rng.integers(0, 256, B, dtype=np.uint8) for _ in range(W)]
        outs = [np.ones(W * B, dtype=np.uint8) for _ in range(W)]
        cases.append((B, ref._ptrs(ins), ref._ptrs(outs), ins, outs))
    moved, passes = 0, 0
    t0 = time.perf_counter()
    while True:
        for B, pi, po, _, _ in cases:
            rc = lib.ref_allgather(pi, po, W, B)
            assert rc == 0
            moved += ag_bytes(B)
        passes += 1
        if time.perf_counter() - t0 >= budget_s and passes >= 2:
            break
    dt = time.perf_counter() - t0
    return {
        "value": moved / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"{passes} passes of the all-gather sweep points 4 KiB..16 MiB per rank (W=8), "
                  f"{moved / 2**30:.1f} GiB moved in {dt:.1f} s, single thread",
        "host_cpus": os.cpu_count(),
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--max-bytes", type=int, default=64 * MiB, help="largest per-rank payload of the sweep")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU baseline leg")
    ap.add_argument("--no-detail", action="store_true", help="skip per-size latency and comparison legs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU (W virtual ranks share its HBM); --gpus must be 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2511_06605_amd as dl
    from paper_2511_06605_amd import benchaid, inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dl.dl_init(0)
    stream = torch.cuda.current_stream()

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

    out = {
        "metric": "all-gather sweep (W=8, 4 KiB..64 MiB per rank) algorithmic read+write throughput",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "all-gather size sweep, W=8 virtual ranks on one GPU, per-rank payload "
                               f"{sizes[0] // KiB} KiB..{big // MiB} MiB in powers of 2, bf16 ~N(0,1) seeded",
                   "W": W, "calls_per_step": len(sizes), "bytes_per_step": step_bytes, "mode": "oneshot"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "dl_exec_list_kernel<dl_fused_item, 8, nontemporal>",
                     "launch": f"all-gather {big // MiB} MiB per rank: {ag_bytes(big)} algorithmic bytes, "
                               f"{big_ms * 1e3:.1f} us average over {len(events)} launches (HIP events)"},
    }

    if not args.no_detail:
        detail = {"allgather": []}
        for B in sizes:
            row = {"bytes_per_rank": B, "device_us": benchaid.time_device(reqs[B], stream, warmup=3,
                                                                          calls=50 if B <= MiB else 10)}
            row["GBps"] = ag_bytes(B) / row["device_us"] / 1e3
            if B <= MiB:
                lat = benchaid.time_host(reqs[B], stream, benchaid.WAIT_STREAM, warmup=50, iters=500)
                row["oneshot_host_us"] = {"p50": pct(lat, .5), "p10": pct(lat, .1), "p90": pct(lat, .9)}
            detail["allgather"].append(row)
        # prelaunch mode: the request is armed ahead of time; timed from the doorbell write to the
        # completion word seen on the host, and from the arming call for comparison
        dl.dl_prelaunch_start()
        dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
        for row in detail["allgather"]:
            B = row["bytes_per_rank"]
            if B > MiB:
                continue
            lat = benchaid.time_host(reqs[B], None, benchaid.WAIT_TRIGGER, warmup=50, iters=500)
            row["prelaunch_trigger_to_done_us"] = {"p50": pct(lat, .5), "p10": pct(lat, .1), "p90": pct(lat, .9)}
            lat = benchaid.time_host(reqs[B], None, benchaid.WAIT_ARM_AND_TRIGGER, warmup=50, iters=500)
            row["prelaunch_arm_to_done_us"] = {"p50": pct(lat, .5), "p10": pct(lat, .1), "p90": pct(lat, .9)}
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_prelaunch_stop()
        out["detail"] = detail
        small = detail["allgather"][0]
        out["latency_us_4KiB_allgather"] = {
            "oneshot_call_to_stream_sync_p50": small["oneshot_host_us"]["p50"],
            "oneshot_device": small["device_us"],
            "prelaunch_trigger_to_done_p50": small["prelaunch_trigger_to_done_us"]["p50"],
            "prelaunch_arm_to_done_p50": small["prelaunch_arm_to_done_us"]["p50"],
        }

    dl.dl_shutdown()
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(sizes)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
