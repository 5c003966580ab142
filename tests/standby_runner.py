"""GPU parity of standby mode (requests handed to a kernel that is already waiting on the device), run as a
script in a process of its own: exit status 0 = every check held.

Why its own process: a waiting kernel holds the hardware queue of its stream, and the HIP runtime maps all
streams of a process to a few hardware queues.  In a process that has created more streams than there are
queues (a long test session does) other work can land behind a waiting kernel and stall until that kernel gives
up, which makes such a session slow, not wrong.  Here the streams are the default one, the library's and the
two of standby mode: one hardware queue each.

Every waiting kernel gives up by itself after 2 ms, so nothing stays on the device."""

import faulthandler
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import paper_2511_06605_amd as dl  # noqa: E402
from paper_2511_06605_amd import inputs  # noqa: E402
from paper_2511_06605_amd.inputs import KiB, MiB  # noqa: E402

from gpu_util import DevBuf, stream, sync  # noqa: E402
from oracle import ref  # noqa: E402

ARM_US = 300_000


class standby:
    """A prelaunch session in standby mode."""

    def __enter__(self):
        dl.dl_set_config(arm_timeout_us=ARM_US)
        dl.dl_prelaunch_start()
        dl.dl_set_mode(dl.DL_MODE_STANDBY)

    def __exit__(self, *exc):
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_prelaunch_stop()


def allgather(W, B, seed, shifts=None):
    ins = inputs.allgather_inputs(W, B, seed)
    shifts = shifts or [0] * (2 * W)
    d_in = [DevBuf(B, fill=ins[r], shift=shifts[r]) for r in range(W)]
    d_out = [DevBuf(W * B, shift=shifts[W + r]) for r in range(W)]
    sync()
    before = dl.dl_last_ticket()
    dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B)
    assert dl.dl_last_ticket() == before + (1 if B else 0)
    dl.dl_wait()
    want = ref.allgather(ins)
    for r in range(W):
        assert np.array_equal(d_out[r].host(), want[r]), f"rank {r} (W={W}, B={B})"
        assert d_out[r].guards_intact()


def allgather_sizes():
    """Requests that fit a waiting kernel (at most 8 items and 64 tiles of 8 KiB; up to 16 tiles each tile reports
    for itself, above that they are counted) and requests that do not (more items, more tiles: they take the
    ordinary launch), with no other synchronisation than dl_wait."""
    for W, B in [(8, 4096), (8, 1), (8, 1000), (8, 16 * KiB), (8, 16 * KiB + 16), (8, 20000), (8, 32 * KiB),
                 (8, 64 * KiB), (8, 64 * KiB + 16), (8, 0), (3, 40000), (1, 100000), (2, 250000), (1, 512 * KiB),
                 (1, 512 * KiB + 1), (9, 4096), (16, 512), (8, 1 * MiB)]:
        with standby():
            allgather(W, B, seed=W * 131 + B)


def allgather_misaligned():
    for shifts in ([5] * 8, [0, 4, 8, 12, 0, 4, 8, 12], [0, 1, 2, 3, 7, 9, 11, 13]):
        with standby():
            allgather(4, 9000, seed=3, shifts=shifts)


def other_operations():
    with standby():
        # broadcast, 7 destinations, 100 KiB: one read-once/write-7 item, 13 tiles; then 300 KiB: 38 tiles, counted
        for nbytes in (100 * KiB + 5, 300 * KiB):
            src = inputs.payload(np.random.default_rng(nbytes), nbytes)
            d_src = DevBuf(src.size, fill=src, shift=nbytes % 2)
            d_dst = [DevBuf(src.size) for _ in range(7)]
            sync()
            dl.dl_broadcast(d_src.ptr(), [b.ptr() for b in d_dst], src.size)
            dl.dl_wait()
            for b in d_dst:
                assert np.array_equal(b.host(), src) and b.guards_intact()
        src = inputs.payload(np.random.default_rng(1), 100 * KiB + 5)
        d_src = DevBuf(src.size, fill=src)
        d_dst = [DevBuf(src.size) for _ in range(7)]
        sync()
        dl.dl_broadcast(d_src.ptr(), [b.ptr() for b in d_dst], src.size)
        dl.dl_wait()
        for b in d_dst:
            assert np.array_equal(b.host(), src) and b.guards_intact()
        # a batch of 6 copies of unequal sizes and alignments
        arena, descs = inputs.mixed_batch(6, 9000, 1 * MiB, seed=4)
        want = ref.batch_copy([arena.copy()], [(0, s, 0, d, m) for s, d, m in descs])[0]
        d = DevBuf(arena.size, fill=arena)
        sync()
        dl.dl_batch_copy([(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs])
        dl.dl_wait()
        assert np.array_equal(d.host(), want) and d.guards_intact()
        # all-to-all between two ranks (4 chunks), between eight (64 plain copies of up to 5000 bytes: one tile each),
        # between eight with chunks of up to three tiles (too many tiles: the ordinary launch) and between nine
        # (81 copies: too many)
        for W, top in ((2, 5000), (8, 5000), (8, 8192), (8, 20000), (9, 3000)):
            C = inputs.random_chunks(W, top, seed=W + top, zero_frac=0.2)
            ins = inputs.alltoall_inputs(C, seed=W + 1)
            want = ref.alltoall(ins, C)
            d_in = [DevBuf(a.size, fill=a) for a in ins]
            d_out = [DevBuf(w.size) for w in want]
            sync()
            dl.dl_alltoall([b.ptr() for b in d_in], [b.ptr() for b in d_out], C)
            dl.dl_wait()
            for j in range(W):
                assert np.array_equal(d_out[j].host(), want[j]) and d_out[j].guards_intact()
        # batches of 9, 40 and 64 copies of unequal sizes and alignments (plain lists), and 65 (too many)
        for n in (9, 40, 64, 65):
            arena, descs = inputs.mixed_batch(n, 6000, 2 * MiB, seed=100 + n)
            want = ref.batch_copy([arena.copy()], [(0, s, 0, t, m) for s, t, m in descs])[0]
            d = DevBuf(arena.size, fill=arena)
            sync()
            dl.dl_batch_copy([(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs])
            dl.dl_wait()
            assert np.array_equal(d.host(), want) and d.guards_intact(), f"batch of {n}"
        # an in-place all-to-all (swaps): never handed to a waiting kernel, same result
        bufs = inputs.alltoall_inputs(inputs.uniform_chunks(4, 3000), seed=9)
        d_buf = [DevBuf(a.size, fill=a) for a in bufs]
        sync()
        dl.dl_alltoall_inplace([b.ptr() for b in d_buf], 3000)
        dl.dl_wait()
        for b, w in zip(d_buf, ref.alltoall_inplace(bufs, 3000)):
            assert np.array_equal(b.host(), w) and b.guards_intact()


def many_requests_with_changing_sources():
    """3000 requests in a row over the same buffers, sizes cycling between what a waiting kernel takes and what
    it does not, the sources rewritten before every call and two receive buffers checked after every dl_wait."""
    import torch
    W = 8
    sizes = [4 * KiB, 16 * KiB, 48 * KiB, 1000, 80 * KiB, 64 * KiB]
    d_in = {B: [torch.zeros(B, dtype=torch.uint8, device="cuda") for _ in range(W)] for B in sizes}
    d_out = {B: [torch.zeros(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)] for B in sizes}
    bad = torch.zeros(1, dtype=torch.int64, device="cuda")
    with standby():
        t0 = time.monotonic()
        for it in range(3000):
            B = sizes[it % len(sizes)]
            for j in range(W):
                d_in[B][j].fill_((it * 7 + j * 31) % 251)
            sync()
            dl.dl_allgather(d_in[B], d_out[B], B)
            dl.dl_wait()
            for r in (it % W, (it + 3) % W):
                got = d_out[B][r].view(W, B)
                want = torch.tensor([(it * 7 + j * 31) % 251 for j in range(W)], dtype=torch.uint8, device="cuda")
                bad += (got != want[:, None]).sum()
            if it % 500 == 499:
                print(f"  {it + 1} requests, {time.monotonic() - t0:.1f} s", flush=True)
        sync()
    assert int(bad.item()) == 0


def kernels_that_gave_up_are_replaced():
    """While the caller idles the waiting kernels give up (2 ms, or the arm limit if that is shorter); the next
    requests must still be served (by the ordinary launch, then by fresh kernels), and none may be lost."""
    for limit_us in (ARM_US, 1000):
        dl.dl_set_config(arm_timeout_us=limit_us)
        try:
            dl.dl_prelaunch_start()
            dl.dl_set_mode(dl.DL_MODE_STANDBY)
            for pause in (0.0, 0.02, 0.0, 0.0, 0.0008, 0.0012, 0.0016, 0.002, 0.0024, 0.02, 0.0):
                time.sleep(pause)
                allgather(8, 4096, seed=int(pause * 1e4))
        finally:
            dl.dl_set_mode(dl.DL_MODE_ONESHOT)
            dl.dl_prelaunch_stop()
            dl.dl_set_config(arm_timeout_us=ARM_US)


def requests_close_to_the_limit():
    """With a limit of 150 us, requests that come some 20 .. 120 us apart find the waiting kernel young (handed
    over), close to its limit (handed over, then the library makes sure that the kernel did serve it) or too old
    (ordinary launch); every one of them must be served exactly as asked."""
    import torch
    W, B, SETS = 8, 4 * KiB, 5
    d_in = [[torch.full((B,), 16 * k + j, dtype=torch.uint8, device="cuda") for j in range(W)] for k in range(SETS)]
    want = [torch.tensor([16 * k + j for j in range(W)], dtype=torch.uint8, device="cuda")[:, None] for k in range(SETS)]
    d_out = [torch.zeros(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)]
    bad = torch.zeros(1, dtype=torch.int64, device="cuda")
    dl.dl_set_config(arm_timeout_us=150)
    try:
        dl.dl_prelaunch_start()
        dl.dl_set_mode(dl.DL_MODE_STANDBY)
        sync()
        for it in range(1500):
            t_end = time.perf_counter() + (it % 41) * 2.5e-6
            while time.perf_counter() < t_end:
                pass
            k = it % SETS
            dl.dl_allgather(d_in[k], d_out, B)
            dl.dl_wait()
            bad += (d_out[it % W].view(W, B) != want[k]).sum()
            sync()   # the comparison has read the receive buffer before the next request rewrites it
        sync()
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_prelaunch_stop()
        dl.dl_set_config(arm_timeout_us=ARM_US)
    assert int(bad.item()) == 0


def mode_switches_and_stop():
    dl.dl_prelaunch_start()
    try:
        for mode in (dl.DL_MODE_STANDBY, dl.DL_MODE_SIGNAL, dl.DL_MODE_STANDBY, dl.DL_MODE_ONESHOT, dl.DL_MODE_STANDBY):
            dl.dl_set_mode(mode)
            ins = inputs.allgather_inputs(8, 4096, seed=mode)
            d_in = [DevBuf(4096, fill=a) for a in ins]
            d_out = [DevBuf(8 * 4096) for _ in range(8)]
            sync()
            dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], 4096, stream() if mode == dl.DL_MODE_ONESHOT else None)
            if mode == dl.DL_MODE_ONESHOT:
                sync()
            else:
                dl.dl_wait()
            for r, w in zip(d_out, ref.allgather(ins)):
                assert np.array_equal(r.host(), w)
    finally:
        dl.dl_prelaunch_stop()          # with kernels waiting: they are cancelled
    assert dl.dl_get_mode() == dl.DL_MODE_ONESHOT
    try:
        dl.dl_set_mode(dl.DL_MODE_STANDBY)   # needs dl_prelaunch_start
    except dl.DlError as e:
        assert e.status == dl.DL_ERR_STATE
    else:
        raise AssertionError("standby mode accepted without a prelaunch session")


def armed_requests_of_every_grid_size():
    """Prelaunch mode beside the standby checks, so that both ways of placing the doorbell (device memory, host
    memory with a hop through device flags above 16 workgroups) get the same requests: all-gathers from one
    workgroup to the capped grid, and a long list."""
    dl.dl_set_config(arm_timeout_us=ARM_US)
    dl.dl_prelaunch_start()
    try:
        dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
        for W, B in [(8, 512), (8, 4 * KiB), (8, 16 * KiB), (8, 24 * KiB + 48), (8, 64 * KiB), (8, 256 * KiB),
                     (8, 1 * MiB + 16), (3, 5 * MiB + 7)]:
            ins = inputs.allgather_inputs(W, B, seed=B + W)
            d_in = [DevBuf(B, fill=a) for a in ins]
            d_out = [DevBuf(W * B) for _ in range(W)]
            sync()
            dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B)
            dl.dl_trigger()
            dl.dl_wait()
            for r, w in zip(d_out, ref.allgather(ins)):
                assert np.array_equal(r.host(), w) and r.guards_intact(), f"armed all-gather W={W} B={B}"
        arena, descs = inputs.mixed_batch(300, 5000, 4 * MiB, seed=11)
        want = ref.batch_copy([arena.copy()], [(0, s, 0, d, m) for s, d, m in descs])[0]
        d = DevBuf(arena.size, fill=arena)
        sync()
        dl.dl_batch_copy([(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs])
        dl.dl_trigger()
        dl.dl_wait()
        assert np.array_equal(d.host(), want) and d.guards_intact()
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_prelaunch_stop()


def random_requests():
    """The seeded random requests of test_gpu_random.py with standby mode among the modes drawn."""
    import test_gpu_random as rnd
    dl.dl_set_config(arm_timeout_us=ARM_US)
    dl.dl_prelaunch_start()
    try:
        for seed in range(5000, 5000 + int(os.environ.get("DL_TEST_RANDOM_CASES", "150"))):
            rnd.run_case(ref, seed, modes=("standby", "standby", "standby", "signal", "oneshot", "prelaunch", "auto", "auto"))
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_prelaunch_stop()


def auto_mode_across_the_table():
    """DL_MODE_AUTO: the four operations (and swaps, and a token dispatch) at sizes on both sides of every row of
    the size -> mode table, each compared with the CPU checker; dl_last_mode() must say what the table says (a
    request for a waiting kernel may also have taken the ordinary launch, if none was free), and dl_complete()
    waits in the way that fits."""
    one, sig, sb = dl.DL_MODE_ONESHOT, dl.DL_MODE_SIGNAL, dl.DL_MODE_STANDBY
    seen = set()

    def done(expect, what):
        got = dl.dl_last_mode()
        assert got == expect or (expect == sb and got == sig), f"{what}: executed in mode {got}, table says {expect}"
        seen.add(got)
        dl.dl_complete(stream())

    dl.dl_set_config(arm_timeout_us=ARM_US)
    dl.dl_prelaunch_start()
    try:
        dl.dl_set_mode(dl.DL_MODE_AUTO)
        W = 8
        for B, expect in [(4 * KiB, sb), (64 * KiB, sb), (64 * KiB + 16, sig), (1 * MiB, sig), (4 * MiB, sig),
                          (4 * MiB + 16, one), (5 * MiB + 3, one)]:
            ins = inputs.allgather_inputs(W, B, seed=B % 1000)
            d_in = [DevBuf(B, fill=a) for a in ins]
            d_out = [DevBuf(W * B) for _ in range(W)]
            sync()
            dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B, stream())
            done(expect, f"all-gather {B}")
            for r, w in zip(d_out, ref.allgather(ins)):
                assert np.array_equal(r.host(), w) and r.guards_intact(), f"auto all-gather B={B}"
        for c, expect in [(8 * KiB, sb), (16 * KiB, sig), (2 * MiB, sig), (4 * MiB, one)]:
            C = inputs.uniform_chunks(W, c)
            ins = inputs.alltoall_inputs(C, seed=c % 1000, kind="fp16")
            want = ref.alltoall(ins, C)
            d_in = [DevBuf(a.size, fill=a) for a in ins]
            d_out = [DevBuf(w.size) for w in want]
            sync()
            dl.dl_alltoall([b.ptr() for b in d_in], [b.ptr() for b in d_out], C, stream())
            done(expect, f"all-to-all {c}")
            for j in range(W):
                assert np.array_equal(d_out[j].host(), want[j]) and d_out[j].guards_intact(), f"auto all-to-all c={c}"
        for nbytes, expect in [(512 * KiB, sb), (512 * KiB + 16, sig), (2 * MiB, sig), (40 * MiB, one)]:
            src = inputs.payload(np.random.default_rng(nbytes), nbytes, "bf16")
            d_src = DevBuf(src.size, fill=src)
            d_dst = [DevBuf(src.size) for _ in range(7)]
            sync()
            dl.dl_broadcast(d_src.ptr(), [b.ptr() for b in d_dst], src.size, stream())
            done(expect, f"broadcast {nbytes}")
            for b in d_dst:
                assert np.array_equal(b.host(), src) and b.guards_intact(), f"auto broadcast {nbytes}"
        for n, nb, expect in [(64, 100, sb), (65, 100, sig), (64, 16 * KiB, sig), (40, 5 * MiB, one)]:
            arena, descs = inputs.b2b_batch(n, nb, max(4 * MiB, 3 * n * nb), seed=n + nb)
            want = ref.batch_copy([arena.copy()], [(0, s, 0, t, m) for s, t, m in descs])[0]
            d = DevBuf(arena.size, fill=arena)
            sync()
            dl.dl_batch_copy([(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs], stream())
            done(expect, f"batch {n} x {nb}")
            assert np.array_equal(d.host(), want) and d.guards_intact(), f"auto batch {n} x {nb}"
        for Wn, c, expect in [(4, 3000, sig), (4, 16 * MiB, one)]:
            bufs = inputs.alltoall_inputs(inputs.uniform_chunks(Wn, c), seed=9)
            d_buf = [DevBuf(a.size, fill=a) for a in bufs]
            sync()
            dl.dl_alltoall_inplace([b.ptr() for b in d_buf], c, stream())
            done(expect, f"in-place all-to-all {c}")
            for b, w in zip(d_buf, ref.alltoall_inplace(bufs, c)):
                assert np.array_equal(b.host(), w) and b.guards_intact(), f"auto in-place all-to-all c={c}"
        for T, expect in [(16, sig), (128, one)]:
            row = 14336
            ins = inputs.token_rows(W, T, row, seed=T + 1, kind="bf16")
            dest = inputs.moe_token_destinations(W, T, seed=T)
            want = ref.token_dispatch(ins, row, dest)
            d_in = [DevBuf(a.size, fill=a) for a in ins]
            d_out = [DevBuf(w.size) for w in want]
            sync()
            dl.dl_token_dispatch([b.ptr() for b in d_in], [b.ptr() for b in d_out], [T] * W, row, dest, stream())
            done(expect, f"token dispatch {T}")
            for j in range(W):
                assert np.array_equal(d_out[j].host(), want[j]) and d_out[j].guards_intact(), f"auto token dispatch T={T}"
        assert {one, sig} <= seen, f"modes executed: {seen}"
        if os.environ.get("DL_NO_BAR") != "1":
            assert sb in seen, "no request was handed to a waiting kernel"
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_prelaunch_stop()


CHECKS = [allgather_sizes, allgather_misaligned, other_operations, many_requests_with_changing_sources,
          kernels_that_gave_up_are_replaced, requests_close_to_the_limit, mode_switches_and_stop,
          armed_requests_of_every_grid_size, auto_mode_across_the_table, random_requests]


def main():
    import torch
    faulthandler.enable()   # a crash in native code names the Python line it came from
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    ref.build()
    dl.dl_init(0)
    try:
        for fn in CHECKS:
            print(f"standby: {fn.__name__} ...", flush=True)
            t0 = time.monotonic()
            fn()
            print(f"standby: {fn.__name__} ok ({time.monotonic() - t0:.2f} s)", flush=True)
    finally:
        dl.dl_shutdown()
    print("standby: all ok", flush=True)


if __name__ == "__main__":
    main()
