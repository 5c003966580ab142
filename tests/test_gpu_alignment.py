"""GPU parity at every position of a destination on the 128-byte grid that tiles are cut on, with sources and
further destinations that disagree with it in every way, and lengths on both sides of every boundary the kernels
know (16 bytes, a 1 KiB row, a tile): the bytes that were to move moved, and no other byte of the arena changed.
Every kind of kernel is driven: short lists in the kernel arguments (row path), lists of tens of items (the
two-dimensional grid and the general path), long lists (tables), read-once/write-k items, swaps, and the same
under the armed, signal and standby kernels, whose loads and stores are the system-scope forms."""

import os

import numpy as np
import pytest

import paper_2511_06605_amd as dl
from paper_2511_06605_amd.inputs import KiB

from gpu_util import DevBuf, sync

pytestmark = pytest.mark.gpu

SLOT = 16 * KiB          # every range of a case lies in a slot of its own, 256 bytes in from the slot's start
LENGTHS = [1, 2, 15, 16, 17, 31, 33, 127, 128, 129, 1023, 1024, 1025, 4095, 4096, 4097, 8191, 8192, 8193, 12345]


@pytest.fixture(scope="module", autouse=True)
def library():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    dl.dl_init(0)
    dl.dl_set_config(arm_timeout_us=300_000)
    # DL_TEST_CONFIG="max_blocks=64,fan_split=1" runs every test with those tunables as the defaults
    forced = dict(kv.split("=") for kv in os.environ.get("DL_TEST_CONFIG", "").split(",") if kv)
    if forced:
        dl.dl_set_config(**{k: int(v) for k, v in forced.items()})
    dl.dl_prelaunch_start()
    yield
    dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    dl.dl_prelaunch_stop()
    dl.dl_shutdown()


MODES = {"oneshot": dl.DL_MODE_ONESHOT, "prelaunch": dl.DL_MODE_PRELAUNCH, "signal": dl.DL_MODE_SIGNAL,
         "standby": dl.DL_MODE_STANDBY}


def finish(mode, ticket_before):
    if mode == "oneshot" or dl.dl_last_ticket() == ticket_before:
        sync()
    elif mode == "prelaunch":
        dl.dl_trigger()
        dl.dl_wait()
    else:
        dl.dl_wait()


def lengths_near(shift, tile):
    """Lengths that end just before, on and just behind the first boundaries of a grid entered `shift` bytes in."""
    out = set(LENGTHS)
    for edge in (16, 128, 1024, tile, 2 * tile):
        for d in (-1, 0, 1):
            n = edge - shift % edge + d
            if n > 0:
                out.add(n)
    return sorted(out)


def cases(tile, src_offsets):
    """(first destination's shift, source offset, length) over all 128 shifts."""
    out = []
    for shift in range(128):
        for q, n in enumerate(lengths_near(shift, tile)):
            out.append((shift, src_offsets[(shift + q) % len(src_offsets)], n))
    return out


def arena_for(ncase, ranges_per_case, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(0, 256, size=ncase * ranges_per_case * SLOT, dtype=np.uint8)


@pytest.mark.parametrize("mode,per_call", [(m, n) for n in (1, 8, 40, 500) for m in MODES if n > 1 or m == "oneshot"])
def test_plain_copies_at_every_shift(ref, mode, per_call):
    """per_call copies per request: 1 (one-shot only) and 8 take the row path, 40 the longer argument list, 500 a
    table."""
    cs = cases(4096, [0, 1, 5, 16, 77, 128])
    if per_call == 1:
        cs = cs[::7]
    arena = arena_for(len(cs), 2, seed=per_call)
    d = DevBuf(arena.size, fill=arena)
    descs = []
    for i, (shift, so, n) in enumerate(cs):
        descs.append(((2 * i) * SLOT + 256 + so, (2 * i + 1) * SLOT + 256 + shift, n))
    want = ref.batch_copy([arena.copy()], [(0, s, 0, t, n) for s, t, n in descs])[0]
    sync()
    dl.dl_set_mode(MODES[mode])
    try:
        for at in range(0, len(descs), per_call):
            before = dl.dl_last_ticket()
            dl.dl_batch_copy([(d.ptr(s), d.ptr(t), n) for s, t, n in descs[at:at + per_call]], None)
            finish(mode, before)
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    sync()
    got = d.host()
    if not np.array_equal(got, want):
        bad = int(np.flatnonzero(got != want)[0])
        i = bad // (2 * SLOT)
        raise AssertionError(f"first wrong byte at arena offset {bad}: case {cs[i]} (shift, source offset, length)")
    assert d.guards_intact()


@pytest.mark.parametrize("policy", [dict(nontemporal_min_bytes=1), dict(write_through_max_bytes=0)])
@pytest.mark.parametrize("per_call", [8, 40, 500])
def test_plain_copies_at_every_shift_with_the_other_store_policies(ref, policy, per_call):
    """The default for requests this small is the write-through store; here the streaming and the plain forms."""
    base = dl.dl_get_config()
    saved = {f[0]: getattr(base, f[0]) for f in base._fields_}
    dl.dl_set_config(**policy)
    try:
        test_plain_copies_at_every_shift(ref, "oneshot", per_call)
    finally:
        dl.dl_set_config(**saved)


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("per_call", [2, 8, 200])
def test_read_once_write_k_at_every_shift(ref, mode, per_call):
    """One source, three destinations that stand differently on the grid; the first decides the cut."""
    cs = cases(1024, [0, 3, 16, 50])[::2]
    arena = arena_for(len(cs), 4, seed=100 + per_call)
    d = DevBuf(arena.size, fill=arena)
    items, copies = [], []
    for i, (shift, so, n) in enumerate(cs):
        src = (4 * i) * SLOT + 256 + so
        dsts = [(4 * i + 1) * SLOT + 256 + shift, (4 * i + 2) * SLOT + 256 + (shift * 5 + 9) % 128,
                (4 * i + 3) * SLOT + 256 + (shift + so) % 16]
        items.append((src, dsts, n))
        copies += [(0, src, 0, t, n) for t in dsts]
    want = ref.batch_copy([arena.copy()], copies)[0]
    sync()
    dl.dl_set_mode(MODES[mode])
    try:
        for at in range(0, len(items), per_call):
            before = dl.dl_last_ticket()
            dl.dl_batch_fanout([dict(src=d.ptr(s), dst=[d.ptr(t) for t in ts], bytes=n) for s, ts, n in items[at:at + per_call]], None)
            finish(mode, before)
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    sync()
    got = d.host()
    if not np.array_equal(got, want):
        bad = int(np.flatnonzero(got != want)[0])
        raise AssertionError(f"first wrong byte at arena offset {bad}: case {cs[bad // (4 * SLOT)]} (shift, source offset, length)")
    assert d.guards_intact()


@pytest.mark.parametrize("mode", ["oneshot", "prelaunch", "signal"])
@pytest.mark.parametrize("per_call", [1, 8, 40, 300])
def test_swaps_at_every_shift(ref, mode, per_call):
    cs = cases(4096, [0, 1, 16, 100])[::3]
    if per_call == 1:
        cs = cs[::5]
    arena = arena_for(len(cs), 2, seed=200 + per_call)
    d = DevBuf(arena.size, fill=arena)
    swaps = [((2 * i) * SLOT + 256 + so, (2 * i + 1) * SLOT + 256 + shift, n) for i, (shift, so, n) in enumerate(cs)]
    want = ref.batch_swap([arena.copy()], [(0, a, 0, b, n) for a, b, n in swaps])[0]
    sync()
    dl.dl_set_mode(MODES[mode])
    try:
        for at in range(0, len(swaps), per_call):
            before = dl.dl_last_ticket()
            dl.dl_batch_swap([(d.ptr(a), d.ptr(b), n) for a, b, n in swaps[at:at + per_call]], None)
            finish(mode, before)
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    sync()
    got = d.host()
    if not np.array_equal(got, want):
        bad = int(np.flatnonzero(got != want)[0])
        raise AssertionError(f"first wrong byte at arena offset {bad}: case {cs[bad // (2 * SLOT)]} (shift, source offset, length)")
    assert d.guards_intact()


@pytest.mark.parametrize("mode", ["oneshot", "prelaunch", "signal"])
@pytest.mark.parametrize("shift_in,shift_out,cut", [(0, 32, 0), (0, 0, 32), (1, 0, 0), (0, 1, 0), (5, 2, 7), (16, 48, 16),
                                                    (3, 127, 1), (64, 64, 64)])
def test_allgather_large_off_the_grid(ref, mode, shift_in, shift_out, cut):
    """An all-gather big enough for many passes of a capped grid (the armed kernels keep several rows in flight
    there), with send and receive buffers off the grid and a length that leaves every rank's share off it too."""
    from paper_2511_06605_amd import inputs
    W, B = 8, 1024 * KiB - cut
    ins = inputs.allgather_inputs(W, B, seed=shift_in * 131 + shift_out, kind="u8")
    want = ref.allgather(ins)
    d_in = [DevBuf(B, fill=ins[r], shift=shift_in) for r in range(W)]
    d_out = [DevBuf(W * B, shift=shift_out) for _ in range(W)]
    sync()
    dl.dl_set_mode(MODES[mode])
    try:
        before = dl.dl_last_ticket()
        dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B, None)
        finish(mode, before)
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    sync()
    for r in range(W):
        assert np.array_equal(d_out[r].host(), want[r]), f"rank {r}"
        assert d_out[r].guards_intact()
