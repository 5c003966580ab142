"""The entry point that allocates nothing (dl_batch_copy_static), through the C boundary: its result against
that of dl_batch_copy on the same batch, byte for byte (and both against the CPU checker), on calls in a row
that shrink, so that the static table still holds the previous call's entries behind the current ones."""

import numpy as np
import pytest

import paper_2511_06605_amd as dl
from paper_2511_06605_amd import inputs
from paper_2511_06605_amd.inputs import KiB, MiB

from gpu_util import DevBuf, stream, sync

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def library():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    dl.dl_init(0)
    yield
    dl.dl_shutdown()


def both_ways(ref, arena, descs):
    """The batch through dl_batch_copy and through dl_batch_copy_static, each on a device copy of the arena."""
    want = ref.batch_copy([arena.copy()], [(0, s, 0, d, m) for s, d, m in descs])[0]
    a, b = DevBuf(arena.size, fill=arena), DevBuf(arena.size, fill=arena)
    dl.dl_batch_copy([(a.ptr(int(s)), a.ptr(int(t)), int(m)) for s, t, m in descs], stream())
    dl.dl_batch_copy_static([(b.ptr(int(s)), b.ptr(int(t)), int(m)) for s, t, m in descs], stream())
    sync()
    got_a, got_b = a.host(), b.host()
    assert np.array_equal(got_b, got_a), "the two entry points disagree"
    assert np.array_equal(got_b, want), "differs from the CPU checker"
    assert a.guards_intact() and b.guards_intact()


def test_static_entry_point_matches_batch_copy_on_shrinking_calls(ref):
    # 3000 copies of 4 KiB, then 500 of unequal sizes and alignments, then 10: the table shrinks every time
    arena, descs = inputs.b2b_batch(3000, 4 * KiB, 64 * MiB, seed=11)
    both_ways(ref, arena, descs)
    arena, descs = inputs.mixed_batch(500, 60000, 48 * MiB, seed=12, shared_sources=0.2)
    both_ways(ref, arena, descs)
    arena, descs = inputs.b2b_batch(10, 100 * KiB + 3, 8 * MiB, seed=13, align=1)
    both_ways(ref, arena, descs)


def test_static_entry_point_large_copies_and_limits(ref):
    # copies that are cut into many tiles each (70 x 3 MiB: 64 KiB tiles, 3360 entries)
    arena, descs = inputs.b2b_batch(70, 3 * MiB, 512 * MiB, seed=14, align=4096)
    both_ways(ref, arena, descs)
    # the most copies the table holds, one byte each; one more is refused and nothing is enqueued
    n = dl.DL_STATIC_MAX_COPIES
    src = np.random.default_rng(15).integers(0, 256, n + 1, dtype=np.uint8)
    d_src, d_dst = DevBuf(n + 1, fill=src), DevBuf(n + 1, fill=np.zeros(n + 1, dtype=np.uint8))
    dl.dl_batch_copy_static([(d_src.ptr(i), d_dst.ptr(i), 1) for i in range(n)], stream())
    sync()
    got = d_dst.host()
    assert np.array_equal(got[:n], src[:n]) and got[n] == 0 and d_dst.guards_intact()
    with pytest.raises(dl.DlError) as e:
        dl.dl_batch_copy_static([(d_src.ptr(i), d_dst.ptr(i), 1) for i in range(n + 1)], stream())
    assert e.value.status == dl.DL_ERR_CAPACITY
    # empty batches and empty copies enqueue nothing
    dl.dl_batch_copy_static([], stream())
    dl.dl_batch_copy_static([(d_src.ptr(0), d_dst.ptr(0), 0)], stream())
    sync()
    assert got[n] == 0


def test_static_entry_point_replays_from_a_graph(ref):
    """What the entry point is for: a long list (500 copies: a table on the device) issued on a stream that is
    being captured.  Only kernel launches are recorded (the fills of the static table and the table kernel), so
    the graph can be replayed with new bytes in the arena; every replay is compared with the CPU checker, with
    eager work and synchronisations in between."""
    import torch
    arena, descs = inputs.b2b_batch(500, 3000, 8 * MiB, seed=21, align=16)
    d = DevBuf(arena.size, fill=arena)
    dlist = [(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        dl.dl_batch_copy_static(dlist, torch.cuda.current_stream())
    rng = np.random.default_rng(22)
    for replay in range(4):
        fresh = rng.integers(0, 256, arena.size, dtype=np.uint8)
        d.view().copy_(torch.from_numpy(fresh))
        sync()
        g.replay()
        torch.cuda.synchronize()
        want = ref.batch_copy([fresh.copy()], [(0, s, 0, t, m) for s, t, m in descs])[0]
        assert np.array_equal(d.host(), want) and d.guards_intact(), f"replay {replay}"
