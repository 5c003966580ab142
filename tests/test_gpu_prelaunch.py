"""GPU parity of the prelaunched mode: a request armed ahead of time and then
triggered through the doorbell gives the same bytes as the CPU checker; an
untriggered or cancelled request copies nothing and says so.

Every armed kernel gives up by itself after the arm limit set below, so no
test can leave waves on the device."""

import os

import numpy as np
import pytest

import paper_2511_06605_amd as dl
from paper_2511_06605_amd import inputs
from paper_2511_06605_amd.inputs import KiB, MiB

from gpu_util import CANARY, DevBuf, stream, sync

pytestmark = pytest.mark.gpu

ARM_US = 300_000  # generous for a Python caller, still far below any watchdog


@pytest.mark.skip(reason="a long-lived resident kernel (one launch serving many requests) ended its first run on a GPU with a "
                         "fault or hung queue; no cause could be shown from the code, so that variant was taken "
                         "out and must not run on a GPU.  Armed per-request kernels below replace it")
def test_resident_kernel_variant_withdrawn():
    pass


@pytest.fixture(scope="module", autouse=True)
def library():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    dl.dl_init(0)
    dl.dl_set_config(arm_timeout_us=ARM_US)
    dl.dl_set_validate(os.environ.get("DL_TEST_VALIDATE") == "1")   # see test_gpu_parity.py
    forced = dict(kv.split("=") for kv in os.environ.get("DL_TEST_CONFIG", "").split(",") if kv)
    if forced:
        dl.dl_set_config(**{k: int(v) for k, v in forced.items()})
    yield
    dl.dl_shutdown()


@pytest.fixture()
def armed():
    dl.dl_prelaunch_start()
    dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
    yield
    if dl.dl_get_mode() == dl.DL_MODE_PRELAUNCH:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    try:
        dl.dl_prelaunch_stop()
    except dl.DlError as e:  # a test may already have stopped it
        assert e.status == dl.DL_ERR_STATE


def fire():
    dl.dl_trigger()
    dl.dl_wait()


def allgather_case(ref, W, B, seed, kind="u8"):
    ins = inputs.allgather_inputs(W, B, seed, kind)
    d_in = [DevBuf(B, fill=ins[r]) for r in range(W)]
    d_out = [DevBuf(W * B) for _ in range(W)]
    sync()
    dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B)
    fire()
    want = ref.allgather(ins)
    for r in range(W):
        assert np.array_equal(d_out[r].host(), want[r]), f"rank {r} (W={W}, B={B})"
        assert d_out[r].guards_intact()


def test_allgather_config0(ref, armed):
    allgather_case(ref, 8, 64 * KiB, seed=0)


@pytest.mark.parametrize("B", [1, 17, 4096, 4097, 8192, 8192 - 16, 8192 + 16, 256 * KiB + 5, 16 * MiB])
def test_allgather_sizes(ref, armed, B):
    allgather_case(ref, 8, B, seed=B, kind="bf16" if B % 2 == 0 else "u8")


@pytest.mark.parametrize("W", [1, 3, 13, 64])
def test_allgather_rank_counts(ref, armed, W):
    allgather_case(ref, W, 5000, seed=W)


def test_alltoall_and_back(ref, armed):
    W = 8
    C = inputs.random_chunks(W, 60000, seed=1, zero_frac=0.2)
    ins = inputs.alltoall_inputs(C, seed=2)
    want = ref.alltoall(ins, C)
    d_in = [DevBuf(a.size, fill=a) for a in ins]
    d_mid = [DevBuf(w.size) for w in want]
    d_back = [DevBuf(a.size) for a in ins]
    sync()
    dl.dl_alltoall([b.ptr() for b in d_in], [b.ptr() for b in d_mid], C)
    dl.dl_alltoall([b.ptr() for b in d_mid], [b.ptr() for b in d_back], C.T)  # same stream: runs after the first
    fire()                                                                    # rings for both tickets
    for j in range(W):
        assert np.array_equal(d_mid[j].host(), want[j]) and d_mid[j].guards_intact()
        assert np.array_equal(d_back[j].host(), ins[j]) and d_back[j].guards_intact()


@pytest.mark.parametrize("T", [16, 128])
def test_alltoall_moe(ref, armed, T):
    C = inputs.moe_dispatch_chunks(8, T, seed=T)
    ins = inputs.alltoall_inputs(C, seed=T + 1, kind="bf16")
    want = ref.alltoall(ins, C)
    d_in = [DevBuf(a.size, fill=a) for a in ins]
    d_out = [DevBuf(w.size) for w in want]
    sync()
    dl.dl_alltoall([b.ptr() for b in d_in], [b.ptr() for b in d_out], C)
    fire()
    for j in range(8):
        assert np.array_equal(d_out[j].host(), want[j]) and d_out[j].guards_intact()


def test_alltoall_long_list_goes_through_table(ref, armed):
    W = 16
    C = inputs.random_chunks(W, 100000, seed=3, zero_frac=0.1)
    ins = inputs.alltoall_inputs(C, seed=4)
    want = ref.alltoall(ins, C)
    d_in = [DevBuf(a.size, fill=a) for a in ins]
    d_out = [DevBuf(w.size) for w in want]
    sync()
    dl.dl_alltoall([b.ptr() for b in d_in], [b.ptr() for b in d_out], C)
    fire()
    for j in range(W):
        assert np.array_equal(d_out[j].host(), want[j]) and d_out[j].guards_intact()


@pytest.mark.parametrize("k,n", [(7, 2 * MiB), (1, 333), (20, 70001), (1, 64 * KiB), (2, 1 * MiB), (4, 48 * KiB)])
def test_broadcast(ref, armed, k, n):
    src = inputs.payload(np.random.default_rng(k), n, "bf16" if n % 2 == 0 else "u8")
    d_src = DevBuf(n, fill=src)
    d_dst = [DevBuf(n) for _ in range(k)]
    sync()
    dl.dl_broadcast(d_src.ptr(), [b.ptr() for b in d_dst], n)
    fire()
    for b, w in zip(d_dst, ref.broadcast(src, k)):
        assert np.array_equal(b.host(), w) and b.guards_intact()


@pytest.mark.parametrize("n,nb,arena,align", [(64, 16 * KiB, 64 * MiB, 256), (300, 5001, 8 * MiB, 1)])
def test_batch(ref, armed, n, nb, arena, align):
    a, descs = inputs.b2b_batch(n, nb, arena, seed=n, align=align)
    want = ref.batch_copy([a.copy()], [(0, s, 0, d, m) for s, d, m in descs])[0]
    d = DevBuf(arena, fill=a)
    sync()
    dl.dl_batch_copy([(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs])
    fire()
    assert np.array_equal(d.host(), want) and d.guards_intact()


@pytest.mark.parametrize("n,max_bytes,shared", [(7, 3000, 0.0), (40, 200000, 0.0), (64, 70000, 0.5), (300, 40000, 0.3)])
def test_batch_of_unequal_sizes_and_alignments_armed(ref, armed, n, max_bytes, shared):
    a, descs = inputs.mixed_batch(n, max_bytes, 48 * MiB, seed=n, shared_sources=shared)
    want = ref.batch_copy([a.copy()], [(0, s, 0, d, m) for s, d, m in descs])[0]
    d = DevBuf(a.size, fill=a)
    sync()
    dl.dl_batch_copy([(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs])
    fire()
    assert np.array_equal(d.host(), want) and d.guards_intact()


def test_item_longer_than_4GiB_armed(ref, armed):
    """Byte offsets past 2^32 in the armed kernels, whose capped grid strides over the tiles."""
    import torch
    n = (4 << 30) + 4112
    src, dst = DevBuf(n), DevBuf(n)
    src.view().random_(0, 256)
    sync()
    dl.dl_batch_copy([(src.ptr(), dst.ptr(), n)])
    fire()
    assert torch.equal(dst.view(), src.view()) and dst.guards_intact()
    lo = (1 << 32) - 2048
    win = src.view()[lo:lo + 4096].cpu().numpy()
    assert np.array_equal(dst.view()[lo:lo + 4096].cpu().numpy(), ref.broadcast(win, 1)[0])


@pytest.mark.parametrize("W,c", [(8, 64 * KiB), (8, 1000), (3, 300 * KiB + 16), (13, 5001)])
def test_alltoall_inplace_armed(ref, armed, W, c):
    bufs = inputs.alltoall_inputs(inputs.uniform_chunks(W, c), seed=W + c, kind="fp16" if c % 2 == 0 else "u8")
    d = [DevBuf(W * c, fill=bufs[i]) for i in range(W)]
    sync()
    dl.dl_alltoall_inplace([b.ptr() for b in d], c)
    fire()
    want = ref.alltoall_inplace(bufs, c)
    for i in range(W):
        assert np.array_equal(d[i].host(), want[i]) and d[i].guards_intact()


@pytest.mark.parametrize("T", [16, 128])
def test_token_dispatch_armed(ref, armed, T):
    W, row = 8, 14336
    ins = inputs.token_rows(W, T, row, seed=T, kind="bf16")
    dest = inputs.moe_token_destinations(W, T, seed=T + 1)
    want = ref.token_dispatch(ins, row, dest)
    d_in = [DevBuf(a.size, fill=a) for a in ins]
    d_out = [DevBuf(w.size) for w in want]
    sync()
    dl.dl_token_dispatch([b.ptr() for b in d_in], [b.ptr() for b in d_out], [T] * W, row, dest)
    fire()
    for j in range(W):
        assert np.array_equal(d_out[j].host(), want[j]) and d_out[j].guards_intact()


def test_batch_swap_armed_twice_restores(ref, armed):
    arena, descs = inputs.swap_batch(30, 20000, 8 * MiB, seed=9, align=16)
    d = DevBuf(8 * MiB, fill=arena)
    sw = [(d.ptr(int(a)), d.ptr(int(b)), int(m)) for a, b, m in descs]
    sync()
    dl.dl_batch_swap(sw)
    fire()
    want = ref.batch_swap([arena.copy()], [(0, a, 0, b, m) for a, b, m in descs])[0]
    assert np.array_equal(d.host(), want)
    dl.dl_batch_swap(sw)
    fire()
    assert np.array_equal(d.host(), arena) and d.guards_intact()


def test_sources_written_after_arming_are_seen(ref, armed):
    """The point of prelaunch: the request is armed first, its inputs are
    produced afterwards, and only then is the doorbell rung.  The same device
    buffers get new contents every round, so a stale cached copy would show."""
    import torch
    W, B = 8, 48 * KiB
    d_in = [DevBuf(B) for _ in range(W)]
    d_out = [DevBuf(W * B) for _ in range(W)]
    up = torch.cuda.Stream()   # uploads must not queue behind the armed kernel
    for rnd in range(6):
        dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B)
        dl.dl_wait_armed()
        ins = inputs.allgather_inputs(W, B, seed=100 + rnd)
        with torch.cuda.stream(up):
            for r in range(W):
                d_in[r].view().copy_(torch.from_numpy(ins[r]))
        up.synchronize()
        fire()
        want = ref.allgather(ins)
        for r in range(W):
            assert np.array_equal(d_out[r].host(), want[r]), f"round {rnd} rank {r}"


@pytest.mark.parametrize("B", [1 * MiB, 8 * MiB])
def test_large_armed_request_leaves_room_for_its_producers(ref, armed, B):
    """A request with more tiles than the armed grid holds is armed first; then kernels on another stream
    produce its sources, and only then is the doorbell rung.  The armed kernel, resident and polling all the
    while, must not take every wavefront slot: the producers have to run beside it, or the request can only
    expire.  Unfused (64 copies), so that the grid is at its cap."""
    import torch
    W = 8
    dl.dl_set_config(fuse_broadcast=0)
    try:
        d_in = [torch.zeros(B, dtype=torch.uint8, device="cuda") for _ in range(W)]
        d_out = [torch.zeros(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)]
        sync()
        dl.dl_allgather(d_in, d_out, B)
        dl.dl_wait_armed()
        for round_ in range(20):                      # producers that need many workgroups of their own
            for j in range(W):
                d_in[j].fill_((round_ * 13 + j * 29) % 251)
        sync()
        fire()
        for r in (0, 5):
            got = d_out[r].view(W, B)
            want = torch.tensor([(19 * 13 + j * 29) % 251 for j in range(W)], dtype=torch.uint8, device="cuda")
            assert bool((got == want[:, None]).all())
    finally:
        dl.dl_set_config(fuse_broadcast=1)


def test_armed_request_waits_beside_a_matrix_multiplication(armed):
    """The producer of an armed request's input is a large bf16 matrix multiplication, whose wavefronts take all
    the vector registers of a SIMD and so cannot share one with a waiting wavefront.  It must run, and in its own
    time, while a request with more tiles than the armed grid holds waits for the doorbell (a grid with a
    workgroup on every compute unit kept it from starting until the request expired)."""
    import time
    import torch
    W, B, n = 8, 2 * MiB, 4096
    a = torch.randn(n, n, dtype=torch.bfloat16, device="cuda")
    b = torch.randn(n, n, dtype=torch.bfloat16, device="cuda")
    torch.matmul(a, b)                                   # library set-up stays outside
    sync()
    d_in = [torch.zeros(B, dtype=torch.uint8, device="cuda") for _ in range(W)]
    d_out = [torch.zeros(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)]
    sync()
    dl.dl_allgather(d_in, d_out, B)
    dl.dl_wait_armed()
    t0 = time.perf_counter()
    c = torch.matmul(a, b)
    src = c.view(torch.uint8).reshape(-1)                # 32 MiB of results: the request's sources
    for j in range(W):
        d_in[j].copy_(src[j * B:(j + 1) * B])
    sync()
    waited = time.perf_counter() - t0
    fire()
    assert waited < ARM_US * 1e-6 / 3, f"the producers took {waited * 1e3:.1f} ms beside the waiting request"
    for r in (0, 6):
        assert torch.equal(d_out[r], src[:W * B])


def test_many_requests_armed_at_once(ref, armed):
    """A full set of 64 armed requests on one stream, one doorbell write for all."""
    W, B, N = 4, 3000, 64
    cases = []
    for i in range(N):
        ins = inputs.allgather_inputs(W, B, seed=200 + i)
        cases.append((ins, [DevBuf(B, fill=a) for a in ins], [DevBuf(W * B) for _ in range(W)]))
    sync()
    first = None
    for ins, d_in, d_out in cases:
        dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B)
        first = first or dl.dl_last_ticket()
    last = dl.dl_last_ticket()
    assert last == first + N - 1
    dl.dl_trigger(last)
    dl.dl_wait(last)
    dl.dl_wait(first)
    for ins, d_in, d_out in cases:
        want = ref.allgather(ins)
        for r in range(W):
            assert np.array_equal(d_out[r].host(), want[r])


@pytest.mark.parametrize("push,count", [(1, 40), (0, 4)])
def test_many_long_lists_armed_at_once(ref, armed, push, count):
    """Armed requests whose copy lists are too long for the kernel arguments keep their tables in memory that
    is reused in turn: 40 of them at once with the tables written through the BAR; through the pinned ring four,
    and the fifth is refused at once (it could only get its slot by outwaiting an untriggered request) and can
    be armed after the others have run."""
    if push and os.environ.get("DL_NO_BAR") == "1":
        pytest.skip("tables are kept in the pinned ring: four at a time")
    base = dl.dl_get_config()
    saved = {f[0]: getattr(base, f[0]) for f in base._fields_}
    dl.dl_set_config(table_push=push)
    try:
        cases = []
        for i in range(count + 1):
            arena, descs = inputs.mixed_batch(90 + i, 3000, 2 * MiB, seed=300 + i)
            want = ref.batch_copy([arena.copy()], [(0, s, 0, d, m) for s, d, m in descs])[0]
            d = DevBuf(arena.size, fill=arena)
            cases.append((d, [(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs], want))
        sync()
        for d, copies, want in cases[:count]:
            dl.dl_batch_copy(copies)
        last = dl.dl_last_ticket()
        extra = cases[count]
        if not push:
            with pytest.raises(dl.DlError) as e:
                dl.dl_batch_copy(extra[1])
            assert e.value.status == dl.DL_ERR_STATE
            assert dl.dl_last_ticket() == last        # and it took no ticket
        dl.dl_trigger(last)
        dl.dl_wait(last)
        dl.dl_batch_copy(extra[1])
        fire()
        for d, copies, want in cases:
            assert np.array_equal(d.host(), want) and d.guards_intact()
    finally:
        dl.dl_set_config(**saved)


def test_slots_reused_by_requests_with_other_completion_words(ref, armed):
    """200 requests, more than three rounds over the 64 slots, their grids cycling through 1, 3, 13 and 40
    workgroups, so that a slot's next request reports in fewer or more completion words than the one before;
    waiting for a ticket whose slot has long been reused is not an error."""
    sizes = [100, 10000, 100000, 160 * KiB]
    srcs = {n: inputs.payload(np.random.default_rng(n), n) for n in sizes}
    d_src = {n: DevBuf(n, fill=srcs[n]) for n in sizes}
    d_dst = {n: DevBuf(n) for n in sizes}
    sync()
    first = None
    for i in range(200):
        n = sizes[(i * 7 + i // 5) % len(sizes)]
        d_dst[n].view().zero_()
        sync()
        dl.dl_broadcast(d_src[n].ptr(), [d_dst[n].ptr()], n)
        first = first or dl.dl_last_ticket()
        fire()
        assert np.array_equal(d_dst[n].host(), srcs[n]), (i, n)
    dl.dl_wait(first)
    dl.dl_wait(first + 100)


def test_trigger_in_ticket_order(ref, armed):
    """Ringing for ticket t releases t and everything before it, nothing after it."""
    B = 2000
    bufs = []
    for i in range(3):
        src = inputs.payload(np.random.default_rng(i), B)
        bufs.append((src, DevBuf(B, fill=src), DevBuf(B)))
    sync()
    tickets = []
    for src, d_src, d_dst in bufs:
        dl.dl_broadcast(d_src.ptr(), [d_dst.ptr()], B)
        tickets.append(dl.dl_last_ticket())
    dl.dl_trigger(tickets[1])
    dl.dl_wait(tickets[1])
    with pytest.raises(dl.DlError) as e:
        dl.dl_wait(tickets[2], 0)            # polls once: the third is still armed
    assert e.value.status == dl.DL_ERR_TIMEOUT
    dl.dl_trigger(tickets[2])
    dl.dl_wait(tickets[2])
    for src, d_src, d_dst in bufs:
        assert np.array_equal(d_dst.host(), src)


def test_armed_on_callers_stream_after_its_producer(ref, armed):
    """On the caller's stream the armed kernel is ordered after the kernel that
    produces its input, so the doorbell may be rung at once."""
    import torch
    s = torch.cuda.Stream()
    n = 1 * MiB
    with torch.cuda.stream(s):
        x = torch.arange(n, device="cuda", dtype=torch.int32)
        y = (x * 3 + 1).to(torch.uint8)           # producer kernels on s
        outs = [torch.zeros(n, dtype=torch.uint8, device="cuda") for _ in range(3)]
        dl.dl_broadcast(y, outs, n, s)
    dl.dl_trigger()
    dl.dl_wait()
    want = ((np.arange(n, dtype=np.int64) * 3 + 1) % 256).astype(np.uint8)
    for o in outs:
        assert np.array_equal(o.cpu().numpy(), want)


@pytest.mark.parametrize("k", [3, 4, 7])
def test_forced_shape_with_sub_groups_and_several_passes(ref, armed, k):
    """A forced tile and workgroup size under which a fan-out of 3 or 4 is shared out over two sub-groups of
    the workgroup, in a request long enough for several passes of the waiting grid: every destination is written."""
    base = dl.dl_get_config()
    saved = {f[0]: getattr(base, f[0]) for f in base._fields_}
    dl.dl_set_config(tile_bytes=2048, block_threads=256)
    try:
        n = 1 * MiB + 48
        src = inputs.payload(np.random.default_rng(k), n)
        d_src = DevBuf(n, fill=src)
        d_dst = [DevBuf(n) for _ in range(k)]
        sync()
        dl.dl_broadcast(d_src.ptr(), [b.ptr() for b in d_dst], n)
        fire()
    finally:
        dl.dl_set_config(**saved)
    for j, b in enumerate(d_dst):
        assert np.array_equal(b.host(), src), f"destination {j}"
        assert b.guards_intact()


def test_phase_stamps_are_ordered_and_clock_relates_to_host(ref, armed):
    import time
    rate, host_ns_at_tick0 = dl.dl_trace_clock()
    assert 1.0 <= rate <= 10000.0                       # ticks per microsecond
    dl.dl_set_trace(True)
    try:
        for B in (4 * KiB, 1 * MiB):                    # every workgroup polls / one polls and fans out
            W = 8
            ins = inputs.allgather_inputs(W, B, seed=B)
            d_in = [DevBuf(B, fill=a) for a in ins]
            d_out = [DevBuf(W * B) for _ in range(W)]
            sync()
            dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B)
            dl.dl_wait_armed()
            t0 = time.clock_gettime_ns(time.CLOCK_MONOTONIC)
            fire()
            t1 = time.clock_gettime_ns(time.CLOCK_MONOTONIC)
            tr = dl.dl_get_trace()
            assert tr["doorbell_seen"] <= tr["copy_begin"] <= tr["copy_end"] <= tr["completion_issued"]
            assert (tr["completion_issued"] - tr["doorbell_seen"]) / rate <= (t1 - t0) / 1e3   # inside the host's window
            for name in ("doorbell_seen", "completion_issued"):
                at = host_ns_at_tick0 + tr[name] * 1e3 / rate
                assert t0 - 50_000 <= at <= t1 + 50_000, name                 # within 50 us of the host's window
            for r, w in zip(d_out, ref.allgather(ins)):
                assert np.array_equal(r.host(), w)
    finally:
        dl.dl_set_trace(False)
    with pytest.raises(dl.DlError) as e:
        dl.dl_get_trace(dl.dl_last_ticket() + 1)
    assert e.value.status == dl.DL_ERR_INVALID


@pytest.mark.parametrize("blocks", [1, 5, 300])
def test_armed_grid_cap(ref, armed, blocks):
    """armed_blocks caps an armed kernel's grid: 1 workgroup (it polls and copies everything), a handful (all
    poll), hundreds (one polls, the rest follow its flags)."""
    dl.dl_set_config(armed_blocks=blocks)
    try:
        allgather_case(ref, 8, 200 * KiB + 16, seed=blocks, kind="bf16")
        allgather_case(ref, 5, 7001, seed=blocks + 1)
    finally:
        dl.dl_set_config(armed_blocks=0)


def test_armed_requests_back_to_back_with_changing_sources(armed):
    """10000 armed all-gathers in a row over the same buffers, the sources rewritten (by another stream) before
    every doorbell and the receive buffers checked (by that stream) right after every completion word: a load
    served from a stale cache line, or a store not yet visible when the completion word is, shows up as a
    wrong byte.  Sizes cycle through both doorbell schemes (every workgroup polls / one polls and fans out)."""
    import torch
    W = 8
    sizes = [4 * KiB, 48 * KiB, 256 * KiB]
    d_in = {B: [torch.zeros(B, dtype=torch.uint8, device="cuda") for _ in range(W)] for B in sizes}
    d_out = {B: [torch.zeros(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)] for B in sizes}
    bad = torch.zeros(1, dtype=torch.int64, device="cuda")
    for it in range(10000):
        B = sizes[it % len(sizes)]
        dl.dl_allgather(d_in[B], d_out[B], B)              # armed on the library's stream, polling
        for j in range(W):
            d_in[B][j].fill_((it * 7 + j * 31) % 251)      # sources written after arming, on torch's stream
        sync()
        fire()
        for r in (it % W, (it + 3) % W):                   # two receive buffers per round, checked on the device
            got = d_out[B][r].view(W, B)
            want = torch.tensor([(it * 7 + j * 31) % 251 for j in range(W)], dtype=torch.uint8, device="cuda")
            bad += (got != want[:, None]).sum()
    sync()
    assert int(bad.item()) == 0


def test_signal_mode_completes_without_trigger_or_stream_sync(ref):
    """DL_MODE_SIGNAL: the kernel starts at once; dl_wait on the ticket is the only synchronisation used here
    between the library's stream and the reads below."""
    import torch
    dl.dl_prelaunch_start()
    dl.dl_set_mode(dl.DL_MODE_SIGNAL)
    try:
        for W, B in ((8, 4 * KiB), (8, 300 * KiB + 16), (3, 7001), (13, 5000)):
            ins = inputs.allgather_inputs(W, B, seed=B)
            d_in = [DevBuf(B, fill=a) for a in ins]
            d_out = [DevBuf(W * B) for _ in range(W)]
            sync()
            before = dl.dl_last_ticket()
            dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B)
            assert dl.dl_last_ticket() == before + 1
            dl.dl_wait()
            for r, w in zip(d_out, ref.allgather(ins)):
                assert np.array_equal(r.host(), w) and r.guards_intact()
        C = inputs.moe_dispatch_chunks(8, 16, seed=4)
        ins = inputs.alltoall_inputs(C, seed=5, kind="bf16")
        want = ref.alltoall(ins, C)
        d_in = [DevBuf(a.size, fill=a) for a in ins]
        d_out = [DevBuf(w.size) for w in want]
        sync()
        dl.dl_alltoall([b.ptr() for b in d_in], [b.ptr() for b in d_out], C)
        dl.dl_wait()
        for r, w in zip(d_out, want):
            assert np.array_equal(r.host(), w) and r.guards_intact()
        # a request issued in prelaunch mode right after still waits for its doorbell
        dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
        src = DevBuf(4096, fill=inputs.payload(np.random.default_rng(1), 4096))
        dst = DevBuf(4096)
        sync()
        dl.dl_batch_copy([(src.ptr(), dst.ptr(), 4096)])
        with pytest.raises(dl.DlError) as e:
            dl.dl_wait(timeout_ns=2_000_000)
        assert e.value.status == dl.DL_ERR_TIMEOUT
        assert (dst.host() == CANARY).all()
        fire()
        assert np.array_equal(dst.host(), src.host())
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_prelaunch_stop()


@pytest.mark.parametrize("n", [3000, 100000, 1 * MiB])
def test_untriggered_request_expires_and_copies_nothing(ref, n):
    """One workgroup, a grid whose workgroups each report in a completion word of their own, and a grid whose
    arrivals are counted."""
    dl.dl_set_config(arm_timeout_us=3000)
    try:
        dl.dl_prelaunch_start()
        dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
        src = DevBuf(n, fill=inputs.payload(np.random.default_rng(1), n))
        dst = [DevBuf(n) for _ in range(8)]
        sync()
        dl.dl_broadcast(src.ptr(), [b.ptr() for b in dst], n)
        with pytest.raises(dl.DlError) as e:
            dl.dl_wait()                       # never triggered
        assert e.value.status == dl.DL_ERR_EXPIRED
        for b in dst:
            assert (b.host() == CANARY).all()
        # a late doorbell does nothing, and the next request works
        dl.dl_trigger()
        dl.dl_set_config(arm_timeout_us=ARM_US)
        dl.dl_broadcast(src.ptr(), [b.ptr() for b in dst], n)
        fire()
        for b in dst:
            assert np.array_equal(b.host(), src.host())
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_prelaunch_stop()
        dl.dl_set_config(arm_timeout_us=ARM_US)


def test_stop_cancels_what_is_still_armed(ref):
    import time
    dl.dl_prelaunch_start()
    dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
    src = DevBuf(5000, fill=inputs.payload(np.random.default_rng(2), 5000))
    dst = DevBuf(5000)
    sync()
    dl.dl_broadcast(src.ptr(), [dst.ptr()], 5000)
    dl.dl_wait_armed()
    t0 = time.perf_counter()
    dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    dl.dl_prelaunch_stop()                       # cancels: well before the 300 ms arm limit
    assert time.perf_counter() - t0 < 0.2
    assert (dst.host() == CANARY).all()
    assert dl.dl_get_mode() == dl.DL_MODE_ONESHOT


def test_one_shot_calls_between_armed_ones(ref, armed):
    dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    ins = inputs.allgather_inputs(8, 10000, seed=9)
    d_in = [DevBuf(10000, fill=a) for a in ins]
    d_out = [DevBuf(80000) for _ in range(8)]
    dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], 10000, stream())
    sync()
    for r, w in enumerate(ref.allgather(ins)):
        assert np.array_equal(d_out[r].host(), w)
    dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
    allgather_case(ref, 8, 10000, seed=10)


def test_empty_request_takes_no_ticket(armed):
    d = DevBuf(256)
    before = dl.dl_last_ticket()
    dl.dl_broadcast(d.ptr(), [d.ptr(128)], 0)
    dl.dl_batch_copy([])
    assert dl.dl_last_ticket() == before


def test_lifecycle_errors():
    with pytest.raises(dl.DlError) as e:
        dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)          # not started
    assert e.value.status == dl.DL_ERR_STATE
    for fn in (dl.dl_prelaunch_stop, lambda: dl.dl_trigger(1), lambda: dl.dl_wait(1, 0)):
        with pytest.raises(dl.DlError) as e:
            fn()
        assert e.value.status == dl.DL_ERR_STATE
    dl.dl_prelaunch_start()
    try:
        with pytest.raises(dl.DlError) as e:
            dl.dl_prelaunch_start()                   # twice
        assert e.value.status == dl.DL_ERR_STATE
        for fn in (lambda: dl.dl_wait(1, 1000), lambda: dl.dl_trigger(1), lambda: dl.dl_wait_armed(1, 0)):
            with pytest.raises(dl.DlError) as e:
                fn()                                  # a ticket never issued
            assert e.value.status == dl.DL_ERR_INVALID
        with pytest.raises(dl.DlError) as e:
            dl.dl_set_config(arm_timeout_us=0)
        assert e.value.status == dl.DL_ERR_INVALID
        with pytest.raises(dl.DlError) as e:
            dl.dl_set_config(arm_timeout_us=2_000_000)
        assert e.value.status == dl.DL_ERR_INVALID
    finally:
        dl.dl_prelaunch_stop()
    assert dl.dl_get_mode() == dl.DL_MODE_ONESHOT


# ------------------------------------------ large armed requests: a gate kernel waits, the copy kernel follows

def test_large_armed_request_sources_written_after_arming(ref, armed):
    """4 MiB per rank (288 MiB moved: above the 256 MiB from which a one-workgroup gate kernel does the waiting and a
    full-grid copy kernel follows it on the stream).  Armed first, sources produced afterwards on another stream,
    then the doorbell; twice over the same buffers with new contents."""
    import torch
    W, B = 8, 4 * MiB
    d_in = [DevBuf(B) for _ in range(W)]
    d_out = [DevBuf(W * B) for _ in range(W)]
    up = torch.cuda.Stream()
    for rnd in range(2):
        dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B)
        dl.dl_wait_armed()
        ins = inputs.allgather_inputs(W, B, seed=300 + rnd, kind="bf16")
        with torch.cuda.stream(up):
            for r in range(W):
                d_in[r].view().copy_(torch.from_numpy(ins[r]))
        up.synchronize()
        fire()
        want = ref.allgather(ins)
        for r in range(W):
            assert np.array_equal(d_out[r].host(), want[r]) and d_out[r].guards_intact(), f"round {rnd} rank {r}"


@pytest.mark.parametrize("what", ["misaligned", "long_list", "swap"])
def test_large_armed_requests_of_other_kinds(ref, armed, what):
    """The gate in front of the general path (addresses that disagree modulo 16), of a table kernel (300 copies of
    512 KiB) and of swaps (an in-place all-to-all of 12 MiB chunks between four ranks); each moves 280 MiB or more."""
    if what == "misaligned":
        W, B = 4, 14 * MiB + 5
        ins = inputs.allgather_inputs(W, B, seed=41)
        d_in = [DevBuf(B, fill=ins[r], shift=r + 1) for r in range(W)]
        d_out = [DevBuf(W * B, shift=2 * r) for r in range(W)]
        sync()
        dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B)
        fire()
        for got, want in zip(d_out, ref.allgather(ins)):
            assert np.array_equal(got.host(), want) and got.guards_intact()
    elif what == "long_list":
        arena, descs = inputs.b2b_batch(300, 512 * KiB, 400 * MiB, seed=42, align=4096)
        want = ref.batch_copy([arena.copy()], [(0, s, 0, t, m) for s, t, m in descs])[0]
        d = DevBuf(arena.size, fill=arena)
        sync()
        dl.dl_batch_copy([(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs])
        fire()
        assert np.array_equal(d.host(), want) and d.guards_intact()
    else:
        W, c = 4, 12 * MiB
        bufs = inputs.alltoall_inputs(inputs.uniform_chunks(W, c), seed=43)
        d_buf = [DevBuf(a.size, fill=a) for a in bufs]
        sync()
        dl.dl_alltoall_inplace([b.ptr() for b in d_buf], c)
        fire()
        for b, w in zip(d_buf, ref.alltoall_inplace(bufs, c)):
            assert np.array_equal(b.host(), w) and b.guards_intact()


def test_large_untriggered_request_expires_and_copies_nothing(ref):
    """The gate kernel gives up at the arm limit; the copy kernel behind it reads that and reports the request as
    expired without touching a byte.  A request that follows works."""
    dl.dl_set_config(arm_timeout_us=3000)
    try:
        dl.dl_prelaunch_start()
        dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
        n = 32 * MiB                                      # 1 + 8 destinations: 288 MiB moved
        src = DevBuf(n, fill=inputs.payload(np.random.default_rng(1), n))
        dst = [DevBuf(n) for _ in range(8)]
        sync()
        dl.dl_broadcast(src.ptr(), [b.ptr() for b in dst], n)
        with pytest.raises(dl.DlError) as e:
            dl.dl_wait()                                  # never triggered
        assert e.value.status == dl.DL_ERR_EXPIRED
        for b in dst:
            assert (b.host() == CANARY).all()
        dl.dl_trigger()                                   # a late doorbell does nothing
        dl.dl_set_config(arm_timeout_us=ARM_US)
        dl.dl_broadcast(src.ptr(), [b.ptr() for b in dst], n)
        fire()
        for b in dst:
            assert np.array_equal(b.host(), src.host()) and b.guards_intact()
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_prelaunch_stop()
        dl.dl_set_config(arm_timeout_us=ARM_US)


def test_stop_cancels_a_large_armed_request(ref):
    import time
    dl.dl_prelaunch_start()
    dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
    n = 160 * MiB
    src = DevBuf(n, fill=inputs.payload(np.random.default_rng(2), n))
    dst = DevBuf(n)
    sync()
    dl.dl_broadcast(src.ptr(), [dst.ptr()], n)
    dl.dl_wait_armed()
    t0 = time.perf_counter()
    dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    dl.dl_prelaunch_stop()                       # cancels: well before the 300 ms arm limit
    assert time.perf_counter() - t0 < 0.2
    assert (dst.host() == CANARY).all()
