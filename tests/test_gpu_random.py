"""Seeded random requests: operation, rank count, sizes, alignments, mode and tunables drawn per case,
every result compared byte for byte with the CPU checker.  The fixed-shape tests cover each path on its
own; these cover the combinations.  A failing case names its seed and prints what it drew."""

import os

import numpy as np
import pytest

import paper_2511_06605_amd as dl
from paper_2511_06605_amd import inputs
from paper_2511_06605_amd.inputs import KiB

from gpu_util import DevBuf, sync

pytestmark = pytest.mark.gpu

TUNABLES = [
    {}, {}, {},
    {"fan_split": 1}, {"fan_split": 2}, {"fan_split": 4},
    {"tile_bytes": 1024, "block_threads": 64}, {"tile_bytes": 8192, "block_threads": 512},
    {"tile_bytes": 65536, "block_threads": 256},
    {"max_blocks": 7}, {"armed_blocks": 5},
    {"fuse_broadcast": 0}, {"infer_broadcast": 0}, {"device_lowering": 0},
    {"write_through_max_bytes": 0}, {"nontemporal_min_bytes": 1}, {"table_push": 0},
]


@pytest.fixture(scope="module", autouse=True)
def library():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    dl.dl_init(0)
    dl.dl_set_config(arm_timeout_us=300_000)
    dl.dl_prelaunch_start()
    yield
    dl.dl_set_mode(dl.DL_MODE_ONESHOT)
    dl.dl_prelaunch_stop()
    dl.dl_shutdown()


def size(rng, top):
    """Log-uniform in [1, top], now and then 0 or a round number."""
    u = rng.random()
    if u < 0.05:
        return 0
    n = int(np.exp(rng.uniform(0.0, np.log(top))))
    if u < 0.35:
        n = max(16, n // 16 * 16)
    if u < 0.15:
        n = max(1024, n // 1024 * 1024)
    return n


def shifts(rng, n):
    """Per-buffer misalignment (DevBuf allows up to 127 bytes): mostly none; else all alike, or multiples of 4 or
    of 16 (off the 128-byte grid that tiles are cut on, whole vectors), or arbitrary."""
    kind = rng.choice(["none", "none", "same", "mod4", "mod16", "any"])
    if kind == "none":
        return [0] * n
    if kind == "same":
        return [int(rng.integers(1, 128))] * n
    if kind == "mod4":
        return [4 * int(rng.integers(0, 32)) for _ in range(n)]
    if kind == "mod16":
        return [16 * int(rng.integers(0, 8)) for _ in range(n)]
    return [int(rng.integers(0, 128)) for _ in range(n)]


def finish(mode, ticket_before):
    """Wait for the request just issued.  An empty request enqueues nothing and takes no ticket."""
    if mode == "oneshot" or dl.dl_last_ticket() == ticket_before:
        sync()
    elif mode == "prelaunch":
        dl.dl_trigger()
        dl.dl_wait()
    else:
        dl.dl_wait()


def check(bufs, want, what):
    for i, (b, w) in enumerate(zip(bufs, want)):
        assert np.array_equal(b.host(), w), f"{what}: buffer {i} differs"
        assert b.guards_intact(), f"{what}: guard band of buffer {i} written"


MODES = ("oneshot", "oneshot", "prelaunch", "signal")


def run_case(ref, seed, scale=1, modes=MODES):
    import torch
    rng = np.random.default_rng(seed)
    op = str(rng.choice(["allgather", "alltoall", "broadcast", "batch", "swap", "inplace", "token", "fanout"]))
    mode = str(rng.choice(list(modes)))
    tun = dict(TUNABLES[int(rng.integers(0, len(TUNABLES)))])
    W = int(rng.choice([1, 2, 3, 4, 7, 8, 8, 8, 9, 16]))
    what = f"seed {seed}: {op}, W={W}, {mode}, {tun}"
    st = torch.cuda.current_stream()
    base = dl.dl_get_config()
    saved = {f[0]: getattr(base, f[0]) for f in base._fields_}
    dl.dl_set_config(**tun)
    dl.dl_set_mode({"oneshot": dl.DL_MODE_ONESHOT, "prelaunch": dl.DL_MODE_PRELAUNCH, "signal": dl.DL_MODE_SIGNAL,
                    "standby": dl.DL_MODE_STANDBY, "auto": dl.DL_MODE_AUTO}[mode])
    s_arg = st if mode == "oneshot" else None
    before = dl.dl_last_ticket()
    try:
        if op == "allgather":
            B = size(rng, scale * 300 * KiB)
            sh = shifts(rng, 2 * W)
            ins = inputs.allgather_inputs(W, B, seed)
            d_in = [DevBuf(B, fill=ins[r], shift=sh[r]) for r in range(W)]
            d_out = [DevBuf(W * B, shift=sh[W + r]) for r in range(W)]
            sync()
            dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B, s_arg)
            finish(mode, before)
            check(d_out, ref.allgather(ins), what)
            check(d_in, ins, what + " (sources)")
        elif op == "alltoall":
            C = np.array([[size(rng, scale * 40 * KiB) for _ in range(W)] for _ in range(W)], dtype=np.uint64)
            ins = inputs.alltoall_inputs(C, seed)
            want = ref.alltoall(ins, C)
            sh = shifts(rng, 2 * W)
            d_in = [DevBuf(ins[i].size, fill=ins[i], shift=sh[i]) for i in range(W)]
            d_out = [DevBuf(want[j].size, shift=sh[W + j]) for j in range(W)]
            sync()
            dl.dl_alltoall([b.ptr() for b in d_in], [b.ptr() for b in d_out], C, s_arg)
            finish(mode, before)
            check(d_out, want, what)
        elif op == "broadcast":
            k, n = int(rng.integers(1, 20)), size(rng, scale * 600 * KiB)
            src = inputs.payload(rng, n)
            sh = shifts(rng, k + 1)
            d_src = DevBuf(n, fill=src, shift=sh[0])
            d_dst = [DevBuf(n, shift=sh[1 + q]) for q in range(k)]
            sync()
            dl.dl_broadcast(d_src.ptr(), [b.ptr() for b in d_dst], n, s_arg)
            finish(mode, before)
            check(d_dst, ref.broadcast(src, k), what)
        elif op == "batch":
            n = int(rng.choice([1, 3, 8, 9, 40, 64, 65, 300, 700]))
            arena, descs = inputs.mixed_batch(n, int(rng.choice([200, 5000, 120000])) * (scale if n <= 65 else 1), scale * (24 << 20), seed=seed,
                                              shared_sources=float(rng.choice([0.0, 0.0, 0.4])))
            want = ref.batch_copy([arena.copy()], [(0, s, 0, d, m) for s, d, m in descs])[0]
            d = DevBuf(arena.size, fill=arena)
            sync()
            dl.dl_batch_copy([(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs], s_arg)
            finish(mode, before)
            check([d], [want], what)
        elif op == "swap":
            n = int(rng.choice([1, 5, 30, 70, 200]))
            arena, descs = inputs.swap_batch(n, max(1, size(rng, (scale if n <= 70 else 1) * 30 * KiB)), scale * (16 << 20), seed=seed,
                                             align=int(rng.choice([1, 4, 16, 256])))
            want = ref.batch_swap([arena.copy()], [(0, a, 0, b, m) for a, b, m in descs])[0]
            d = DevBuf(arena.size, fill=arena)
            sync()
            dl.dl_batch_swap([(d.ptr(int(a)), d.ptr(int(b)), int(m)) for a, b, m in descs], s_arg)
            finish(mode, before)
            check([d], [want], what)
        elif op == "inplace":
            c = size(rng, scale * 100 * KiB)
            bufs = inputs.alltoall_inputs(inputs.uniform_chunks(W, c), seed=seed)
            d = [DevBuf(W * c, fill=bufs[i]) for i in range(W)]
            sync()
            dl.dl_alltoall_inplace([b.ptr() for b in d], c, s_arg)
            finish(mode, before)
            check(d, ref.alltoall_inplace(bufs, c), what)
        elif op == "token":
            row = int(rng.choice([16, 48, 100, 1024, 1040, 4097, 14336]))
            top = int(rng.choice([3, 40, 200])) * (4 if scale > 1 else 1)
            counts = [int(rng.integers(0, top)) for _ in range(W)]
            ins = inputs.token_rows(W, counts, row, seed=seed)
            dest = inputs.moe_token_destinations(W, counts, seed=seed + 1, n_experts=16 * W, top_k=int(rng.integers(1, min(8, W) + 1)))
            if rng.random() < 0.3 and len(dest):
                dest[::int(rng.integers(2, 6))] = 0
            want = ref.token_dispatch(ins, row, dest)
            d_in = [DevBuf(a.size, fill=a) for a in ins]
            d_out = [DevBuf(w.size) for w in want]
            sync()
            dl.dl_token_dispatch([b.ptr() for b in d_in], [b.ptr() for b in d_out], counts, row, dest, s_arg)
            finish(mode, before)
            check(d_out, want, what)
        else:  # fanout
            n_items, slot = int(rng.choice([1, 6, 24, 40, 150])), int(rng.choice([300, 20000]))
            arena = rng.integers(0, 256, (n_items * 9 + 1) * slot, dtype=np.uint8)
            d = DevBuf(arena.size, fill=arena)
            items, copies = [], []
            for i in range(n_items):
                k, nb = int(rng.integers(1, 9)), int(rng.integers(1, slot))
                s0 = i * 9 * slot + int(rng.integers(0, 4)) * int(rng.choice([0, 1, 4]))
                dsts = [i * 9 * slot + (q + 1) * slot for q in range(k)]
                items.append(dict(src=d.ptr(s0), bytes=min(nb, slot - 16), dst=[d.ptr(t) for t in dsts]))
                copies += [(0, s0, 0, t, min(nb, slot - 16)) for t in dsts]
            want = ref.batch_copy([arena.copy()], copies)[0]
            sync()
            dl.dl_batch_fanout(items, s_arg)
            finish(mode, before)
            check([d], [want], what)
    except Exception:
        print(what, flush=True)
        raise
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_set_config(**saved)


N_CASES = int(os.environ.get("DL_TEST_RANDOM_CASES", "240"))


@pytest.mark.parametrize("first", range(0, N_CASES, 20))
def test_random_requests(ref, first):
    for seed in range(first, min(first + 20, N_CASES)):
        run_case(ref, seed)


N_LARGE = int(os.environ.get("DL_TEST_RANDOM_LARGE_CASES", "24"))


@pytest.mark.parametrize("first", range(0, N_LARGE, 8))
def test_random_requests_large(ref, first):
    """The same draws with sizes up to 16 times larger: across the thresholds of the store policies, of the row
    kernel over staged tables and of the armed grid's cap."""
    for seed in range(first, min(first + 8, N_LARGE)):
        run_case(ref, 1_000_000 + seed, scale=16)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_requests_back_to_back_depend_on_each_other_in_stream_order(ref, seed):
    """Thirty batches on one stream with no synchronisation between them, each reading what earlier ones wrote
    (inside one arena): lists in the kernel arguments, table kernels reading the pinned ring, tables staged in
    device memory and swaps, so that the ring's four slots are reused while earlier requests are still queued.
    The checker applies the same batches one after the other."""
    import torch
    rng = np.random.default_rng(seed)
    size_ = 12 << 20
    arena = rng.integers(0, 256, size_, dtype=np.uint8)
    want = arena.copy()
    d = DevBuf(size_, fill=arena)
    sync()
    st = torch.cuda.current_stream()
    for step in range(30):
        n = int(rng.choice([3, 8, 60, 100, 700, 3000]))
        if rng.random() < 0.25:
            _, descs = inputs.swap_batch(min(n, 200), int(rng.choice([48, 1000, 20000])), size_, seed=1000 * seed + step,
                                         align=int(rng.choice([1, 16])))
            ref.batch_swap([want], [(0, a, 0, b, m) for a, b, m in descs])
            dl.dl_batch_swap([(d.ptr(int(a)), d.ptr(int(b)), int(m)) for a, b, m in descs], st)
        else:
            _, descs = inputs.mixed_batch(n, int(rng.choice([300, 6000, 60000] if n < 1000 else [300])), size_,
                                          seed=1000 * seed + step, shared_sources=float(rng.choice([0.0, 0.3])))
            ref.batch_copy([want], [(0, s, 0, t, m) for s, t, m in descs])
            dl.dl_batch_copy([(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs], st)
    sync()
    assert np.array_equal(d.host(), want) and d.guards_intact()


def test_token_dispatches_back_to_back_reuse_the_staging_ring(ref):
    """Twelve token dispatches on one stream without synchronisation, each with its own mask and receive
    buffers; three times as many as the staging ring has slots, alternating between the device-side lowering
    (mask staged) and the host lowering (item table staged)."""
    import torch
    W, row = 8, 1024
    st = torch.cuda.current_stream()
    ins = inputs.token_rows(W, 100, row, seed=5)
    d_in = [DevBuf(a.size, fill=a) for a in ins]
    runs = []
    sync()
    for k in range(12):
        dest = inputs.moe_token_destinations(W, 100, seed=50 + k, top_k=1 + k % 8)
        want = ref.token_dispatch(ins, row, dest)
        d_out = [DevBuf(w.size) for w in want]
        dl.dl_set_config(device_lowering=k % 2)
        dl.dl_token_dispatch([b.ptr() for b in d_in], [b.ptr() for b in d_out], [100] * W, row, dest, st)
        runs.append((d_out, want))
    dl.dl_set_config(device_lowering=1)
    sync()
    for k, (d_out, want) in enumerate(runs):
        check(d_out, want, f"dispatch {k}")
