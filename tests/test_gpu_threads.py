"""Several host threads driving the library at once (its host state sits behind one lock; "the most recent
request" is the calling thread's own).  The foreign calls run outside the interpreter lock, so the threads
really overlap inside the library.  Every result is compared with the CPU checker."""

import threading

import numpy as np
import pytest

import paper_2511_06605_amd as dl
from paper_2511_06605_amd import inputs
from paper_2511_06605_amd.inputs import KiB

from gpu_util import DevBuf

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def library():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    dl.dl_init(0)
    dl.dl_set_config(arm_timeout_us=300_000)
    yield
    dl.dl_shutdown()


def run_threads(workers):
    errors = []

    def guard(fn, k):
        try:
            fn(k)
        except BaseException as e:   # reported by the test's own thread
            errors.append((k, repr(e)))

    threads = [threading.Thread(target=guard, args=(fn, k)) for k, fn in enumerate(workers)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(120)
    assert not any(t.is_alive() for t in threads), "a worker thread did not finish"
    assert not errors, errors


def test_threads_issue_one_shot_requests_on_streams_of_their_own(ref):
    """Four threads, each with a stream and buffers of its own: all-gathers (kernel-argument lists) in two of
    them, long-list batches (table memory, events) in the other two, 40 requests each."""
    import torch
    W, ROUNDS = 8, 40
    cases = []
    for k in range(4):
        per = []
        for r in range(ROUNDS):
            if k % 2 == 0:
                B = int(np.random.default_rng(100 * k + r).choice([512, 4 * KiB, 48 * KiB, 200 * KiB + 16]))
                ins = inputs.allgather_inputs(W, B, seed=1000 * k + r)
                per.append(("ag", B, ins, [DevBuf(B, fill=a) for a in ins], [DevBuf(W * B) for _ in range(W)]))
            else:
                arena, descs = inputs.b2b_batch(70 + r, 3000, 2 * 1024 * KiB, seed=1000 * k + r)
                per.append(("batch", descs, arena, DevBuf(arena.size, fill=arena), None))
        cases.append(per)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(4)]

    def worker(k):
        torch.cuda.set_device(0)
        st = streams[k]
        for case in cases[k]:
            if case[0] == "ag":
                _, B, _, d_in, d_out = case
                dl.dl_allgather([b.ptr() for b in d_in], [b.ptr() for b in d_out], B, st)
            else:
                _, descs, _, d, _ = case
                dl.dl_batch_copy([(d.ptr(int(s)), d.ptr(int(t)), int(m)) for s, t, m in descs], st)
        st.synchronize()

    run_threads([worker] * 4)
    torch.cuda.synchronize()
    for k in range(4):
        for r, case in enumerate(cases[k]):
            if case[0] == "ag":
                _, B, ins, _, d_out = case
                for got, want in zip(d_out, ref.allgather(ins)):
                    assert np.array_equal(got.host(), want) and got.guards_intact(), f"thread {k} request {r}"
            else:
                _, descs, arena, d, _ = case
                want = ref.batch_copy([arena.copy()], [(0, s, 0, t, m) for s, t, m in descs])[0]
                assert np.array_equal(d.host(), want) and d.guards_intact(), f"thread {k} request {r}"


def test_threads_wait_for_their_own_tickets_in_signal_mode(ref):
    """Three threads in signal mode: each issues a request and waits for the ticket of its own most recent
    request (dl_last_ticket is per thread), 60 times, checking its receive buffers after every wait."""
    import torch
    W, ROUNDS = 8, 60
    sizes = [4 * KiB, 24 * KiB + 16, 96 * KiB]
    d_in = [[torch.zeros(B, dtype=torch.uint8, device="cuda") for _ in range(W)] for B in sizes]
    d_out = [[torch.zeros(W * B, dtype=torch.uint8, device="cuda") for _ in range(W)] for B in sizes]
    streams = [torch.cuda.Stream() for _ in sizes]
    bad = [torch.zeros(1, dtype=torch.int64, device="cuda") for _ in sizes]
    tickets = [[] for _ in sizes]
    torch.cuda.synchronize()
    dl.dl_prelaunch_start()
    try:
        dl.dl_set_mode(dl.DL_MODE_SIGNAL)

        def worker(k):
            torch.cuda.set_device(0)
            B, st = sizes[k], streams[k]
            with torch.cuda.stream(st):
                for it in range(ROUNDS):
                    for j in range(W):
                        d_in[k][j].fill_((it * 5 + j * 17 + k) % 251)
                    dl.dl_allgather(d_in[k], d_out[k], B, st)     # ordered on st behind the fills
                    tickets[k].append(dl.dl_last_ticket())
                    dl.dl_wait()
                    want = torch.tensor([(it * 5 + j * 17 + k) % 251 for j in range(W)], dtype=torch.uint8, device="cuda")
                    for r in (it % W, (it + 5) % W):
                        bad[k] += (d_out[k][r].view(W, B) != want[:, None]).sum()
                    st.synchronize()   # the comparison has read the buffers before the next fill

        run_threads([worker] * len(sizes))
    finally:
        dl.dl_set_mode(dl.DL_MODE_ONESHOT)
        dl.dl_prelaunch_stop()
    torch.cuda.synchronize()
    assert [int(b.item()) for b in bad] == [0] * len(sizes)
    # every request took a ticket of its own: 180 distinct ones over the three threads, increasing per thread
    every = [t for per in tickets for t in per]
    assert len(set(every)) == len(sizes) * ROUNDS and 0 not in every
    assert all(per == sorted(per) for per in tickets)
