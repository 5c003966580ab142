"""Token dispatch with the routing mask in device memory (dl_token_dispatch_device), through the C boundary,
byte for byte against the CPU checker on the same seeded inputs (the checker gets the mask as a host array)."""

import numpy as np
import pytest

import paper_2511_06605_amd as dl
from paper_2511_06605_amd import inputs

from gpu_util import DevBuf, stream, sync

pytestmark = pytest.mark.gpu

W = 8


@pytest.fixture(scope="module", autouse=True)
def library():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    dl.dl_init(0)
    yield
    dl.dl_shutdown()


def run(ref, counts, row, seed, top_k=8, mask_value=1, drop=None, kind="u8", check_host_entry=False, shifts=None):
    import torch
    ins = inputs.token_rows(W, counts, row, seed=seed, kind=kind)
    dest = inputs.moe_token_destinations(W, counts, seed=seed + 1, n_experts=256, top_k=top_k) * np.uint8(mask_value)
    if drop:
        dest[::drop] = 0
    want = ref.token_dispatch(ins, row, dest)
    shifts = shifts or [0] * (2 * W)
    d_in = [DevBuf(a.size, fill=a, shift=shifts[i]) for i, a in enumerate(ins)]
    d_out = [DevBuf(w.size, shift=shifts[W + j]) for j, w in enumerate(want)]
    d_mask = torch.from_numpy(np.ascontiguousarray(dest)).cuda()
    tok = [counts] * W if np.isscalar(counts) else list(counts)
    sync()
    dl.dl_token_dispatch_device([b.ptr() for b in d_in], [b.ptr() for b in d_out], tok, row, d_mask, stream())
    sync()
    for j in range(W):
        assert np.array_equal(d_out[j].host(), want[j]), f"receiver {j} differs"
        assert d_out[j].guards_intact()
    for b, a in zip(d_in, ins):
        assert np.array_equal(b.host(), a) and b.guards_intact()
    if check_host_entry:   # the entry point with the mask on the host gives the same bytes
        again = [DevBuf(w.size) for w in want]
        dl.dl_token_dispatch([b.ptr() for b in d_in], [b.ptr() for b in again], tok, row, dest, stream())
        sync()
        for a, b in zip(again, d_out):
            assert np.array_equal(a.host(), b.host())


@pytest.mark.parametrize("T", [16, 128, 512])
def test_moe_hidden_7168_bf16_top8(ref, T):
    """The task's dispatch workload: 256 experts over 8 ranks, top-8, rows of 14336 bytes."""
    run(ref, T, 14336, seed=T, kind="bf16", check_host_entry=True)


@pytest.mark.parametrize("counts,row,top_k,mask_value,drop", [
    ([1] * 8, 16, 8, 1, None),                              # eight tokens: one block, mostly empty
    ([0, 0, 0, 5, 0, 0, 0, 0], 48, 2, 1, None),             # a single sender
    ([257, 255, 256, 1, 0, 511, 64, 63], 1040, 3, 1, None),  # rank boundaries off the 256-token blocks
    ([100] * 8, 2048, 64, 7, None),                         # (nearly) every token to all eight ranks; mask bytes of 7
    ([300] * 8, 64, 4, 0x80, 3),                            # only the highest bit set; every third token goes nowhere
    ([700, 1, 0, 300, 0, 0, 29, 2], 1024, 1, 255, None),    # every token to exactly one rank
    ([1280] * 8, 16, 2, 1, 5),                              # 10 240 tokens: the most the entry point takes
])
def test_edges(ref, counts, row, top_k, mask_value, drop):
    run(ref, counts, row, seed=sum(counts) + row, top_k=top_k, mask_value=mask_value, drop=drop)


@pytest.mark.parametrize("counts,row,top_k,shifts", [
    ([40] * 8, 1000, 3, None),                                   # rows of whole 8 bytes: every second one off the 16
    ([100] * 8, 14336 + 2, 8, None),                             # the task's row and one bf16 element more
    ([64] * 8, 777, 2, None),                                    # an odd row length
    ([90] * 8, 4096, 4, [0, 1, 2, 3, 16, 32, 64, 127] * 2),      # whole rows, buffers anywhere
    ([33, 0, 257, 5, 64, 1, 300, 12], 3001, 5, [7, 0, 100, 16, 1, 4, 8, 2, 0, 127, 3, 64, 16, 5, 9, 48]),
])
def test_rows_and_buffers_of_any_length_and_alignment(ref, counts, row, top_k, shifts):
    """Neither the row length nor any buffer address has to be a multiple of anything; the same through the entry point
    with the mask on the host, which lowers on the device from 512 tokens."""
    run(ref, counts, row, seed=row + sum(counts), top_k=top_k, shifts=shifts, check_host_entry=True)


def test_mask_produced_on_the_stream_just_before(ref):
    """The mask is written by a kernel on the same stream and the dispatch follows without a synchronisation in
    between: the three launches are ordered behind it.  Twice, with the mask buffer reused."""
    import torch
    counts, row = [200] * W, 512
    ins = inputs.token_rows(W, counts, row, seed=3)
    d_in = [DevBuf(a.size, fill=a) for a in ins]
    total = sum(counts)
    d_mask = torch.zeros((total, W), dtype=torch.uint8, device="cuda")
    cap = [DevBuf(total * row) for _ in range(W)]          # room for every token: the host does not know the counts
    for rnd in range(2):
        dest = inputs.moe_token_destinations(W, counts, seed=40 + rnd, n_experts=64, top_k=3)
        scores = torch.from_numpy(dest.astype(np.float32)).cuda()
        sync()
        d_mask.copy_((scores > 0.5).to(torch.uint8))       # the "router": a kernel on the current stream
        dl.dl_token_dispatch_device([b.ptr() for b in d_in], [b.ptr() for b in cap], counts, row, d_mask, stream())
        sync()
        want = ref.token_dispatch(ins, row, dest)
        for j in range(W):
            assert np.array_equal(cap[j].host()[:want[j].size], want[j]), f"round {rnd} receiver {j}"
            assert cap[j].guards_intact()


def test_limits_and_malformed_requests():
    """Every buffer here is large enough for the largest request named, so that a request which ought to be
    refused could not reach outside them if it were accepted."""
    import torch
    most = dl.DL_DISPATCH_DEVICE_MAX_TOKENS
    rows = most + 8
    d = DevBuf(rows * 16)
    mask = torch.zeros((rows, W), dtype=torch.uint8, device="cuda")
    ok = dict(ins=[d.ptr()] * W, outs=[d.ptr()] * W, tokens=[2] * W, row_bytes=16, dest_device=mask, stream=stream())

    def status(**kw):
        try:
            dl.dl_token_dispatch_device(**{**ok, **kw})
        except dl.DlError as e:
            return e.status
        return dl.DL_OK

    assert status(ins=[d.ptr()] * 4, outs=[d.ptr()] * 4, tokens=[2] * 4) == dl.DL_ERR_INVALID   # eight ranks only
    assert status(row_bytes=24) == dl.DL_OK and status(ins=[d.ptr(4)] * W) == dl.DL_OK          # any row length, any address (the mask is empty: nothing moves)
    assert status(dest_device=mask.data_ptr() + 4) == dl.DL_ERR_INVALID                         # 8-byte aligned mask
    assert status(dest_device=None) == dl.DL_ERR_INVALID
    assert status(tokens=[most // W] * (W - 1) + [most // W + 1]) == dl.DL_ERR_CAPACITY         # one token too many
    assert status(tokens=[0] * W) == dl.DL_OK and status(row_bytes=0) == dl.DL_OK               # nothing to move
    sync()
    assert d.guards_intact() and not bool(mask.any())
