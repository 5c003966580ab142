"""CPU tests of the library's host side: the exported symbols, the lowering of
collectives to copy lists, the hazard validator and the tile count.

The lowering entry points treat pointers as opaque addresses, so here they are
given the addresses of numpy buffers and the resulting copy list is replayed
with ctypes.memmove and compared with the CPU checker.  No GPU call is made.
"""

import ctypes
import os
import re

import numpy as np
import pytest

import paper_2511_06605_amd as dl
from paper_2511_06605_amd import binding, inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def golden_counts():
    out = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "paper_copy_counts.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = int(line[1])
    return out


def replay(items):
    for it in items:
        for d in it["dst"]:
            ctypes.memmove(d, it["src"], it["bytes"])


def addr(a, off=0):
    return a.ctypes.data + off


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "dmalatte.h")).read()
    declared = set(re.findall(r"\b(dl_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    L = binding.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_header_is_plain_c(tmp_path):
    """The boundary is a C header: it must compile as C99 on its own, with nothing but the standard headers,
    and every declared function must link against the built library from a C program."""
    import subprocess
    header = open(os.path.join(ROOT, "include", "dmalatte.h")).read()
    names = sorted(set(re.findall(r"\b(dl_[a-z_]+)\s*\(", header)))
    src = tmp_path / "uses_header.c"
    src.write_text('#include "dmalatte.h"\n'
                   "typedef void (*fn)(void);\n"
                   "fn table[] = {" + ", ".join(f"(fn){n}" for n in names) + "};\n"
                   "int main(void) { return sizeof(dl_plan_item) == 88 && sizeof(dl_copy_desc) == 24 && "
                   "sizeof(dl_config) == 72 && sizeof(table) > 0 ? 0 : 1; }\n")
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I" + inc, "-fsyntax-only", str(src)],
                   check=True)
    libdir = os.path.dirname(binding.LIB_PATH)
    exe = tmp_path / "uses_header"
    subprocess.run(["gcc", "-std=c99", "-I" + inc, str(src), "-L" + libdir, "-ldmalatte", "-Wl,-rpath," + libdir,
                    "-Wl,--allow-shlib-undefined", "-o", str(exe)], check=True)


def test_binding_structs_have_the_layout_of_the_header():
    """Sizes and offsets the C side asserts or implies: a mismatch here silently corrupts every call."""
    assert ctypes.sizeof(binding.PlanItem) == 88 and binding.PlanItem.dst.offset == 24
    assert ctypes.sizeof(binding.CopyDesc) == 24 and ctypes.sizeof(binding.SwapDesc) == 24
    assert ctypes.sizeof(binding.Trace) == 32
    assert ctypes.sizeof(binding.Config) == 72 and binding.Config.write_through_max_bytes.offset == 48
    assert binding.Config.stream_plain_min_bytes.offset == 56
    header = open(os.path.join(ROOT, "include", "dmalatte.h")).read()
    body = header[header.index("typedef struct dl_config {"):header.index("} dl_config;")]
    names = re.findall(r"^\s*uint(?:32|64)_t\s+(\w+);", body, flags=re.M)
    assert names == [f[0] for f in binding.Config._fields_]


def test_strerror_and_state_without_gpu():
    assert dl.binding.strerror(dl.DL_OK) == "ok"
    assert "overlap" in dl.binding.strerror(dl.DL_ERR_OVERLAP)
    # nothing initialised: operations refuse instead of touching the GPU
    a = np.zeros(64, dtype=np.uint8)
    with pytest.raises(dl.DlError) as e:
        dl.dl_batch_copy([(addr(a), addr(a, 32), 16)])
    assert e.value.status == dl.DL_ERR_STATE
    with pytest.raises(dl.DlError) as e:
        dl.dl_set_mode(dl.DL_MODE_PRELAUNCH)
    assert e.value.status == dl.DL_ERR_STATE


def test_paper_counts_inplace_allgather():
    """The paper's all-gather is in place and needs n(n-1) copies, one per peer."""
    g = golden_counts()
    W, B = g["n_devices"], 4096
    bufs = [np.zeros(W * B, dtype=np.uint8) for _ in range(W)]
    ins = [addr(bufs[r], r * B) for r in range(W)]
    outs = [addr(b) for b in bufs]
    plain = dl.dl_plan_allgather(ins, outs, B, fuse_broadcast=False)
    assert len(plain) == g["copies_per_collective"]
    for j in range(W):
        assert sum(1 for it in plain if it["src"] == ins[j]) == g["peers_per_device"]
    fused = dl.dl_plan_allgather(ins, outs, B, fuse_broadcast=True)
    # one read-once/write-many command per device instead of one per peer;
    # with the paper's two-destination command that is ceil(7/2) commands
    assert len(fused) == W and all(it["k"] == g["peers_per_device"] for it in fused)
    assert -(-g["peers_per_device"] // g["bcst_destinations"]) == g["bcst_commands_per_device"]
    # out of place adds the W self-copies
    ins2 = [addr(np.zeros(B, dtype=np.uint8)) for _ in range(W)]
    assert len(dl.dl_plan_allgather(ins2, outs, B, fuse_broadcast=False)) == W * W


@pytest.mark.parametrize("W", [1, 2, 3, 8, 13])
@pytest.mark.parametrize("B", [0, 1, 17, 4096])
@pytest.mark.parametrize("fuse", [False, True])
def test_allgather_lowering_replays_to_oracle(ref, W, B, fuse):
    ins = inputs.allgather_inputs(W, B, seed=W + B)
    outs = [np.zeros(W * B, dtype=np.uint8) for _ in range(W)]
    items = dl.dl_plan_allgather([addr(a) for a in ins], [addr(a) for a in outs], B, fuse)
    if B == 0:
        assert items == []
        return
    assert len(items) == (W * -(-W // dl.DL_PLAN_FANOUT) if fuse else W * W)
    replay(items)
    want = ref.allgather(ins)
    for r in range(W):
        assert np.array_equal(outs[r], want[r])
    assert dl.dl_plan_first_hazard(items) == -1


def test_allgather_inplace_lowering_replays_to_oracle(ref):
    W, B = 5, 333
    ins = inputs.allgather_inputs(W, B, seed=1)
    bufs = [np.zeros(W * B, dtype=np.uint8) for _ in range(W)]
    for r in range(W):
        bufs[r][r * B:(r + 1) * B] = ins[r]
    items = dl.dl_plan_allgather([addr(bufs[r], r * B) for r in range(W)], [addr(b) for b in bufs], B)
    assert all(it["k"] == W - 1 for it in items)
    replay(items)
    want = ref.allgather(ins)
    for r in range(W):
        assert np.array_equal(bufs[r], want[r])


@pytest.mark.parametrize("W", [1, 2, 3, 8])
@pytest.mark.parametrize("seed", [0, 1])
def test_alltoall_lowering_replays_to_oracle(ref, W, seed):
    C = inputs.random_chunks(W, 700, seed=seed + W, zero_frac=0.25)
    ins = inputs.alltoall_inputs(C, seed=seed)
    outs = [np.zeros(int(C[:, j].sum()), dtype=np.uint8) for j in range(W)]
    items = dl.dl_plan_alltoall([addr(a) if a.size else 0 for a in ins], [addr(a) if a.size else 0 for a in outs], C)
    assert len(items) == int((C > 0).sum())
    assert all(it["k"] == 1 for it in items)
    replay(items)
    want = ref.alltoall(ins, C)
    for j in range(W):
        assert np.array_equal(outs[j], want[j])


@pytest.mark.parametrize("k", [1, 7, 8, 9, 20, 64])
def test_broadcast_lowering(ref, k):
    src = inputs.payload(np.random.default_rng(k), 1000)
    dsts = [np.zeros(1000, dtype=np.uint8) for _ in range(k)]
    items = dl.dl_plan_broadcast(addr(src), [addr(d) for d in dsts], 1000)
    assert len(items) == -(-k // dl.DL_PLAN_FANOUT)
    assert sum(it["k"] for it in items) == k
    replay(items)
    for d, w in zip(dsts, ref.broadcast(src, k)):
        assert np.array_equal(d, w)


def test_batch_lowering_drops_empty_and_identical(ref):
    arena, descs = inputs.b2b_batch(16, 512, 64 * 1024, seed=3, align=16)
    work = arena.copy()
    lst = [(addr(work, int(s)), addr(work, int(d)), int(n)) for s, d, n in descs]
    lst += [(addr(work, 0), addr(work, 0), 100), (addr(work, 5), addr(work, 900), 0)]
    items = dl.dl_plan_batch(lst)
    assert len(items) == 16
    replay(items)
    want = ref.batch_copy([arena.copy()], [(0, s, 0, d, n) for s, d, n in descs])[0]
    assert np.array_equal(work, want)


@pytest.mark.parametrize("n,max_bytes,shared", [(7, 3000, 0.0), (64, 70000, 0.5), (500, 9000, 0.3)])
def test_batch_lowering_of_unequal_copies_with_and_without_inference(ref, n, max_bytes, shared):
    arena, descs = inputs.mixed_batch(n, max_bytes, 8 * 1024 * 1024, seed=n, shared_sources=shared)
    want = ref.batch_copy([arena.copy()], [(0, s, 0, d, m) for s, d, m in descs])[0]
    live = sum(1 for s, d, m in descs if m and s != d)
    for plan in (dl.dl_plan_batch, dl.dl_plan_batch_inferred):
        work = arena.copy()
        items = plan([(addr(work, int(s)), addr(work, int(d)), int(m)) for s, d, m in descs])
        assert sum(len(it["dst"]) for it in items) == live     # every live copy appears exactly once
        if plan is dl.dl_plan_batch:
            assert len(items) == live
        elif shared:
            assert len(items) < live                            # copies of one source were merged
        replay(items)
        assert np.array_equal(work, want)


def test_invalid_arguments():
    a = np.zeros(64, dtype=np.uint8)
    with pytest.raises(dl.DlError) as e:
        dl.dl_plan_broadcast(addr(a), [], 8)
    assert e.value.status == dl.DL_ERR_INVALID
    with pytest.raises(dl.DlError):
        dl.dl_plan_broadcast(addr(a), [addr(a, 8)] * 65, 1)
    with pytest.raises(dl.DlError):
        dl.dl_plan_broadcast(0, [addr(a, 8)], 8)
    with pytest.raises(dl.DlError):
        dl.dl_plan_allgather([0], [addr(a)], 8)
    with pytest.raises(dl.DlError):
        dl.dl_plan_batch([(0, addr(a), 8)])
    with pytest.raises(dl.DlError):
        dl.dl_plan_alltoall([0, addr(a)], [addr(a, 32), addr(a, 48)], [[4, 4], [4, 4]])
    assert dl.dl_plan_allgather([0], [0], 0) == []


def test_hazard_validator_agrees_with_oracle(ref):
    rng = np.random.default_rng(0)
    buf = np.zeros(4096, dtype=np.uint8)
    n_haz = 0
    for trial in range(300):
        n = int(rng.integers(1, 7))
        descs = []
        for _ in range(n):
            nb = int(rng.integers(0, 200))
            descs.append((int(rng.integers(0, 4096 - nb)), int(rng.integers(0, 4096 - nb)), nb))
        descs = [d for d in descs if d[0] != d[1]]  # identical ranges are dropped by the lowering
        want = ref.first_hazard([buf], [(0, s, 0, d, nb) for s, d, nb in descs])
        items = dl.dl_plan_batch([(addr(buf, s), addr(buf, d), nb) for s, d, nb in descs])
        got = dl.dl_plan_first_hazard(items)
        # the lowering drops empty copies: the checker's index counts them, the library's does not
        kept = [q for q, d in enumerate(descs) if d[2] > 0]
        assert got == (kept.index(want) if want >= 0 else -1), (trial, descs, got, want)
        n_haz += want >= 0
    assert 30 < n_haz < 270  # both outcomes are exercised


def test_hazard_validator_reports_the_first_offender_of_either_kind(ref):
    """A destination that lies before another one by address but later in the list, both under one source; and a
    destination/source overlap at a lower index than a destination/destination overlap."""
    buf = np.zeros(4096, dtype=np.uint8)

    def both(descs):
        want = ref.first_hazard([buf], [(0, s, 0, d, nb) for s, d, nb in descs])
        got = dl.dl_plan_first_hazard(dl.dl_plan_batch([(addr(buf, s), addr(buf, d), nb) for s, d, nb in descs]))
        return got, want

    # item 0 writes [100,110), item 1 writes [90,100), item 2 reads [95,105): both destinations are hit, 0 is first
    assert both([(2000, 100, 10), (2100, 90, 10), (95, 3000, 10)]) == (0, 0)
    # item 0's destination lies under item 3's source only; items 1 and 2 write the same bytes
    assert both([(2000, 500, 10), (2100, 700, 20), (2200, 710, 20), (505, 3000, 10)]) == (0, 0)
    # one source over many destinations, the first of the list last by address
    assert both([(2000, 140, 10), (2100, 100, 10), (2200, 120, 10), (90, 3000, 100)]) == (0, 0)


def test_hazard_validator_fanout_and_touching():
    a = np.zeros(1024, dtype=np.uint8)
    ok = [dict(src=addr(a), bytes=100, dst=[addr(a, 100), addr(a, 200), addr(a, 300)])]
    assert dl.dl_plan_first_hazard(ok) == -1
    bad = [dict(src=addr(a), bytes=100, dst=[addr(a, 100), addr(a, 199)])]
    assert dl.dl_plan_first_hazard(bad) == 0
    bad2 = ok + [dict(src=addr(a, 350), bytes=10, dst=[addr(a, 600)])]
    assert dl.dl_plan_first_hazard(bad2) == 0
    nested = [dict(src=addr(a, 900), bytes=10, dst=[addr(a, 0)]),
              dict(src=addr(a, 910), bytes=500, dst=[addr(a, 20)]),
              dict(src=addr(a, 800), bytes=10, dst=[addr(a, 400)])]
    assert dl.dl_plan_first_hazard(nested) == 1


def test_tile_count():
    """Tiles lie on the grid of the first destination: an item whose first destination stands s bytes behind a
    128-byte boundary takes ceil((bytes + s) / tile) tiles, whatever the source and the other destinations are."""
    a = 1 << 20  # an opaque address on every grid
    it = lambda s, d, n: dict(src=s, bytes=n, dst=list(d))
    T = 4096
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16)], 4096)], T) == 1
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16)], 4097)], T) == 2        # one byte in a tile of its own
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16)], 4096 + 16)], T) == 2
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16)], 5)], T) == 1
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16)], 0)], T) == 0
    # the first destination decides: 3 bytes behind a boundary, the first tile holds 4093 bytes
    assert dl.dl_plan_tiles([it(a + 3, [a + (1 << 16) + 3], 4093)], T) == 1
    assert dl.dl_plan_tiles([it(a + 3, [a + (1 << 16) + 3], 4094)], T) == 2
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16) + 127], 1)], T) == 1
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16) + 127], 3 * 4096 - 127)], T) == 3
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16) + 127], 3 * 4096 - 126)], T) == 4
    # the grid repeats every 128 bytes, not every tile: 128 bytes behind a tile boundary is on the grid
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16) + 128], 4096)], T) == 1
    # neither the source nor the later destinations matter
    assert dl.dl_plan_tiles([it(a + 77, [a + (1 << 16), a + (1 << 17) + 5], 3 * 4096)], T) == 3
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16) + 4], 3 * 4096)], T) == 4
    # items add up; a tile size that is not a multiple of 128 is refused
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16)], 4097), it(a, [a + (1 << 17) + 1], 4096)], T) == 4
    assert dl.dl_plan_tiles([it(a, [a + (1 << 16)], 4096)], 100) == 0
    # all-gather at 64 MiB per rank, fused, 16 KiB tiles
    B = 64 << 20
    ins = [a + r * B for r in range(8)]
    outs = [(1 << 40) + r * 8 * B for r in range(8)]
    items = dl.dl_plan_allgather(ins, outs, B)
    assert dl.dl_plan_tiles(items, 16384) == 8 * B // 16384


# ------------------------------------------------- swap / in-place all-to-all (Sec. IV-C)

@pytest.mark.parametrize("W", [1, 2, 3, 8, 13])
def test_inplace_alltoall_lowers_to_one_swap_per_pair_and_replays_to_the_checker(ref, W):
    """W(W-1)/2 swaps, i.e. half the n(n-1) copies of the out-of-place form (for the paper's n = 8:
    28 instead of 56), nothing on the diagonal; replayed on the CPU through a temporary and three
    moves each (what a swap replaces), the list gives the checker's result."""
    c = 40
    g = golden_counts()
    bufs = inputs.alltoall_inputs(inputs.uniform_chunks(W, c), seed=W)
    work = [b.copy() for b in bufs]
    swaps = dl.dl_plan_alltoall_inplace([addr(b) for b in work], c)
    assert len(swaps) == W * (W - 1) // 2
    if W == g["n_devices"]:
        assert 2 * len(swaps) == g["copies_per_collective"]
    assert dl.dl_plan_swap_first_hazard(swaps) == -1
    moves = 0
    for a, b, n in swaps:
        tmp = (ctypes.c_char * n)()
        ctypes.memmove(tmp, a, n)
        ctypes.memmove(a, b, n)
        ctypes.memmove(b, tmp, n)
        moves += 3
    assert moves == g["swap_copies_replaced"] * len(swaps)
    for x, y in zip(work, ref.alltoall_inplace(bufs, c)):
        assert np.array_equal(x, y)
    assert dl.dl_plan_alltoall_inplace([addr(b) for b in work], 0) == []


def test_swap_hazard_validator_agrees_with_the_checker(ref):
    buf = np.zeros(4096, dtype=np.uint8)
    base = addr(buf)
    cases = {
        "disjoint": [(0, 100, 50), (200, 300, 50)],
        "touching": [(0, 50, 50), (100, 150, 50)],
        "own ranges overlap": [(0, 30, 50)],
        "a hits other b": [(0, 100, 50), (500, 40, 50)],
        "b hits other a": [(0, 100, 50), (120, 600, 50)],
        "a hits other a": [(0, 100, 50), (30, 600, 50)],
        "b hits other b": [(0, 100, 50), (600, 130, 50)],
        "empty range inside another": [(0, 100, 50), (700, 120, 0)],
        "contained": [(0, 1000, 500), (100, 2000, 10)],
        "identical range is a no-op": [(10, 10, 100), (20, 300, 50)],
        "empty ranges never collide": [(0, 10, 0), (0, 100, 50)],
    }
    for name, sw in cases.items():
        got = dl.dl_plan_swap_first_hazard([(base + a, base + b, n) for a, b, n in sw])
        try:
            ref.batch_swap([buf.copy()], [(0, a, 0, b, n) for a, b, n in sw])
            want_ok = True
        except ValueError:
            want_ok = False
        assert (got == -1) == want_ok, name
    rng = np.random.default_rng(5)
    for _ in range(200):
        sw = [(int(rng.integers(0, 900)), int(rng.integers(0, 900)), int(rng.integers(0, 60))) for _ in range(3)]
        got = dl.dl_plan_swap_first_hazard([(base + a, base + b, n) for a, b, n in sw])
        try:
            ref.batch_swap([buf.copy()], [(0, a, 0, b, n) for a, b, n in sw])
            want_ok = True
        except ValueError:
            want_ok = False
        assert (got == -1) == want_ok, sw


# --------------------------------------- token dispatch and broadcast inference (Sec. IV-B, VI)

@pytest.mark.parametrize("W,counts,row", [(8, [16] * 8, 14336), (3, [5, 0, 7], 100), (13, [3] * 13, 48), (1, [4], 9)])
def test_token_dispatch_lowers_to_one_fanout_copy_per_token_and_replays_to_the_checker(ref, W, counts, row):
    ins = inputs.token_rows(W, counts, row, seed=W)
    dest = inputs.moe_token_destinations(W, counts, seed=W + 1, n_experts=16 * W, top_k=min(8, W))
    dest[1::7] = 0
    want = ref.token_dispatch(ins, row, dest)
    outs = [np.zeros(w.size, dtype=np.uint8) for w in want]
    items = dl.dl_plan_token_dispatch([addr(a) for a in ins], [addr(o) if o.size else 0 for o in outs], counts, row, dest)
    k = dest.sum(axis=1)
    # one item per group of up to 8 destinations of a token; none for a token that goes nowhere
    assert len(items) == int(np.ceil(k / 8).sum())
    assert sum(len(it["dst"]) for it in items) == int(dest.sum())
    assert all(it["bytes"] == row for it in items)
    assert dl.dl_plan_first_hazard(items) == -1
    replay(items)
    for o, w in zip(outs, want):
        assert np.array_equal(o, w)


def test_broadcast_inference_merges_copies_with_same_source_and_size(ref):
    W, B = 8, 96
    ins = inputs.allgather_inputs(W, B, seed=4)
    outs = [np.zeros(W * B, dtype=np.uint8) for _ in range(W)]
    # an all-gather written as n x n plain copies, receiver-major (so equal sources are not adjacent)
    descs = [(addr(ins[j]), addr(outs[r], j * B), B) for r in range(W) for j in range(W)]
    items = dl.dl_plan_batch_inferred(descs)
    assert len(items) == W and all(len(it["dst"]) == W for it in items)
    assert [it["src"] for it in items] == [addr(a) for a in ins]        # order of first appearance
    replay(items)
    for o, w in zip(outs, ref.allgather(ins)):
        assert np.array_equal(o, w)
    # more than 8 destinations: a second item; other size or other source: not merged; empty and identical: dropped
    buf = np.zeros(4096, dtype=np.uint8)
    p = addr(buf)
    descs = [(p, p + 1000 + 100 * d, 50) for d in range(11)] + [(p, p + 3000, 40), (p + 8, p + 3100, 50),
                                                                 (p, p + 3200, 0), (p + 500, p + 500, 20)]
    items = dl.dl_plan_batch_inferred(descs)
    assert [(it["src"] - p, it["bytes"], len(it["dst"])) for it in items] == [(0, 50, 8), (0, 40, 1), (8, 50, 1), (0, 50, 3)] \
        or [(it["src"] - p, it["bytes"], len(it["dst"])) for it in items] == [(0, 50, 8), (0, 50, 3), (0, 40, 1), (8, 50, 1)]
    assert sorted(d - p for it in items if it["bytes"] == 50 and it["src"] == p for d in it["dst"]) == \
        [1000 + 100 * d for d in range(11)]


@pytest.mark.parametrize("seed", range(6))
def test_broadcast_inference_gives_the_same_items_into_any_capacity(seed):
    """The lowering builds its items where they are wanted if there is room for one item per copy, and in a
    buffer of its own otherwise: the same items either way, and the same count with no room at all."""
    from paper_2511_06605_amd import binding
    lib = binding.lib()
    n = [1, 7, 64, 300, 1000, 2500][seed]
    arena, descs = inputs.mixed_batch(n, 4000, 8 << 20, seed=seed, shared_sources=0.5)
    p = addr(arena)
    d = binding._desc_array([(p + int(s), p + int(t), int(m)) for s, t, m in descs])

    def items_with_capacity(cap):
        arr = (binding.PlanItem * max(cap, 1))()
        m = lib.dl_plan_batch_inferred(d, n, arr, cap)
        return m, [(arr[i].src, arr[i].bytes, arr[i].k, tuple(arr[i].dst[j] for j in range(arr[i].k))) for i in range(min(m, cap))]

    count, none = items_with_capacity(0)
    exact = items_with_capacity(count)
    roomy = items_with_capacity(n + 5)
    assert count <= n and none == []
    assert exact == roomy and exact[0] == count and len(exact[1]) == count
    if count > 1:
        short = items_with_capacity(count - 1)
        assert short[0] == count and short[1] == exact[1][:count - 1]


# ------------------------------------------------------- size -> mode table (paper Tables II / III, Sec. V-B)

def _header_constants():
    text = open(os.path.join(ROOT, "include", "dmalatte.h")).read()
    tiles = int(re.search(r"#define DL_AUTO_STANDBY_TILES (\d+)", text).group(1))
    sig = int(re.search(r"#define DL_AUTO_SIGNAL_MAX_BYTES \((\d+)ull << 20\)", text).group(1)) << 20
    pre = int(re.search(r"#define DL_AUTO_PRELAUNCH_MAX_BYTES \((\d+)ull << 20\)", text).group(1)) << 20
    return tiles, sig, pre


def test_mode_table_constants_agree_with_the_header():
    assert _header_constants() == (dl.DL_AUTO_STANDBY_TILES, dl.DL_AUTO_SIGNAL_MAX_BYTES, dl.DL_AUTO_PRELAUNCH_MAX_BYTES)


def test_mode_table_at_every_threshold():
    """dl_plan_mode on both sides of every row of the table, one tile / one item / one byte apart."""
    T, SIG, PRE = _header_constants()
    AG, AA, BC, BT, SW, TD = (dl.DL_OP_ALLGATHER, dl.DL_OP_ALLTOALL, dl.DL_OP_BROADCAST, dl.DL_OP_BATCH, dl.DL_OP_SWAP,
                              dl.DL_OP_TOKEN_DISPATCH)
    one, pre, sig, sb = dl.DL_MODE_ONESHOT, dl.DL_MODE_PRELAUNCH, dl.DL_MODE_SIGNAL, dl.DL_MODE_STANDBY
    plan = dl.dl_plan_mode
    # known ahead: prelaunch up to the limit, one-shot above; tiles and items play no part
    for op in (AG, AA, BC, BT, SW, TD):
        assert plan(op, 8, 8 if op == AG else 1, PRE, 10 ** 6, True) == pre
        assert plan(op, 8, 8 if op == AG else 1, PRE + 1, 1, True) == one
        assert plan(op, 1, 1, 1, 1, True) == pre
    # known on issue: the waiting kernel's record holds 64 tiles, 8 items with several destinations or 64 plain ones
    assert plan(AG, 8, 8, 72 * 65536, T, False) == sb
    assert plan(AG, 8, 8, 72 * 65536 + 72 * 16, T + 1, False) == sig
    assert plan(AG, 9, 8, 9 * 10 * 4096, 9, False) == sig          # nine fan-out items do not fit
    assert plan(BC, 1, 7, 8 * 512 * 1024, T, False) == sb
    assert plan(AA, 64, 1, 128 * 8192, T, False) == sb
    assert plan(AA, 64, 1, 128 * 8208, 2 * T, False) == sig
    assert plan(BT, 64, 1, 2 * 64 * 100, 64, False) == sb
    assert plan(BT, 65, 1, 2 * 65 * 100, 65, False) == sig
    assert plan(BT, 9, 2, 3 * 9 * 100, 9, False) == sig            # broadcast inference made fan-out items: 8 at most
    assert plan(BT, 8, 2, 3 * 8 * 100, 8, False) == sb
    # swaps and token dispatches are never handed to a waiting kernel, however small
    assert plan(SW, 1, 1, 4 * 1024, 1, False) == sig
    assert plan(TD, 16, 8, 16 * 9 * 1024, 16, False) == sig
    assert plan(TD, 511, 8, 511 * 9 * 1024, 511, False) == sig
    assert plan(TD, 512, 8, 512 * 9 * 1024, 512, False) == one     # lowered on the device, one-shot
    # above the record: signal up to the limit, one-shot beyond
    for op in (AG, AA, BC, BT, SW):
        assert plan(op, 8, 8 if op in (AG, BC) else 1, SIG, 10 ** 5, False) == sig
        assert plan(op, 8, 8 if op in (AG, BC) else 1, SIG + 1, 10 ** 5, False) == one
    # malformed questions
    for bad in ((-1, 1, 1, 1, 1, False), (6, 1, 1, 1, 1, False), (AG, 1, 0, 1, 1, False), (AG, 1, 9, 1, 1, False)):
        with pytest.raises(dl.DlError):
            plan(*bad)


def test_mode_table_applied_to_the_lowered_collectives():
    """The table fed with what the lowering of the task's workloads gives: all-gather sweep points on both sides
    of each threshold (W = 8), the uniform all-to-all, the 2 MiB -> 7 broadcast, the 64 x 16 KiB batch."""
    W = 8
    a = np.zeros(1, dtype=np.uint8)
    base = addr(a) & ~127  # opaque addresses on the 128-byte grid that tiles are cut on

    def ag_mode(B, ahead):
        ins = [base + (1 << 32) * (1 + j) for j in range(W)]
        outs = [base + (1 << 32) * (20 + j) for j in range(W)]
        items = dl.dl_plan_allgather(ins, outs, B)
        return dl.dl_plan_mode(dl.DL_OP_ALLGATHER, len(items), max(i["k"] for i in items), (W + W * W) * B,
                               dl.dl_plan_tiles(items, 8192), ahead)

    assert [ag_mode(B, False) for B in (4096, 64 * 1024, 64 * 1024 + 16, 1 << 20, 4 << 20, (4 << 20) + 16, 64 << 20)] == \
        [dl.DL_MODE_STANDBY, dl.DL_MODE_STANDBY, dl.DL_MODE_SIGNAL, dl.DL_MODE_SIGNAL, dl.DL_MODE_SIGNAL,
         dl.DL_MODE_ONESHOT, dl.DL_MODE_ONESHOT]
    assert [ag_mode(B, True) for B in (4096, 4 << 20, (4 << 20) + 16, 64 << 20)] == \
        [dl.DL_MODE_PRELAUNCH, dl.DL_MODE_PRELAUNCH, dl.DL_MODE_ONESHOT, dl.DL_MODE_ONESHOT]

    def aa_mode(c):
        ins = [base + (1 << 32) * (1 + j) for j in range(W)]
        outs = [base + (1 << 32) * (20 + j) for j in range(W)]
        items = dl.dl_plan_alltoall(ins, outs, [[c] * W] * W)
        return dl.dl_plan_mode(dl.DL_OP_ALLTOALL, len(items), 1, 2 * W * W * c, dl.dl_plan_tiles(items, 8192), False)

    assert [aa_mode(c) for c in (1024, 8192, 16384, 2 << 20, 4 << 20)] == \
        [dl.DL_MODE_STANDBY, dl.DL_MODE_STANDBY, dl.DL_MODE_SIGNAL, dl.DL_MODE_SIGNAL, dl.DL_MODE_ONESHOT]
    items = dl.dl_plan_broadcast(base + (1 << 32), [base + (1 << 32) * (2 + d) for d in range(7)], 2 << 20)
    assert dl.dl_plan_mode(dl.DL_OP_BROADCAST, len(items), 7, 8 * (2 << 20), dl.dl_plan_tiles(items, 8192), False) == dl.DL_MODE_SIGNAL
    assert dl.dl_plan_mode(dl.DL_OP_BATCH, 64, 1, 2 * 64 * 16384, 128, False) == dl.DL_MODE_SIGNAL


def test_config_from_text():
    """dl_parse_config (what dl_init does with the DL_CONFIG environment variable): every tunable by name, C
    integer literals, refusal of anything it does not understand without touching the struct."""
    c = dl.dl_parse_config("tile_bytes=4096, block_threads=256,fan_split=2,table_push=0,write_through_max_bytes=0x100000,"
                           "stream_plain_min_bytes=18446744073709551615,armed_chain_min_bytes=0,arm_timeout_us=500")
    assert (c.tile_bytes, c.block_threads, c.fan_split, c.table_push) == (4096, 256, 2, 0)
    assert c.write_through_max_bytes == 1 << 20 and c.stream_plain_min_bytes == (1 << 64) - 1
    assert c.armed_chain_min_bytes == 0 and c.arm_timeout_us == 500
    names = [f[0] for f in binding.Config._fields_]
    c = dl.dl_parse_config(",".join(f"{n}={1 if n != 'tile_bytes' and n != 'block_threads' else 0}" for n in names))
    assert all(getattr(c, n) == (0 if n in ("tile_bytes", "block_threads") else 1) for n in names)   # every field has a name
    base = binding.Config(arm_timeout_us=7, fan_split=4)
    for bad in ("tile_bytes=3000", "nosuch=1", "fan_split=3", "fan_split", "=4", "block_threads=abc", "tile_bytes=4096;fan_split=2",
                "arm_timeout_us=0", "fan_split=99999999999"):
        with pytest.raises(dl.DlError):
            dl.dl_parse_config(bad, base)
        assert (base.arm_timeout_us, base.fan_split, base.tile_bytes) == (7, 4, 0), bad
    assert dl.dl_parse_config("", base).fan_split == 4
