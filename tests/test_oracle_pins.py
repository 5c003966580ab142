"""Pins of the CPU checker to things other than itself.

Each pin is independent of ``oracle/dl_oracle.c``:
  * per-byte index formulas evaluated by pure-Python loops (brute force),
  * reductions to numpy library routines (tile/concatenate, reshape+transpose,
    broadcast_to),
  * the invariants of the collectives (identical all-gather outputs,
    all-to-all twice with the transposed chunk matrix is the identity,
    broadcast destinations equal the source, byte-multiset conservation),
  * W = 1, where every operation is a plain copy,
  * the hazard rule of back-to-back copies (Sec. IV-D) on hand-built cases,
  * swap and the in-place all-to-all (Sec. IV-C): slice exchange, the three
    copies through a temporary that a swap replaces, reshape+transpose, the
    out-of-place all-to-all, the series of pairwise swaps, involution.
The paper prints no worked numeric example for these operations, so there is
no golden fixture of printed values; tests/golden holds only the copy counts
the paper states.
"""

import itertools

import numpy as np
import pytest

from paper_2511_06605_amd import inputs

SIZES = [0, 1, 2, 15, 16, 17, 255, 256, 4097]
WS = [1, 2, 3, 5, 8]


# ---------------------------------------------------------------- brute force

def brute_allgather(ins):
    W, B = len(ins), len(ins[0])
    outs = []
    for r in range(W):
        o = bytearray(W * B)
        for p in range(W * B):
            o[p] = ins[p // B][p % B]
        outs.append(np.frombuffer(bytes(o), dtype=np.uint8))
    return outs


def brute_alltoall(ins, C):
    """For each receiver j walk its buffer byte by byte; find which sender's
    chunk the byte falls in by scanning column j; locate it in the sender's
    buffer by scanning row i.  No prefix arrays."""
    W = len(ins)
    outs = []
    for j in range(W):
        total = sum(int(C[i][j]) for i in range(W))
        o = bytearray(total)
        for p in range(total):
            i, q = 0, p
            while q >= int(C[i][j]):
                q -= int(C[i][j])
                i += 1
            s = q
            for jj in range(j):
                s += int(C[i][jj])
            o[p] = ins[i][s]
        outs.append(np.frombuffer(bytes(o), dtype=np.uint8))
    return outs


@pytest.mark.parametrize("W", WS)
@pytest.mark.parametrize("B", [0, 1, 2, 15, 16, 17, 255, 256])
def test_allgather_bruteforce(ref, W, B):
    ins = inputs.allgather_inputs(W, B, seed=W * 1000 + B)
    got = ref.allgather(ins)
    want = brute_allgather(ins)
    for r in range(W):
        assert got[r].tobytes() == want[r].tobytes()


@pytest.mark.parametrize("W", WS)
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_alltoall_bruteforce_nonsymmetric(ref, W, seed):
    C = inputs.random_chunks(W, 300, seed=seed * 17 + W, zero_frac=0.25)
    if W > 1:
        assert not np.array_equal(C, C.T)  # a symmetric C cannot tell i from j
    ins = inputs.alltoall_inputs(C, seed=seed)
    got = ref.alltoall(ins, C)
    want = brute_alltoall(ins, C)
    for j in range(W):
        assert got[j].tobytes() == want[j].tobytes()


@pytest.mark.parametrize("W", [2, 3, 8])
@pytest.mark.parametrize("c", [1, 15, 16, 17, 256])
def test_alltoall_bruteforce_uniform(ref, W, c):
    C = inputs.uniform_chunks(W, c)
    ins = inputs.alltoall_inputs(C, seed=c)
    got = ref.alltoall(ins, C)
    want = brute_alltoall(ins, C)
    for j in range(W):
        assert got[j].tobytes() == want[j].tobytes()


# ------------------------------------------------- reductions to numpy routines

@pytest.mark.parametrize("W", WS)
@pytest.mark.parametrize("B", SIZES)
def test_allgather_is_tile_of_concatenation(ref, W, B):
    ins = inputs.allgather_inputs(W, B, seed=B + 7 * W, kind="bf16" if B % 2 == 0 else "u8")
    got = ref.allgather(ins)
    want = np.tile(np.concatenate(ins), (W, 1))
    assert np.array_equal(np.stack(got), want)


@pytest.mark.parametrize("W", WS)
@pytest.mark.parametrize("c", SIZES)
def test_uniform_alltoall_is_transpose(ref, W, c):
    C = inputs.uniform_chunks(W, c)
    ins = inputs.alltoall_inputs(C, seed=c + W, kind="fp16" if c % 2 == 0 else "u8")
    got = ref.alltoall(ins, C)
    x = np.stack(ins).reshape(W, W, c)           # [sender i][chunk j][t]
    want = x.transpose(1, 0, 2).reshape(W, W * c)  # [receiver j][chunk i][t]
    assert np.array_equal(np.stack(got), want)


@pytest.mark.parametrize("k", [1, 2, 7, 8, 13])
@pytest.mark.parametrize("n", SIZES)
def test_broadcast_is_broadcast_to(ref, k, n):
    src = inputs.payload(np.random.default_rng(n * 31 + k), n)
    got = ref.broadcast(src, k)
    assert np.array_equal(np.stack(got), np.broadcast_to(src, (k, n)))


@pytest.mark.parametrize("n", SIZES)
def test_W1_everything_is_a_plain_copy(ref, n):
    x = inputs.payload(np.random.default_rng(n), n)
    assert ref.allgather([x])[0].tobytes() == x.tobytes()
    assert ref.alltoall([x], np.array([[n]]))[0].tobytes() == x.tobytes()
    assert ref.broadcast(x, 1)[0].tobytes() == x.tobytes()
    bufs = [x.copy(), np.zeros(n, dtype=np.uint8)]
    ref.batch_copy(bufs, [(0, 0, 1, 0, n)])
    assert bufs[1].tobytes() == x.tobytes()


# ------------------------------------------------------------------ invariants

@pytest.mark.parametrize("W,B", [(8, 64 * 1024), (8, 4096), (5, 12345), (3, 1)])
def test_allgather_invariants(ref, W, B):
    ins = inputs.allgather_inputs(W, B, seed=0)
    outs = ref.allgather(ins)
    for r in range(1, W):
        assert np.array_equal(outs[r], outs[0])
    assert outs[0].tobytes() == b"".join(a.tobytes() for a in ins)
    # conservation: every input byte value appears W times as often in the outputs
    hin = np.bincount(np.concatenate(ins), minlength=256)
    hout = np.bincount(np.concatenate(outs), minlength=256)
    assert np.array_equal(hout, W * hin)


@pytest.mark.parametrize("W", [2, 3, 8])
@pytest.mark.parametrize("seed", [3, 4])
def test_alltoall_twice_with_transposed_chunks_is_identity(ref, W, seed):
    C = inputs.random_chunks(W, 5000, seed=seed, zero_frac=0.2)
    assert not np.array_equal(C, C.T)
    ins = inputs.alltoall_inputs(C, seed=seed + 100)
    mid = ref.alltoall(ins, C)
    back = ref.alltoall(mid, C.T)
    for i in range(W):
        assert back[i].tobytes() == ins[i].tobytes()
    hin = np.bincount(np.concatenate(ins), minlength=256)
    hmid = np.bincount(np.concatenate(mid), minlength=256)
    assert np.array_equal(hin, hmid)


def test_alltoall_moe_shape_matches_index_formula(ref):
    """MoE-dispatch chunk sizes (whole token rows, some zero chunks): check
    sampled output bytes against the closed-form source location."""
    W = 8
    C = inputs.moe_dispatch_chunks(W, tokens_per_rank=16, seed=5, hidden=64)
    assert (C % 128 == 0).all() and int(C.sum()) == W * 8 * 16 * 128
    ins = inputs.alltoall_inputs(C, seed=6, kind="bf16")
    outs = ref.alltoall(ins, C)
    rng = np.random.default_rng(0)
    for _ in range(2000):
        i, j = int(rng.integers(W)), int(rng.integers(W))
        if C[i, j] == 0:
            continue
        t = int(rng.integers(int(C[i, j])))
        assert outs[j][int(C[:i, j].sum()) + t] == ins[i][int(C[i, :j].sum()) + t]


def test_broadcast_destinations_equal_source(ref):
    src = inputs.payload(np.random.default_rng(1), 2 * 1024 * 1024, "bf16")
    for d in ref.broadcast(src, 7):
        assert np.array_equal(d, src)


# ------------------------------------------------------------- batched copies

def test_batch_copy_matches_slice_assignment(ref):
    arena, descs = inputs.b2b_batch(64, 16 * 1024, 4 * 1024 * 1024, seed=2)
    want = arena.copy()
    before = arena.copy()
    for s, d, n in descs.astype(np.int64):
        want[d:d + n] = before[s:s + n]
    got = ref.batch_copy([arena], [(0, s, 0, d, n) for s, d, n in descs])[0]
    assert np.array_equal(got, want)
    # bytes outside every destination are untouched
    mask = np.ones(arena.size, dtype=bool)
    for _, d, n in descs.astype(np.int64):
        mask[d:d + n] = False
    assert np.array_equal(got[mask], before[mask])


@pytest.mark.parametrize("perm_seed", [0, 1, 2])
def test_batch_copy_order_does_not_matter(ref, perm_seed):
    arena, descs = inputs.b2b_batch(32, 1000, 256 * 1024, seed=9, align=8)
    a = ref.batch_copy([arena.copy()], [(0, s, 0, d, n) for s, d, n in descs])[0]
    p = np.random.default_rng(perm_seed).permutation(len(descs))
    b = ref.batch_copy([arena.copy()], [(0, s, 0, d, n) for s, d, n in descs[p]])[0]
    assert np.array_equal(a, b)


def test_hazard_rule(ref):
    buf = np.arange(256, dtype=np.uint8)
    ok = [(0, 0, 0, 100, 50), (0, 10, 0, 160, 40)]            # overlapping sources are fine
    assert ref.first_hazard([buf], ok) == -1
    assert ref.first_hazard([buf], [(0, 0, 0, 100, 50), (0, 60, 0, 149, 10)]) == 0   # dst-dst, 1 byte
    assert ref.first_hazard([buf], [(0, 0, 0, 100, 50), (0, 60, 0, 150, 10)]) == -1  # touching, disjoint
    assert ref.first_hazard([buf], [(0, 0, 0, 100, 50), (0, 120, 0, 200, 10)]) == 0  # dst of 0 hits src of 1
    assert ref.first_hazard([buf], [(0, 0, 0, 10, 50)]) == 0                         # src-dst of one copy
    assert ref.first_hazard([buf], [(0, 5, 0, 5, 50)]) == -1                         # identical range: no-op
    assert ref.first_hazard([buf], [(0, 0, 0, 100, 0), (0, 0, 0, 100, 10)]) == -1    # empty copies never collide
    assert ref.first_hazard([buf], [(0, 0, 0, 105, 0), (0, 0, 0, 100, 10)]) == -1    # ... not even from inside a range
    assert ref.first_hazard([buf], [(0, 0, 0, 100, 10), (0, 105, 0, 200, 0)]) == -1
    with pytest.raises(ValueError):
        ref.batch_copy([buf.copy()], [(0, 0, 0, 100, 50), (0, 60, 0, 149, 10)])
    same = buf.copy()
    ref.batch_copy([same], [(0, 5, 0, 5, 50)])
    assert np.array_equal(same, buf)


@pytest.mark.parametrize("n,max_bytes,shared", [(7, 3000, 0.0), (64, 70000, 0.5), (500, 9000, 0.2)])
def test_batch_of_unequal_sizes_matches_slice_assignment(ref, n, max_bytes, shared):
    arena, descs = inputs.mixed_batch(n, max_bytes, 8 * 1024 * 1024, seed=n, shared_sources=shared)
    assert ref.first_hazard([arena], [(0, s, 0, d, m) for s, d, m in descs]) == -1
    want = arena.copy()
    for s, d, m in descs.astype(np.int64):
        want[d:d + m] = arena[s:s + m]
    got = ref.batch_copy([arena.copy()], [(0, s, 0, d, m) for s, d, m in descs])[0]
    assert np.array_equal(got, want)


def test_generated_batches_are_hazard_free(ref):
    for seed in range(5):
        arena, descs = inputs.b2b_batch(64, 16 * 1024, 8 * 1024 * 1024, seed=seed)
        d = [(0, s, 0, t, n) for s, t, n in descs]
        assert ref.first_hazard([arena], d) == -1
        # and every pair is checked independently of the C validator
        iv = [(int(t), int(t + n)) for _, t, n in descs]
        sv = [(int(s), int(s + n)) for s, _, n in descs]
        for (a0, a1), (b0, b1) in itertools.combinations(iv, 2):
            assert a1 <= b0 or b1 <= a0
        for (a0, a1) in iv:
            for (b0, b1) in sv:
                assert a1 <= b0 or b1 <= a0


# ------------------------------------------- swap and in-place all-to-all (Sec. IV-C)

def test_swap_is_slice_exchange(ref):
    arena, descs = inputs.swap_batch(9, 70, 8192, seed=1, align=2)
    want = arena.copy()
    for a, b, n in descs.astype(np.int64):
        want[a:a + n], want[b:b + n] = arena[b:b + n].copy(), arena[a:a + n].copy()
    got = ref.batch_swap([arena.copy()], [(0, a, 0, b, n) for a, b, n in descs])[0]
    assert np.array_equal(got, want)
    assert not np.array_equal(got, arena)


@pytest.mark.parametrize("n", [0, 1, 15, 16, 17, 4097])
def test_swap_equals_three_copies_through_a_temporary(ref, n):
    """What the swap command replaces (Sec. IV-C): copy a to a temporary, b to a, the temporary to b."""
    rng = np.random.default_rng(n)
    a, b = inputs.payload(rng, n), inputs.payload(rng, n)
    x, y, tmp = a.copy(), b.copy(), np.zeros(n, dtype=np.uint8)
    ref.batch_copy([x, y, tmp], [(0, 0, 2, 0, n)])
    ref.batch_copy([x, y, tmp], [(1, 0, 0, 0, n)])
    ref.batch_copy([x, y, tmp], [(2, 0, 1, 0, n)])
    p, q = a.copy(), b.copy()
    ref.batch_swap([p, q], [(0, 0, 1, 0, n)])
    assert np.array_equal(p, x) and np.array_equal(q, y)
    assert np.array_equal(p, b) and np.array_equal(q, a)


def test_swap_twice_is_identity_and_order_is_free(ref):
    arena, descs = inputs.swap_batch(12, 100, 16384, seed=2, align=4)
    d = [(0, a, 0, b, n) for a, b, n in descs]
    once = ref.batch_swap([arena.copy()], d)[0]
    assert np.array_equal(ref.batch_swap([once.copy()], d)[0], arena)
    assert np.array_equal(ref.batch_swap([arena.copy()], d[::-1])[0], once)
    # exchanging the two locations of a descriptor changes nothing
    assert np.array_equal(ref.batch_swap([arena.copy()], [(0, b, 0, a, n) for a, b, n in descs])[0], once)


def test_swap_rejects_overlapping_ranges(ref):
    buf = np.arange(256, dtype=np.uint8)
    with pytest.raises(ValueError):
        ref.batch_swap([buf.copy()], [(0, 0, 0, 10, 20)])                      # its own two ranges overlap
    with pytest.raises(ValueError):
        ref.batch_swap([buf.copy()], [(0, 0, 0, 100, 20), (0, 110, 0, 200, 20)])  # b of one, a of the other
    with pytest.raises(ValueError):
        ref.batch_swap([buf.copy()], [(0, 0, 0, 100, 20), (0, 200, 0, 19, 20)])   # a of one, b of the other
    ok = ref.batch_swap([buf.copy()], [(0, 0, 0, 20, 20), (0, 40, 0, 60, 20), (0, 90, 0, 90, 10)])[0]  # touching; identical
    assert np.array_equal(ok[:20], buf[20:40]) and np.array_equal(ok[40:60], buf[60:80]) and np.array_equal(ok[90:100], buf[90:100])


@pytest.mark.parametrize("W", WS)
@pytest.mark.parametrize("c", [0, 1, 16, 17, 255])
def test_alltoall_inplace_is_transpose_and_matches_out_of_place(ref, W, c):
    bufs = inputs.alltoall_inputs(inputs.uniform_chunks(W, c), seed=W + c)
    got = ref.alltoall_inplace(bufs, c)
    want = np.stack(bufs).reshape(W, W, c).transpose(1, 0, 2).reshape(W, W * c)
    assert np.array_equal(np.stack(got), want)
    for g, o in zip(got, ref.alltoall(bufs, inputs.uniform_chunks(W, c))):
        assert np.array_equal(g, o)
    back = ref.alltoall_inplace(got, c)
    for x, y in zip(back, bufs):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("W,c", [(2, 3), (3, 5), (5, 2)])
def test_alltoall_inplace_bruteforce(ref, W, c):
    bufs = inputs.alltoall_inputs(inputs.uniform_chunks(W, c), seed=7 * W + c)
    got = ref.alltoall_inplace(bufs, c)
    for j in range(W):
        for p in range(W * c):
            assert got[j][p] == bufs[p // c][j * c + p % c]


@pytest.mark.parametrize("W", [2, 3, 8])
def test_alltoall_inplace_is_a_series_of_swaps(ref, W):
    """The paper's realisation (Sec. IV-C): one swap per pair of ranks, W(W-1)/2 in all, nothing on the diagonal."""
    c = 48
    bufs = inputs.alltoall_inputs(inputs.uniform_chunks(W, c), seed=W)
    work = [b.copy() for b in bufs]
    swaps = [(i, j * c, j, i * c, c) for i in range(W) for j in range(i + 1, W)]
    assert len(swaps) == W * (W - 1) // 2
    ref.batch_swap(work, swaps)
    for x, y in zip(work, ref.alltoall_inplace(bufs, c)):
        assert np.array_equal(x, y)


# ------------------------------------------------- token dispatch (Sec. II-A1, IV-B)

def brute_token_dispatch(ins, row, dest):
    W = len(ins)
    outs = []
    for j in range(W):
        o = bytearray()
        g = 0
        for i in range(W):
            for t in range(len(ins[i]) // row if row else 0):
                if dest[g][j]:
                    for q in range(row):
                        o.append(int(ins[i][t * row + q]))
                g += 1
        outs.append(np.frombuffer(bytes(o), dtype=np.uint8))
    return outs


@pytest.mark.parametrize("W,counts,row", [(1, [3], 5), (2, [2, 3], 1), (3, [4, 0, 2], 7), (5, [1, 2, 3, 2, 1], 16),
                                          (8, [3] * 8, 17)])
def test_token_dispatch_bruteforce(ref, W, counts, row):
    ins = inputs.token_rows(W, counts, row, seed=W)
    dest = inputs.moe_token_destinations(W, counts, seed=W + 1, n_experts=8 * W, top_k=min(3, W))
    dest[::5] = 0                      # some tokens go nowhere
    got = ref.token_dispatch(ins, row, dest)
    for g, w in zip(got, brute_token_dispatch(ins, row, dest)):
        assert np.array_equal(g, w)


@pytest.mark.parametrize("W,T,row", [(8, 16, 64), (4, 33, 100), (8, 5, 14336)])
def test_token_dispatch_is_boolean_row_selection(ref, W, T, row):
    """Receive buffer j is the stacked token rows filtered by column j of the destination mask."""
    ins = inputs.token_rows(W, T, row, seed=T, kind="bf16")
    dest = inputs.moe_token_destinations(W, T, seed=T + 1)
    rows = np.concatenate(ins).reshape(W * T, row)
    got = ref.token_dispatch(ins, row, dest)
    for j in range(W):
        assert np.array_equal(got[j].reshape(-1, row), rows[dest[:, j] != 0])
    # top-8 over 256 experts: every token reaches between 1 and min(8, W) ranks
    k = dest.sum(axis=1)
    assert k.min() >= 1 and k.max() <= min(8, W)


def test_token_dispatch_to_every_rank_is_an_allgather(ref):
    W, T, row = 4, 6, 24
    ins = inputs.token_rows(W, T, row, seed=3)
    got = ref.token_dispatch(ins, row, np.ones((W * T, W), dtype=np.uint8))
    for g, w in zip(got, ref.allgather(ins)):
        assert np.array_equal(g, w)


def test_token_dispatch_with_one_destination_sorted_by_rank_is_the_alltoall(ref):
    """Tokens that each go to exactly one rank, stored grouped by that rank: the packed all-to-all."""
    W, row = 5, 12
    rng = np.random.default_rng(11)
    counts = rng.integers(0, 4, (W, W))                  # tokens rank i sends to rank j
    ins = inputs.token_rows(W, [int(c.sum()) for c in counts], row, seed=12)
    dest = np.zeros((int(counts.sum()), W), dtype=np.uint8)
    g = 0
    for i in range(W):
        for j in range(W):
            dest[g:g + counts[i, j], j] = 1
            g += counts[i, j]
    got = ref.token_dispatch(ins, row, dest)
    for x, y in zip(got, ref.alltoall(ins, counts * row)):
        assert np.array_equal(x, y)
