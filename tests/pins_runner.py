"""A condensed pass over the pins of test_oracle_pins.py against one build of
the CPU checker.  Run as a script with the library path as its argument so
that a build with a planted mistake (which may write out of bounds) cannot
damage the test process: exit status 0 = all pins hold."""

import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

from oracle import ref  # noqa: E402
from paper_2511_06605_amd import inputs  # noqa: E402


def run_pins(lib):
    W = 3
    ins = inputs.allgather_inputs(W, 17, seed=1)
    got = ref.allgather(ins, lib=lib)
    assert np.array_equal(np.stack(got), np.tile(np.concatenate(ins), (W, 1)))

    C = inputs.random_chunks(W, 40, seed=5, zero_frac=0.2)
    assert not np.array_equal(C, C.T)
    ins = inputs.alltoall_inputs(C, seed=2)
    mid = ref.alltoall(ins, C, lib=lib)
    for j in range(W):
        for i in range(W):
            a = mid[j][int(C[:i, j].sum()): int(C[:i + 1, j].sum())]
            b = ins[i][int(C[i, :j].sum()): int(C[i, :j + 1].sum())]
            assert np.array_equal(a, b)
    back = ref.alltoall(mid, C.T, lib=lib)
    for i in range(W):
        assert np.array_equal(back[i], ins[i])

    src = inputs.payload(np.random.default_rng(3), 100)
    for d in ref.broadcast(src, 4, lib=lib):
        assert np.array_equal(d, src)

    arena, descs = inputs.b2b_batch(8, 64, 4096, seed=4, align=8)
    want = arena.copy()
    for s, d, n in descs.astype(np.int64):
        want[d:d + n] = arena[s:s + n]
    got = ref.batch_copy([arena.copy()], [(0, s, 0, d, n) for s, d, n in descs], lib=lib)[0]
    assert np.array_equal(got, want)

    buf = np.arange(256, dtype=np.uint8)
    assert ref.first_hazard([buf], [(0, 0, 0, 100, 50), (0, 60, 0, 150, 10)], lib=lib) == -1
    assert ref.first_hazard([buf], [(0, 0, 0, 100, 50), (0, 120, 0, 200, 10)], lib=lib) == 0
    assert ref.first_hazard([buf], [(0, 0, 0, 100, 50), (0, 60, 0, 149, 10)], lib=lib) == 0   # two destinations share a byte
    assert ref.first_hazard([buf], [(0, 0, 0, 10, 50)], lib=lib) == 0                         # a copy onto its own source
    assert ref.first_hazard([buf], [(0, 5, 0, 5, 50)], lib=lib) == -1                         # identical range: no-op
    assert ref.first_hazard([buf], [(0, 0, 0, 105, 0), (0, 0, 0, 100, 10)], lib=lib) == -1    # an empty copy collides with nothing,
    assert ref.first_hazard([buf], [(0, 0, 0, 100, 10), (0, 105, 0, 200, 0)], lib=lib) == -1  # not even from inside a range
    kept = buf.copy()
    try:                                                     # a batch with a hazard is refused and moves nothing
        ref.batch_copy([kept], [(0, 0, 0, 100, 50), (0, 60, 0, 149, 10)], lib=lib)
    except ValueError:
        pass
    else:
        raise AssertionError("hazard accepted")
    assert np.array_equal(kept, buf)

    arena, descs = inputs.swap_batch(5, 30, 2048, seed=6, align=2)
    want = arena.copy()
    for a, b, n in descs.astype(np.int64):
        want[a:a + n], want[b:b + n] = arena[b:b + n].copy(), arena[a:a + n].copy()
    got = ref.batch_swap([arena.copy()], [(0, a, 0, b, n) for a, b, n in descs], lib=lib)[0]
    assert np.array_equal(got, want)
    for bad in ([(0, 0, 0, 100, 20), (0, 110, 0, 200, 20)], [(0, 0, 0, 100, 20), (0, 200, 0, 19, 20)],
                [(0, 0, 0, 10, 20)],
                [(0, 0, 0, 100, 20), (0, 10, 0, 200, 20)],      # the two first ranges share bytes
                [(0, 0, 0, 100, 20), (0, 200, 0, 110, 20)]):    # the two second ranges share bytes
        try:
            ref.batch_swap([buf.copy()], bad, lib=lib)
        except ValueError:
            pass
        else:
            raise AssertionError("overlapping swap ranges accepted")
    ref.batch_swap([buf.copy()], [(0, 0, 0, 20, 20), (0, 40, 0, 60, 20)], lib=lib)   # touching ranges are fine

    c = 7
    bufs = inputs.alltoall_inputs(inputs.uniform_chunks(W, c), seed=8)
    got = ref.alltoall_inplace(bufs, c, lib=lib)
    assert np.array_equal(np.stack(got), np.stack(bufs).reshape(W, W, c).transpose(1, 0, 2).reshape(W, W * c))

    empty = [np.zeros(0, dtype=np.uint8) for _ in range(W)]
    assert all(b.size == 0 for b in ref.alltoall_inplace(empty, 0, lib=lib))                   # empty chunks: a no-op, not an error

    counts, row = [3, 0, 4], 6
    tin = inputs.token_rows(W, counts, row, seed=9)
    dest = inputs.moe_token_destinations(W, counts, seed=10, n_experts=12, top_k=2)
    dest[2] = 0
    rows = np.concatenate(tin).reshape(sum(counts), row)
    got = ref.token_dispatch(tin, row, dest, lib=lib)
    for j in range(W):
        assert np.array_equal(got[j].reshape(-1, row), rows[dest[:, j] != 0])


if __name__ == "__main__":
    run_pins(ref.load(sys.argv[1]))
