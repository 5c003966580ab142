"""Each plausible mistake, planted in a patched copy of the CPU checker's
source (compiled to a temporary library, on the CPU only), must be caught by
at least one pin.  This guards the pins, not the checker: a mutant that
survives means the pins could not tell a wrong checker from a right one."""

import os

import numpy as np
import pytest

from paper_2511_06605_amd import inputs

MUTANTS = {
    # all-gather: wrong source rank, wrong slot, dropped last rank
    "ag_src_rank": ("memcpy((char *)out[r] + (size_t)j * B, in[j], B);",
                    "memcpy((char *)out[r] + (size_t)j * B, in[r], B);"),
    "ag_slot": ("memcpy((char *)out[r] + (size_t)j * B, in[j], B);",
                "memcpy((char *)out[r] + (size_t)r * B, in[j], B);"),
    "ag_drop_last": ("for (int j = 0; j < W; ++j) {\n            if (B && (!in[j] || !out[r]))",
                     "for (int j = 0; j < W - 1; ++j) {\n            if (B && (!in[j] || !out[r]))"),
    # all-to-all: transposed chunk matrix, swapped offsets, swapped operands, off-by-one prefix
    "aa_transposed_size": ("size_t n = C[(size_t)i * W + j];", "size_t n = C[(size_t)j * W + i];"),
    "aa_send_uses_column": ("send += C[(size_t)i * W + jj];", "send += C[(size_t)jj * W + i];"),
    "aa_recv_uses_row": ("recv += C[(size_t)ii * W + j];", "recv += C[(size_t)j * W + ii];"),
    "aa_swapped_offsets": ("memcpy((char *)out[j] + recv, (const char *)in[i] + send, n);",
                           "memcpy((char *)out[j] + send, (const char *)in[i] + recv, n);"),
    "aa_prefix_inclusive": ("for (int jj = 0; jj < j; ++jj)", "for (int jj = 0; jj <= j; ++jj)"),
    "aa_wrong_receiver": ("memcpy((char *)out[j] + recv, (const char *)in[i] + send, n);",
                          "memcpy((char *)out[i] + recv, (const char *)in[i] + send, n);"),
    # broadcast: one destination skipped, short copy
    "bc_skip_first": ("for (int d = 0; d < k; ++d) {\n        if (bytes && !dsts[d])",
                      "for (int d = 1; d < k; ++d) {\n        if (bytes && !dsts[d])"),
    "bc_short": ("memcpy(dsts[d], src, bytes);", "memcpy(dsts[d], src, bytes - (bytes > 16));"),
    # batch: swapped operands, hazard check that ignores sources
    "bt_swapped": ("memcpy(d[k].dst, d[k].src, d[k].bytes);", "memcpy((void *)d[k].src, d[k].dst, d[k].bytes);"),
    "hz_ignores_sources": ("if (ranges_overlap(d[a].dst, d[a].bytes, d[b].src, d[b].bytes))\n                return (long)a;",
                           "if (0)\n                return (long)a;"),
    "hz_closed_interval": ("return (uintptr_t)a < (uintptr_t)b + bn && (uintptr_t)b < (uintptr_t)a + an;",
                           "return (uintptr_t)a <= (uintptr_t)b + bn && (uintptr_t)b <= (uintptr_t)a + an;"),
}


def run_pins(ref, lib):
    """A condensed pass over the pins of test_oracle_pins.py against ``lib``."""
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


def test_unpatched_checker_passes(ref):
    run_pins(ref, ref.load())


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(ref, tmp_path, name):
    old, new = MUTANTS[name]
    text = open(ref.SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    out = str(tmp_path / f"libmutant_{name}.so")
    ref.build(str(src), out, force=True)
    lib = ref.load(out)
    with pytest.raises((AssertionError, ValueError, RuntimeError)):
        run_pins(ref, lib)
