"""Each plausible mistake, planted in a patched copy of the CPU checker's
source (compiled to a temporary library, on the CPU only), must be caught by
at least one pin.  This guards the pins, not the checker: a mutant that
survives means the pins could not tell a wrong checker from a right one."""

import os
import subprocess
import sys

import pytest

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
    # swap: one copy of the three dropped, exchange in one direction only, hazard check between swaps incomplete
    "sw_no_restore": ("memcpy(d[k].b, tmp, d[k].bytes);", "memcpy(d[k].b, d[k].a, d[k].bytes);"),
    "sw_one_way": ("memcpy(d[k].a, d[k].b, d[k].bytes);\n", "\n"),
    "sw_hazard_ab_only": ("ranges_overlap(d[k].b, d[k].bytes, d[m].a, d[m].bytes) ||", "0 ||"),
    "sw_hazard_self": ("if (d[k].a != d[k].b && ranges_overlap(d[k].a, d[k].bytes, d[k].b, d[k].bytes))", "if (0)"),
    # in-place all-to-all: not transposed, chunk index and rank exchanged on one side only, wrong stride
    "ip_not_transposed": ("memcpy((char *)buf[j] + (size_t)i * c, old + (size_t)i * row + (size_t)j * c, c);",
                          "memcpy((char *)buf[i] + (size_t)j * c, old + (size_t)i * row + (size_t)j * c, c);"),
    "ip_wrong_slot": ("memcpy((char *)buf[j] + (size_t)i * c, old + (size_t)i * row + (size_t)j * c, c);",
                      "memcpy((char *)buf[j] + (size_t)j * c, old + (size_t)i * row + (size_t)j * c, c);"),
    "ip_reads_new": ("memcpy((char *)buf[j] + (size_t)i * c, old + (size_t)i * row + (size_t)j * c, c);",
                     "memcpy((char *)buf[j] + (size_t)i * c, (char *)buf[i] + (size_t)j * c, c);"),
    # token dispatch: mask read transposed, rows placed by token number instead of packed, row index of the wrong rank
    "td_mask_transposed": ("if (!dest[g * (size_t)W + (size_t)j])", "if (!dest[(size_t)j * (size_t)W + g % (size_t)W])"),
    "td_not_packed": ("memcpy((char *)out[j] + placed * row_bytes, (const char *)in[i] + (size_t)t * row_bytes, row_bytes);",
                      "memcpy((char *)out[j] + (placed ? placed - 1 : 0) * row_bytes, (const char *)in[i] + (size_t)t * row_bytes, row_bytes);"),
    "td_global_row": ("(const char *)in[i] + (size_t)t * row_bytes, row_bytes);\n                }\n                ++placed;",
                      "(const char *)in[i] + (size_t)(t ? t - 1 : 0) * row_bytes, row_bytes);\n                }\n                ++placed;"),
    "td_local_token_index": ("if (!dest[g * (size_t)W + (size_t)j])", "if (!dest[(size_t)t * (size_t)W + (size_t)j])"),
    "aa_stops_at_empty_chunk": ("            if (n == 0)\n                continue;", "            if (n == 0)\n                break;"),
    "hz_ignores_destinations": ("if (a != b && ranges_overlap(d[a].dst, d[a].bytes, d[b].dst, d[b].bytes))\n                return (long)a;",
                                "if (0)\n                return (long)a;"),
    "hz_noop_copy_flagged": ("            if (a == b && d[a].src == d[a].dst)\n                continue;\n", ""),
    "bt_no_hazard_check": ("    if (ref_first_hazard(d, n) >= 0)\n        return -2;\n", ""),
    "bc_always_first_destination": ("memcpy(dsts[d], src, bytes);", "memcpy(dsts[0], src, bytes);"),
    "sw_hazard_skips_neighbour": ("for (size_t m = k + 1; m < n; ++m) {", "for (size_t m = k + 2; m < n; ++m) {"),
    "td_rows_counted_across_receivers": ("size_t placed = 0; /* rows already written to out[j] */",
                                         "static size_t placed; if (j == 0) placed = 0;"),
    "ag_rank_stride_off": ("memcpy((char *)out[r] + (size_t)j * B, in[j], B);",
                           "memcpy((char *)out[r] + (size_t)j * B, in[j], B - (j == W - 1 && B > 1));"),
    "ro_empty_ranges_collide": ("    if (an == 0 || bn == 0)\n        return 0;\n", ""),
    "sw_hazard_aa": ("if (ranges_overlap(d[k].a, d[k].bytes, d[m].a, d[m].bytes) ||", "if (0 ||"),
    "sw_hazard_a_with_later_b": ("ranges_overlap(d[k].a, d[k].bytes, d[m].b, d[m].bytes) ||", "0 ||"),
    "sw_hazard_bb": ("ranges_overlap(d[k].b, d[k].bytes, d[m].b, d[m].bytes))", "0)"),
    "ip_empty_chunks_not_noop": ("    if (c == 0)\n        return 0;\n", "    if (c == 0)\n        return -1;\n"),
    "td_counts_skipped": ("                if (!dest[g * (size_t)W + (size_t)j])\n                    continue;",
                          "                if (!dest[g * (size_t)W + (size_t)j]) {\n                    ++placed;\n                    continue;\n                }"),
}


RUNNER = os.path.join(os.path.dirname(os.path.abspath(__file__)), "pins_runner.py")


def pins_hold(lib_path) -> bool:
    return subprocess.run([sys.executable, RUNNER, lib_path], capture_output=True).returncode == 0


def test_unpatched_checker_passes(ref):
    assert pins_hold(ref.build())


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(ref, tmp_path, name):
    old, new = MUTANTS[name]
    text = open(ref.SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    out = str(tmp_path / f"libmutant_{name}.so")
    ref.build(str(src), out, force=True)
    assert not pins_hold(out)
