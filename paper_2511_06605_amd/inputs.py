"""Seeded synthetic inputs for the copy collectives (all-gather, all-to-all,
broadcast, batched back-to-back copies).

This module only draws random payloads, chunk-size matrices and copy offsets.
It holds none of the data-movement logic: it never computes where a byte ends
up.  Both the CPU checker and the HIP path are fed from here, and neither one
is imported here.

Every payload is returned as a contiguous ``numpy.uint8`` array; the element
type named by a workload (uint8, bf16, fp16) only decides the bit patterns.
One ``numpy.random.default_rng(seed)`` generator is used per case and ranks
are filled in rank order.
"""

from __future__ import annotations

import numpy as np

KiB = 1024
MiB = 1024 * 1024


def _normal16_bytes(rng: np.random.Generator, n_bytes: int, kind: str) -> np.ndarray:
    """``n_bytes`` of N(0,1) samples rounded to a 16-bit float type, as bytes.

    kind = "bf16": float32 rounded to nearest-even on the upper 16 bits.
    kind = "fp16": IEEE half via numpy's cast.
    An odd ``n_bytes`` gets one extra uniform byte at the end.
    """
    n_el = n_bytes // 2
    x = rng.standard_normal(n_el, dtype=np.float32)
    if kind == "fp16":
        b = x.astype(np.float16).view(np.uint8)
    elif kind == "bf16":
        u = x.view(np.uint32)
        u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
        b = u.astype(np.uint16).view(np.uint8)
    else:
        raise ValueError(kind)
    if n_bytes & 1:
        b = np.concatenate([b, rng.integers(0, 256, 1, dtype=np.uint8)])
    return np.ascontiguousarray(b)


def payload(rng: np.random.Generator, n_bytes: int, kind: str = "u8") -> np.ndarray:
    """One buffer of ``n_bytes`` bytes of the given element kind."""
    if n_bytes == 0:
        return np.zeros(0, dtype=np.uint8)
    if kind == "u8":
        return rng.integers(0, 256, n_bytes, dtype=np.uint8)
    return _normal16_bytes(rng, n_bytes, kind)


def allgather_inputs(W: int, bytes_per_rank: int, seed: int, kind: str = "u8"):
    """W send buffers of ``bytes_per_rank`` bytes each."""
    rng = np.random.default_rng(seed)
    return [payload(rng, bytes_per_rank, kind) for _ in range(W)]


def uniform_chunks(W: int, c: int) -> np.ndarray:
    """W x W matrix with every entry c: rank i sends c bytes to every rank j."""
    return np.full((W, W), c, dtype=np.uint64)


def random_chunks(W: int, max_chunk: int, seed: int, zero_frac: float = 0.2,
                  multiple_of: int = 1) -> np.ndarray:
    """A non-symmetric W x W chunk-size matrix with some zero entries."""
    rng = np.random.default_rng(seed)
    C = rng.integers(0, max_chunk // multiple_of + 1, (W, W)).astype(np.uint64) * np.uint64(multiple_of)
    C[rng.random((W, W)) < zero_frac] = 0
    return C


def moe_dispatch_chunks(W: int, tokens_per_rank: int, seed: int, hidden: int = 7168,
                        n_experts: int = 256, top_k: int = 8, elem_bytes: int = 2,
                        skew_alpha: float | None = None) -> np.ndarray:
    """Chunk-size matrix of an expert-parallel MoE dispatch.

    Each sender draws top_k * tokens_per_rank expert assignments from a
    multinomial over the experts (uniform, or Dirichlet(skew_alpha) weights),
    the experts are split evenly over the W ranks, and every assignment ships
    one token row of hidden * elem_bytes bytes.
    """
    rng = np.random.default_rng(seed)
    per_rank = n_experts // W
    if skew_alpha is None:
        p = np.full(n_experts, 1.0 / n_experts)
    else:
        p = rng.dirichlet(np.full(n_experts, skew_alpha))
    C = np.zeros((W, W), dtype=np.uint64)
    for i in range(W):
        counts = rng.multinomial(top_k * tokens_per_rank, p)
        C[i] = counts.reshape(W, per_rank).sum(axis=1).astype(np.uint64) * np.uint64(hidden * elem_bytes)
    return C


def alltoall_inputs(C: np.ndarray, seed: int, kind: str = "u8"):
    """W send buffers; buffer i has sum_j C[i][j] bytes."""
    rng = np.random.default_rng(seed)
    return [payload(rng, int(C[i].sum()), kind) for i in range(C.shape[0])]


def tp_decode_bytes_per_rank(tokens: int, hidden: int = 8192, W: int = 8, elem_bytes: int = 2) -> int:
    """Per-rank payload of a tensor-parallel decode all-gather."""
    return hidden * tokens * elem_bytes // W


def b2b_batch(n: int, copy_bytes: int, arena_bytes: int, seed: int, align: int = 256):
    """n independent copies inside one arena.

    Returns (arena, descs) with descs an (n, 3) uint64 array of
    (src_offset, dst_offset, bytes).  Offsets are multiples of ``align``.
    Candidates are rejected until every destination range is disjoint from
    every other destination range and from every source range; sources may
    overlap each other.
    """
    rng = np.random.default_rng(seed)
    arena = rng.integers(0, 256, arena_bytes, dtype=np.uint8)
    slots = (arena_bytes - copy_bytes) // align + 1
    srcs: list[tuple[int, int]] = []
    dsts: list[tuple[int, int]] = []

    def hits(a0, a1, ranges):
        return any(a0 < b1 and b0 < a1 for b0, b1 in ranges)

    out = np.zeros((n, 3), dtype=np.uint64)
    i = 0
    while i < n:
        s = int(rng.integers(0, slots)) * align
        d = int(rng.integers(0, slots)) * align
        sr, dr = (s, s + copy_bytes), (d, d + copy_bytes)
        if hits(*dr, dsts) or hits(*dr, srcs) or hits(*sr, dsts) or hits(*dr, [sr]):
            continue
        srcs.append(sr)
        dsts.append(dr)
        out[i] = (s, d, copy_bytes)
        i += 1
    return arena, out


def mixed_batch(n: int, max_bytes: int, arena_bytes: int, seed: int, shared_sources: float = 0.0):
    """n independent copies of unequal sizes and alignments inside one arena.

    Sizes are log-uniform in [1, max_bytes] (one in ten is 0); source and
    destination offsets are multiples of 1, 4, 16 or 256 drawn per copy and
    per side, so one list mixes every element width, with heads and tails.
    With probability ``shared_sources`` a copy reuses the previous copy's
    source and size (what a fan-out looks like when handed over as plain
    copies).  Same return value and the same disjointness as ``b2b_batch``.
    """
    rng = np.random.default_rng(seed)
    arena = rng.integers(0, 256, arena_bytes, dtype=np.uint8)
    srcs: list[tuple[int, int]] = []
    dsts: list[tuple[int, int]] = []

    def hits(a0, a1, ranges):
        return a1 > a0 and any(a0 < b1 and b0 < a1 for b0, b1 in ranges)

    out = np.zeros((n, 3), dtype=np.uint64)
    i = 0
    while i < n:
        if i and rng.random() < shared_sources:
            s, nb = int(out[i - 1][0]), int(out[i - 1][2])
        else:
            nb = 0 if rng.random() < 0.1 else int(np.exp(rng.uniform(0.0, np.log(max_bytes))))
            sa = int(rng.choice([1, 4, 16, 256]))
            s = int(rng.integers(0, (arena_bytes - nb) // sa + 1)) * sa
        da = int(rng.choice([1, 4, 16, 256]))
        d = int(rng.integers(0, (arena_bytes - nb) // da + 1)) * da
        sr, dr = (s, s + nb), (d, d + nb)
        if hits(*dr, dsts) or hits(*dr, srcs) or hits(*sr, dsts) or hits(*dr, [sr]):
            continue
        srcs.append(sr)
        dsts.append(dr)
        out[i] = (s, d, nb)
        i += 1
    return arena, out


def swap_batch(n: int, swap_bytes: int, arena_bytes: int, seed: int, align: int = 256):
    """n independent swaps inside one arena.

    Returns (arena, descs) with descs an (n, 3) uint64 array of
    (a_offset, b_offset, bytes); all 2n ranges are pairwise disjoint.
    """
    rng = np.random.default_rng(seed)
    arena = rng.integers(0, 256, arena_bytes, dtype=np.uint8)
    slots = (arena_bytes - swap_bytes) // align + 1
    taken: list[tuple[int, int]] = []
    out = np.zeros((n, 3), dtype=np.uint64)
    i = 0
    while i < n:
        a = int(rng.integers(0, slots)) * align
        b = int(rng.integers(0, slots)) * align
        ra, rb = (a, a + swap_bytes), (b, b + swap_bytes)
        if ra[0] < rb[1] and rb[0] < ra[1]:
            continue
        if any(x0 < y1 and y0 < x1 for x0, x1 in (ra, rb) for y0, y1 in taken):
            continue
        taken += [ra, rb]
        out[i] = (a, b, swap_bytes)
        i += 1
    return arena, out


def kv_fetch_blocks(n_blocks: int, host_pool_blocks: int, device_pool_blocks: int, seed: int) -> np.ndarray:
    """Which blocks a paged KV-cache fetch moves: an (n_blocks, 2) array of
    (host pool block index, device pool block index), each column without
    repeats, drawn uniformly (the blocks of one request are dispersed in both
    pools)."""
    rng = np.random.default_rng(seed)
    src = rng.choice(host_pool_blocks, n_blocks, replace=False)
    dst = rng.choice(device_pool_blocks, n_blocks, replace=False)
    return np.stack([src, dst], axis=1).astype(np.int64)


def moe_token_destinations(W: int, tokens_per_rank, seed: int, n_experts: int = 256, top_k: int = 8,
                           skew_alpha: float | None = None) -> np.ndarray:
    """Which ranks each token of an expert-parallel MoE layer goes to.

    Every token picks ``top_k`` distinct experts (uniformly, or by Dirichlet
    (skew_alpha) weights); the experts are split evenly over the W ranks; a
    token goes once to every rank that owns at least one of its experts.
    ``tokens_per_rank`` is one number or a list of W.  Returns a
    (total tokens, W) uint8 array with 1 where the token goes to the rank.
    """
    rng = np.random.default_rng(seed)
    counts = [int(tokens_per_rank)] * W if np.isscalar(tokens_per_rank) else [int(t) for t in tokens_per_rank]
    total = sum(counts)
    if skew_alpha is None:
        keys = rng.random((total, n_experts))
    else:
        p = rng.dirichlet(np.full(n_experts, skew_alpha))
        keys = rng.random((total, n_experts)) ** (1.0 / np.maximum(p, 1e-12))   # weighted sampling without replacement
    experts = np.argsort(-keys, axis=1)[:, :top_k]
    per_rank = n_experts // W
    dest = np.zeros((total, W), dtype=np.uint8)
    np.put_along_axis(dest, np.minimum(experts // per_rank, W - 1), 1, axis=1)
    return dest


def token_rows(W: int, tokens_per_rank, row_bytes: int, seed: int, kind: str = "u8"):
    """W send buffers of tokens_i rows of ``row_bytes`` bytes."""
    rng = np.random.default_rng(seed)
    counts = [int(tokens_per_rank)] * W if np.isscalar(tokens_per_rank) else [int(t) for t in tokens_per_rank]
    return [payload(rng, c * row_bytes, kind) for c in counts]
