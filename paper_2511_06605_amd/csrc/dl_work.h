// Internal: the unit of device work and the geometry of cutting it into tiles.
// Shared by the host side (grid sizing) and the kernels (tile -> byte range) of
// the library, so both always agree.  Not part of the C boundary.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define DL_HD __host__ __device__ __forceinline__
#else
#define DL_HD inline
#endif

constexpr int DL_FAN = 8;  // destinations one work item can write from a single read

// A slot of device memory that the host fills through the BAR (short copy tables, masks): the payload, and in the
// last 8 bytes a stamp that is written after it.
constexpr uint32_t DL_PUSH_SLOT_BYTES = 64u << 10;
constexpr uint32_t DL_PUSH_PAYLOAD_BYTES = DL_PUSH_SLOT_BYTES - 8;

// What a kernel that reads a table written through the BAR needs besides the table: the stamp that the slot
// holds once the table is complete, how often to look for it, and where to report that it never came.
struct dl_pushed {
    uint64_t stamp;
    uint32_t tries;
    uint32_t pad;
    uint64_t *lost;  // host-coherent: the library's device error word
};

// Plain copy: one source, one destination.
struct dl_plain_item {
    const char *src;
    char *dst;
    uint64_t bytes;
};

// Swap (Sec. IV-C): the ranges [src, src + bytes) and [dst, dst + bytes), which
// do not overlap, exchange their contents.  Same layout and geometry as a plain
// copy; only what the device does with a tile differs.
struct dl_swap_item : dl_plain_item {};

// Fused broadcast copy: one source read once, k <= DL_FAN destinations.
struct dl_fused_item {
    const char *src;
    uint64_t bytes;
    uint32_t k;
    uint32_t pad;
    char *dst[DL_FAN];
};

// How one item is moved.  The widest element size E in {16, 4, 1} for which the
// source and every destination agree modulo E; `head` bytes bring the source
// (and so every destination) to an E boundary, `body` counts E-byte elements,
// `tail` bytes remain.  Tiles cut the body only; tile 0 also moves head and tail.
struct dl_geom {
    uint32_t esize;  // 16, 4 or 1
    uint32_t head;   // < esize
    uint32_t tail;   // < esize
    uint64_t body;   // elements
};

DL_HD dl_geom dl_make_geom(uint64_t src, uint64_t diff_or, uint64_t bytes)
{
    // diff_or = OR over destinations of (src XOR dst): its low bits are zero
    // exactly where all addresses agree.
    dl_geom g;
    g.esize = ((diff_or & 15) == 0) ? 16u : ((diff_or & 3) == 0) ? 4u : 1u;
    uint64_t head = (0 - src) & (g.esize - 1);
    if (head > bytes) head = bytes;
    g.head = (uint32_t)head;
    g.body = (bytes - head) / g.esize;
    g.tail = (uint32_t)(bytes - head - g.body * g.esize);
    return g;
}

// Number of tiles of an item (at least 1 for a non-empty item, so that head and
// tail bytes always have an owner).
DL_HD uint64_t dl_geom_tiles(const dl_geom &g, uint32_t tile_bytes)
{
    uint64_t per_tile = tile_bytes / g.esize;
    uint64_t t = (g.body + per_tile - 1) / per_tile;
    return t ? t : 1;
}

DL_HD uint64_t dl_item_diff(const dl_plain_item &it)
{
    return (uint64_t)it.src ^ (uint64_t)it.dst;
}

DL_HD uint64_t dl_item_diff(const dl_fused_item &it)
{
    uint64_t d = 0;
    for (uint32_t j = 0; j < it.k && j < (uint32_t)DL_FAN; ++j) d |= (uint64_t)it.src ^ (uint64_t)it.dst[j];
    return d;
}

template <class Item>
DL_HD uint64_t dl_item_tiles(const Item &it, uint32_t tile_bytes)
{
    if (it.bytes == 0) return 0;
    return dl_geom_tiles(dl_make_geom((uint64_t)it.src, dl_item_diff(it), it.bytes), tile_bytes);
}
