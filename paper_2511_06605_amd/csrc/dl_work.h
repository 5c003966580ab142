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

// How an item is cut into tiles.  Tiles lie on a grid of DL_CUT bytes of the item's first destination: with
// shift = that address modulo DL_CUT, tile t of a tile size T (a multiple of DL_CUT) covers the item's bytes
// [t T - shift, (t + 1) T - shift), clipped to [0, bytes).  So every tile but an item's first begins on a
// DL_CUT boundary of the first destination, whatever the addresses are, and no two workgroups write into the
// same 128 bytes of it (partly written lines that two compute units share cost a third of the all-gather rate);
// the other destinations and the source may lie anywhere relative to that grid (16-byte accesses need no
// alignment on this hardware).
constexpr uint32_t DL_CUT = 128;

DL_HD uint32_t dl_item_shift(const dl_plain_item &it)
{
    return (uint32_t)((uint64_t)it.dst & (DL_CUT - 1u));
}

DL_HD uint32_t dl_item_shift(const dl_fused_item &it)
{
    return (uint32_t)((uint64_t)it.dst[0] & (DL_CUT - 1u));
}

// Number of tiles of an item (0 for an empty one).
template <class Item>
DL_HD uint64_t dl_item_tiles(const Item &it, uint32_t tile_bytes)
{
    if (it.bytes == 0) return 0;
    const uint64_t span = it.bytes + dl_item_shift(it);
    return span / tile_bytes + (span % tile_bytes ? 1u : 0u);
}

// Bytes [*lo, *hi) of an item that tile `tile` covers (*lo >= *hi: none).
DL_HD void dl_tile_range(uint32_t shift, uint64_t bytes, uint64_t tile, uint32_t tile_bytes, uint64_t *lo, uint64_t *hi)
{
    const uint64_t begin = tile * tile_bytes;  // on the grid; the item starts `shift` bytes into tile 0
    *lo = begin > shift ? begin - shift : 0;
    const uint64_t end = begin + tile_bytes - shift;
    *hi = end < bytes ? end : bytes;
}
