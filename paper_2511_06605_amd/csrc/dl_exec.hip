// One-shot execution: a whole lowered copy list in ONE kernel launch (the
// compute-unit analogue of queueing many copies back to back on one engine with
// a single completion, Sec. IV-D, and of spreading one large copy over many
// engines, Sec. IV-A).
//
// Short lists travel by value in the kernel-argument segment, so the device
// needs no extra memory round trip to find its work: workgroup b finds its
// (item, tile) from an inclusive prefix sum of tile counts with one wavefront
// ballot.  Long lists are cut into one-tile items on the host and read by the
// device straight from a pinned host ring, workgroup b taking item b.
#include "dl_device.h"
#include "dl_internal.h"

#include <string.h>

#include <vector>

// ------------------------------------------------------------------- kernels

__device__ __forceinline__ uint64_t dl_uniform64(uint64_t v)
{
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

template <bool NT>
__device__ __forceinline__ void dl_run_item(const dl_plain_item &it, uint64_t tile, uint32_t tile_bytes)
{
    char *d[1] = {(char *)dl_uniform64((uint64_t)it.dst)};
    dl_move_tile<1, NT>((const char *)dl_uniform64((uint64_t)it.src), d, 1u, dl_uniform64(it.bytes), tile, tile_bytes,
                        threadIdx.x, blockDim.x);
}

template <bool NT>
__device__ __forceinline__ void dl_run_item(const dl_fused_item &it, uint64_t tile, uint32_t tile_bytes)
{
    char *d[DL_FAN];
#pragma unroll
    for (int j = 0; j < DL_FAN; ++j) d[j] = (char *)dl_uniform64((uint64_t)it.dst[j]);
    dl_move_tile<DL_FAN, NT>((const char *)dl_uniform64((uint64_t)it.src), d, __builtin_amdgcn_readfirstlane(it.k),
                             dl_uniform64(it.bytes), tile, tile_bytes, threadIdx.x, blockDim.x);
}

template <class Item, int NMAX>
struct dl_klist {
    uint32_t n;
    uint32_t tile_bytes;
    uint32_t tile_end[NMAX];  // inclusive prefix sum of tiles per item
    Item item[NMAX];
};

template <class Item, int NMAX, bool NT>
__global__ void __launch_bounds__(512) dl_exec_list_kernel(const dl_klist<Item, NMAX> p)
{
    const uint32_t b = blockIdx.x;
    const uint32_t lane = threadIdx.x & 63u;
    // item index = number of items whose last tile lies before b
    uint32_t d = 0;
#pragma unroll
    for (int base = 0; base < NMAX; base += 64) {
        const uint32_t idx = base + lane;
        const uint32_t e = (idx < p.n) ? p.tile_end[idx < NMAX ? idx : 0] : 0xFFFFFFFFu;
        d += (uint32_t)__popcll(__ballot(e <= b));
    }
    d = __builtin_amdgcn_readfirstlane(d);
    if (d >= p.n) return;
    const uint32_t first = d ? p.tile_end[d - 1] : 0u;
    dl_run_item<NT>(p.item[d], (uint64_t)(b - first), p.tile_bytes);
}

// Same, with a capped grid: workgroup b takes tiles b, b + grid, b + 2 grid, ...
template <class Item, int NMAX, bool NT>
__global__ void __launch_bounds__(512) dl_exec_list_strided_kernel(const dl_klist<Item, NMAX> p)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t total = p.tile_end[p.n - 1];
    for (uint32_t b = blockIdx.x; b < total; b += gridDim.x) {
        uint32_t d = 0;
#pragma unroll
        for (int base = 0; base < NMAX; base += 64) {
            const uint32_t idx = base + lane;
            const uint32_t e = (idx < p.n) ? p.tile_end[idx < NMAX ? idx : 0] : 0xFFFFFFFFu;
            d += (uint32_t)__popcll(__ballot(e <= b));
        }
        d = __builtin_amdgcn_readfirstlane(d);
        if (d >= p.n) return;
        const uint32_t first = d ? p.tile_end[d - 1] : 0u;
        dl_run_item<NT>(p.item[d], (uint64_t)(b - first), p.tile_bytes);
    }
}

template <class Item, bool NT>
__global__ void __launch_bounds__(512) dl_exec_table_kernel(const Item *__restrict__ items, uint32_t n,
                                                            uint32_t tile_bytes)
{
    const uint32_t b = blockIdx.x;
    if (b >= n) return;
    const Item it = items[b];
    dl_run_item<NT>(it, 0, tile_bytes);
}

// ---------------------------------------------------------------- host side

namespace {

constexpr int NMAX_SMALL = 8;
template <class Item> struct list_cap;
template <> struct list_cap<dl_plain_item> { static constexpr int big = 64; };
template <> struct list_cap<dl_fused_item> { static constexpr int big = 32; };

constexpr size_t RING_SLOTS = 4;
constexpr size_t RING_SLOT_BYTES = 1u << 20;

struct ring_t {
    char *base = nullptr;
    hipEvent_t ev[RING_SLOTS]{};
    bool used[RING_SLOTS]{};
    size_t next = 0;
} g_ring;

inline uint32_t item_k(const dl_plain_item &) { return 1; }
inline uint32_t item_k(const dl_fused_item &it) { return it.k; }

template <class Item, int NMAX>
int launch_klist(const Item *items, size_t n, const uint64_t *tile_end, const dl_launch_shape &sh, hipStream_t stream)
{
    dl_klist<Item, NMAX> p;
    p.n = (uint32_t)n;
    p.tile_bytes = sh.tile_bytes;
    for (size_t i = 0; i < n; ++i) {
        p.tile_end[i] = (uint32_t)tile_end[i];
        p.item[i] = items[i];
    }
    const uint32_t grid = (uint32_t)tile_end[n - 1];
    if (sh.max_blocks && grid > sh.max_blocks) {
        if (sh.nontemporal)
            hipLaunchKernelGGL((dl_exec_list_strided_kernel<Item, NMAX, true>), dim3(sh.max_blocks),
                               dim3(sh.block_threads), 0, stream, p);
        else
            hipLaunchKernelGGL((dl_exec_list_strided_kernel<Item, NMAX, false>), dim3(sh.max_blocks),
                               dim3(sh.block_threads), 0, stream, p);
    } else if (sh.nontemporal)
        hipLaunchKernelGGL((dl_exec_list_kernel<Item, NMAX, true>), dim3(grid), dim3(sh.block_threads), 0, stream, p);
    else
        hipLaunchKernelGGL((dl_exec_list_kernel<Item, NMAX, false>), dim3(grid), dim3(sh.block_threads), 0, stream, p);
    DL_HIP(hipGetLastError());
    return DL_OK;
}

inline void advance(dl_plain_item &it, uint64_t off)
{
    it.src += off;
    it.dst += off;
}
inline void advance(dl_fused_item &it, uint64_t off)
{
    it.src += off;
    for (uint32_t j = 0; j < it.k; ++j) it.dst[j] += off;
}

template <class Item>
int launch_table(const Item *items, size_t n, const dl_launch_shape &sh, hipStream_t stream)
{
    if (!g_ring.base) return DL_ERR_STATE;
    const size_t cap = RING_SLOT_BYTES / sizeof(Item);
    size_t i = 0;
    uint64_t off = 0;  // progress inside items[i]
    while (i < n) {
        const size_t s = g_ring.next++ % RING_SLOTS;
        if (g_ring.used[s]) DL_HIP(hipEventSynchronize(g_ring.ev[s]));
        Item *slot = (Item *)(g_ring.base + s * RING_SLOT_BYTES);
        size_t m = 0;
        while (i < n && m < cap) {
            const uint64_t left = items[i].bytes - off;
            if (left == 0) {
                ++i;
                off = 0;
                continue;
            }
            Item it = items[i];
            advance(it, off);
            it.bytes = left < sh.tile_bytes ? left : sh.tile_bytes;
            slot[m++] = it;
            off += it.bytes;
        }
        if (m == 0) break;
        if (sh.nontemporal)
            hipLaunchKernelGGL((dl_exec_table_kernel<Item, true>), dim3((uint32_t)m), dim3(sh.block_threads), 0,
                               stream, slot, (uint32_t)m, sh.tile_bytes);
        else
            hipLaunchKernelGGL((dl_exec_table_kernel<Item, false>), dim3((uint32_t)m), dim3(sh.block_threads), 0,
                               stream, slot, (uint32_t)m, sh.tile_bytes);
        DL_HIP(hipGetLastError());
        DL_HIP(hipEventRecord(g_ring.ev[s], stream));
        g_ring.used[s] = true;
    }
    return DL_OK;
}

template <class Item>
int exec_list(const Item *items, size_t n, hipStream_t stream)
{
    if (n == 0) return DL_OK;
    uint64_t total = 0, biggest = 0;
    uint32_t kmax = 1;
    for (size_t i = 0; i < n; ++i) {
        total += items[i].bytes;
        if (items[i].bytes > biggest) biggest = items[i].bytes;
        if (item_k(items[i]) > kmax) kmax = item_k(items[i]);
    }
    if (total == 0) return DL_OK;
    dl_launch_shape sh = dl_choose_shape(total, biggest, kmax);

    constexpr int NBIG = list_cap<Item>::big;
    if (n <= (size_t)NBIG) {
        uint64_t tile_end[NBIG];
        for (;;) {
            uint64_t acc = 0;
            for (size_t i = 0; i < n; ++i) {
                acc += dl_item_tiles(items[i], sh.tile_bytes);
                tile_end[i] = acc;
            }
            if (acc < (1ull << 30)) break;
            sh.tile_bytes *= 2;  // keep the grid inside the launch limit
        }
        if (n <= (size_t)NMAX_SMALL) return launch_klist<Item, NMAX_SMALL>(items, n, tile_end, sh, stream);
        return launch_klist<Item, NBIG>(items, n, tile_end, sh, stream);
    }
    return launch_table(items, n, sh, stream);
}

uint32_t floor_pow2(uint64_t v)
{
    uint32_t p = 1;
    while ((uint64_t)p * 2 <= v && p < (1u << 30)) p *= 2;
    return p;
}

}  // namespace

// Tile and workgroup size for a request.  Measured on MI355X (all-gather of
// 64 MiB per rank, 1:1 copies of 2 GiB): the finest cut wins.  For fused
// fan-out, one wavefront per workgroup moving one 1 KiB row (one 16-byte load
// and k stores per lane) beat every larger tile; for 1:1 copies 4 KiB tiles of
// 256 threads did.  Larger tiles, capped grids and streaming hints were slower.
dl_launch_shape dl_choose_shape(uint64_t src_bytes, uint64_t max_item_bytes, uint32_t max_k)
{
    const dl_config &c = g_dl.cfg;
    dl_launch_shape sh;
    uint32_t tile = c.tile_bytes;
    if (tile == 0) tile = max_k > 2 ? 1024u : 4096u;
    sh.tile_bytes = tile;
    uint32_t bt = c.block_threads;
    if (bt == 0) {
        const uint64_t span = max_item_bytes < tile ? max_item_bytes : tile;
        bt = floor_pow2(span / 16 ? span / 16 : 1);
        if (bt > 256) bt = 256;
        if (bt < 64) bt = 64;
    }
    sh.block_threads = bt;
    sh.max_blocks = c.max_blocks;
    sh.nontemporal = src_bytes * (1ull + max_k) >= c.nontemporal_min_bytes;
    return sh;
}

int dl_exec_plain(const dl_plain_item *items, size_t n, hipStream_t stream) { return exec_list(items, n, stream); }
int dl_exec_fused(const dl_fused_item *items, size_t n, hipStream_t stream) { return exec_list(items, n, stream); }

int dl_exec_init()
{
    if (g_ring.base) return DL_OK;
    DL_HIP(hipHostMalloc((void **)&g_ring.base, RING_SLOTS * RING_SLOT_BYTES, hipHostMallocDefault));
    for (size_t s = 0; s < RING_SLOTS; ++s) {
        DL_HIP(hipEventCreateWithFlags(&g_ring.ev[s], hipEventDisableTiming));
        g_ring.used[s] = false;
    }
    g_ring.next = 0;
    return DL_OK;
}

int dl_exec_shutdown()
{
    if (!g_ring.base) return DL_OK;
    for (size_t s = 0; s < RING_SLOTS; ++s) {
        if (g_ring.used[s]) (void)hipEventSynchronize(g_ring.ev[s]);
        (void)hipEventDestroy(g_ring.ev[s]);
    }
    (void)hipHostFree(g_ring.base);
    g_ring.base = nullptr;
    return DL_OK;
}
