// dl_batch_copy_static: the batched copy for callers that cannot allocate (code under stream capture, tight
// serving loops, harnesses that forbid it).  The table that a long list needs on the device lives in a
// file-scope device array instead of memory that the library allocates and recycles with events; the host
// carries the table there in the kernel arguments of small fill kernels, 64 entries at a time, on the caller's
// stream, and the table kernel of the ordinary path then executes it.  Nothing here calls hipMalloc, hipFree,
// an event or a memset, and the host side works on the stack.
#include "dl_device.h"
#include "dl_internal.h"

namespace {

constexpr uint32_t MAX_ENTRIES = DL_STATIC_MAX_COPIES;  // one-tile entries the array holds (a copy is at least one)
constexpr int MAX_DEVICES = 64;

// Each GPU holds its own copy of this array, at its own address, until the process ends.  In host code the name
// is only a handle for hipGetSymbolAddress: the kernels get the address that call returned.
static __device__ __align__(256) unsigned char scratch[(size_t)MAX_ENTRIES * sizeof(dl_plain_item)];

dl_plain_item *g_table[MAX_DEVICES] = {};  // per device: where its copy of `scratch` lives

struct fill_chunk {
    uint32_t n;
    uint32_t first;
    dl_plain_item item[64];
};

// Entries first .. first + n - 1 of the table, one per thread, from the kernel arguments.
__global__ void __launch_bounds__(64) dl_static_fill_kernel(const fill_chunk c, dl_plain_item *__restrict__ table)
{
    const uint32_t i = threadIdx.x;
    if (i < c.n) table[c.first + i] = c.item[i];
}

}  // namespace

// Once per device, with that device current (called by dl_init).
int dl_static_init(int device)
{
    if (device < 0 || device >= MAX_DEVICES) return DL_OK;  // the entry point will say that it has no table there
    if (g_table[device]) return DL_OK;
    void *p = nullptr;
    DL_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    g_table[device] = (dl_plain_item *)p;
    return DL_OK;
}

extern "C" int dl_batch_copy_static(const dl_copy_desc *desc, size_t n, void *stream)
{
    DL_LOCKED;  // a mutex, not an allocation: calls of several threads on one stream stay whole
    if (!g_dl.inited) return DL_ERR_STATE;
    if (dl_device_error_pending()) return DL_ERR_LOST;
    if (n && !desc) return DL_ERR_INVALID;
    if (n > MAX_ENTRIES) return DL_ERR_CAPACITY;
    dl_plain_item *const table = g_dl.device >= 0 && g_dl.device < MAX_DEVICES ? g_table[g_dl.device] : nullptr;
    if (!table) return DL_ERR_STATE;
    hipStream_t hs = (hipStream_t)stream;

    // pass 1: what there is to move, and the tile that cuts it into few enough entries
    uint64_t total = 0, biggest = 0;
    for (size_t i = 0; i < n; ++i) {
        if (desc[i].bytes == 0 || desc[i].src == desc[i].dst) continue;
        if (!desc[i].src || !desc[i].dst) return DL_ERR_INVALID;
        total += desc[i].bytes;
        if (desc[i].bytes > biggest) biggest = desc[i].bytes;
    }
    if (total == 0) return DL_OK;
    auto entries = [&](uint64_t tile) {  // a copy is cut on the grid of its destination, like everywhere (see dl_work.h)
        uint64_t m = 0;
        for (size_t i = 0; i < n; ++i)
            if (desc[i].bytes && desc[i].src != desc[i].dst)
                m += dl_item_tiles(dl_plain_item{(const char *)desc[i].src, (char *)desc[i].dst, desc[i].bytes}, (uint32_t)tile);
        return m;
    };
    // as for the ordinary long list: one entry per copy up to 64 KiB, 64 KiB tiles above that, coarser while
    // that leaves more entries than a table kernel likes; and in any case no more than the array holds
    uint64_t tile = 4096;
    while (tile < 65536u && tile < biggest) tile *= 2;
    while (tile < (1u << 20) && entries(tile) > 8192u) tile *= 2;
    while (entries(tile) > MAX_ENTRIES) {
        if (tile >= (1u << 30)) return DL_ERR_CAPACITY;
        tile *= 2;
    }

    // pass 2: cut, and carry the entries to the table 64 at a time
    fill_chunk c;
    c.n = 0;
    c.first = 0;
    uint32_t m = 0;
    auto flush = [&]() -> int {
        if (c.n == 0) return DL_OK;
        hipLaunchKernelGGL(dl_static_fill_kernel, dim3(1), dim3(64), 0, hs, c, table);
        DL_HIP(hipGetLastError());
        c.first += c.n;
        c.n = 0;
        return DL_OK;
    };
    for (size_t i = 0; i < n; ++i) {
        if (desc[i].bytes == 0 || desc[i].src == desc[i].dst) continue;
        uint64_t piece = tile - ((uint64_t)desc[i].dst & (DL_CUT - 1u));  // the first one ends on the grid
        for (uint64_t off = 0; off < desc[i].bytes; off += piece, piece = tile) {
            const uint64_t left = desc[i].bytes - off;
            c.item[c.n++] = dl_plain_item{(const char *)desc[i].src + off, (char *)desc[i].dst + off, left < piece ? left : piece};
            ++m;
            if (c.n == 64) {
                const int rc = flush();
                if (rc != DL_OK) return rc;
            }
        }
    }
    const int rc = flush();
    if (rc != DL_OK) return rc;
    return dl_launch_plain_table(table, m, (uint32_t)tile, 2 * total, hs);
}
