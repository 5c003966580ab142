// One-shot execution: a whole lowered copy list in ONE kernel launch (the
// compute-unit analogue of queueing many copies back to back on one engine with
// a single completion, Sec. IV-D, and of spreading one large copy over many
// engines, Sec. IV-A).
//
// Short lists travel by value in the kernel-argument segment, so the device
// needs no extra memory round trip to find its work: workgroup b finds its
// (item, tile) from an inclusive prefix sum of tile counts.  Long lists are cut
// into one-tile entries on the host and become a table, workgroup b taking
// entry b: written straight into device memory through the BAR where that is
// possible (see push_acquire), else into a pinned host ring (and copied to
// device memory first when there are many entries).
#include "dl_device.h"
#include "dl_internal.h"

#include <immintrin.h>
#include <stdlib.h>
#include <string.h>

#include <type_traits>
#include <vector>

// ------------------------------------------------------------------- kernels

// Row path only (see dl_run_rows).  A kernel of its own: sharing one kernel with
// the general path cost 5 % of the all-gather rate through its register count.
// ON_GRID: see dl_rows_body.
template <class Item, int NMAX, int POL, bool ON_GRID>
__global__ void __launch_bounds__(512) dl_exec_rows_kernel(const dl_klist<Item, NMAX> p)
{
    dl_run_rows<POL, ON_GRID>(p, blockIdx.x);
}

// Row path over a list too long for the scalar compares of dl_find_item (the 64 chunks of an all-to-all between
// eight ranks): a two-dimensional grid, blockIdx.y the item, blockIdx.x the tile within it, so nothing is
// searched and nothing divided.  The grid is as wide as the longest item; a workgroup beyond its item's last
// row leaves at once (the host takes this path only while few workgroups are wasted that way).  Consecutive
// workgroups walk along one item, so the chip-wide stream of addresses stays sequential.
template <class Item, int NMAX, int POL, bool ON_GRID>
__global__ void __launch_bounds__(512) dl_exec_rows2d_kernel(const dl_klist<Item, NMAX> p)
{
    dl_rows_body<POL, ON_GRID>(p.item[blockIdx.y], blockIdx.x, p.wpg_log2, p.split_log2);
}

// Entry i of a table that the host wrote into device memory through the BAR just before the launch.  A line
// of the table that used this memory before may still sit in a cache, so the entry is read past every cache,
// once per workgroup (8 bytes per lane), and handed on through LDS; before that, one lane has seen the slot's
// stamp.  Call with the whole workgroup.  Null if the stamp never came (reported by the caller).
template <class Item>
__device__ __forceinline__ const Item *dl_pushed_entry(const Item *items, uint32_t i, const dl_pushed &ps)
{
    constexpr uint32_t WORDS = sizeof(Item) / 8;
    static_assert(sizeof(Item) % 8 == 0 && WORDS < 64, "one 8-byte load per lane of the first wavefront");
    __shared__ uint64_t raw[WORDS];
    __shared__ uint32_t sealed;
    if (threadIdx.x == 0) sealed = dl_pushed_sealed(items, ps) ? 1u : 0u;
    __syncthreads();
    if (!sealed) return nullptr;
    if (threadIdx.x < WORDS) raw[threadIdx.x] = dl_ld<DL_POL_COHERENT>(dl_global<uint64_t>(items + i) + threadIdx.x);
    __syncthreads();
    return reinterpret_cast<const Item *>(raw);
}

// Row path over a table of equally sized items in device memory (long lists: thousands of token
// rows, hundreds of cache blocks) on a two-dimensional grid: blockIdx.y is the item (at most DL_UROWS_MAX_ITEMS,
// the grid's limit in that dimension), which every workgroup of that item finds in the scalar cache, blockIdx.x
// the tile within it; nothing is divided.  PUSHED: see dl_pushed_entry.
template <class Item, int POL, bool PUSHED, bool ON_GRID>
__global__ void __launch_bounds__(512) dl_exec_urows_kernel(const Item *__restrict__ items, uint32_t wpg_log2,
                                                            uint32_t split_log2, const dl_pushed ps)
{
    const uint32_t d = blockIdx.y;
    if constexpr (PUSHED) {
        const Item *it = dl_pushed_entry(items, d, ps);
        if (it)
            dl_rows_body<POL, ON_GRID>(*it, blockIdx.x, wpg_log2, split_log2);
        else if (threadIdx.x == 0)
            dl_pushed_report_lost(ps);  // nothing copied by this workgroup; the host hears of it
    } else
        dl_rows_body<POL, ON_GRID>(items[d], blockIdx.x, wpg_log2, split_log2);
}

// General path: any tile size, one workgroup per tile.
template <class Item, int NMAX, int POL>
__global__ void __launch_bounds__(512) dl_exec_list_kernel(const dl_klist<Item, NMAX> p)
{
    dl_run_tile<POL>(p, blockIdx.x);
}

// Same, with a capped grid: workgroup b takes tiles b, b + grid, b + 2 grid, ...
template <class Item, int NMAX, int POL>
__global__ void __launch_bounds__(512) dl_exec_list_strided_kernel(const dl_klist<Item, NMAX> p)
{
    const uint32_t total = p.tile_end[p.n - 1];
    for (uint32_t b = blockIdx.x; b < total; b += gridDim.x) dl_run_tile<POL>(p, b);
}

template <class Item, int POL, bool PUSHED = false>
__global__ void __launch_bounds__(512) dl_exec_table_kernel(const Item *__restrict__ items, uint32_t n, uint32_t split,
                                                            const dl_pushed ps)
{
    const uint32_t b = blockIdx.x;
    if (b >= n) return;
    if constexpr (PUSHED) {
        const Item *pushed = dl_pushed_entry(items, b, ps);
        if (!pushed) {
            if (threadIdx.x == 0) dl_pushed_report_lost(ps);  // nothing copied by this workgroup; the host hears of it
            return;
        }
        const Item it = *pushed;
        dl_run_entry<POL>(it, split);
    } else {
        const Item it = items[b];
        dl_run_entry<POL>(it, split);
    }
}

// ------------------------------------------------------------ armed kernels
//
// The compute-unit analogue of a poll command queued in front of the copies
// (Sec. IV-E): the kernel is enqueued ahead of time, its workgroups wait until
// the doorbell word (in device memory that the host writes through the BAR, else
// in host-coherent memory) reaches their ticket, then copy.
// No workgroup ever waits for another one to make progress, and every wait is
// bounded by a wall-clock limit, so every wave leaves the kernel.

enum : uint32_t { DL_GO_WAIT = 0, DL_GO_RUN = 1, DL_GO_SKIP = 2 };

// Housekeeping of a request, done by one thread where its stores' round trips delay nothing: clear the
// counters that the slot's next request will count on, and tell the host that the kernel is resident.
__device__ __forceinline__ void dl_arm_housekeeping(const dl_arm &a)
{
    for (uint32_t g = 0; a.arrive_clear && g <= DL_ARM_GROUPS; ++g)
        __hip_atomic_store((uint32_t *)((char *)a.arrive_clear + g * DL_ARM_STRIDE), 0u, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(a.armed, a.ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Returns DL_GO_RUN once the doorbell has been rung for this ticket, DL_GO_SKIP
// if the request was cancelled or the limit ran out.  Uniform over the workgroup.
__device__ __forceinline__ uint32_t dl_arm_wait(const dl_arm &a)
{
    __shared__ uint32_t s_go;
    if (a.nowait && a.gated) {
        // uniform over the grid: the waiting was done by the gate kernel that ran before this one on the stream
        // (see dl_arm_gate_kernel); what it decided lies in the slot's first flag
        if (threadIdx.x == 0) {
            const uint64_t g = __hip_atomic_load(a.go, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_go = (g >> 2) == a.ticket ? (uint32_t)(g & 3u) : (uint32_t)DL_GO_SKIP;
            if (a.trace_host && blockIdx.x == 0 && s_go == DL_GO_RUN)
                __hip_atomic_store(a.trace_host + 1, (uint64_t)wall_clock64(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        __syncthreads();
        return s_go;
    }
    if (a.nowait) {  // uniform over the grid: started without a doorbell; housekeeping follows the copy
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            if (a.trace_host) {
                const uint64_t t = (uint64_t)wall_clock64();
                __hip_atomic_store(a.trace_host, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                __hip_atomic_store(a.trace_host + 1, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
        }
        return DL_GO_RUN;
    }
    if (threadIdx.x == 0) {
        uint32_t go = DL_GO_SKIP;
        const uint64_t t0 = wall_clock64();
        if (blockIdx.x == 0) dl_arm_housekeeping(a);  // before the wait: off the critical path
        if (a.direct || blockIdx.x == 0) {
            // poll the doorbell (system-scope loads past every cache: device memory, or host memory over the link)
            for (uint32_t spins = 1;; ++spins) {
                // doorbell and cancel word sit side by side in one aligned 16 bytes: one read over the link
                // (each is an aligned 8-byte word that the host writes with one store, so neither can tear)
                const dl_u32x4 w = dl_ld<DL_POL_COHERENT>(dl_global<dl_u32x4>(a.bell));
                const uint64_t bell = (uint64_t)w.x | ((uint64_t)w.y << 32);
                const uint64_t cancel = (uint64_t)w.z | ((uint64_t)w.w << 32);
                if (cancel >= a.ticket) break;
                if (bell >= a.ticket) {
                    go = DL_GO_RUN;
                    if (a.trace_host && blockIdx.x == 0)
                        __hip_atomic_store(a.trace_host, (uint64_t)wall_clock64(), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_SYSTEM);
                    break;
                }
                if ((spins & 3u) == 0 && (uint64_t)wall_clock64() - t0 > a.limit_ticks) break;
                if (spins >= a.max_spins) break;
                if (blockIdx.x && !a.direct) __builtin_amdgcn_s_sleep(8);
            }
            if (!a.direct) {
                // pass the word on: one flag per group of workgroups, each in its own cache line
                // (the flag carries everything the others need, so it is not ordered against anything)
                const uint32_t groups = gridDim.x < DL_ARM_GROUPS ? gridDim.x : DL_ARM_GROUPS;
                for (uint32_t g = 0; g < groups; ++g)
                    __hip_atomic_store((uint64_t *)((char *)a.go + g * DL_ARM_STRIDE), (a.ticket << 2) | go,
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        } else {
            // wait for workgroup 0 to pass the word on through device memory
            const uint64_t *flag = (const uint64_t *)((const char *)a.go + (blockIdx.x % DL_ARM_GROUPS) * DL_ARM_STRIDE);
            for (uint32_t spins = 1;; ++spins) {
                const uint64_t g = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((g >> 2) == a.ticket) {
                    go = (uint32_t)(g & 3u);
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
                if ((spins & 15u) == 0 && (uint64_t)wall_clock64() - t0 > a.limit_ticks + a.margin_ticks) break;
                if (spins >= a.max_spins) break;
            }
        }
        if (a.trace_host && blockIdx.x == 0 && go == DL_GO_RUN)  // the polling workgroup is the first to begin its copy
            __hip_atomic_store(a.trace_host + 1, (uint64_t)wall_clock64(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        s_go = go;
    }
    __syncthreads();
    // No cache invalidate here: the copy that follows loads at system scope (DL_POL_COHERENT), so
    // it sees everything that was written before the doorbell was rung.
    return s_go;
}

// Count this workgroup in; the last one to arrive publishes the completion word.
// Arrivals are counted per group first (a counter per cache line), and the last
// of each group is counted at the top, so no counter sees more than
// grid / DL_ARM_GROUPS + DL_ARM_GROUPS updates.  The low 16 bits of a counter
// count arrivals, the high bits count workgroups that skipped the copy.
//
// No cache write-back anywhere: the copy stored at system scope, so once every
// wavefront has drained its memory counter the workgroup's bytes are visible to
// the host and to every later kernel, and relaxed counters suffice.  (With
// ordinary stores each workgroup had to write the L2 back before counting
// itself in; that serialised per XCD and cost ~0.5 us per workgroup.)
__device__ __forceinline__ void dl_arm_finish(const dl_arm &a, uint32_t go)
{
    // without a doorbell there was no wait to hide the housekeeping behind: its stores go out behind the copy's
    // and share their round trip
    if (a.nowait && blockIdx.x == 0 && threadIdx.x == 0) dl_arm_housekeeping(a);
    dl_drain_stores();
    __syncthreads();
    if (threadIdx.x == 0 && a.own_word) {
        // a small grid: the host waits for one word per workgroup, no count in between
        __hip_atomic_store(a.done + blockIdx.x, a.ticket | (go == DL_GO_RUN ? 0ull : DL_DONE_SKIPPED), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
        return;
    }
    if (threadIdx.x == 0) {
        const uint32_t grid = gridDim.x;
        const bool flat = grid <= DL_ARM_FLAT_MAX;  // few enough to count at one word without queueing there
        const uint32_t groups = flat ? grid : DL_ARM_GROUPS;
        const uint32_t g = blockIdx.x % DL_ARM_GROUPS;
        const uint32_t gsize = (grid - g + DL_ARM_GROUPS - 1) / DL_ARM_GROUPS;
        uint32_t *gcount = (uint32_t *)((char *)a.arrive + g * DL_ARM_STRIDE);
        uint32_t *top = (uint32_t *)((char *)a.arrive + DL_ARM_GROUPS * DL_ARM_STRIDE);
        // this workgroup's stores have drained; the workgroup that turns out to be the last of all reports
        // its own reading as the end of the last copy (no extra traffic for the others)
        const uint64_t t_end = a.trace_host ? (uint64_t)wall_clock64() : 0ull;
        uint32_t add = 1u + (go == DL_GO_RUN ? 0u : 0x10000u);
        uint32_t old;
        if (!flat) {
            old = __hip_atomic_fetch_add(gcount, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((old & 0xFFFFu) != gsize - 1u) return;
            // last of the group: carry the result to the top
            add = 1u + (((old >> 16) + (add >> 16)) << 16);
        }
        // a small grid is counted at the top directly
        old = __hip_atomic_fetch_add(top, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((old & 0xFFFFu) != groups - 1u) return;
        // last of all
        // The counters stay as they are: the slot's next request counts on the other set and clears this one
        // (see dl_arm).  Nothing is in flight from this wavefront here except, when tracing, the stamps, which
        // must have landed before the completion word.
        const uint32_t skipped = (old >> 16) + (add >> 16);
        if (a.trace_host) {
            __hip_atomic_store(a.trace_host + 2, t_end, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            __hip_atomic_store(a.trace_host + 3, (uint64_t)wall_clock64(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            dl_drain_stores();
        }
        __hip_atomic_store(a.done, a.ticket | (skipped ? DL_DONE_SKIPPED : 0ull), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// Gate of a large prelaunched request.  A grid that waits for a doorbell must stay small (see armed_grid), and a
// small grid is what bounds a large copy.  So the waiting is done by this kernel, one workgroup, and the copy by
// an ordinary signal-style kernel with a full grid that is enqueued behind it on the same stream: it starts when
// this one ends, reads what this one decided, and copies or reports that the request gave up.  One more kernel
// start (0.5-1.5 us measured) on the critical path, which pays from about 256 MiB moved; and while the request waits it
// holds one workgroup instead of one on every other compute unit.
__global__ void __launch_bounds__(64) dl_arm_gate_kernel(const dl_arm a)
{
    const uint32_t go = dl_arm_wait(a);
    if (threadIdx.x == 0)
        __hip_atomic_store(a.go, (a.ticket << 2) | (uint64_t)go, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <class Item, int NMAX, bool ROWS>
__global__ void __launch_bounds__(512) dl_armed_list_kernel(const dl_klist<Item, NMAX> p, const dl_arm a)
{
    {
        // Before the wait: read what the workgroup's first tile will need from the list, so that after the
        // doorbell those scalar loads hit the scalar cache instead of going to memory one after the other.
        uint32_t first;
        const uint32_t d = dl_find_item(p, blockIdx.x, &first);
        uint64_t touched = first + p.n + p.tile_end[p.n - 1];
        if (d < p.n) {
            const Item &it = p.item[d];
            touched += (uint64_t)it.src + it.bytes + (uint64_t)dl_item_dst(it, 0) + (uint64_t)dl_item_dst(it, DL_FAN - 1);
        }
        asm volatile("" ::"s"(touched));
    }
    const uint32_t go = dl_arm_wait(a);
    if (go == DL_GO_RUN) {
        const uint32_t total = p.tile_end[p.n - 1];
        if constexpr (ROWS && !std::is_same<Item, dl_swap_item>::value) {
            // A grid that makes several passes (it is capped while it waits) keeps four rows in flight per
            // wavefront, or two: a coherent load takes a microsecond or two, and one per pass left the memory idle.
            const uint32_t grid = gridDim.x;
            if (total <= grid)
                dl_run_rows<DL_POL_COHERENT>(p, blockIdx.x);
            else if (p.split_log2 != 0)  // (a forced shape: the several-rows form knows one sub-group only)
                for (uint32_t b = blockIdx.x; b < total; b += grid) dl_run_rows<DL_POL_COHERENT>(p, b);
            else if (total <= 2u * grid)
                dl_run_rows_coherent<2>(p, blockIdx.x, grid, total, a.go);
            else
                for (uint32_t b = blockIdx.x; b < total; b += 4u * grid) dl_run_rows_coherent<4>(p, b, grid, total, a.go);
        } else {
            for (uint32_t b = blockIdx.x; b < total; b += gridDim.x) {
                if constexpr (ROWS)
                    dl_run_rows<DL_POL_COHERENT>(p, b);
                else
                    dl_run_tile<DL_POL_COHERENT>(p, b);
            }
        }
    }
    dl_arm_finish(a, go);
}

// What a standby executor reads once its doorbell has rung.  The two copies of the ticket and the activation
// number let the executor refuse a record that is not the one its doorbell announced.
struct dl_standby_rec {
    uint64_t ticket_front;
    uint64_t activation;  // which arming of this pool slot the record is for (the executor's doorbell value)
    uint64_t *done;       // the request's completion words (host-coherent): one per tile up to DL_DONE_WORDS tiles, else one
    uint64_t arrivals;    // written as 0; requests of more than DL_DONE_WORDS tiles count their workgroups in here
    // The ticket's slot has two sets of arrival counters that its requests use in turn, each clearing the set it
    // does not use (see dl_arm).  A request served here counts nothing there, but it keeps that chain: this is
    // the set it clears.
    uint32_t *arrive_clear;
    uint64_t plain;       // 1: `copies` holds the request (up to 64 plain copies); 0: `list` (up to 8 read-once/write-k items)
    union {
        dl_klist<dl_fused_item, 8> list;
        dl_klist<dl_plain_item, 64> copies;
    };
    uint64_t ticket_back;
};
static_assert(sizeof(dl_standby_rec) <= DL_STANDBY_REC_BYTES && sizeof(dl_standby_rec) % 8 == 0, "record size");
static_assert(offsetof(dl_standby_rec, list.tile_end) == offsetof(dl_standby_rec, copies.tile_end) &&
                  offsetof(dl_standby_rec, list.n) == offsetof(dl_standby_rec, copies.n),
              "the two kinds of list start alike");

// Standby executor: a generic armed kernel (see dl_internal.h).  Its doorbell is its pool slot's, its "ticket"
// the slot's activation number; the request's own ticket and completion words come with the record.  Workgroup b
// copies tile b of the request; workgroups beyond its last tile have nothing to do and nothing to report.
__global__ void __launch_bounds__(DL_STANDBY_THREADS) dl_standby_kernel(dl_standby_rec *rec_mem, const dl_arm a)
{
    constexpr uint32_t VEC = (uint32_t)((sizeof(dl_standby_rec) + 15) / 16);
    static_assert(VEC <= DL_STANDBY_THREADS, "one 16-byte load per thread fetches the record");
    __shared__ dl_u32x4 raw[VEC];
    if (dl_arm_wait(a) != DL_GO_RUN) return;  // cancelled or never used: no request, nothing to report
    // the record was complete before the doorbell was rung; these loads go to where it lies (device or host
    // memory), past every cache
    if (threadIdx.x < VEC) raw[threadIdx.x] = dl_ld<DL_POL_COHERENT>(dl_global<dl_u32x4>(rec_mem) + threadIdx.x);
    __syncthreads();
    const dl_standby_rec &rec = *reinterpret_cast<const dl_standby_rec *>(raw);
    // n, tile_bytes, split and tile_end[] sit at the same offsets in both kinds of list
    const uint32_t n_max = rec.plain ? 64u : 8u;
    const bool ok = rec.ticket_front != 0 && rec.ticket_front == rec.ticket_back && rec.activation == a.ticket &&
                    rec.done != nullptr && rec.list.n >= 1 && rec.list.n <= n_max && rec.list.tile_bytes == DL_STANDBY_TILE &&
                    rec.list.split == 1 && rec.copies.tile_end[rec.list.n - 1] <= gridDim.x;
    if (!ok) return;  // not the announced record: touch nothing (the host's wait for the request times out)
    const uint32_t tiles = rec.copies.tile_end[rec.list.n - 1];
    if (blockIdx.x >= tiles) return;
    if (blockIdx.x == 0 && threadIdx.x == 0)  // in flight beside the copy, drained with it before the completion word
        for (uint32_t g = 0; rec.arrive_clear && g <= DL_ARM_GROUPS; ++g)
            __hip_atomic_store((uint32_t *)((char *)rec.arrive_clear + g * DL_ARM_STRIDE), 0u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    if (rec.plain)
        dl_run_rows<DL_POL_COHERENT>(rec.copies, blockIdx.x);
    else
        dl_run_rows<DL_POL_COHERENT>(rec.list, blockIdx.x);
    // the copy stored at system scope: once the memory counters have drained, the bytes are where everybody sees them
    dl_drain_stores();
    __syncthreads();
    if (threadIdx.x != 0) return;
    if (tiles <= DL_DONE_WORDS) {
        // the host waits for one word per tile, no count in between
        __hip_atomic_store(rec.done + blockIdx.x, rec.ticket_front, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    } else {
        // count in at the record (device memory: the host sends such requests only there); the last one reports
        const uint64_t before = __hip_atomic_fetch_add(&rec_mem->arrivals, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (before == tiles - 1u)
            __hip_atomic_store(rec.done, rec.ticket_front, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// Entry i of a table written through the BAR (see dl_pushed_entry), read by every lane for itself: all lanes
// load the same 8 bytes, which costs one request per wavefront, and no barrier.  For kernels that walk a table.
// *sealed: the slot's stamp has been seen (looked for here, before the entry is read, unless an earlier call
// saw it already: once the stamp is there the whole table is); if it is not, the entry is not to be used.
template <class Item>
__device__ __forceinline__ Item dl_pushed_entry_per_lane(const Item *items, uint32_t i, const dl_pushed &ps, bool *sealed)
{
    static_assert(sizeof(Item) % 8 == 0, "whole 8-byte words");
    union {
        Item it;
        uint64_t w[sizeof(Item) / 8];
    } u;
    if (!*sealed) *sealed = dl_uniform64(dl_pushed_sealed(items, ps) ? 1ull : 0ull) != 0;
#pragma unroll
    for (uint32_t q = 0; q < sizeof(Item) / 8; ++q) {
        const uint64_t v = *sealed ? dl_ld<DL_POL_COHERENT>(dl_global<uint64_t>(items + i) + q) : 0ull;
        u.w[q] = dl_uniform64(v);  // the same in every lane: keep it in scalar registers
    }
    return u.it;
}

// PUSHED: the table was written through the BAR when the request was armed; the workgroup's first entry is
// fetched before the wait.
template <class Item, bool PUSHED = false>
__global__ void __launch_bounds__(512) dl_armed_table_kernel(const Item *__restrict__ items, uint32_t n, uint32_t split,
                                                             const dl_pushed ps, const dl_arm a)
{
    if constexpr (PUSHED) {
        Item it{};
        bool sealed = blockIdx.x >= n;  // looked for with the first entry; once the stamp has been seen the whole table is there
        if (blockIdx.x < n) it = dl_pushed_entry_per_lane(items, blockIdx.x, ps, &sealed);
        uint32_t go = dl_arm_wait(a);
        if (!sealed && go == DL_GO_RUN) go = DL_GO_SKIP;  // reported like a request that gave up
        if (go == DL_GO_RUN) {
            for (uint32_t b = blockIdx.x; b < n; b += gridDim.x) {
                if (b != blockIdx.x) it = dl_pushed_entry_per_lane(items, b, ps, &sealed);
                dl_run_entry<DL_POL_COHERENT>(it, split);
            }
        }
        dl_arm_finish(a, go);
    } else {
        const uint32_t go = dl_arm_wait(a);
        if (go == DL_GO_RUN) {
            for (uint32_t b = blockIdx.x; b < n; b += gridDim.x) {
                const Item it = items[b];
                dl_run_entry<DL_POL_COHERENT>(it, split);
            }
        }
        dl_arm_finish(a, go);
    }
}

// ---------------------------------------------------------------- host side

namespace {

constexpr int NMAX_SMALL = 8;
template <class Item> struct list_cap;
template <> struct list_cap<dl_plain_item> { static constexpr int big = 64; };
template <> struct list_cap<dl_swap_item> { static constexpr int big = 64; };
template <> struct list_cap<dl_fused_item> { static constexpr int big = 32; };

constexpr uint32_t DL_UROWS_MAX_ITEMS = 65535;    // a grid's second dimension goes no further
constexpr uint64_t TABLE_ENTRIES_TARGET = 8192;  // table kernels: aim for at most this many one-tile entries
constexpr uint64_t UNIFORM_ROWS_MIN_BYTES = 4ull << 20;  // source bytes from which a uniform long list takes the row kernel
constexpr uint64_t UNIFORM_ROWS_STAGE_BYTES = 768ull << 20;  // bytes moved (read + written) from which its table is staged even where it could be pushed
constexpr size_t TABLE_STAGE_MIN = 512;          // tables at least this long are staged in device memory first
constexpr size_t RING_SLOTS = 4;
constexpr size_t RING_SLOT_BYTES = DL_RING_SLOT_BYTES;

constexpr size_t PUSH_SLOT_BYTES = DL_PUSH_SLOT_BYTES;        // a slot of the tables written through the BAR
constexpr size_t PUSH_PAYLOAD_BYTES = DL_PUSH_PAYLOAD_BYTES;  // the longest such table
constexpr size_t PUSH_SLOTS = 64, PUSH_BATCH = PUSH_SLOTS / 2;

struct ring_t {
    char *base = nullptr;  // pinned host memory: the host writes tables here
    char *dev = nullptr;   // device memory of the same shape: long tables are staged here before they are used
    // Tables written through the BAR (see push_acquire): PUSH_SLOTS slots of device memory that the host can
    // store into, used in turn.  Before a slot is used again the kernel that read its table must have ended:
    // cover[s] names the slot whose event was recorded behind that kernel.  On a stream that cannot go away
    // between calls (the default stream, the library's own) the launches of up to PUSH_BATCH calls in a row
    // share one event, recorded behind the last of them; on a caller's stream every launch gets its own, while
    // the handle is known to be good.
    char *push = nullptr;
    size_t push_next = 0;                 // slot that the next table takes
    hipEvent_t push_ev[PUSH_SLOTS]{};
    int push_cover[PUSH_SLOTS]{};         // -1: never used, or used in the batch that is still open
    bool push_used[PUSH_SLOTS]{};
    uint64_t push_armed[PUSH_SLOTS]{};    // ticket of the armed (prelaunch mode) request whose table is in the slot, or 0
    size_t batch_first = 0, batch_len = 0;  // the open batch: slots batch_first .. batch_first + batch_len - 1 (mod PUSH_SLOTS)
    hipStream_t batch_stream = nullptr;
    hipStream_t own_stream = nullptr;     // the library's stream for armed requests, while it exists
    // the pinned ring: an event per slot, recorded behind the kernel that reads it
    hipEvent_t ev[RING_SLOTS]{};
    bool used[RING_SLOTS]{};
    uint64_t armed[RING_SLOTS]{};         // ticket of the armed (prelaunch mode) request whose table is in the slot, or 0
    size_t next = 0;
} g_ring;

// Calls f with the cache policy as a compile-time constant.
template <class F>
inline void with_policy(int policy, F f)
{
    switch (policy) {
    case DL_POL_STREAM: f(std::integral_constant<int, DL_POL_STREAM>{}); break;
    case DL_POL_WT: f(std::integral_constant<int, DL_POL_WT>{}); break;
    default: f(std::integral_constant<int, DL_POL_PLAIN>{}); break;
    }
}

// ... and with whether every item lies on the grid (see dl_rows_body) as one too.
template <class F>
inline void with_policy_and_grid(int policy, bool on_grid, F f)
{
    with_policy(policy, [&](auto pol) {
        if (on_grid)
            f(pol, std::true_type{});
        else
            f(pol, std::false_type{});
    });
}

// The item's first destination stands on a DL_CUT boundary, its length is a multiple of 16 and its source one of 4.
template <class Item>
inline bool item_on_grid(const Item &it)
{
    return dl_item_shift(it) == 0 && (it.bytes & 15u) == 0 && ((uint64_t)it.src & 3u) == 0;
}

inline uint32_t log2u(uint32_t v)
{
    uint32_t l = 0;
    while ((2u << l) <= v) ++l;
    return l;
}

// Row path layout of a fused item's destinations: sub-group g of `split` owns
// slots g * (DL_FAN / split) onwards and gets destinations g * per ..
// g * per + per - 1 (per = ceil(k / split)), filled from the front; unused
// slots are null, which is what ends a sub-group's store loop on the device.
inline void slots_by_subgroup(dl_plain_item &, uint32_t) {}
inline void slots_by_subgroup(dl_fused_item &it, uint32_t split)
{
    char *by_group[DL_FAN] = {};
    const uint32_t slots = (uint32_t)DL_FAN / split, per = (it.k + split - 1) / split;
    for (uint32_t g = 0; g < split; ++g)
        for (uint32_t q = 0; q < per && g * per + q < it.k; ++q) by_group[g * slots + q] = it.dst[g * per + q];
    for (int j = 0; j < DL_FAN; ++j) it.dst[j] = by_group[j];
}

inline uint32_t item_k(const dl_plain_item &) { return 1; }
inline uint32_t item_k(const dl_fused_item &it) { return it.k; }

constexpr uint32_t ARMED_DIRECT_MAX = 16;  // grids up to this size report in a completion word per workgroup; the shape rule below aims for them

// Workgroups of an armed kernel.  While it waits for its doorbell the kernel must leave room for other
// kernels, above all for the ones that produce what it is going to copy.  Room means whole compute units: a
// kernel whose wavefronts take all the vector registers of a SIMD (a large matrix multiplication's do) cannot
// share that SIMD with even one waiting wavefront, and behind a grid that had a workgroup on every compute
// unit such a kernel did not start until the armed request expired.  Unless the caller sets the cap, the grid
// has at most one workgroup for every other compute unit.
// A kernel that does not wait (signal mode) is in nobody's way: it gets half of the wavefront slots.
uint32_t armed_grid(uint64_t tiles, uint32_t block_threads, bool waits)
{
    const uint32_t cus = (uint32_t)(g_dl.num_cu > 0 ? g_dl.num_cu : 256);
    uint32_t cap = g_dl.cfg.armed_blocks ? g_dl.cfg.armed_blocks : waits ? cus / 2u : 16u * cus / (block_threads / 64u);
    if (cap < 1u) cap = 1u;
    if (cap > 32768u) cap = 32768u;  // the arrival counter keeps 16 bits for the count
    return (uint32_t)(tiles < cap ? tiles : cap);
}

// Enqueue the gate of a chained request and turn `a` into what the copy kernel behind it gets.
int launch_gate(dl_arm &a, hipStream_t stream)
{
    dl_arm gate = a;
    gate.direct = 1;  // one workgroup: it polls the doorbell itself wherever that lies
    gate.own_word = 0;
    gate.gated = 0;
    hipLaunchKernelGGL(dl_arm_gate_kernel, dim3(1), dim3(64), 0, stream, gate);
    DL_HIP(hipGetLastError());
    a.nowait = 1;
    a.gated = 1;
    return DL_OK;
}

template <class Item, int NMAX>
int launch_klist(const Item *items, size_t n, const uint64_t *tile_end, const dl_launch_shape &sh, hipStream_t stream,
                 const dl_arm *arm)
{
    dl_klist<Item, NMAX> p;
    p.n = (uint32_t)n;
    p.tile_bytes = sh.tile_bytes;
    p.split = sh.split;
    p.split_log2 = log2u(sh.split);
    p.wpg_log2 = log2u(sh.block_threads / 64u / sh.split);
    for (size_t i = 0; i < n; ++i) {
        p.tile_end[i] = (uint32_t)tile_end[i];
        p.item[i] = items[i];
    }
    for (size_t i = n; i < (size_t)NMAX; ++i) p.tile_end[i] = 0xFFFFFFFFu;  // the device compares without looking at n
    bool on_grid = true;
    for (size_t i = 0; i < n; ++i) on_grid = on_grid && item_on_grid(items[i]);
    if (sh.rows)
        for (size_t i = 0; i < n; ++i) slots_by_subgroup(p.item[i], sh.split);
    const uint32_t grid = (uint32_t)tile_end[n - 1];
    if (arm) {
        dl_arm a = *arm;
        if (sh.chain && !a.nowait) {
            const int rc = launch_gate(a, stream);
            if (rc != DL_OK) return rc;
        }
        const uint32_t g = armed_grid(grid, sh.block_threads, !a.nowait);
        a.direct = g <= a.direct_max ? 1u : 0u;
        a.own_word = g <= DL_DONE_WORDS && !a.trace_host ? 1u : 0u;  // the stamps come from the last arriver
        g_dl.armed_words = a.own_word ? g : 1u;
        if (sh.rows)
            hipLaunchKernelGGL((dl_armed_list_kernel<Item, NMAX, true>), dim3(g), dim3(sh.block_threads), 0, stream, p, a);
        else
            hipLaunchKernelGGL((dl_armed_list_kernel<Item, NMAX, false>), dim3(g), dim3(sh.block_threads), 0, stream, p, a);
    } else if (sh.rows && sh.rows2d_width) {
        with_policy_and_grid(sh.policy, on_grid, [&](auto pol, auto og) {
            hipLaunchKernelGGL((dl_exec_rows2d_kernel<Item, NMAX, decltype(pol)::value, decltype(og)::value>),
                               dim3(sh.rows2d_width, (uint32_t)n), dim3(sh.block_threads), 0, stream, p);
        });
    } else if (sh.rows) {
        with_policy_and_grid(sh.policy, on_grid, [&](auto pol, auto og) {
            hipLaunchKernelGGL((dl_exec_rows_kernel<Item, NMAX, decltype(pol)::value, decltype(og)::value>), dim3(grid),
                               dim3(sh.block_threads), 0, stream, p);
        });
    } else if (sh.max_blocks && grid > sh.max_blocks) {
        with_policy(sh.policy, [&](auto pol) {
            hipLaunchKernelGGL((dl_exec_list_strided_kernel<Item, NMAX, decltype(pol)::value>), dim3(sh.max_blocks),
                               dim3(sh.block_threads), 0, stream, p);
        });
    } else {
        with_policy(sh.policy, [&](auto pol) {
            hipLaunchKernelGGL((dl_exec_list_kernel<Item, NMAX, decltype(pol)::value>), dim3(grid),
                               dim3(sh.block_threads), 0, stream, p);
        });
    }
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

// Short tables skip the pinned ring.  Where the device exposes all of its memory through a PCIe BAR the host
// writes the table straight into device memory (write-combined stores, nothing is ever read back), fences, and
// launches: posted writes reach the device in order, the launch's doorbell is one of them, so the kernel finds
// the table complete, and in its own memory.  (Through the pinned ring every workgroup fetched its entry over
// the host link, or a staging kernel ran in front.)
//
// push_acquire: a slot for a table of table_bytes whose kernel will be launched on `stream` next, or null if
// this table cannot go that way (*rc says whether that is an error).  push_commit: after that launch.
// Wait for `ev`, behind which the memory that is about to be reused was last read.  If that reader is an armed
// request that nobody has triggered yet, the wait could only end with that request's expiry: refuse instead.
int wait_for_readers(hipEvent_t ev, uint64_t armed_ticket)
{
    if (armed_ticket && dl_armed_untriggered(armed_ticket)) return DL_ERR_STATE;
    DL_HIP(hipEventSynchronize(ev));
    return DL_OK;
}

// Record one event behind everything the open batch has launched; its slots are covered by it from now on.
int push_close_batch()
{
    if (g_ring.batch_len == 0) return DL_OK;
    const size_t last = (g_ring.batch_first + g_ring.batch_len - 1) % PUSH_SLOTS;
    DL_HIP(hipEventRecord(g_ring.push_ev[last], g_ring.batch_stream));
    for (size_t q = 0; q < g_ring.batch_len; ++q) g_ring.push_cover[(g_ring.batch_first + q) % PUSH_SLOTS] = (int)last;
    g_ring.batch_len = 0;
    return DL_OK;
}

char *push_acquire(size_t table_bytes, hipStream_t stream, int *rc)
{
    *rc = DL_OK;
    if (!g_ring.push || !g_dl.cfg.table_push || table_bytes > PUSH_PAYLOAD_BYTES) return nullptr;
    // a batch is one stream's: another stream ends it (on its own stream, which is one that cannot have gone)
    if (g_ring.batch_len && (stream != g_ring.batch_stream || g_ring.batch_len >= PUSH_BATCH))
        if ((*rc = push_close_batch()) != DL_OK) return nullptr;
    const size_t s = g_ring.push_next;
    if (g_ring.push_used[s]) {  // the kernel that read this slot's previous table must have ended
        if (g_ring.push_cover[s] < 0) {
            *rc = DL_ERR_STATE;  // cannot happen: a batch is shorter than the ring
            return nullptr;
        }
        if ((*rc = wait_for_readers(g_ring.push_ev[g_ring.push_cover[s]], g_ring.push_armed[s])) != DL_OK) return nullptr;
    }
    g_ring.push_used[s] = false;  // free until push_commit: a call that fails in between leaves it so
    g_ring.push_armed[s] = 0;
    return g_ring.push + s * PUSH_SLOT_BYTES;
}

// After the last write into the slot: the payload leaves the write-combining buffers, then the stamp, then
// whatever the caller does next (the launch).
uint64_t push_seal(char *slot)
{
    static uint64_t stamps = 0;
    const uint64_t stamp = ++stamps;
    _mm_sfence();
    *(volatile uint64_t *)(slot + PUSH_PAYLOAD_BYTES) = stamp;
    _mm_sfence();
    return stamp;
}

// After the launch that reads the slot push_acquire gave out last (only then is the slot taken).  armed_ticket: that launch is a request armed
// in prelaunch mode (0: it is not).
int push_commit(hipStream_t stream, uint64_t armed_ticket)
{
    const size_t s = g_ring.push_next;
    g_ring.push_next = (s + 1) % PUSH_SLOTS;
    g_ring.push_used[s] = true;
    g_ring.push_cover[s] = -1;
    g_ring.push_armed[s] = armed_ticket;
    if (stream == nullptr || stream == g_ring.own_stream) {
        if (g_ring.batch_len == 0) {
            g_ring.batch_first = s;
            g_ring.batch_stream = stream;
        }
        ++g_ring.batch_len;
        return DL_OK;
    }
    // a caller's stream: it may be gone by the next call, so its event is recorded now
    DL_HIP(hipEventRecord(g_ring.push_ev[s], stream));
    g_ring.push_cover[s] = (int)s;
    return DL_OK;
}

// Copy `bytes` (a multiple of 16) from a slot of the pinned ring to the same slot of its device
// mirror with a 1:1 row kernel of our own, enqueued on `stream` in front of the kernel that reads it.
int stage_slot(size_t s, uint64_t bytes, hipStream_t stream)
{
    dl_plain_item stage{g_ring.base + s * RING_SLOT_BYTES, g_ring.dev + s * RING_SLOT_BYTES, bytes};
    dl_launch_shape ssh = dl_choose_shape(stage.bytes, stage.bytes, 1);
    ssh.split = 1;
    ssh.tile_bytes = 16u * ssh.block_threads;  // the row path's tile: one 1 KiB row per wavefront
    ssh.rows = true;
    uint64_t stage_tiles = dl_item_tiles(stage, ssh.tile_bytes);
    return launch_klist<dl_plain_item, NMAX_SMALL>(&stage, 1, &stage_tiles, ssh, stream, nullptr);
}

// Long list of equally sized items that moves enough bytes to pay for staging
// its table: the items themselves (not cut into tiles) go to device memory and the row kernel
// above works on them.  Returns false if the list does not qualify.  (Lists that still fit the
// kernel arguments, such as the 64 chunks of a uniform all-to-all, were 5-25 % slower this way than
// on the general path and do not come here.)
template <class Item>
bool launch_uniform_rows(const Item *items, size_t n, const dl_launch_shape &sh, hipStream_t stream, int *rc)
{
    const dl_config &c = g_dl.cfg;
    if (c.tile_bytes || sh.max_blocks) return false;
    // Read-once/write-k items with a mix of fan-outs (token rows: 1 to 8 destinations, 5.3 on average) go
    // fastest with two wavefronts per 1 KiB row, each storing to up to four destinations, in workgroups of
    // just those two: 5-20 % faster over mean fan-outs 1.9 .. 8 than four wavefronts with two stores each,
    // of which the ones without a destination are dead weight at the rate wavefronts can be started.
    const bool fused = std::is_same<Item, dl_fused_item>::value;
    const uint32_t split = c.fan_split ? sh.split : fused ? DL_TABLE_ROWS_SPLIT : 1u;
    const uint32_t threads = c.block_threads ? c.block_threads : fused && !c.fan_split ? DL_TABLE_ROWS_THREADS : 256u;
    if (threads > 512u || threads % (64u * split) || ((threads / 64u / split) & (threads / 64u / split - 1u)))
        return false;  // whole sub-groups of a power-of-two number of wavefronts
    if (n * sizeof(Item) > RING_SLOT_BYTES) return false;
    const uint64_t bytes = items[0].bytes;
    uint32_t kmax = 1;
    for (size_t i = 0; i < n; ++i) {
        if (items[i].bytes != bytes) return false;
        if (item_k(items[i]) > kmax) kmax = item_k(items[i]);
    }
    // a table that needs staging must move enough bytes to pay for it; one written through the BAR needs none.
    // But every workgroup that reads a pushed table looks for the stamp and fetches its entry past the caches, two
    // round trips that cost a large request 12 % of its kernel time, against 4 us for the staging kernel and the
    // gap behind it: from UNIFORM_ROWS_STAGE_BYTES moved, the table is staged (256 copies of 4 MiB: 368 -> 345 us).
    const bool pushable = g_ring.push && c.table_push && n * sizeof(Item) <= PUSH_PAYLOAD_BYTES &&
                          bytes * n * (1u + kmax) < UNIFORM_ROWS_STAGE_BYTES;
    if (!pushable && bytes * n < UNIFORM_ROWS_MIN_BYTES) return false;
    const uint32_t tile = 16u * threads / split;  // one 1 KiB row per wavefront of a sub-group
    uint64_t tpi = 0;  // of the item that lies worst on its grid; the others leave a workgroup without work
    bool on_grid = true;
    for (size_t i = 0; i < n; ++i) {
        const uint64_t t = dl_item_tiles(items[i], tile);
        if (t > tpi) tpi = t;
        on_grid = on_grid && item_on_grid(items[i]);
    }
    if (tpi * n >= (1ull << 30) || tpi >= (1ull << 31) || n > DL_UROWS_MAX_ITEMS) return false;

    char *pushed = pushable ? push_acquire(n * sizeof(Item), stream, rc) : nullptr;
    if (*rc != DL_OK) return true;
    size_t s = 0;
    *rc = DL_ERR_HIP;
    if (!pushed) {
        s = g_ring.next++ % RING_SLOTS;
        if (g_ring.used[s]) {
            if ((*rc = wait_for_readers(g_ring.ev[s], g_ring.armed[s])) != DL_OK) {
                --g_ring.next;
                return true;
            }
            *rc = DL_ERR_HIP;
        }
        g_ring.armed[s] = 0;
    }
    Item *slot = (Item *)(pushed ? pushed : g_ring.base + s * RING_SLOT_BYTES);
    for (size_t i = 0; i < n; ++i) {
        Item it = items[i];
        slots_by_subgroup(it, split);
        slot[i] = it;  // write only: the slot may be device memory behind the BAR
    }
    const Item *dslot = slot;
    uint64_t stamp = 0;
    if (pushed) {
        stamp = push_seal(pushed);
    } else {
        *rc = stage_slot(s, (n * sizeof(Item) + 15u) & ~(uint64_t)15u, stream);
        if (*rc != DL_OK) return true;
        dslot = (const Item *)(g_ring.dev + s * RING_SLOT_BYTES);
    }
    const dl_pushed ps = dl_push_kernel_args(stamp);
    with_policy_and_grid(sh.policy, on_grid, [&](auto pol, auto og) {
        if (pushed)
            hipLaunchKernelGGL((dl_exec_urows_kernel<Item, decltype(pol)::value, true, decltype(og)::value>),
                               dim3((uint32_t)tpi, (uint32_t)n), dim3(threads), 0, stream, dslot,
                               log2u(threads / 64u / split), log2u(split), ps);
        else
            hipLaunchKernelGGL((dl_exec_urows_kernel<Item, decltype(pol)::value, false, decltype(og)::value>),
                               dim3((uint32_t)tpi, (uint32_t)n), dim3(threads), 0, stream, dslot,
                               log2u(threads / 64u / split), log2u(split), ps);
    });
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && !pushed) e = hipEventRecord(g_ring.ev[s], stream);
    if (e != hipSuccess) {
        g_dl.last_hip = (int)e;
        *rc = DL_ERR_HIP;
        return true;
    }
    if (pushed) {
        *rc = push_commit(stream, 0);
        return true;
    }
    g_ring.used[s] = true;
    *rc = DL_OK;
    return true;
}

template <class Item>
int launch_table(const Item *items, size_t n, dl_launch_shape sh, hipStream_t stream, const dl_arm *arm)
{
    if (!g_ring.base) return DL_ERR_STATE;
    if (!arm) {
        int rc = DL_OK;
        if (launch_uniform_rows(items, n, sh, stream, &rc)) return rc;
    }
    const size_t cap = RING_SLOT_BYTES / sizeof(Item);
    auto entries = [&](uint32_t tile) {  // one per tile of the first destination's grid, like everywhere
        uint64_t m = 0;
        for (size_t i = 0; i < n; ++i) m += dl_item_tiles(items[i], tile);
        return m;
    };
    // Entries are what a long list pays for (a table in the pinned ring: every workgroup fetches its
    // entry over the host link, ~1.5 us each, a few hundred in flight): with one entry per 4 KiB,
    // 256 copies of 1 MiB ran at 2.3 TB/s and 256 copies of 16 KiB took 11.6 us.  Unless the caller
    // fixed the tile: one entry per item up to 64 KiB (7.6 us for the same 256 copies), 64 KiB tiles
    // for larger items (4.7 TB/s), and coarser still when that leaves more than a few thousand
    // entries.  The workgroup loops over its tile.  (With the table in device memory, through the BAR,
    // tiles from 4 to 64 KiB were within 1 us of each other; the same rule is kept.)
    if (g_dl.cfg.tile_bytes == 0) {
        uint64_t biggest = 0;
        for (size_t i = 0; i < n; ++i) biggest = items[i].bytes > biggest ? items[i].bytes : biggest;
        while (sh.tile_bytes < 65536u && sh.tile_bytes < biggest) sh.tile_bytes *= 2;
        sh.block_threads = 256;
        if (sh.block_threads / sh.split < 64) sh.split = 1;
    }
    while (sh.tile_bytes < (1u << 20) && entries(sh.tile_bytes) > TABLE_ENTRIES_TARGET) sh.tile_bytes *= 2;
    if (arm) {
        // an armed request is exactly one kernel: grow the tile until the cut list fits one ring slot
        while (entries(sh.tile_bytes) > cap) {
            if (sh.tile_bytes >= (1u << 30)) return DL_ERR_INVALID;
            sh.tile_bytes *= 2;
        }
    }
    const uint64_t all_entries = entries(sh.tile_bytes);
    size_t i = 0;
    uint64_t off = 0;  // progress inside items[i]
    while (i < n) {
        // a short table that is all of the request
        char *pushed = nullptr;
        uint64_t pushed_armed_ticket = 0;
        if (i == 0 && off == 0) {
            int rc = DL_OK;
            pushed = push_acquire(all_entries * sizeof(Item), stream, &rc);
            if (rc != DL_OK) return rc;
        }
        size_t s = 0;
        if (!pushed) {
            s = g_ring.next++ % RING_SLOTS;
            if (g_ring.used[s]) {
                const int rc = wait_for_readers(g_ring.ev[s], g_ring.armed[s]);
                if (rc != DL_OK) {
                    --g_ring.next;
                    return rc;
                }
            }
            g_ring.armed[s] = 0;
        }
        Item *slot = (Item *)(pushed ? pushed : g_ring.base + s * RING_SLOT_BYTES);
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
            const uint64_t room = sh.tile_bytes - dl_item_shift(it);  // up to the next tile boundary of the grid
            it.bytes = left < room ? left : room;
            slot[m++] = it;  // write only: the slot may be device memory behind the BAR
            off += it.bytes;
        }
        if (m == 0) break;
        uint64_t stamp = 0;
        if (pushed) {
            stamp = push_seal(pushed);
        } else if (m >= TABLE_STAGE_MIN) {
            // Stage the table in device memory, in front of the kernel that uses it (the copy does not
            // wait for a doorbell: the table is final now).  The workgroups then find their entries in
            // HBM instead of each fetching one over the host link.
            const int rc = stage_slot(s, (m * sizeof(Item) + 15u) & ~(uint64_t)15u, stream);
            if (rc != DL_OK) return rc;
            slot = (Item *)(g_ring.dev + s * RING_SLOT_BYTES);
        }
        const dl_pushed ps = dl_push_kernel_args(stamp);
        if (arm) {
            dl_arm a = *arm;
            if (sh.chain && !a.nowait) {
                const int rc = launch_gate(a, stream);
                if (rc != DL_OK) return rc;
            }
            const uint32_t g = armed_grid(m, sh.block_threads, !a.nowait);
            a.direct = g <= a.direct_max ? 1u : 0u;
            a.own_word = g <= DL_DONE_WORDS && !a.trace_host ? 1u : 0u;
            g_dl.armed_words = a.own_word ? g : 1u;
            if (pushed)
                hipLaunchKernelGGL((dl_armed_table_kernel<Item, true>), dim3(g), dim3(sh.block_threads), 0, stream, slot,
                                   (uint32_t)m, sh.split, ps, a);
            else
                hipLaunchKernelGGL((dl_armed_table_kernel<Item, false>), dim3(g), dim3(sh.block_threads), 0, stream, slot,
                                   (uint32_t)m, sh.split, ps, a);
            // whoever wants this memory next must not wait for a request that nobody has triggered
            // (arm->nowait: a chained request's copy kernel does not wait itself, but its gate does)
            if (!arm->nowait) {
                if (pushed)
                    pushed_armed_ticket = a.ticket;
                else
                    g_ring.armed[s] = a.ticket;
            }
        } else {
            with_policy(sh.policy, [&](auto pol) {
                if (pushed)
                    hipLaunchKernelGGL((dl_exec_table_kernel<Item, decltype(pol)::value, true>), dim3((uint32_t)m),
                                       dim3(sh.block_threads), 0, stream, slot, (uint32_t)m, sh.split, ps);
                else
                    hipLaunchKernelGGL((dl_exec_table_kernel<Item, decltype(pol)::value, false>), dim3((uint32_t)m),
                                       dim3(sh.block_threads), 0, stream, slot, (uint32_t)m, sh.split, ps);
            });
        }
        DL_HIP(hipGetLastError());
        if (pushed) {
            const int rc = push_commit(stream, pushed_armed_ticket);
            if (rc != DL_OK) return rc;
            continue;
        }
        DL_HIP(hipEventRecord(g_ring.ev[s], stream));
        g_ring.used[s] = true;
    }
    return DL_OK;
}

template <class Item>
int exec_list(const Item *items, size_t n, hipStream_t stream, const dl_arm *arm, bool *launched)
{
    *launched = false;
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
    if (arm && !arm->nowait && g_dl.cfg.armed_blocks == 0) {
        // prelaunch mode, and the caller has not fixed the waiting grid: large requests wait in a gate kernel
        uint64_t moved = 0;
        for (size_t i = 0; i < n; ++i)
            moved += items[i].bytes * (std::is_same<Item, dl_swap_item>::value ? 4ull : 1ull + item_k(items[i]));
        sh.chain = moved > g_dl.cfg.armed_chain_min_bytes;
    }
    if (arm && g_dl.cfg.tile_bytes == 0 && g_dl.cfg.block_threads == 0) {
        // armed kernels pay per workgroup for the doorbell fan-out and the arrival count:
        // four wavefronts per workgroup, each still moving 1 KiB rows
        sh.tile_bytes = 4096;
        sh.block_threads = biggest >= 4096 ? 256u : sh.block_threads;
        sh.split = 1;
        // Up to ARMED_DIRECT_MAX workgroups report each in a completion word of its own, and with the doorbell
        // in host memory only that many poll it themselves (32 or 64 pollers over the link took 7 and 9.5 us,
        // the hop through device flags 6.5, against 5.0-5.2).  A request too long for that takes eight
        // wavefronts per workgroup where that cuts the number of workgroups: more of them stay below the limit,
        // and above it arrivals and passes over a capped grid halve (1 MiB per rank: 17.1 -> 14.6 us).
        uint64_t t4 = 0, t8 = 0;
        for (size_t i = 0; i < n; ++i) {
            t4 += dl_item_tiles(items[i], 4096);
            t8 += dl_item_tiles(items[i], 8192);
        }
        if (sh.block_threads == 256u && t4 > ARMED_DIRECT_MAX && 3u * t8 <= 2u * t4) {
            sh.tile_bytes = 8192;
            sh.block_threads = 512;
        }
    }

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
        // row path: a short list (found by a few scalar compares; bisecting a long one per wavefront
        // measured slower than the general path) and a tile that is exactly one 1 KiB row per
        // wavefront of a sub-group
        sh.rows = n <= (size_t)NMAX_SMALL && sh.tile_bytes == 16u * (sh.block_threads / sh.split) &&
                  !(sh.max_blocks && !arm);
        // ... or, one-shot, a longer list whose items are about equally long: item by item on a
        // two-dimensional grid (see dl_exec_rows2d_kernel), while at most a fifth of its workgroups find nothing to do
        if (n > (size_t)NMAX_SMALL && !arm && !sh.max_blocks && sh.tile_bytes == 16u * (sh.block_threads / sh.split)) {
            uint64_t widest = 0;
            for (size_t i = 0; i < n; ++i) {
                const uint64_t t = i ? tile_end[i] - tile_end[i - 1] : tile_end[0];
                if (t > widest) widest = t;
            }
            if (widest * n <= tile_end[n - 1] + tile_end[n - 1] / 4 && widest < (1ull << 31)) {
                sh.rows = true;
                sh.rows2d_width = (uint32_t)widest;
            }
        }
        *launched = true;
        if (n <= (size_t)NMAX_SMALL) return launch_klist<Item, NMAX_SMALL>(items, n, tile_end, sh, stream, arm);
        return launch_klist<Item, NBIG>(items, n, tile_end, sh, stream, arm);
    }
    *launched = true;
    return launch_table(items, n, sh, stream, arm);
}

uint32_t floor_pow2(uint64_t v)
{
    uint32_t p = 1;
    while ((uint64_t)p * 2 <= v && p < (1u << 30)) p *= 2;
    return p;
}

}  // namespace

// Tile, workgroup size and fan split for a request.  Measured on MI355X
// (all-gather of 8 .. 64 MiB per rank, 1:1 copies of 2 GiB): the finest cut
// wins, with 256-thread workgroups in which every wavefront moves one 1 KiB row
// with one 16-byte load and at most two stores per lane.  So a fan-out of 5..8
// takes 1 KiB tiles shared out over four wavefronts, 3..4 takes 2 KiB tiles and
// two sub-groups, 1:1 and 1:2 copies take 4 KiB tiles.  Larger tiles, larger or
// smaller workgroups, capped grids and streaming hints were all slower.
dl_launch_shape dl_choose_shape(uint64_t src_bytes, uint64_t max_item_bytes, uint32_t max_k)
{
    const dl_config &c = g_dl.cfg;
    dl_launch_shape sh;
    uint32_t split = c.fan_split;
    if (split == 0) split = max_k > 4 ? 4u : max_k > 2 ? 2u : 1u;
    if (max_k == 1) split = 1;
    uint32_t tile = c.tile_bytes;
    if (tile == 0) tile = 4096u / split;
    sh.tile_bytes = tile;
    uint32_t bt = c.block_threads;
    if (bt == 0) {
        // threads of one sub-group: enough for the tile (or the largest item if that is smaller)
        const uint64_t span = max_item_bytes < tile ? max_item_bytes : tile;
        uint32_t sub = floor_pow2(span / 16 ? span / 16 : 1);
        if (sub > 256u / split) sub = 256u / split;
        if (sub < 64) sub = 64;
        bt = sub * split;
    }
    while (split > 1 && bt / split < 64) split /= 2;  // sub-groups are whole wavefronts
    sh.block_threads = bt;
    sh.split = split;
    sh.max_blocks = c.max_blocks;
    const uint64_t moved = src_bytes * (1ull + max_k);  // upper bound on bytes read + written
    // Streaming hints: where the caller asks for them; and for lists of plain copies too large for anything of
    // them to stay in the on-die caches (cold and warm alike 3-6 % faster at 512 MiB moved; copies with several
    // destinations were 10 % slower with them, smaller plain lists slower when their buffers are reused).
    const bool stream = moved >= c.nontemporal_min_bytes || (max_k == 1 && moved >= c.stream_plain_min_bytes);
    sh.policy = stream ? DL_POL_STREAM : moved <= c.write_through_max_bytes ? DL_POL_WT : DL_POL_PLAIN;
    return sh;
}

int dl_exec_plain(const dl_plain_item *items, size_t n, hipStream_t stream, const dl_arm *arm, bool *launched)
{
    return exec_list(items, n, stream, arm, launched);
}
int dl_exec_fused(const dl_fused_item *items, size_t n, hipStream_t stream, const dl_arm *arm, bool *launched)
{
    return exec_list(items, n, stream, arm, launched);
}
int dl_exec_swap(const dl_swap_item *items, size_t n, hipStream_t stream, const dl_arm *arm, bool *launched)
{
    return exec_list(items, n, stream, arm, launched);
}

template <class Item, int NMAX, class Get>
uint64_t standby_list(dl_klist<Item, NMAX> &l, size_t n, uint32_t max_tiles, Get get)
{
    uint64_t acc = 0;
    for (size_t i = 0; i < (size_t)NMAX; ++i) {
        if (i < n) {
            const Item it = get(i);
            acc += dl_item_tiles(it, DL_STANDBY_TILE);
            if (acc > max_tiles) return 0;  // one tile per workgroup, one pass
            l.item[i] = it;
        }
        l.tile_end[i] = i < n ? (uint32_t)acc : 0xFFFFFFFFu;
    }
    l.n = (uint32_t)n;
    l.tile_bytes = DL_STANDBY_TILE;
    l.split = 1;
    l.split_log2 = 0;
    l.wpg_log2 = log2u(DL_STANDBY_THREADS / 64u);
    return acc;
}

uint32_t dl_standby_fill(void *rec_mem, const dl_plan_item *items, size_t n, uint64_t activation, uint64_t ticket,
                         uint64_t *done, uint32_t *arrive_clear, uint32_t max_tiles)
{
    const dl_config &c = g_dl.cfg;
    if (n == 0 || n > 64 || c.tile_bytes || c.block_threads || c.max_blocks || c.armed_blocks) return 0;
    static_assert(sizeof(dl_plan_item) == sizeof(dl_fused_item), "plan items are fused items");
    const dl_fused_item *it = reinterpret_cast<const dl_fused_item *>(items);
    static dl_standby_rec r;  // 2 KiB: not on the stack of every call
    uint64_t acc, used;
    if (n <= 8) {
        r.plain = 0;
        acc = standby_list(r.list, n, max_tiles, [&](size_t i) { return it[i]; });
        used = offsetof(dl_standby_rec, list) + sizeof r.list;
    } else {
        for (size_t i = 0; i < n; ++i)
            if (it[i].k != 1) return 0;
        r.plain = 1;
        acc = standby_list(r.copies, n, max_tiles,
                           [&](size_t i) { return dl_plain_item{it[i].src, it[i].dst[0], it[i].bytes}; });
        used = offsetof(dl_standby_rec, copies) + sizeof r.copies;
    }
    if (acc == 0) return 0;
    r.ticket_front = r.ticket_back = ticket;
    r.activation = activation;
    r.done = done;
    r.arrive_clear = arrive_clear;
    r.arrivals = 0;
    // The record may live in device memory mapped write-combined: plain 8-byte stores in ascending order, of the
    // part that this kind of list uses and of the closing ticket.
    static uint64_t words[sizeof r / 8];
    memcpy(words, &r, sizeof r);
    volatile uint64_t *out = (volatile uint64_t *)rec_mem;
    for (size_t q = 0; q < (used + 7) / 8; ++q) out[q] = words[q];
    out[sizeof r / 8 - 1] = words[sizeof r / 8 - 1];
    return acc <= DL_DONE_WORDS ? (uint32_t)acc : 1u;
}

int dl_standby_launch(void *rec_mem, const dl_arm *a, hipStream_t stream)
{
    hipLaunchKernelGGL(dl_standby_kernel, dim3(DL_STANDBY_GRID), dim3(DL_STANDBY_THREADS), 0, stream,
                       (dl_standby_rec *)rec_mem, *a);
    DL_HIP(hipGetLastError());
    return DL_OK;
}

int dl_launch_fused_rows_table(const dl_fused_item *dev_items, uint32_t n, uint64_t item_bytes, uint32_t max_shift,
                               bool on_grid, hipStream_t stream)
{
    // the table's destinations are laid out for DL_TABLE_ROWS_SPLIT sub-groups (see slots_by_subgroup)
    const uint32_t split = DL_TABLE_ROWS_SPLIT, threads = DL_TABLE_ROWS_THREADS, tile = 16u * threads / split;
    const uint64_t tpi = (item_bytes + max_shift + tile - 1) / tile;
    if (n == 0 || n > DL_UROWS_MAX_ITEMS || max_shift >= DL_CUT || tpi * n >= (1ull << 30)) return DL_ERR_INVALID;
    const dl_launch_shape sh = dl_choose_shape((uint64_t)n * item_bytes, item_bytes, 8);
    with_policy_and_grid(sh.policy, on_grid && max_shift == 0, [&](auto pol, auto og) {
        hipLaunchKernelGGL((dl_exec_urows_kernel<dl_fused_item, decltype(pol)::value, false, decltype(og)::value>),
                           dim3((uint32_t)tpi, n), dim3(threads), 0, stream, dev_items, log2u(threads / 64u / split),
                           log2u(split), dl_push_kernel_args(0));
    });
    DL_HIP(hipGetLastError());
    return DL_OK;
}

int dl_launch_plain_table(const dl_plain_item *dev_items, uint32_t m, uint32_t entry_bytes, uint64_t moved, hipStream_t stream)
{
    if (m == 0) return DL_OK;
    const dl_launch_shape sh = dl_choose_shape(moved / 2, entry_bytes, 1);  // for the cache policy
    with_policy(sh.policy, [&](auto pol) {
        hipLaunchKernelGGL((dl_exec_table_kernel<dl_plain_item, decltype(pol)::value, false>), dim3(m), dim3(256), 0,
                           stream, dev_items, m, 1u, dl_push_kernel_args(0));
    });
    DL_HIP(hipGetLastError());
    return DL_OK;
}

int dl_ring_acquire(size_t *slot, char **host, char **dev)
{
    if (!g_ring.base) return DL_ERR_STATE;
    const size_t s = g_ring.next++ % RING_SLOTS;
    if (g_ring.used[s]) {
        const int rc = wait_for_readers(g_ring.ev[s], g_ring.armed[s]);
        if (rc != DL_OK) {
            --g_ring.next;
            return rc;
        }
    }
    g_ring.armed[s] = 0;
    *slot = s;
    *host = g_ring.base + s * RING_SLOT_BYTES;
    *dev = g_ring.dev + s * RING_SLOT_BYTES;
    return DL_OK;
}

int dl_ring_stage(size_t slot, uint64_t bytes, hipStream_t stream) { return stage_slot(slot, bytes, stream); }

void dl_ring_forget_armed()
{
    for (size_t s = 0; s < RING_SLOTS; ++s) g_ring.armed[s] = 0;
    for (size_t s = 0; s < PUSH_SLOTS; ++s) g_ring.push_armed[s] = 0;
}

void dl_ring_own_stream(hipStream_t stream)
{
    if (!stream && g_ring.batch_len && g_ring.batch_stream == g_ring.own_stream) (void)push_close_batch();
    g_ring.own_stream = stream;
}

// The device error word: host-coherent memory that a kernel writes when it gives up on a table that never
// became complete (see dl_pushed).  Read, and cleared, by dl_last_device_error().
static uint64_t *g_lost = nullptr;
// Test hook (dl_debug_lose_next_table): the kernel of the next table that goes through the BAR is told a stamp
// that its slot will never hold and this many looks, so that the give-up path runs, every wait still bounded.
static uint32_t g_debug_lose_tries = 0;

dl_pushed dl_push_kernel_args(uint64_t stamp)
{
    dl_pushed ps{stamp, DL_PUSHED_TRIES, 0u, g_lost};
    if (stamp && g_debug_lose_tries) {
        ps.stamp = stamp | (1ull << 62);
        ps.tries = g_debug_lose_tries;
        g_debug_lose_tries = 0;
    }
    return ps;
}

bool dl_device_error_pending() { return g_lost && __atomic_load_n(g_lost, __ATOMIC_ACQUIRE) != 0; }

extern "C" int dl_last_device_error(void)
{
    if (!g_lost) return DL_OK;
    return __atomic_exchange_n(g_lost, 0ull, __ATOMIC_ACQ_REL) ? DL_ERR_LOST : DL_OK;
}

extern "C" int dl_debug_lose_next_table(uint32_t tries)
{
    if (!g_dl.inited) return DL_ERR_STATE;
    if (!g_ring.push || !g_dl.cfg.table_push) return DL_ERR_STATE;  // no table goes through the BAR here
    if (tries > 1024) return DL_ERR_INVALID;  // 0 disarms the hook
    g_debug_lose_tries = tries;
    return DL_OK;
}

char *dl_push_acquire(size_t bytes, hipStream_t stream, int *rc) { return push_acquire(bytes, stream, rc); }
uint64_t dl_push_seal(char *slot) { return push_seal(slot); }
int dl_push_commit(hipStream_t stream) { return push_commit(stream, 0); }

int dl_ring_release(size_t slot, hipStream_t stream)
{
    DL_HIP(hipEventRecord(g_ring.ev[slot], stream));
    g_ring.used[slot] = true;
    return DL_OK;
}

// Device memory that the host can store into: only where one PCIe BAR covers all of the device's memory.  Made
// once per process and kept until it ends.
void *dl_bar_memory(size_t bytes)
{
    const char *off = getenv("DL_NO_BAR");  // "1": keep everything the host writes in host memory
    if (off && off[0] == '1') return nullptr;
    int large_bar = 0;
    if (hipDeviceGetAttribute(&large_bar, hipDeviceAttributeIsLargeBar, g_dl.device) != hipSuccess || large_bar != 1) {
        (void)hipGetLastError();
        return nullptr;
    }
    void *p = nullptr;
    if (hipExtMallocWithFlags(&p, bytes, hipDeviceMallocFinegrained) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    if (hipMemset(p, 0, bytes) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;  // left allocated and unused
    }
    return p;
}

int dl_exec_init()
{
    // kept for the life of the process, per device: what was made for another device is left behind
    static int push_device = -1;
    static char *push_memory = nullptr;
    if (push_device != g_dl.device) {
        push_device = g_dl.device;
        push_memory = (char *)dl_bar_memory(PUSH_SLOTS * PUSH_SLOT_BYTES);
    }
    if (g_ring.base) return DL_OK;
    g_ring.push = push_memory;
    g_ring.push_next = 0;
    g_ring.batch_len = 0;
    g_ring.own_stream = nullptr;
    for (size_t q = 0; q < PUSH_SLOTS; ++q) {
        DL_HIP(hipEventCreateWithFlags(&g_ring.push_ev[q], hipEventDisableTiming));
        g_ring.push_used[q] = false;
        g_ring.push_cover[q] = -1;
        g_ring.push_armed[q] = 0;
    }
    DL_HIP(hipHostMalloc((void **)&g_lost, 64, hipHostMallocCoherent | hipHostMallocMapped));
    *g_lost = 0;
    g_debug_lose_tries = 0;
    DL_HIP(hipHostMalloc((void **)&g_ring.base, RING_SLOTS * RING_SLOT_BYTES, hipHostMallocDefault));
    DL_HIP(hipMalloc((void **)&g_ring.dev, RING_SLOTS * RING_SLOT_BYTES));
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
    // everything launched has ended before the tables' memory is handed out again after the next dl_exec_init
    // (the open batch has no event yet; its stream is the default one or the library's, which is gone by now)
    (void)hipDeviceSynchronize();
    for (size_t q = 0; q < PUSH_SLOTS; ++q) (void)hipEventDestroy(g_ring.push_ev[q]);
    (void)hipHostFree(g_ring.base);
    (void)hipFree(g_ring.dev);
    (void)hipHostFree(g_lost);
    g_lost = nullptr;
    g_ring.base = nullptr;
    g_ring.dev = nullptr;
    return DL_OK;
}
