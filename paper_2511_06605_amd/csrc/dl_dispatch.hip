// Token dispatch lowered on the device (Sec. IV-B: a token that goes to several experts is one
// source with several destinations).  The host-side lowering writes one 88-byte item per token and
// ships that table over the host link; for thousands of tokens that "control" work (Sec. III-B2) is
// as long as the copy.  Here only the destination mask (W bytes per token) crosses the link:
//   1. the mask goes to device memory (written there by the host through the BAR where that is possible, else
//      through the pinned ring and a copy),
//   2. a small kernel builds the item table there, one token per thread: its source row and, for
//      every rank it goes to, the row it lands on (receive buffers are packed in token order, so
//      that is an exclusive prefix count per column of the mask; the host, which touches every mask
//      word anyway, sends along the counts at every 256th token, the kernel counts inside its 256),
//   3. the row kernel for long lists of equal items executes the table.
#include "dl_device.h"
#include "dl_internal.h"

#include <string.h>

namespace {

constexpr int DISPATCH_W = 8;            // ranks this path handles: exactly 8 (one 64-bit mask word per token)
constexpr uint32_t BUILD_THREADS = 256;  // tokens per workgroup of the build kernel
constexpr uint32_t BUILD_WAVES = BUILD_THREADS / 64;

struct build_args {
    const char *in[DISPATCH_W];
    char *out[DISPATCH_W];
    uint32_t first_token[DISPATCH_W + 1];  // tokens before rank i; entries past W hold the total
    uint32_t W;
    uint32_t tokens;  // over all ranks
    uint64_t row_bytes;
};

// Workgroup b builds the items of tokens 256 b .. 256 b + 255, one token per thread.  No workgroup
// waits for another: the rows that earlier blocks' tokens took in each receive buffer come with the
// mask (block_rows: W counts per block, written by the host), the rows taken inside the block come
// from wavefront ballots.
//
// PUSHED: the host wrote the mask into device memory just before the launch; it is read past the caches, where
// a line of whatever used that memory before may linger.
// Per block of 256 tokens and per rank: how many of the block's tokens go to that rank (any non-zero mask byte
// counts).  For a mask that is already in device memory: what the host otherwise counts while it folds the mask.
__global__ void __launch_bounds__(BUILD_THREADS) dl_dispatch_count_kernel(const uint8_t *__restrict__ mask, uint32_t tokens,
                                                                          uint32_t *__restrict__ counts)
{
    __shared__ uint32_t in_wave[BUILD_WAVES][DISPATCH_W];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t token = blockIdx.x * BUILD_THREADS + tid;
    const uint64_t mine = token < tokens ? dl_global<uint64_t>(mask)[token] : 0ull;
#pragma unroll
    for (int j = 0; j < DISPATCH_W; ++j) {
        const uint64_t votes = __ballot(((mine >> (8 * j)) & 0xFFu) != 0);
        if (lane == 0) in_wave[wave][j] = (uint32_t)__popcll(votes);
    }
    __syncthreads();
    if (tid < DISPATCH_W) {
        uint32_t c = 0;
#pragma unroll
        for (uint32_t w = 0; w < BUILD_WAVES; ++w) c += in_wave[w][tid];
        counts[blockIdx.x * DISPATCH_W + tid] = c;
    }
}

// COUNTS: block_rows holds every block's own counts (dl_dispatch_count_kernel), and the rows taken by earlier
// blocks are summed up here; else it holds those sums already (the host's).
template <bool PUSHED, bool COUNTS = false>
__global__ void __launch_bounds__(BUILD_THREADS) dl_dispatch_build_kernel(const uint8_t *__restrict__ mask,
                                                                          const uint32_t *__restrict__ block_rows,
                                                                          const build_args a,
                                                                          dl_fused_item *__restrict__ items,
                                                                          const dl_pushed ps)
{
    constexpr int POL = PUSHED ? DL_POL_COHERENT : DL_POL_PLAIN;
    __shared__ uint32_t before_block[DISPATCH_W];          // rows taken by the tokens of earlier blocks
    __shared__ uint32_t in_wave[BUILD_WAVES][DISPATCH_W];  // per wavefront: destinations of its own 64 tokens
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    constexpr uint32_t W = DISPATCH_W;
    const uint32_t block0 = blockIdx.x * BUILD_THREADS;
    const uint32_t token = block0 + tid;
    const bool valid = token < a.tokens;
    uint64_t mine = 0;
    if constexpr (PUSHED) {
        // one lane sees the slot's stamp first: only what is read after that is known to be this request's
        __shared__ uint32_t sealed;
        if (tid == 0) sealed = dl_pushed_sealed(mask, ps) ? 1u : 0u;
        __syncthreads();
        if (!sealed) {
            // The mask never became complete (the writes were on their way before the launch, so: never).  The row
            // kernel behind this one executes whatever the table holds: give it an entry that moves nothing for
            // every token of this block, and let the host hear of the loss.
            if (valid) {
                dl_fused_item none;
                none.src = nullptr;
                none.bytes = 0;
                none.k = 0;
                none.pad = 0;
#pragma unroll
                for (int q = 0; q < DL_FAN; ++q) none.dst[q] = nullptr;
                items[token] = none;
            }
            if (tid == 0) dl_pushed_report_lost(ps);
            return;
        }
        if (tid < DISPATCH_W)
            before_block[tid] = dl_ld<POL>(dl_global<uint32_t>(block_rows) + blockIdx.x * DISPATCH_W + tid);
        mine = valid ? dl_ld<POL>(dl_global<uint64_t>(mask) + token) : 0ull;
    } else if constexpr (COUNTS) {
        if (tid < DISPATCH_W) {
            uint32_t before = 0;
            for (uint32_t b = 0; b < blockIdx.x; ++b) before += block_rows[b * DISPATCH_W + tid];
            before_block[tid] = before;
        }
        mine = valid ? dl_ld<POL>(dl_global<uint64_t>(mask) + token) : 0ull;
    } else {
        if (tid < DISPATCH_W) before_block[tid] = dl_ld<POL>(dl_global<uint32_t>(block_rows) + blockIdx.x * DISPATCH_W + tid);
        mine = valid ? dl_ld<POL>(dl_global<uint64_t>(mask) + token) : 0ull;
    }
    bool m[DISPATCH_W];
    uint32_t pos[DISPATCH_W], k = 0;
#pragma unroll
    for (int j = 0; j < DISPATCH_W; ++j) {
        m[j] = ((mine >> (8 * j)) & 0xFFu) != 0;
        const uint64_t votes = __ballot(m[j]);
        pos[j] = (uint32_t)__popcll(votes & ((1ull << lane) - 1ull));  // earlier tokens of this wavefront
        if (lane == 0) in_wave[wave][j] = (uint32_t)__popcll(votes);
        k += m[j] ? 1u : 0u;
    }
    __syncthreads();
    if (!valid) return;
#pragma unroll
    for (int j = 0; j < DISPATCH_W; ++j) {
        pos[j] += before_block[j];
#pragma unroll
        for (uint32_t w = 0; w < BUILD_WAVES; ++w) pos[j] += w < wave ? in_wave[w][j] : 0u;
    }

    // the token's rank is the last one that starts at or before it; its send buffer and first token are
    // picked by compares against kernel arguments (no load depends on the token)
    const char *base = a.in[0];
    uint32_t first = 0;
#pragma unroll
    for (int r = 1; r < DISPATCH_W; ++r)
        if ((uint32_t)r < W && a.first_token[r] <= token) {
            base = a.in[r];
            first = a.first_token[r];
        }
    dl_fused_item it;
    it.src = base + (uint64_t)(token - first) * a.row_bytes;
    it.bytes = a.row_bytes;
    it.k = k;
    it.pad = 0;
#pragma unroll
    for (int s = 0; s < DL_FAN; ++s) it.dst[s] = nullptr;
    // destination number d (in rank order) goes to sub-group d / per (0 or 1), slot 4 (d / per) + d % per,
    // per = ceil(k / 2): the layout of slots_by_subgroup for DL_TABLE_ROWS_SPLIT sub-groups
    static_assert(DL_TABLE_ROWS_SPLIT == 2 && DL_FAN == 8, "slot layout below is written for two sub-groups of four");
    const uint32_t per = (k + 1u) >> 1;
    uint32_t d = 0;
#pragma unroll
    for (int j = 0; j < DISPATCH_W; ++j) {
        if (m[j]) {
            char *p = a.out[j] + (uint64_t)pos[j] * a.row_bytes;
            const uint32_t slot = d >= per ? 4u + d - per : d;
#pragma unroll
            for (int s = 0; s < DL_FAN; ++s)
                if ((uint32_t)s == slot) it.dst[s] = p;
            ++d;
        }
    }
    items[token] = it;
}

// How far behind a DL_CUT boundary the first destination of a row can lie: rows stand whole multiples of
// row_bytes into the receive buffers, so every such address is a multiple of the largest power of two that
// divides row_bytes and all of the buffers' addresses.
uint32_t worst_shift(void *const *out, int W, size_t row_bytes)
{
    uint64_t m = row_bytes;
    for (int i = 0; i < W; ++i) m |= (uint64_t)out[i];
    m &= DL_CUT - 1u;
    return m ? DL_CUT - (uint32_t)(m & (0 - m)) : 0u;
}

// Every row lies as the on-grid instance of the row kernel wants it (see dl_rows_body).
bool rows_on_grid(const void *const *in, void *const *out, int W, size_t row_bytes)
{
    uint64_t m = row_bytes & 3u;
    for (int i = 0; i < W; ++i) m |= (uint64_t)in[i] & 3u;
    return m == 0 && (row_bytes & 15u) == 0 && worst_shift(out, W, row_bytes) == 0;
}

}  // namespace

int dl_dispatch_on_device(const void *const *in, void *const *out, int W, const uint32_t *tokens, size_t row_bytes,
                          const uint8_t *dest, hipStream_t stream, bool *taken)
{
    *taken = false;
    const dl_config &c = g_dl.cfg;
    if (W != DISPATCH_W || !in || !out || !tokens || !dest) return DL_OK;
    if (c.tile_bytes || c.block_threads || c.max_blocks || (c.fan_split != 0 && c.fan_split != DL_TABLE_ROWS_SPLIT)) return DL_OK;
    if (row_bytes == 0) return DL_OK;
    uint64_t total = 0;
    for (int i = 0; i < W; ++i) {
        total += tokens[i];
        if ((tokens[i] && !in[i]) || !out[i]) return DL_OK;  // the host lowering reports what is wrong
    }
    // worth two small launches only for many tokens; mask, block counts and item table share one ring slot
    const uint64_t blocks = (total + BUILD_THREADS - 1) / BUILD_THREADS;
    const uint64_t mask_bytes = (total * (uint64_t)W + 255u) & ~(uint64_t)255u;               // then the block counts:
    const uint64_t head_bytes = (mask_bytes + blocks * DISPATCH_W * sizeof(uint32_t) + 255u) & ~(uint64_t)255u;
    if (total < 512 || head_bytes + total * sizeof(dl_fused_item) > DL_RING_SLOT_BYTES)
        return DL_OK;

    size_t slot;
    char *host, *dev;
    int rc = dl_ring_acquire(&slot, &host, &dev);  // the item table's place (and the mask's, if it is staged)
    if (rc != DL_OK) return rc;
    char *pushed = dl_push_acquire(head_bytes, stream, &rc);
    if (rc != DL_OK) return rc;
    *taken = true;
    // One 64-bit word per token, every byte 0 or 1.  Adding words adds the eight columns bytewise: the running
    // sums are unpacked every 128 tokens (a byte holds 255), and before every 256th token they go out as that
    // block's counts of rows already taken.
    static_assert(DISPATCH_W == 8 && BUILD_THREADS == 256, "a token's mask is one 64-bit word; blocks of 256 tokens");
    uint64_t *words = (uint64_t *)(pushed ? pushed : host);
    uint32_t *block_rows = (uint32_t *)((char *)words + mask_bytes);
    uint32_t taken_rows[DISPATCH_W] = {0};
    for (size_t t0 = 0; t0 < total; t0 += 128) {
        if ((t0 & 255u) == 0)
            for (int j = 0; j < DISPATCH_W; ++j) block_rows[(t0 >> 8) * DISPATCH_W + j] = taken_rows[j];
        const size_t t1 = t0 + 128 < total ? t0 + 128 : total;
        uint64_t acc = 0;
        for (size_t t = t0; t < t1; ++t) {  // a plain loop over words: the compiler vectorises it
            uint64_t w;
            memcpy(&w, dest + t * (size_t)DISPATCH_W, sizeof w);
            // a non-zero byte becomes 1: fold its bits into bit 0, keep bit 0 of every byte
            w |= w >> 4;
            w |= w >> 2;
            w |= w >> 1;
            w &= 0x0101010101010101ull;
            words[t] = w;  // write only: the slot may be device memory behind the BAR
            acc += w;
        }
        for (int j = 0; j < DISPATCH_W; ++j) taken_rows[j] += (uint32_t)(acc >> (8 * j)) & 0xFFu;
    }
    uint64_t stamp = 0;
    if (pushed) {
        stamp = dl_push_seal(pushed);
    } else {
        rc = dl_ring_stage(slot, head_bytes, stream);
        if (rc != DL_OK) return rc;
    }
    const char *head = pushed ? pushed : dev;

    build_args a;
    uint32_t first = 0;
    for (int i = 0; i < DISPATCH_W; ++i) {
        a.in[i] = i < W ? (const char *)in[i] : nullptr;
        a.out[i] = i < W ? (char *)out[i] : nullptr;
        a.first_token[i] = first;
        if (i < W) first += tokens[i];
    }
    a.first_token[DISPATCH_W] = first;
    a.W = (uint32_t)W;
    a.tokens = (uint32_t)total;
    a.row_bytes = row_bytes;
    dl_fused_item *items = (dl_fused_item *)(dev + head_bytes);
    const dim3 grid((uint32_t)blocks);
    const uint8_t *mask = (const uint8_t *)head;
    const uint32_t *rows_before = (const uint32_t *)(head + mask_bytes);
    const dl_pushed ps = dl_push_kernel_args(stamp);
    if (pushed)
        hipLaunchKernelGGL(dl_dispatch_build_kernel<true>, grid, dim3(BUILD_THREADS), 0, stream, mask, rows_before, a, items, ps);
    else
        hipLaunchKernelGGL(dl_dispatch_build_kernel<false>, grid, dim3(BUILD_THREADS), 0, stream, mask, rows_before, a, items, ps);
    DL_HIP(hipGetLastError());
    if (pushed) {
        rc = dl_push_commit(stream);
        if (rc != DL_OK) return rc;
    }
    rc = dl_launch_fused_rows_table(items, (uint32_t)total, row_bytes, worst_shift(out, W, row_bytes),
                                    rows_on_grid(in, out, W, row_bytes), stream);
    if (rc != DL_OK) return rc;
    return dl_ring_release(slot, stream);
}

// Token dispatch with the routing mask in device memory (dl_token_dispatch_device): nothing of the request but
// the kernel arguments comes from the host.  Three launches on the caller's stream: count per block, build the
// item table (in a slot of the library's table memory), execute it.
extern "C" int dl_token_dispatch_device(const void *const *in, void *const *out, int W, const uint32_t *tokens,
                                        size_t row_bytes, const uint8_t *dest_device, void *stream)
{
    DL_LOCKED;
    if (!g_dl.inited) return DL_ERR_STATE;
    if (dl_device_error_pending()) return DL_ERR_LOST;
    if (W != DISPATCH_W || !in || !out || !tokens) return DL_ERR_INVALID;
    uint64_t total = 0;
    for (int i = 0; i < W; ++i) total += tokens[i];
    if (total == 0 || row_bytes == 0) return DL_OK;
    if (!dest_device || ((uint64_t)dest_device & 7u)) return DL_ERR_INVALID;
    for (int i = 0; i < W; ++i) {
        if ((tokens[i] && !in[i]) || !out[i]) return DL_ERR_INVALID;
    }
    if (total > DL_DISPATCH_DEVICE_MAX_TOKENS) return DL_ERR_CAPACITY;
    const uint64_t blocks = (total + BUILD_THREADS - 1) / BUILD_THREADS;
    const uint64_t head_bytes = (blocks * DISPATCH_W * sizeof(uint32_t) + 255u) & ~(uint64_t)255u;
    static_assert((((DL_DISPATCH_DEVICE_MAX_TOKENS + BUILD_THREADS - 1) / BUILD_THREADS * DISPATCH_W * sizeof(uint32_t) + 255u) & ~(size_t)255u) +
                          DL_DISPATCH_DEVICE_MAX_TOKENS * sizeof(dl_fused_item) <= DL_RING_SLOT_BYTES,
                  "counts and table of the largest request fit one slot of the table memory");
    hipStream_t hs = (hipStream_t)stream;

    size_t slot;
    char *host, *dev;
    int rc = dl_ring_acquire(&slot, &host, &dev);
    if (rc != DL_OK) return rc;
    uint32_t *counts = (uint32_t *)dev;
    dl_fused_item *items = (dl_fused_item *)(dev + head_bytes);
    hipLaunchKernelGGL(dl_dispatch_count_kernel, dim3((uint32_t)blocks), dim3(BUILD_THREADS), 0, hs, dest_device,
                       (uint32_t)total, counts);
    DL_HIP(hipGetLastError());
    build_args a;
    uint32_t first = 0;
    for (int i = 0; i < DISPATCH_W; ++i) {
        a.in[i] = (const char *)in[i];
        a.out[i] = (char *)out[i];
        a.first_token[i] = first;
        first += tokens[i];
    }
    a.first_token[DISPATCH_W] = first;
    a.W = (uint32_t)W;
    a.tokens = (uint32_t)total;
    a.row_bytes = row_bytes;
    hipLaunchKernelGGL((dl_dispatch_build_kernel<false, true>), dim3((uint32_t)blocks), dim3(BUILD_THREADS), 0, hs,
                       dest_device, (const uint32_t *)counts, a, items, dl_push_kernel_args(0));
    DL_HIP(hipGetLastError());
    rc = dl_launch_fused_rows_table(items, (uint32_t)total, row_bytes, worst_shift(out, W, row_bytes),
                                    rows_on_grid(in, out, W, row_bytes), hs);
    if (rc != DL_OK) return rc;
    t_dl_last.mode = DL_MODE_ONESHOT;
    return dl_ring_release(slot, hs);
}
