// Internal: the device-side copy loop (the "copy" phase of Sec. III-B2 executed
// by compute units) used by both the one-shot and the armed kernels.
//
// One tile = a contiguous run of the item's body, read once with 16-byte
// vector loads (lane l of a wavefront reads bytes 16*l .. 16*l+15 of each
// 1 KiB row, so every wavefront access is one fully coalesced row) and written
// from registers to each of the k destinations (the fused broadcast of
// Sec. IV-B, with k up to 8 instead of 2).  Several loads are issued before the
// first store so each lane keeps UNROLL requests in flight.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dl_work.h"

typedef uint32_t dl_u32x4 __attribute__((ext_vector_type(4)));

// Every buffer the library touches is device (or host-pinned) global memory;
// saying so lets the compiler emit global_* instead of flat_* accesses.
#define DL_GLOBAL __attribute__((address_space(1)))
template <typename V>
__device__ __forceinline__ DL_GLOBAL V *dl_global(const void *p)
{
    return (DL_GLOBAL V *)(uint64_t)p;
}

constexpr int DL_UNROLL = 4;

template <bool NT, typename V>
__device__ __forceinline__ V dl_ld(const DL_GLOBAL V *p)
{
    if constexpr (NT)
        return __builtin_nontemporal_load(p);
    else
        return *p;
}

template <bool NT, typename V>
__device__ __forceinline__ void dl_st(DL_GLOBAL V *p, V v)
{
    if constexpr (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// n 16-byte vectors from s to the first K of the destinations, by nthr threads.
template <int K, int FAN, bool NT>
__device__ __forceinline__ void dl_copy_vec16(const DL_GLOBAL dl_u32x4 *__restrict__ s, char *const (&dsts)[FAN],
                                              uint64_t byte_off, uint32_t n, uint32_t tid, uint32_t nthr)
{
    static_assert(K <= FAN, "fan-out");
    DL_GLOBAL dl_u32x4 *d[K];
#pragma unroll
    for (int j = 0; j < K; ++j) d[j] = dl_global<dl_u32x4>(dsts[j] + byte_off);

    uint32_t i = tid;
    const uint32_t step = nthr * DL_UNROLL;
    for (; i + (DL_UNROLL - 1) * nthr < n; i += step) {
        dl_u32x4 v[DL_UNROLL];
#pragma unroll
        for (int u = 0; u < DL_UNROLL; ++u) v[u] = dl_ld<NT>(s + i + u * nthr);
#pragma unroll
        for (int u = 0; u < DL_UNROLL; ++u)
#pragma unroll
            for (int j = 0; j < K; ++j) dl_st<NT>(d[j] + i + u * nthr, v[u]);
    }
    for (; i < n; i += nthr) {
        dl_u32x4 v = dl_ld<NT>(s + i);
#pragma unroll
        for (int j = 0; j < K; ++j) dl_st<NT>(d[j] + i, v);
    }
}

// Narrow elements (addresses that do not agree modulo 16): correctness path.
template <typename V, int FAN>
__device__ __forceinline__ void dl_copy_narrow(const char *src, char *const (&dsts)[FAN], uint32_t k,
                                               uint64_t byte_off, uint32_t n, uint32_t tid, uint32_t nthr)
{
    const DL_GLOBAL V *s = dl_global<V>(src + byte_off);
    for (uint32_t i = tid; i < n; i += nthr) {
        V v = s[i];
#pragma unroll
        for (int j = 0; j < FAN; ++j)
            if ((uint32_t)j < k) dl_global<V>(dsts[j] + byte_off)[i] = v;
    }
}

// Move tile `tile` of the copy (src -> dsts[0..k)), all threads of the
// workgroup taking part.  src, dsts, k, bytes, tile must be uniform across the
// workgroup; 1 <= k <= FAN; nthr >= 64.
template <int FAN, bool NT>
__device__ __forceinline__ void dl_move_tile(const char *src, char *const (&dsts)[FAN], uint32_t k, uint64_t bytes,
                                             uint64_t tile, uint32_t tile_bytes, uint32_t tid, uint32_t nthr)
{
    uint64_t diff = 0;
#pragma unroll
    for (int j = 0; j < FAN; ++j)
        if ((uint32_t)j < k) diff |= (uint64_t)src ^ (uint64_t)dsts[j];
    const dl_geom g = dl_make_geom((uint64_t)src, diff, bytes);

    if (tile == 0) {
        // head bytes by threads 0..15, tail bytes by threads 32..47
        if (tid < g.head) {
            uint8_t v = dl_global<uint8_t>(src)[tid];
#pragma unroll
            for (int j = 0; j < FAN; ++j)
                if ((uint32_t)j < k) dl_global<uint8_t>(dsts[j])[tid] = v;
        }
        if (tid >= 32 && tid - 32 < g.tail) {
            uint64_t off = (uint64_t)g.head + g.body * g.esize + (tid - 32);
            uint8_t v = dl_global<uint8_t>(src)[off];
#pragma unroll
            for (int j = 0; j < FAN; ++j)
                if ((uint32_t)j < k) dl_global<uint8_t>(dsts[j])[off] = v;
        }
    }

    const uint64_t per_tile = tile_bytes / g.esize;
    const uint64_t first = tile * per_tile;
    if (first >= g.body) return;
    const uint64_t left = g.body - first;
    const uint32_t n = (uint32_t)(left < per_tile ? left : per_tile);
    const uint64_t off = (uint64_t)g.head + first * g.esize;

    if (g.esize == 16) {
        const DL_GLOBAL dl_u32x4 *s = dl_global<dl_u32x4>(src + off);
        if constexpr (FAN == 1) {
            dl_copy_vec16<1, FAN, NT>(s, dsts, off, n, tid, nthr);
        } else {
            static_assert(FAN == 8, "fan-out switch below is written for 8");
            switch (k) {
            case 1: dl_copy_vec16<1, FAN, NT>(s, dsts, off, n, tid, nthr); break;
            case 2: dl_copy_vec16<2, FAN, NT>(s, dsts, off, n, tid, nthr); break;
            case 3: dl_copy_vec16<3, FAN, NT>(s, dsts, off, n, tid, nthr); break;
            case 4: dl_copy_vec16<4, FAN, NT>(s, dsts, off, n, tid, nthr); break;
            case 5: dl_copy_vec16<5, FAN, NT>(s, dsts, off, n, tid, nthr); break;
            case 6: dl_copy_vec16<6, FAN, NT>(s, dsts, off, n, tid, nthr); break;
            case 7: dl_copy_vec16<7, FAN, NT>(s, dsts, off, n, tid, nthr); break;
            default: dl_copy_vec16<8, FAN, NT>(s, dsts, off, n, tid, nthr); break;
            }
        }
    } else if (g.esize == 4) {
        dl_copy_narrow<uint32_t, FAN>(src, dsts, k, off, n, tid, nthr);
    } else {
        dl_copy_narrow<uint8_t, FAN>(src, dsts, k, off, n, tid, nthr);
    }
}

// ------------------------------------------------ items and lists on the device

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

// Global tile b of a list: find its item with one wavefront ballot over the
// prefix sums (item index = number of items whose last tile lies before b),
// then move that tile.  b must be uniform across the workgroup.
template <bool NT, class Item, int NMAX>
__device__ __forceinline__ void dl_run_tile(const dl_klist<Item, NMAX> &p, uint32_t b)
{
    const uint32_t lane = threadIdx.x & 63u;
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
