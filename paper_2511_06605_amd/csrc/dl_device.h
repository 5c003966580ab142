// Internal: the device-side copy loop (the "copy" phase of Sec. III-B2 executed
// by compute units) used by both the one-shot and the armed kernels.
//
// One tile = a contiguous run of an item's bytes on the grid of its first
// destination (see dl_work.h), read once with 16-byte vector loads (lane l of a
// wavefront reads bytes 16*l .. 16*l+15 of each 1 KiB row, so every wavefront
// access is one fully coalesced row) and written from registers to each of the
// k destinations (the fused broadcast of Sec. IV-B, with k up to 8 instead of
// 2).  Several loads are issued before the first store so each lane keeps
// UNROLL requests in flight.  No address needs any alignment.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

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

// Cache policy of the copy loop's loads and stores.
//  PLAIN    ordinary loads and stores (write-back L2): best for the largest requests.
//  STREAM   non-temporal hint on both: kept as a tunable.
//  WT       ordinary loads, write-through 16-byte stores: nothing is left dirty in the
//           L2 for the end of the kernel to write back, which shortens small and
//           medium requests by 10-15 % and costs nothing until the output outgrows
//           the on-die caches.
//  COHERENT every load and store at system scope: loads never hit a stale cache
//           line, stores are written through and are visible to the whole system once
//           the wavefront's memory counter has drained.  Used by the armed kernels,
//           which therefore need no cache invalidate after the doorbell and no cache
//           write-back before the completion word.  A wavefront that used this policy
//           must execute dl_drain_stores() before it signals anything: the compiler
//           does not count the stores issued from inline assembly.
enum : int { DL_POL_PLAIN = 0, DL_POL_STREAM = 1, DL_POL_WT = 2, DL_POL_COHERENT = 3 };

template <int POL, typename V>
__device__ __forceinline__ V dl_ld(const DL_GLOBAL V *p)
{
    if constexpr (POL == DL_POL_STREAM) {
        return __builtin_nontemporal_load(p);
    } else if constexpr (POL == DL_POL_COHERENT && sizeof(V) == 16) {
        V v;
        asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
        return v;
    } else if constexpr (POL == DL_POL_COHERENT) {
        return __hip_atomic_load((const V *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    } else {
        return *p;
    }
}

template <int POL, typename V>
__device__ __forceinline__ void dl_st(DL_GLOBAL V *p, V v)
{
    if constexpr (POL == DL_POL_STREAM)
        __builtin_nontemporal_store(v, p);
    // The s_nop after each store: a store of more than 8 bytes must not be followed directly by a
    // vector ALU write to its data registers (the hardware reads them a cycle late).  The compiler
    // pads its own stores for this, but it cannot see that the assembly below is one, and it is free
    // to reuse v's registers in the very next instruction.
    else if constexpr (POL == DL_POL_WT && sizeof(V) == 16)
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
    else if constexpr (POL == DL_POL_COHERENT && sizeof(V) == 16)
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
    else if constexpr (POL == DL_POL_COHERENT)
        __hip_atomic_store((V *)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    else
        *p = v;
}

// Wait until every vector memory operation of this wavefront has completed.
__device__ __forceinline__ void dl_drain_stores()
{
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
}

// 16 bytes at any address.  A 16-byte global access needs no alignment on this hardware (the runtime enables
// unaligned access for the whole process, and the compiler counts on it: it emits one global_load_dwordx4 for a
// load that it knows nothing about the alignment of).  The pointee type says "alignment 1" so that nothing is
// ever assumed about the low address bits; aligned and unaligned addresses take the same instruction.
typedef dl_u32x4 dl_u32x4u __attribute__((aligned(1)));

template <int POL>
__device__ __forceinline__ dl_u32x4 dl_ld16(const char *p)
{
    const DL_GLOBAL dl_u32x4u *q = (const DL_GLOBAL dl_u32x4u *)(uint64_t)p;
    if constexpr (POL == DL_POL_STREAM) {
        return __builtin_nontemporal_load(q);
    } else if constexpr (POL == DL_POL_COHERENT) {
        dl_u32x4 v;
        asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(q) : "memory");
        return v;
    } else {
        return *q;
    }
}

template <int POL>
__device__ __forceinline__ void dl_st16(char *p, dl_u32x4 v)
{
    DL_GLOBAL dl_u32x4u *q = (DL_GLOBAL dl_u32x4u *)(uint64_t)p;
    if constexpr (POL == DL_POL_STREAM)
        __builtin_nontemporal_store(v, q);
    else if constexpr (POL == DL_POL_WT)  // (the s_nop: see dl_st)
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(q), "v"(v) : "memory");
    else if constexpr (POL == DL_POL_COHERENT)
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(q), "v"(v) : "memory");
    else
        *q = v;
}

// 16 bytes from an address that is not a multiple of 4, as the five aligned 4-byte words that hold them, shifted
// into place.  (A 16-byte load from such an address is legal but takes the memory pipeline about twice as long as
// one from a multiple of 4, which showed where every row is loaded by several wavefronts: the all-gather.)  Up to
// 3 bytes in front of p and behind p + 16 are read with them and dropped; they lie in 4-byte words that also hold
// bytes of the source.  `odd` = p modulo 4, from 1 to 3.  Not meant for the system-scope policy, whose loads each
// wait for their own round trip.
template <int POL>
__device__ __forceinline__ dl_u32x4 dl_ld16_shifted(const char *p, uint32_t odd)
{
    const dl_u32x4 w = dl_ld16<POL>(p - odd);
    const uint32_t w4 = dl_ld<POL>(dl_global<uint32_t>(p - odd + 16));
    dl_u32x4 v;
    v.x = __builtin_amdgcn_alignbyte(w.y, w.x, odd);
    v.y = __builtin_amdgcn_alignbyte(w.z, w.y, odd);
    v.z = __builtin_amdgcn_alignbyte(w.w, w.z, odd);
    v.w = __builtin_amdgcn_alignbyte(w4, w.w, odd);
    return v;
}

// The same for a lane of the row path, where lane l + 1 loads the 16 bytes that follow lane l's: the fifth word is
// the next lane's first one, taken across lanes (a DPP move that shifts the wavefront by one lane) instead of from
// memory.  own_fifth: this lane has no such neighbour (lane 63, or the next lane loads nothing) and fetches the word
// itself, in flight together with the other four.  Every lane of the row that loads calls this together.
// (All-gather of 64 MiB per rank from sources one byte off: unaligned 16-byte loads 4.2 TB/s, five words per lane
// 4.7, this 5.6; aligned sources 6.0.)
template <int POL>
__device__ __forceinline__ dl_u32x4 dl_ld16_shifted_row(const char *p, uint32_t odd, bool own_fifth)
{
    const dl_u32x4 w = dl_ld16<POL>(p - odd);
    uint32_t mine = 0;
    if (own_fifth) mine = dl_ld<POL>(dl_global<uint32_t>(p - odd + 16));
    constexpr int WAVE_SHL1 = 0x130;  // lane l receives lane l + 1's value; lane 63 keeps the first operand
    uint32_t w4 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w.x, WAVE_SHL1, 0xf, 0xf, false);
    if (own_fifth) w4 = mine;
    dl_u32x4 v;
    v.x = __builtin_amdgcn_alignbyte(w.y, w.x, odd);
    v.y = __builtin_amdgcn_alignbyte(w.z, w.y, odd);
    v.z = __builtin_amdgcn_alignbyte(w.w, w.z, odd);
    v.w = __builtin_amdgcn_alignbyte(w4, w.w, odd);
    return v;
}

// One byte from src + i to the same offset of the first k destinations.
template <int FAN, int POL>
__device__ __forceinline__ void dl_copy_byte(const char *src, char *const (&dsts)[FAN], uint32_t k, uint64_t i)
{
    const uint8_t v = dl_ld<POL>(dl_global<uint8_t>(src) + i);
#pragma unroll
    for (int j = 0; j < FAN; ++j)
        if ((uint32_t)j < k) dl_st<POL>(dl_global<uint8_t>(dsts[j]) + i, v);
}

// N 16-byte loads (any alignment) issued back to back, so that a lane has N requests in flight.  For the coherent
// policy the loads and the one wait behind them are a single assembly statement: the compiler cannot see that
// such a load completes later, so its results must not be visible to it before the wait (outputs are
// early-clobber: the addresses of the later loads are still needed when the first result register is written).
// Every address must be readable; what a lane does not want it simply does not store.
template <int POL, int N>
__device__ __forceinline__ void dl_ld_many(dl_u32x4 (&v)[N], const char *const (&p)[N])
{
    static_assert(N == 1 || N == 2 || N == 4, "one, two or four loads in flight");
    if constexpr (POL != DL_POL_COHERENT) {
#pragma unroll
        for (int u = 0; u < N; ++u) v[u] = dl_ld16<POL>(p[u]);
    } else if constexpr (N == 1) {
        v[0] = dl_ld16<POL>(p[0]);
    } else if constexpr (N == 2) {
        asm volatile("global_load_dwordx4 %0, %2, off sc0 sc1\n\t"
                     "global_load_dwordx4 %1, %3, off sc0 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(v[0]), "=&v"(v[1])
                     : "v"(p[0]), "v"(p[1])
                     : "memory");
    } else {
        asm volatile("global_load_dwordx4 %0, %4, off sc0 sc1\n\t"
                     "global_load_dwordx4 %1, %5, off sc0 sc1\n\t"
                     "global_load_dwordx4 %2, %6, off sc0 sc1\n\t"
                     "global_load_dwordx4 %3, %7, off sc0 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
                     : "v"(p[0]), "v"(p[1]), "v"(p[2]), "v"(p[3])
                     : "memory");
    }
}

// n 16-byte vectors from s to d[0..K), by nthr threads.  SHIFTED: s is not a multiple of 4 (see dl_ld16_shifted).
template <int K, int POL, bool SHIFTED>
__device__ __forceinline__ void dl_copy_vec16_loop(const char *__restrict__ s, char *const (&d)[K], uint32_t n, uint32_t tid,
                                                   uint32_t nthr, uint32_t odd)
{
    uint32_t i = tid;
    const uint32_t step = nthr * DL_UNROLL;
    for (; i + (DL_UNROLL - 1) * nthr < n; i += step) {
        dl_u32x4 v[DL_UNROLL];
        const char *from[DL_UNROLL];
#pragma unroll
        for (int u = 0; u < DL_UNROLL; ++u) from[u] = s + 16ull * (i + u * nthr);
        if constexpr (SHIFTED) {
#pragma unroll
            for (int u = 0; u < DL_UNROLL; ++u) v[u] = dl_ld16_shifted<POL>(from[u], odd);
        } else {
            dl_ld_many<POL, DL_UNROLL>(v, from);
        }
#pragma unroll
        for (int u = 0; u < DL_UNROLL; ++u)
#pragma unroll
            for (int j = 0; j < K; ++j) dl_st16<POL>(d[j] + 16ull * (i + u * nthr), v[u]);
    }
    for (; i < n; i += nthr) {
        dl_u32x4 v;
        if constexpr (SHIFTED)
            v = dl_ld16_shifted<POL>(s + 16ull * i, odd);
        else
            v = dl_ld16<POL>(s + 16ull * i);
#pragma unroll
        for (int j = 0; j < K; ++j) dl_st16<POL>(d[j] + 16ull * i, v);
    }
}

// n 16-byte vectors from s to the same offsets of the first K of the destinations, by nthr threads.
template <int K, int FAN, int POL>
__device__ __forceinline__ void dl_copy_vec16(const char *__restrict__ s, char *const (&dsts)[FAN], uint64_t byte_off,
                                              uint32_t n, uint32_t tid, uint32_t nthr)
{
    static_assert(K <= FAN, "fan-out");
    s += byte_off;
    char *d[K];
#pragma unroll
    for (int j = 0; j < K; ++j) d[j] = dsts[j] + byte_off;
    if constexpr (POL != DL_POL_COHERENT) {
        // every load address is the same modulo 4
        const uint32_t odd = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)s & 3u);
        if (odd) {
            dl_copy_vec16_loop<K, POL, true>(s, d, n, tid, nthr, odd);
            return;
        }
    }
    dl_copy_vec16_loop<K, POL, false>(s, d, n, tid, nthr, 0u);
}

// Move bytes [lo, hi) of the copy (src -> dsts[0..k)), all threads of the workgroup taking part: up to 15 bytes
// one by one until the first destination stands on a 16-byte boundary, then 16-byte vectors (aligned stores to
// the first destination; the other addresses are whatever they are), then up to 15 bytes one by one.
// src, dsts, k, lo, hi, split must be uniform across the workgroup; 1 <= k <= FAN; nthr >= 64; hi - lo < 2^32.
//
// split in {1, 2, 4} divides the workgroup into that many sub-groups of whole
// wavefronts.  Every sub-group reads the whole range (the first read brings it
// into the compute unit's cache, the others hit there) and writes it to its
// own share of ceil(k / split) destinations, so a lane issues few stores per
// load.  On MI355X one load followed by two stores per wavefront moved an
// 8-way fan-out about 10 % faster than one load followed by eight stores.
template <int FAN, int POL>
__device__ __forceinline__ void dl_move_range(const char *src, char *const (&dsts)[FAN], uint32_t k, uint64_t lo,
                                              uint64_t hi, uint32_t split, uint32_t tid, uint32_t nthr)
{
    if (lo >= hi) return;
    const uint64_t len = hi - lo;
    uint64_t head = (0 - ((uint64_t)dsts[0] + lo)) & 15u;
    if (head > len) head = len;
    const uint32_t n = (uint32_t)((len - head) >> 4);
    const uint32_t tail = (uint32_t)(len - head) & 15u;
    const uint64_t off = lo + head;
    // head bytes by threads 0..15, tail bytes by threads 32..47
    if (tid < head) dl_copy_byte<FAN, POL>(src, dsts, k, lo + tid);
    if (tid >= 32 && tid - 32 < tail) dl_copy_byte<FAN, POL>(src, dsts, k, off + 16ull * n + (tid - 32));
    if (n == 0) return;

    if constexpr (FAN == 1) {
        dl_copy_vec16<1, FAN, POL>(src, dsts, off, n, tid, nthr);
    } else {
        static_assert(FAN == 8, "fan-out switch and shifter below are written for 8");
        char *my[FAN];
#pragma unroll
        for (int j = 0; j < FAN; ++j) my[j] = dsts[j];
        uint32_t my_k = k;
        if (split > 1) {
            // sub-group `grp` (whole wavefronts) takes destinations first .. first + my_k - 1
            nthr /= split;
            const uint32_t grp = __builtin_amdgcn_readfirstlane(tid / nthr);
            tid -= grp * nthr;
            const uint32_t per = (k + split - 1) / split;
            const uint32_t first = grp * per;
            my_k = first < k ? (k - first < per ? k - first : per) : 0u;
            // my[q] = dsts[first + q]: shift the (uniform) pointer array down by first, bit by bit
#pragma unroll
            for (int sh = 1; sh < FAN; sh *= 2)
                if (first & (uint32_t)sh) {
#pragma unroll
                    for (int j = 0; j + sh < FAN; ++j) my[j] = my[j + sh];
                }
        }
        switch (my_k) {
        case 0: break;
        case 1: dl_copy_vec16<1, FAN, POL>(src, my, off, n, tid, nthr); break;
        case 2: dl_copy_vec16<2, FAN, POL>(src, my, off, n, tid, nthr); break;
        case 3: dl_copy_vec16<3, FAN, POL>(src, my, off, n, tid, nthr); break;
        case 4: dl_copy_vec16<4, FAN, POL>(src, my, off, n, tid, nthr); break;
        case 5: dl_copy_vec16<5, FAN, POL>(src, my, off, n, tid, nthr); break;
        case 6: dl_copy_vec16<6, FAN, POL>(src, my, off, n, tid, nthr); break;
        case 7: dl_copy_vec16<7, FAN, POL>(src, my, off, n, tid, nthr); break;
        default: dl_copy_vec16<8, FAN, POL>(src, my, off, n, tid, nthr); break;
        }
    }
}

// Tile `tile` of the copy: the bytes that lie in that tile of the first destination's grid (see dl_tile_range).
template <int FAN, int POL>
__device__ __forceinline__ void dl_move_tile(const char *src, char *const (&dsts)[FAN], uint32_t k, uint64_t bytes,
                                             uint64_t tile, uint32_t tile_bytes, uint32_t split, uint32_t tid,
                                             uint32_t nthr)
{
    uint64_t lo, hi;
    dl_tile_range((uint32_t)((uint64_t)dsts[0] & (DL_CUT - 1u)), bytes, tile, tile_bytes, &lo, &hi);
    dl_move_range<FAN, POL>(src, dsts, k, lo, hi, split, tid, nthr);
}

// Exchange bytes [lo, hi) of a and b (disjoint ranges): cut like dl_move_range with b in the place of the first
// destination.  Every byte of either range is read and written by exactly one lane, so no lane depends on another.
template <int POL>
__device__ __forceinline__ void dl_swap_byte(char *a, char *b, uint64_t i)
{
    const uint8_t x = dl_ld<POL>(dl_global<uint8_t>(a) + i);
    const uint8_t y = dl_ld<POL>(dl_global<uint8_t>(b) + i);
    dl_st<POL>(dl_global<uint8_t>(a) + i, y);
    dl_st<POL>(dl_global<uint8_t>(b) + i, x);
}

template <int POL>
__device__ __forceinline__ void dl_swap_range(char *a, char *b, uint64_t lo, uint64_t hi, uint32_t tid, uint32_t nthr)
{
    if (lo >= hi) return;
    const uint64_t len = hi - lo;
    uint64_t head = (0 - ((uint64_t)b + lo)) & 15u;
    if (head > len) head = len;
    const uint32_t n = (uint32_t)((len - head) >> 4);
    const uint32_t tail = (uint32_t)(len - head) & 15u;
    const uint64_t off = lo + head;
    if (tid < head) dl_swap_byte<POL>(a, b, lo + tid);
    if (tid >= 32 && tid - 32 < tail) dl_swap_byte<POL>(a, b, off + 16ull * n + (tid - 32));
    for (uint32_t i = tid; i < n; i += nthr) {
        dl_u32x4 xy[2];
        const char *const from[2] = {a + off + 16ull * i, b + off + 16ull * i};
        dl_ld_many<POL, 2>(xy, from);  // both in flight together
        dl_st16<POL>(a + off + 16ull * i, xy[1]);
        dl_st16<POL>(b + off + 16ull * i, xy[0]);
    }
}

template <int POL>
__device__ __forceinline__ void dl_swap_tile(char *a, char *b, uint64_t bytes, uint64_t tile, uint32_t tile_bytes,
                                             uint32_t tid, uint32_t nthr)
{
    uint64_t lo, hi;
    dl_tile_range((uint32_t)((uint64_t)b & (DL_CUT - 1u)), bytes, tile, tile_bytes, &lo, &hi);
    dl_swap_range<POL>(a, b, lo, hi, tid, nthr);
}

// A slot that the host filled through the BAR carries a stamp behind its payload, written after it; writes that
// cross the link arrive in order, so once the stamp is there what was written before it is there too.  The word
// that holds it (`slot` is the slot's first byte):
__device__ __forceinline__ const DL_GLOBAL uint64_t *dl_pushed_stamp(const void *slot)
{
    return dl_global<uint64_t>((const char *)slot + DL_PUSH_PAYLOAD_BYTES);
}
// How often a kernel looks again if the stamp is not there at the first look (the launch overtook the writes
// inside the device; they were on their way before it): bounded, like every wait in this library.
constexpr uint32_t DL_PUSHED_TRIES = 1u << 18;  // a look takes about a microsecond: a quarter of a second in all

// The kernel gave up on its table: say so where the host will look (any non-zero value; the stamp tells which).
__device__ __forceinline__ void dl_pushed_report_lost(const dl_pushed &ps)
{
    __hip_atomic_store(ps.lost, ps.stamp | (1ull << 63), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Wait (bounded) until the slot's stamp is the table's.  The host writes the table, then the stamp; only what is
// read AFTER the stamp has been seen is vouched for by it, so every reader looks at the stamp first and loads
// table words behind this call.  One lane's business; the compiler barrier keeps later loads behind the loop.
__device__ __forceinline__ bool dl_pushed_sealed(const void *slot, const dl_pushed &ps)
{
    bool ok = false;
    for (uint32_t t = 0; t < ps.tries && !ok; ++t) ok = dl_ld<DL_POL_COHERENT>(dl_pushed_stamp(slot)) == ps.stamp;
    asm volatile("" ::: "memory");
    return ok;
}

// ------------------------------------------------ items and lists on the device

__device__ __forceinline__ uint64_t dl_uniform64(uint64_t v)
{
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

template <int POL>
__device__ __forceinline__ void dl_run_item(const dl_plain_item &it, uint64_t tile, uint32_t tile_bytes, uint32_t)
{
    char *d[1] = {(char *)dl_uniform64((uint64_t)it.dst)};
    dl_move_tile<1, POL>((const char *)dl_uniform64((uint64_t)it.src), d, 1u, dl_uniform64(it.bytes), tile, tile_bytes,
                        1u, threadIdx.x, blockDim.x);
}

template <int POL>
__device__ __forceinline__ void dl_run_item(const dl_swap_item &it, uint64_t tile, uint32_t tile_bytes, uint32_t)
{
    dl_swap_tile<POL>((char *)dl_uniform64((uint64_t)it.src), (char *)dl_uniform64((uint64_t)it.dst),
                      dl_uniform64(it.bytes), tile, tile_bytes, threadIdx.x, blockDim.x);
}

template <int POL>
__device__ __forceinline__ void dl_run_item(const dl_fused_item &it, uint64_t tile, uint32_t tile_bytes,
                                            uint32_t split)
{
    char *d[DL_FAN];
#pragma unroll
    for (int j = 0; j < DL_FAN; ++j) d[j] = (char *)dl_uniform64((uint64_t)it.dst[j]);
    dl_move_tile<DL_FAN, POL>((const char *)dl_uniform64((uint64_t)it.src), d, __builtin_amdgcn_readfirstlane(it.k),
                             dl_uniform64(it.bytes), tile, tile_bytes, split, threadIdx.x, blockDim.x);
}

// A whole item by one workgroup (an entry of a table: the host has cut those to a tile's length at most).
template <int POL>
__device__ __forceinline__ void dl_run_entry(const dl_plain_item &it, uint32_t)
{
    char *d[1] = {(char *)dl_uniform64((uint64_t)it.dst)};
    dl_move_range<1, POL>((const char *)dl_uniform64((uint64_t)it.src), d, 1u, 0, dl_uniform64(it.bytes), 1u, threadIdx.x,
                          blockDim.x);
}

template <int POL>
__device__ __forceinline__ void dl_run_entry(const dl_swap_item &it, uint32_t)
{
    dl_swap_range<POL>((char *)dl_uniform64((uint64_t)it.src), (char *)dl_uniform64((uint64_t)it.dst), 0,
                       dl_uniform64(it.bytes), threadIdx.x, blockDim.x);
}

template <int POL>
__device__ __forceinline__ void dl_run_entry(const dl_fused_item &it, uint32_t split)
{
    char *d[DL_FAN];
#pragma unroll
    for (int j = 0; j < DL_FAN; ++j) d[j] = (char *)dl_uniform64((uint64_t)it.dst[j]);
    dl_move_range<DL_FAN, POL>((const char *)dl_uniform64((uint64_t)it.src), d, __builtin_amdgcn_readfirstlane(it.k), 0,
                               dl_uniform64(it.bytes), split, threadIdx.x, blockDim.x);
}

template <class Item, int NMAX>
struct dl_klist {
    uint32_t n;
    uint32_t tile_bytes;
    uint32_t split;           // sub-groups of a workgroup that share out the destinations of a fused item
    uint32_t split_log2;      // row path: log2(split)
    uint32_t wpg_log2;        // row path: log2(wavefronts per sub-group) = log2(rows per tile)
    uint32_t tile_end[NMAX];  // inclusive prefix sum of tiles per item; entries past n hold 0xFFFFFFFF
    Item item[NMAX];
};

// Item of global tile b: the number of items whose last tile lies before b,
// and (in *first) the number of tiles before that item.  A short list is
// compared entry by entry on the scalar unit (b is uniform, the list sits in
// the kernel-argument segment); a long one takes one entry per lane and a
// ballot.
template <class Item, int NMAX>
__device__ __forceinline__ uint32_t dl_find_item(const dl_klist<Item, NMAX> &p, uint32_t b, uint32_t *first)
{
    if constexpr (NMAX <= 8) {
        uint32_t d = 0, f = 0;
#pragma unroll
        for (int i = 0; i < NMAX; ++i) {
            const uint32_t e = p.tile_end[i];  // non-decreasing; 0xFFFFFFFF past the last item
            const bool before = e <= b;
            d += before ? 1u : 0u;
            f = before ? e : f;
        }
        *first = f;
        return d;
    } else {
        // one entry per lane, one ballot: a single memory round trip however long the list
        static_assert(NMAX <= 64, "one wavefront holds the whole prefix sum");
        const uint32_t lane = threadIdx.x & 63u;
        const uint32_t e = lane < (uint32_t)NMAX ? p.tile_end[lane < (uint32_t)NMAX ? lane : 0] : 0xFFFFFFFFu;
        const uint32_t d = __builtin_amdgcn_readfirstlane((uint32_t)__popcll(__ballot(e <= b)));
        *first = d ? (uint32_t)__builtin_amdgcn_readlane((int)e, (int)(d - 1)) : 0u;
        return d;
    }
}

__device__ __forceinline__ const char *dl_item_dst(const dl_plain_item &it, uint32_t) { return it.dst; }
__device__ __forceinline__ const char *dl_item_dst(const dl_fused_item &it, uint32_t j) { return it.dst[j]; }

// The bytes of an item that no lane of the row path moves inside a whole vector: up to 15 in front of the first
// destination's first 16-byte boundary and up to 15 behind its last one (or the whole of an item that lies inside
// one vector).  Every wavefront calls this for its row with uniform arguments; if the item begins in that row,
// lanes 0..14 move the leading bytes, if it ends there, lanes 16..30 move the trailing ones, a byte each, so all of
// them are in flight together.  each(i) moves byte i of the item.
template <class Each>
__device__ __forceinline__ void dl_row_edges(uint32_t shift, uint64_t bytes, uint64_t row, uint32_t lane, Each each)
{
    // positions on the grid: the item occupies [shift, end)
    const uint64_t end = shift + bytes;
    const uint64_t first_whole = ((uint64_t)shift + 15u) & ~(uint64_t)15u;  // where the first vector inside the item would begin
    const uint64_t last_part = end & ~(uint64_t)15u;                        // where a trailing partial vector begins
    if (row == 0 && (shift & 15u)) {
        const uint64_t n = first_whole < end ? first_whole - shift : bytes;
        if (lane < n) each((uint64_t)lane);
    }
    if ((end & 15u) && last_part >= first_whole && (last_part >> 10) == row) {
        const uint32_t n = (uint32_t)end & 15u;
        if (lane >= 16u && lane - 16u < n) each(last_part - shift + (lane - 16u));
    }
}

template <class Item>
__device__ __forceinline__ bool dl_item_ragged(const Item &it)
{
    return __builtin_amdgcn_readfirstlane((dl_item_shift(it) | (uint32_t)it.bytes) & 15u) != 0;
}

// How a row lies in its item, for the lanes' question "are my 16 bytes wholly inside?".  The answer costs vector
// compares only where it has to: in an item that is not ragged (see dl_item_ragged) one compare per lane decides; in a
// ragged one every lane of a row between the item's first and last row is inside, and only those two rows look
// closely (and have bytes to move singly, see dl_row_edges).
enum : uint32_t { DL_ROW_PLAIN = 0, DL_ROW_INNER = 1, DL_ROW_EDGE = 2, DL_ROW_NONE = 3 };

__device__ __forceinline__ uint32_t dl_row_kind(bool ragged, uint32_t shift, uint64_t bytes, uint64_t row)
{
    if (!ragged) return DL_ROW_PLAIN;
    const uint64_t last = (shift + bytes - 1u) >> 10;  // (bytes >= 1: empty items have no tiles)
    return row > last ? DL_ROW_NONE : (row == 0 || row == last) ? DL_ROW_EDGE : DL_ROW_INNER;
}

// A lane whose 16 bytes begin at offset `byte` of an item of `bytes` bytes (an offset in front of the item has
// wrapped below zero) has a whole vector inside the item.  kind: the row's, uniform.
__device__ __forceinline__ bool dl_lane_whole(uint64_t byte, uint64_t bytes, uint32_t kind)
{
    if (kind == DL_ROW_INNER) return true;
    if (kind == DL_ROW_PLAIN) return byte < bytes;
    return kind == DL_ROW_EDGE && byte < bytes && bytes - byte >= 16u;
}

// Row path: the hot loop of large requests, kept to a few dozen instructions and two scalar round trips per
// wavefront.  Rows are the 1 KiB rows of the grid of the item's first destination (see dl_tile_range; a tile
// is (1 << wpg_log2) rows), and lane l of a row moves the 16 bytes at row * 1024 + 16 l - shift of the item:
// one 16-byte load, then one store per destination.  No address needs any alignment.  Where an item begins or
// ends in mid-vector (its first destination or its length is not a multiple of 16: one scalar test), the
// wavefront of that row moves those bytes one per lane (dl_row_edges).
// The destinations of a fused item are stored by sub-group (established on the host): sub-group g owns slots
// g * (DL_FAN >> split_log2) onwards, filled from the front, the rest null; slot 0 is the first destination.
// Wavefront w of the workgroup belongs to sub-group w >> wpg_log2 and moves row w & (rows - 1) of the tile, to
// the destinations in its sub-group's slots.  At this granularity (a wavefront lives for one load and one or two
// stores) the per-wavefront instruction count and the dependent scalar loads in front of the vector load decide
// the rate.  `tile` is the tile's index within the item.
// ON_GRID: the host has seen that every item's first destination stands on a DL_CUT boundary, that every
// length is a multiple of 16 and every source a multiple of 4.  Nothing of the above is computed then; the dozen
// scalar instructions that it takes cost the all-gather of 4 .. 64 MiB per rank 1-2.5 % of its rate.
template <int POL, bool ON_GRID = false, class Item>
__device__ __forceinline__ void dl_rows_body(const Item &it, uint32_t tile, uint32_t wl, uint32_t sl)
{
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t row = ((uint64_t)tile << wl) + (wave & ((1u << wl) - 1u));
    // everything the wavefront needs from the item is requested before the first use
    const char *src = it.src;
    const uint64_t bytes = it.bytes;
    const bool ragged = ON_GRID ? false : dl_item_ragged(it);
    const uint32_t shift = ON_GRID ? 0u : dl_item_shift(it);
    const uint32_t kind = ON_GRID ? (uint32_t)DL_ROW_PLAIN : dl_row_kind(ragged, shift, bytes, row);
    const uint64_t byte = ((row << 10) - shift) + (lane << 4);
    // every lane's source address is the same modulo 4: not zero -> dl_ld16_shifted_row (not at system scope, and not
    // for swaps, which load both sides)
    uint32_t odd = 0;
    if constexpr (POL != DL_POL_COHERENT && !ON_GRID)
        odd = __builtin_amdgcn_readfirstlane(((uint32_t)(uint64_t)src - shift) & 3u);
    if constexpr (std::is_same<Item, dl_swap_item>::value) {
        char *pa = const_cast<char *>(src);
        char *pb = it.dst;
        if (kind == DL_ROW_EDGE) dl_row_edges(shift, bytes, row, lane, [&](uint64_t i) { dl_swap_byte<POL>(pa, pb, i); });
        if (!dl_lane_whole(byte, bytes, kind)) return;
        dl_u32x4 xy[2];
        const char *const from[2] = {pa + byte, pb + byte};
        dl_ld_many<POL, 2>(xy, from);
        dl_st16<POL>(pa + byte, xy[1]);
        dl_st16<POL>(pb + byte, xy[0]);
    } else if constexpr (std::is_same<Item, dl_plain_item>::value) {
        char *dst = it.dst;
        if (kind == DL_ROW_EDGE)
            dl_row_edges(shift, bytes, row, lane, [&](uint64_t i) {
                dl_st<POL>(dl_global<uint8_t>(dst) + i, dl_ld<POL>(dl_global<uint8_t>(src) + i));
            });
        if (!dl_lane_whole(byte, bytes, kind)) return;
        if (odd)
            dl_st16<POL>(dst + byte, dl_ld16_shifted_row<POL>(src + byte, odd, lane == 63u || !dl_lane_whole(byte + 16u, bytes, kind)));
        else
            dl_st16<POL>(dst + byte, dl_ld16<POL>(src + byte));
    } else {
        const uint32_t slots = (uint32_t)DL_FAN >> sl;
        const uint32_t base = (wave >> wl) * slots;
        char *d0 = it.dst[base];
        char *d1 = slots > 1 ? it.dst[base + 1] : nullptr;
        if (!d0) return;
        if (kind == DL_ROW_EDGE)
            dl_row_edges(shift, bytes, row, lane, [&](uint64_t i) {
                const uint8_t v = dl_ld<POL>(dl_global<uint8_t>(src) + i);
                for (uint32_t q = 0; q < slots; ++q) {
                    char *dq = it.dst[base + q];
                    if (!dq) break;
                    dl_st<POL>(dl_global<uint8_t>(dq) + i, v);
                }
            });
        if (!dl_lane_whole(byte, bytes, kind)) return;
        dl_u32x4 v;
        if (odd)
            v = dl_ld16_shifted_row<POL>(src + byte, odd, lane == 63u || !dl_lane_whole(byte + 16u, bytes, kind));
        else
            v = dl_ld16<POL>(src + byte);
        dl_st16<POL>(d0 + byte, v);
        if (!d1) return;
        dl_st16<POL>(d1 + byte, v);
#pragma unroll
        for (uint32_t q = 2; q < (uint32_t)DL_FAN; ++q) {
            if (q >= slots) break;
            char *dq = it.dst[base + q];
            if (!dq) break;
            dl_st16<POL>(dq + byte, v);
        }
    }
}

// Row path over a list in the kernel arguments: global tile b -> (item, tile).
template <int POL, bool ON_GRID = false, class Item, int NMAX>
__device__ __forceinline__ void dl_run_rows(const dl_klist<Item, NMAX> &p, uint32_t b)
{
    uint32_t first_tile;
    const uint32_t d = dl_find_item(p, b, &first_tile);
    if (d >= p.n) return;
    dl_rows_body<POL, ON_GRID>(p.item[d], b - first_tile, p.wpg_log2, p.split_log2);
}

// Row path of the armed kernels, whose loads go to memory at system scope and take long to come back: a
// wavefront takes up to R global tiles per pass (b0, b0 + stride, ...; those below `total`), issues the loads
// of all of them, waits once and stores.  Rows and lanes as in dl_rows_body, with one sub-group per workgroup
// (every wavefront stores its row to all of the item's destinations).  b0 < total.  Not for swaps.
// spare: 16 readable bytes of device memory, for the lanes that have no vector of their own to load.
template <int R, class Item, int NMAX>
__device__ __forceinline__ void dl_run_rows_coherent(const dl_klist<Item, NMAX> &p, uint32_t b0, uint32_t stride,
                                                     uint32_t total, const void *spare)
{
    static_assert(!std::is_same<Item, dl_swap_item>::value, "a swap has two loads per row already");
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wl = p.wpg_log2;
    uint32_t first;
    const uint32_t d0 = dl_find_item(p, b0, &first);
    // what a lane without a vector loads instead: the first 16 bytes of tile b0's item, if it has that many
    const char *const safe = p.item[d0].bytes >= 16u ? p.item[d0].src : (const char *)spare;
    uint32_t d[R];
    uint64_t byte[R];
    bool whole[R];
    const char *from[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t b = b0 + (uint32_t)r * stride;
        d[r] = p.n;
        byte[r] = 0;
        whole[r] = false;
        from[r] = safe;
        if (b < total && b >= b0) {  // (b >= b0: no wrap-around)
            d[r] = dl_find_item(p, b, &first);
            if (d[r] < p.n) {
                const Item &it = p.item[d[r]];
                const uint64_t row = ((uint64_t)(b - first) << wl) + (wave & ((1u << wl) - 1u));
                const uint32_t shift = dl_item_shift(it);
                byte[r] = ((row << 10) - shift) + (lane << 4);
                const uint32_t kind = dl_row_kind(dl_item_ragged(it), shift, it.bytes, row);
                whole[r] = dl_lane_whole(byte[r], it.bytes, kind);
                if (whole[r]) from[r] = it.src + byte[r];
                if (kind == DL_ROW_EDGE)  // the bytes in front of and behind the item's whole vectors
                    dl_row_edges(shift, it.bytes, row, lane, [&](uint64_t i) {
                        const uint8_t x = dl_ld<DL_POL_COHERENT>(dl_global<uint8_t>(it.src) + i);
                        if constexpr (std::is_same<Item, dl_plain_item>::value) {
                            dl_st<DL_POL_COHERENT>(dl_global<uint8_t>(it.dst) + i, x);
                        } else {
                            for (uint32_t q = 0; q < (uint32_t)DL_FAN; ++q) {
                                char *dq = it.dst[q];  // filled from the front, the rest null
                                if (!dq) break;
                                dl_st<DL_POL_COHERENT>(dl_global<uint8_t>(dq) + i, x);
                            }
                        }
                    });
            }
        }
    }
    dl_u32x4 v[R];
    dl_ld_many<DL_POL_COHERENT, R>(v, from);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (!whole[r]) continue;
        const Item &it = p.item[d[r]];
        if constexpr (std::is_same<Item, dl_plain_item>::value) {
            dl_st16<DL_POL_COHERENT>(it.dst + byte[r], v[r]);
        } else {
#pragma unroll
            for (uint32_t q = 0; q < (uint32_t)DL_FAN; ++q) {
                char *dq = it.dst[q];  // filled from the front, the rest null
                if (!dq) break;
                dl_st16<DL_POL_COHERENT>(dq + byte[r], v[r]);
            }
        }
    }
}

// Global tile b of a list, any alignment and tile size: find its item, then
// move that tile.  b must be uniform across the workgroup.
template <int POL, class Item, int NMAX>
__device__ __forceinline__ void dl_run_tile(const dl_klist<Item, NMAX> &p, uint32_t b)
{
    uint32_t first;
    const uint32_t d = dl_find_item(p, b, &first);
    if (d >= p.n) return;
    dl_run_item<POL>(p.item[d], (uint64_t)(b - first), p.tile_bytes, p.split);
}
