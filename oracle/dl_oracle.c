/*
 * CPU checker for the copy collectives of the DMA-offload paper
 * (all-gather, all-to-all, broadcast, batched back-to-back copies).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain definition of each operation
 * written with memcpy on host buffers, single-threaded, with no blocking,
 * fusion or reordering.  It shares no code with the HIP library and is never
 * called by it; only the tests, the smoke check and the benchmark's CPU
 * baseline use it.
 *
 * Every result is pinned by the CPU tests (per-byte index formulas on tiny
 * inputs, reductions to numpy library routines, and the invariants of the
 * collectives), so no function here is "parity unpinned".
 *
 * Every function returns 0 on success and a negative value on a malformed
 * request.  Buffers are host memory owned by the caller.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    const void *src;
    void *dst;
    size_t bytes;
} ref_copy;

static int ranges_overlap(const char *a, size_t an, const char *b, size_t bn)
{
    if (an == 0 || bn == 0)
        return 0;
    return (uintptr_t)a < (uintptr_t)b + bn && (uintptr_t)b < (uintptr_t)a + an;
}

/*
 * Hazard rule of back-to-back copies (Sec. IV-D): queued copies may overlap in
 * time only if they have unique source and destination buffers, i.e. no
 * destination range touches another destination range or any source range.
 * Sources may overlap each other.  A copy whose source and destination are the
 * identical range is a no-op and is not a hazard against itself.
 * Returns -1 if the list is hazard-free, else the index of the first copy
 * whose destination collides with something.
 */
long ref_first_hazard(const ref_copy *d, size_t n)
{
    for (size_t a = 0; a < n; ++a) {
        for (size_t b = 0; b < n; ++b) {
            if (a != b && ranges_overlap(d[a].dst, d[a].bytes, d[b].dst, d[b].bytes))
                return (long)a;
            if (a == b && d[a].src == d[a].dst)
                continue;
            if (ranges_overlap(d[a].dst, d[a].bytes, d[b].src, d[b].bytes))
                return (long)a;
        }
    }
    return -1;
}

/*
 * Batch of independent copies with no ordering among them (Sec. IV-D, and the
 * batched-copy runtime call of Sec. VI): copy k moves bytes_k bytes from src_k
 * to dst_k.  Defined only for a hazard-free list; -2 otherwise.
 */
int ref_batch_copy(const ref_copy *d, size_t n)
{
    if (n && !d)
        return -1;
    for (size_t k = 0; k < n; ++k)
        if (d[k].bytes && (!d[k].src || !d[k].dst))
            return -1;
    if (ref_first_hazard(d, n) >= 0)
        return -2;
    for (size_t k = 0; k < n; ++k)
        if (d[k].bytes && d[k].src != d[k].dst)
            memcpy(d[k].dst, d[k].src, d[k].bytes);
    return 0;
}

/*
 * Broadcast (Sec. IV-B): one source, k destinations, every destination ends up
 * holding the source's bytes.  (The hardware command has k = 2; any k >= 1
 * here.)
 */
int ref_broadcast(const void *src, void *const *dsts, int k, size_t bytes)
{
    if (k < 1 || !dsts || (bytes && !src))
        return -1;
    for (int d = 0; d < k; ++d) {
        if (bytes && !dsts[d])
            return -1;
        if (bytes)
            memcpy(dsts[d], src, bytes);
    }
    return 0;
}

/*
 * All-gather (Sec. II-A1, Fig. 2 left): rank j starts with a sub-array of B
 * bytes; afterwards every rank r holds all W sub-arrays in rank order:
 *   out[r][j*B + t] = in[j][t].
 */
int ref_allgather(const void *const *in, void *const *out, int W, size_t B)
{
    if (W < 1 || !in || !out)
        return -1;
    for (int r = 0; r < W; ++r) {
        for (int j = 0; j < W; ++j) {
            if (B && (!in[j] || !out[r]))
                return -1;
            if (B)
                memcpy((char *)out[r] + (size_t)j * B, in[j], B);
        }
    }
    return 0;
}

/*
 * All-to-all (Sec. II-A1, Fig. 2 right: the ranks collectively transpose).
 * C[i*W + j] = bytes rank i sends to rank j.  in[i] holds rank i's chunks
 * packed in destination order, out[j] holds what rank j receives packed in
 * source order:
 *   send offset of (i,j) = sum of C[i][j'] over j' < j
 *   recv offset of (i,j) = sum of C[i'][j] over i' < i
 *   out[j][recv(i,j) + t] = in[i][send(i,j) + t],  0 <= t < C[i][j].
 */
int ref_alltoall(const void *const *in, void *const *out, int W, const size_t *C)
{
    if (W < 1 || !in || !out || !C)
        return -1;
    for (int i = 0; i < W; ++i) {
        for (int j = 0; j < W; ++j) {
            size_t send = 0, recv = 0;
            for (int jj = 0; jj < j; ++jj)
                send += C[(size_t)i * W + jj];
            for (int ii = 0; ii < i; ++ii)
                recv += C[(size_t)ii * W + j];
            size_t n = C[(size_t)i * W + j];
            if (n == 0)
                continue;
            if (!in[i] || !out[j])
                return -1;
            memcpy((char *)out[j] + recv, (const char *)in[i] + send, n);
        }
    }
    return 0;
}

typedef struct {
    void *a;
    void *b;
    size_t bytes;
} ref_swap;

/*
 * Batch of swaps (Sec. IV-C): swap k exchanges the contents of the two memory
 * locations a_k and b_k.  Written as what the swap command replaces: three
 * copies, to and from a temporary buffer.  The swaps of a batch are independent
 * and unordered, so every range that any of them touches must be disjoint from
 * every other one (the hazard rule of Sec. IV-D applied to ranges that are
 * both read and written); -2 otherwise.  A swap whose two locations are the
 * identical range is a no-op.
 */
int ref_batch_swap(const ref_swap *d, size_t n)
{
    if (n && !d)
        return -1;
    for (size_t k = 0; k < n; ++k)
        if (d[k].bytes && (!d[k].a || !d[k].b))
            return -1;
    for (size_t k = 0; k < n; ++k) {
        if (d[k].a != d[k].b && ranges_overlap(d[k].a, d[k].bytes, d[k].b, d[k].bytes))
            return -2;
        for (size_t m = k + 1; m < n; ++m) {
            if (ranges_overlap(d[k].a, d[k].bytes, d[m].a, d[m].bytes) ||
                ranges_overlap(d[k].a, d[k].bytes, d[m].b, d[m].bytes) ||
                ranges_overlap(d[k].b, d[k].bytes, d[m].a, d[m].bytes) ||
                ranges_overlap(d[k].b, d[k].bytes, d[m].b, d[m].bytes))
                return -2;
        }
    }
    for (size_t k = 0; k < n; ++k) {
        if (d[k].bytes == 0 || d[k].a == d[k].b)
            continue;
        void *tmp = malloc(d[k].bytes);
        if (!tmp)
            return -3;
        memcpy(tmp, d[k].a, d[k].bytes);
        memcpy(d[k].a, d[k].b, d[k].bytes);
        memcpy(d[k].b, tmp, d[k].bytes);
        free(tmp);
    }
    return 0;
}

/*
 * In-place all-to-all with equal chunks (Sec. IV-C; Fig. 2 right): buf[i]
 * holds W chunks of c bytes, chunk j being what rank i sends to rank j.
 * Afterwards buf[j] chunk i holds what buf[i] chunk j held before:
 *   new buf[j][i*c + t] = old buf[i][j*c + t].
 * Written as the definition: every buffer is copied aside first, then every
 * chunk is placed from the copies.  (That the same result is a series of swaps
 * between the buffers, as the paper realises it, is checked by the tests.)
 */
int ref_alltoall_inplace(void *const *buf, int W, size_t c)
{
    if (W < 1 || !buf)
        return -1;
    if (c == 0)
        return 0;
    for (int i = 0; i < W; ++i)
        if (!buf[i])
            return -1;
    const size_t row = (size_t)W * c;
    char *old = malloc((size_t)W * row);
    if (!old)
        return -3;
    for (int i = 0; i < W; ++i)
        memcpy(old + (size_t)i * row, buf[i], row);
    for (int i = 0; i < W; ++i)
        for (int j = 0; j < W; ++j)
            memcpy((char *)buf[j] + (size_t)i * c, old + (size_t)i * row + (size_t)j * c, c);
    free(old);
    return 0;
}

/*
 * Token dispatch of an expert-parallel mixture-of-experts layer (Sec. II-A1:
 * tokens are exchanged between ranks by expert preference; Sec. IV-B: a token
 * that goes to several experts is one source with several destinations).
 * in[i] holds tokens[i] rows of row_bytes bytes.  dest has one byte per (token,
 * rank), tokens numbered over all ranks in rank order: dest[g*W + j] != 0 means
 * token g goes to rank j.  out[j] receives its rows packed in token order
 * (source rank first, then row index):
 *   out[j] row (number of tokens g' < g with dest[g'*W + j] != 0) = row of token g.
 */
int ref_token_dispatch(const void *const *in, void *const *out, int W, const uint32_t *tokens, size_t row_bytes,
                       const uint8_t *dest)
{
    if (W < 1 || !in || !out || !tokens)
        return -1;
    for (int j = 0; j < W; ++j) {
        size_t placed = 0; /* rows already written to out[j] */
        size_t g = 0;      /* global token number */
        for (int i = 0; i < W; ++i) {
            for (uint32_t t = 0; t < tokens[i]; ++t, ++g) {
                if (!dest)
                    return -1;
                if (!dest[g * (size_t)W + (size_t)j])
                    continue;
                if (row_bytes) {
                    if (!in[i] || !out[j])
                        return -1;
                    memcpy((char *)out[j] + placed * row_bytes, (const char *)in[i] + (size_t)t * row_bytes, row_bytes);
                }
                ++placed;
            }
        }
    }
    return 0;
}
