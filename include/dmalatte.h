/*
 * dmalatte.h - C boundary of the MI355X copy-collective library.
 *
 * The library executes the data movement behind DMA-offloaded collectives
 * (all-gather, all-to-all, broadcast, batched back-to-back copies) on the
 * compute units of one GPU.  W "virtual ranks" are W send buffers and W receive
 * buffers that all live in that GPU's memory.
 *
 * Conventions for every entry point
 *  - Data pointers (src, dst, in[r], out[r], dsts[d]) are DEVICE pointers owned
 *    by the caller.  The library never allocates, frees or keeps them.
 *  - Pointer arrays, descriptor arrays and chunk_bytes are HOST arrays.  They
 *    are fully consumed before the call returns.
 *  - Any byte count and any alignment gives the result memcpy would give, and
 *    all of them move as 16-byte vectors (work is cut on the 128-byte lines
 *    of each copy's first destination; sources may stand anywhere).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *  - Calls only enqueue work.  In one-shot mode the result is complete when
 *    the stream reaches the end of the enqueued kernel.  In prelaunch mode the
 *    call enqueues an "armed" kernel that waits for dl_trigger() before it
 *    copies (see "prelaunch mode" below); completion is observed with
 *    dl_wait() on the ticket of the call.
 *  - Stream capture: in one-shot mode a request whose lowered list fits the
 *    kernel arguments (at most 64 plain copies, or 32 read-once/write-k copies;
 *    all-gather up to 16 ranks, every broadcast, all-to-all up to 8 ranks)
 *    is exactly one kernel launch and nothing else, so it may be
 *    issued on a stream that is being captured into a HIP graph.  Longer
 *    lists go through table memory that the library reuses (host writes at
 *    call time, events) and must not be captured; neither may prelaunch,
 *    signal or standby mode.
 *  - Where the device exposes all of its memory to the host through a PCIe
 *    BAR, the library writes what its kernels read first (doorbells, the
 *    tables of long lists, standby records) straight into device memory.
 *    With DL_NO_BAR=1 in the environment at dl_init() it keeps all of that in
 *    host-coherent memory, as it does on a device without such a BAR.
 *  - Return value: DL_OK (0) or a negative dl_status.  No exceptions, no
 *    aborts.  On DL_ERR_HIP, dl_last_hip_error() gives the hipError_t.
 *  - Host threads: the library's host state sits behind one lock, which every
 *    entry point takes for the length of the call, so several threads may
 *    issue requests, trigger and wait at once (the waits spin without the
 *    lock).  Mode, tunables and the prelaunch session are process-wide;
 *    dl_last_ticket(), dl_last_mode() and dl_complete() refer to the most
 *    recent request of the CALLING thread.  dl_prelaunch_stop() and
 *    dl_shutdown() must not run while another thread is inside a wait.
 */
#ifndef DMALATTE_H
#define DMALATTE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum dl_status {
    DL_OK = 0,
    DL_ERR_INVALID = -1,  /* null pointer with non-zero bytes, W < 1, k < 1, k > DL_MAX_FANOUT, bad config */
    DL_ERR_OVERLAP = -2,  /* a destination overlaps another destination or a source (validation on) */
    DL_ERR_HIP = -3,      /* a HIP call failed; see dl_last_hip_error() */
    DL_ERR_TIMEOUT = -4,  /* a host-side wait gave up */
    DL_ERR_STATE = -5,    /* not initialised; prelaunch mode not started; started twice; table memory still held by an armed request that has not been triggered */
    DL_ERR_EXPIRED = -6,  /* an armed request was cancelled or not triggered within its arm limit: nothing, or (triggered at the very limit) only part, was copied */
    DL_ERR_LOST = -7,     /* a kernel of an EARLIER request gave up waiting for the copy table that the host had written into device memory, so that request copied nothing or only part; every operation returns this until dl_last_device_error() has been called */
    DL_ERR_CAPACITY = -8  /* the request is larger than the stated maximum of the entry point (dl_batch_copy_static) */
} dl_status;

/* Largest number of destinations of one dl_broadcast call / ranks of a collective. */
#define DL_MAX_FANOUT 64

typedef enum dl_mode {
    DL_MODE_ONESHOT = 0,   /* one kernel launch per call, ordered on `stream` */
    DL_MODE_PRELAUNCH = 1, /* one armed kernel per call, started by dl_trigger() */
    DL_MODE_SIGNAL = 2,    /* one kernel launch per call that starts at once and writes a completion word: the
                              request has a ticket, dl_wait() observes its end without a stream synchronisation */
    DL_MODE_STANDBY = 3,   /* small requests are handed to a kernel that is already waiting on the device: no
                              launch between the call and the copy (see "standby mode" below); the rest run as in
                              DL_MODE_SIGNAL */
    DL_MODE_AUTO = 4       /* the library picks standby, signal or one-shot execution per request from its size
                              (see "size -> mode table" below) */
} dl_mode;

/* One copy of a batch: `bytes` bytes from device pointer src to device pointer dst. */
typedef struct dl_copy_desc {
    const void *src;
    void *dst;
    size_t bytes;
} dl_copy_desc;

/* ------------------------------------------------------------------ lifecycle */

/* Bind the library to HIP device `device` and create its staging ring.  Calling
 * it again for the same device is a no-op; another device needs dl_shutdown()
 * first (DL_ERR_STATE). */
int dl_init(int device);

/* Leave prelaunch mode if it was started, release the staging memory. */
int dl_shutdown(void);

/* Select how the operations are executed.  Every mode but DL_MODE_ONESHOT
 * requires dl_prelaunch_start() first (DL_ERR_STATE otherwise): they use its
 * completion words. */
int dl_set_mode(int mode);
int dl_get_mode(void);

/* Validation of the hazard rule (see dl_batch_copy).  Off by default: it costs
 * O(n log n) on the host.  on = 0 / 1. */
int dl_set_validate(int on);

const char *dl_strerror(int status);
int dl_last_hip_error(void);

/*
 * Failures that only the device can notice.  The table of a long list (more
 * copies than fit the kernel arguments), and the mask of a token dispatch
 * lowered on the device, are written by the host straight into device memory
 * and sealed with a stamp; the kernel looks for the stamp before it reads
 * (the two cross the host link in order, and the launch follows them; paper
 * Sec. III-B2: the engine fetches its commands after the doorbell).  Every
 * such wait is bounded.  A kernel whose stamp never appears copies nothing
 * from then on, ends normally and sets an error word in host memory; the
 * call that launched it has returned DL_OK long before.
 *   dl_last_device_error() returns DL_ERR_LOST if that has happened since
 * it was last called (and clears the word), else DL_OK.  While the word is
 * set, every operation returns DL_ERR_LOST and enqueues nothing.  For an
 * armed request the same case is reported as DL_ERR_EXPIRED by dl_wait().
 *   dl_debug_lose_next_table(tries) is a test hook for this path: the
 * kernel of the next table that is written through the BAR is told a stamp
 * that its slot will never hold and gives up after `tries` (1..1024) looks;
 * tries == 0 takes the hook back.
 * DL_ERR_STATE where no table goes that way (no BAR, dl_config.table_push 0).
 */
int dl_last_device_error(void);
int dl_debug_lose_next_table(uint32_t tries);

/* ----------------------------------------------------------------- operations */

/*
 * Batched back-to-back copies (paper Sec. IV-D; the batched-copy runtime call
 * of Sec. VI).  n independent copies, no ordering among them, one completion
 * for the whole batch; all of them are packed into one grid.
 * Precondition (hazard rule of Sec. IV-D): no destination range overlaps
 * another destination range or any source range.  Sources may overlap each
 * other.  A descriptor with src == dst is a no-op.  With validation on, a
 * violated precondition returns DL_ERR_OVERLAP and nothing is enqueued; with
 * validation off the result of such a batch is undefined.
 * desc: host array of n descriptors.  n == 0 or all bytes == 0: DL_OK, no work.
 */
int dl_batch_copy(const dl_copy_desc *desc, size_t n, void *stream);

/*
 * dl_batch_copy for callers that cannot allocate: code under HIP stream
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * semantics, arguments and hazard rule as dl_batch_copy, with these
 * differences:
 *  - it calls no hipMalloc, no hipFree, no event, memset or other allocating
 *    routine, on the host or the device side, and keeps nothing of the
 *    caller's after it returns;
 *  - the table of the cut list lives in a static device array of
 *    DL_STATIC_MAX_COPIES entries of 24 bytes (384 KiB, held by every GPU the
 *    library runs on until the process ends).  n > DL_STATIC_MAX_COPIES, or a
 *    batch that cannot be cut into that many pieces of at most 1 GiB, returns
 *    DL_ERR_CAPACITY and enqueues nothing;
 *  - it always executes as in DL_MODE_ONESHOT, on `stream`: ceil(entries/64)
 *    small kernels that carry the table to the device in their arguments,
 *    then the table kernel.  No broadcast inference and no hazard check
 *    (dl_set_validate has no effect here);
 *  - all calls on one GPU share the array: calls on one stream are ordered
 *    by the stream; calls that overlap on different streams race and give
 *    undefined results.  Nothing in the array has to start at zero: a call
 *    reads only the entries it wrote itself.
 */
#define DL_STATIC_MAX_COPIES 16384
int dl_batch_copy_static(const dl_copy_desc *desc, size_t n, void *stream);

/*
 * Broadcast (paper Sec. IV-B, generalised from 2 to k destinations): every
 * dsts[d][0..bytes) becomes src[0..bytes).  The source is read once per group
 * of up to 8 destinations and written to each of them from registers.
 * dsts: host array of k device pointers, 1 <= k <= DL_MAX_FANOUT, pairwise
 * disjoint and disjoint from src.
 */
int dl_broadcast(const void *src, void *const *dsts, int k, size_t bytes, void *stream);

/*
 * All-gather over W virtual ranks (paper Sec. II-A1, Fig. 2 left):
 *   out[r][j*B + t] = in[j][t]   for all r, j in [0,W), t in [0,B), B = bytes_per_rank.
 * in, out: host arrays of W device pointers; in[j] has B bytes, out[r] has W*B.
 * Lowered to W read-once/write-W copies.  The in-place layout of the paper is
 * accepted: if in[j] == out[j] + j*B that self-copy is skipped.  Any other
 * overlap between inputs and outputs is a hazard.
 */
int dl_allgather(const void *const *in, void *const *out, int W, size_t bytes_per_rank, void *stream);

/*
 * All-to-all over W virtual ranks (paper Sec. II-A1, Fig. 2 right: the ranks
 * collectively transpose).  chunk_bytes is a host W x W row-major matrix,
 * C[i][j] = chunk_bytes[i*W + j] = bytes rank i sends to rank j (zero allowed).
 * in[i] is packed in destination order and out[j] in source order:
 *   out[j][roff(i,j) + t] = in[i][soff(i,j) + t],  0 <= t < C[i][j],
 *   soff(i,j) = sum of C[i][j'] for j' < j,  roff(i,j) = sum of C[i'][j] for i' < i.
 * Out of place only.
 */
int dl_alltoall(const void *const *in, void *const *out, int W, const size_t *chunk_bytes, void *stream);

/* One swap of a batch: the `bytes` bytes at device pointer a and the `bytes` bytes at b change places. */
typedef struct dl_swap_desc {
    void *a;
    void *b;
    size_t bytes;
} dl_swap_desc;

/*
 * Batch of swaps (paper Sec. IV-C: the swap command exchanges the contents of
 * two memory locations, which otherwise takes a temporary buffer and three
 * copies).  n independent swaps, no ordering among them, one completion; every
 * 16-byte piece is read from both ranges into registers and written back
 * crossed, so there is no temporary.
 * Precondition: all 2n ranges are pairwise disjoint (each is both read and
 * written).  A descriptor with a == b is a no-op.  With validation on, a
 * violated precondition returns DL_ERR_OVERLAP and nothing is enqueued.
 * desc: host array.  n == 0 or all bytes == 0: DL_OK, no work.
 */
int dl_batch_swap(const dl_swap_desc *desc, size_t n, void *stream);

/*
 * In-place all-to-all with equal chunks (paper Sec. IV-C, Fig. 2 right): buf[i]
 * (device, W * chunk_bytes bytes) holds W chunks, chunk j being what rank i
 * sends to rank j.  Afterwards
 *   buf[j][i*c + t] = old buf[i][j*c + t],  c = chunk_bytes,
 * i.e. the result of dl_alltoall with a uniform chunk matrix, written over the
 * inputs.  Lowered to one swap per pair of ranks, W(W-1)/2 in all; the diagonal
 * chunks stay where they are.  buf: host array of W device pointers to
 * pairwise disjoint buffers, 1 <= W <= DL_MAX_FANOUT.
 */
int dl_alltoall_inplace(void *const *buf, int W, size_t chunk_bytes, void *stream);

/* ------------------------------------------------------------- prelaunch mode */

/*
 * Prelaunch (paper Sec. IV-E: copies pre-enqueued behind a poll command and
 * triggered later by a memory write, which takes the launch off the critical
 * path).  In DL_MODE_PRELAUNCH each of the four operations enqueues ONE kernel
 * immediately, on `stream` (NULL = a non-blocking stream owned by the library),
 * and returns; dl_last_ticket() then names the request.  The kernel's
 * workgroups become resident and poll a doorbell word (in device memory that
 * the host writes through the BAR, else in host-coherent memory).
 *   dl_trigger(t)  rings the doorbell for every ticket <= t: one 8-byte store
 *                  (and one more for the host's own copy).
 *                  Everything the request reads must be complete before it.
 *   dl_wait(t, ns) spins on the host until request t has finished: DL_OK,
 *                  DL_ERR_EXPIRED (the request gave up without copying a byte,
 *                  or copied only part, because it was cancelled or waited
 *                  longer than dl_config.arm_timeout_us), or DL_ERR_TIMEOUT
 *                  (the host gave up waiting; ns == 0 polls once).
 *   dl_wait_armed(t, ns) returns once request t's kernel is resident and
 *                  polling (used to time trigger -> completion).
 * Requests on one stream run in ticket order.  The armed kernel occupies its
 * stream until it is triggered, cancelled or expires; later work on that
 * stream waits for it.  At most 64 requests may be armed and unfinished.
 * While it waits, an armed kernel occupies compute units: at most one
 * workgroup for every other compute unit for one request
 * (dl_config.armed_blocks), so that the kernels which produce its inputs can
 * run beside it, also those that cannot share a SIMD with another wavefront
 * (large matrix multiplications; such a kernel still runs slower beside any
 * waiting kernel, because some compute units are closed to it).  Requests
 * armed on different streams are
 * resident together and their workgroups add up: arm large requests on one
 * stream, where they become resident one after the other.
 * A request that moves more than dl_config.armed_chain_min_bytes (256 MiB)
 * is two kernels: a gate of ONE workgroup that does the waiting, and behind
 * it on the same stream the copy kernel with a full grid, which reads what
 * the gate decided (run, or gave up) when it starts.  The small grid of a
 * waiting kernel is what bounds a large copy; this way the request holds one
 * workgroup while it waits and copies at the rate of a kernel that never
 * waited (all-gather of 4 MiB per rank: 49 us after the doorbell instead of
 * 72).
 * A request whose list is too long for the kernel arguments (more than 64
 * plain copies or swaps, 32 read-once/write-k copies) keeps a table in memory
 * that the library reuses in turn: at least 32 such requests may be armed and
 * unfinished if their tables go through the BAR (dl_config.table_push, tables
 * up to 64 KiB, all armed on one stream), 4 otherwise; a call that could get
 * its table memory only by outwaiting a request that has not been triggered
 * returns DL_ERR_STATE at once and arms nothing.
 * Lists too long for one kernel (hundreds of thousands of tiles) are refused
 * with DL_ERR_INVALID in this mode.  An empty request enqueues nothing and
 * takes no ticket.
 *
 * DL_MODE_SIGNAL is the same kernel without the doorbell: it copies as soon as
 * it starts (still in order on its stream), and the last workgroup writes the
 * completion word (the analogue of the sync command that ends a queue of
 * copies, paper Sec. III-B2).  dl_wait() on its ticket returns about 3 us
 * earlier than a stream synchronisation would for the same kernel.
 *
 * Standby mode (DL_MODE_STANDBY) is prelaunch for requests that are not known
 * ahead of time: the library keeps two generic kernels waiting on the device
 * (64 workgroups each, on streams of its own).  A call whose lowered list is
 * short enough (at most 8 read-once/write-k copies, or at most 64 plain
 * copies, and at most 64 tiles of 8 KiB, every copy starting a tile of its
 * own: an all-gather of up to 64 KiB per rank at W = 8, a broadcast of up to
 * 512 KiB, an all-to-all between 8 ranks with chunks of up to 8 KiB, ...;
 * 16 tiles where the device's memory cannot be written by the host through a
 * BAR) writes that list where the waiting kernel will
 * look for it (device memory, through the BAR, or else host-coherent memory)
 * and rings that kernel's doorbell; the kernel reads the list, copies, and
 * reports in the request's completion words.  The call
 * takes a ticket as in signal mode and dl_wait() observes the end; `stream`
 * plays no part, so everything the request reads must be complete before the
 * call, and two requests are ordered only if the first was waited for.  A
 * waiting kernel serves one request and ends; one that has waited 2 ms (or
 * dl_config.arm_timeout_us, if that is shorter) gives up, so after an idle
 * period no kernel of the library is on the device.  Requests that do not
 * fit, or that find no kernel that is sure to be waiting still (fresh ones
 * are armed at once), run as in DL_MODE_SIGNAL.
 *
 * What waiting costs others.  A standby kernel holds its compute units like an
 * armed request does: kernels that can share a SIMD hardly notice, a large
 * matrix multiplication beside it ran a third to a half slower.  And a kernel
 * that waits (an armed request, a standby kernel) holds the hardware queue that its stream is mapped to, and
 * the HIP runtime maps all streams of a process to a few hardware queues
 * (GPU_MAX_HW_QUEUES, 4 by default): work on another stream that shares the
 * queue starts only when the waiting kernel has ended, i.e. after its
 * doorbell or at its limit.  With at most four streams in use (the default
 * stream, the library's, the two of standby mode) every stream has a queue of
 * its own; a process that uses more should raise GPU_MAX_HW_QUEUES, or keep
 * to DL_MODE_SIGNAL, which never waits on the device.
 *
 * dl_prelaunch_start() allocates the doorbell and completion words and the
 * library's stream; dl_prelaunch_stop() cancels whatever is still armed, waits
 * for it to leave the device and releases them.
 */
int dl_prelaunch_start(void);
int dl_prelaunch_stop(void);
uint64_t dl_last_ticket(void); /* ticket of the calling thread's most recent request that took one (prelaunch, signal, standby mode; 0 = none yet in this session) */
int dl_trigger(uint64_t ticket);
int dl_wait(uint64_t ticket, uint64_t timeout_ns);
int dl_wait_armed(uint64_t ticket, uint64_t timeout_ns);

/*
 * Phase stamps of an armed request (the analogue of splitting one copy into
 * schedule, copy and sync with timestamp commands, paper Sec. III-B1/B2).
 * With dl_set_trace(1), every request armed afterwards records four readings of
 * the device's wall clock; dl_get_trace() returns them once dl_wait() has
 * returned for that ticket (and before 64 later requests reuse its slot):
 *   doorbell_seen      the polling workgroup saw the doorbell
 *   copy_begin         the polling workgroup, the first to do so, began to copy
 *   copy_end           the stores of the workgroup that arrived last had completed
 *   completion_issued  the last workgroup was about to write the completion word
 * dl_trace_clock() relates that clock to the host's CLOCK_MONOTONIC by a short
 * ping-pong through host-coherent memory: device tick t happened at about
 * host_ns_at_tick0 + t * 1000 / ticks_per_us nanoseconds (good to half a
 * round trip over the host link, under a microsecond).  Needs prelaunch mode started.
 */
typedef struct dl_trace {
    uint64_t doorbell_seen;
    uint64_t copy_begin;
    uint64_t copy_end;
    uint64_t completion_issued;
} dl_trace;
int dl_set_trace(int on);
int dl_get_trace(uint64_t ticket, dl_trace *out);
int dl_trace_clock(double *ticks_per_us, double *host_ns_at_tick0);

/* --------------------------------------------------------- size -> mode table */

/*
 * Which way of executing a request is fastest depends on its size; the paper
 * tabulates that choice per collective and size for its DMA features (Tables
 * II and III, Sec. V-B).  The table for this library, measured on MI355X
 * (host-observed time from the call, or from the doorbell for an armed
 * request, to completion seen on the host):
 *
 *   request known ahead of time (the caller can arm it and trigger later):
 *     moved bytes <= DL_AUTO_PRELAUNCH_MAX_BYTES            DL_MODE_PRELAUNCH
 *     larger                                                DL_MODE_ONESHOT
 *   request known only when it is issued:
 *     fits a waiting kernel: at most DL_AUTO_STANDBY_TILES tiles of 8 KiB and
 *     at most 8 items (64 if every item has one destination), not a swap,
 *     not a token dispatch                                  DL_MODE_STANDBY
 *     else moved bytes <= DL_AUTO_SIGNAL_MAX_BYTES          DL_MODE_SIGNAL
 *     larger                                                DL_MODE_ONESHOT
 *     (a token dispatch of 512 tokens or more: DL_MODE_ONESHOT, where the
 *     device derives the copies from the mask)
 *
 * "moved bytes" are the algorithmic bytes read plus written (an all-gather of
 * B bytes per rank over W ranks: (W + W*W) * B); a tile count is what
 * dl_plan_tiles() gives for 8192-byte tiles.  The large requests go one-shot
 * because the kernels of the other modes load and store at system scope and
 * wait on a capped grid, which costs bandwidth once the copy dominates.
 *
 * dl_plan_mode() is that table as a host-only function (no GPU needed).
 * op: a dl_op; items and max_fanout: length of the lowered list and the most
 * destinations any item has (what the dl_plan_* functions return); tiles:
 * dl_plan_tiles(items, n, 8192); known_ahead: 0 / 1.  Returns a dl_mode, or
 * DL_ERR_INVALID.
 *
 * In DL_MODE_AUTO (needs dl_prelaunch_start(), keeps the standby kernels
 * waiting like DL_MODE_STANDBY) every operation applies the table with
 * known_ahead = 0 to its own lowered list.  Because the request may be handed
 * to a waiting kernel, which is not ordered on `stream`, everything it reads
 * must be complete before the call, as in standby mode.  dl_last_mode() tells
 * how the most recent request was executed (a request that the table sends to
 * standby but that no waiting kernel could take runs as DL_MODE_SIGNAL), and
 * dl_complete(stream, ns) waits for it in the way that fits: a stream
 * synchronisation after one-shot execution, dl_wait() on its ticket
 * otherwise.
 */
typedef enum dl_op {
    DL_OP_BATCH = 0,
    DL_OP_BROADCAST = 1,
    DL_OP_ALLGATHER = 2,
    DL_OP_ALLTOALL = 3,
    DL_OP_SWAP = 4,           /* dl_batch_swap, dl_alltoall_inplace */
    DL_OP_TOKEN_DISPATCH = 5
} dl_op;
#define DL_AUTO_STANDBY_TILES 64
#define DL_AUTO_SIGNAL_MAX_BYTES (288ull << 20)     /* an all-gather of 4 MiB per rank over 8 ranks */
#define DL_AUTO_PRELAUNCH_MAX_BYTES (288ull << 20)  /* an all-gather of 4 MiB per rank over 8 ranks */
int dl_plan_mode(int op, size_t items, uint32_t max_fanout, uint64_t moved_bytes, uint64_t tiles, int known_ahead);
int dl_last_mode(void);
int dl_complete(void *stream, uint64_t timeout_ns);

/* -------------------------------------------------------------------- tunables */

typedef struct dl_config {
    uint32_t tile_bytes;         /* bytes of one workgroup tile; 0 = choose from the fan-out; power of two >= 1024 */
    uint32_t block_threads;      /* workgroup size of the one-shot kernel: 64, 128, 256 or 512; 0 = choose */
    uint64_t nontemporal_min_bytes; /* requests moving at least this many bytes use streaming loads/stores; default: never */
    uint32_t armed_blocks;       /* cap on the grid of an armed kernel (its workgroups stride over the tiles); 0 = half as many as the GPU has compute units, so that the kernels that produce the request's inputs can run beside it */
    uint32_t arm_timeout_us;     /* an armed kernel gives up this long after becoming resident; 1 .. 1000000, default 20000 */
    uint32_t fuse_broadcast;     /* 1: all-gather reads each source once (W fused copies); 0: W*W plain copies */
    uint32_t max_blocks;         /* cap on the one-shot grid; workgroups then stride over the tiles; 0 = one workgroup per tile */
    uint32_t fan_split;          /* sub-groups of a workgroup that share out the destinations of a fused copy: 1, 2 or 4; 0 = choose */
    uint32_t infer_broadcast;    /* 1: dl_batch_copy merges copies that share source and size into read-once/write-k copies; default 1 */
    uint32_t device_lowering;    /* 1: dl_token_dispatch with 512 tokens or more (W = 8, one-shot mode, validation off) sends only the mask to the device, which derives the copies itself; default 1 */
    uint32_t table_push;         /* 1: the table of a long list (more copies than fit the kernel arguments) is written by the host straight into device memory, through the BAR, when the device exposes one that covers its memory and the table is short enough; 0: always through pinned host memory; default 1 */
    uint64_t write_through_max_bytes; /* requests moving at most this many bytes (read + written) use write-through stores; default 144 MiB */
    uint64_t stream_plain_min_bytes;  /* lists of plain 1:1 copies (all-to-all, batches) moving at least this many bytes use streaming loads/stores: nothing of such a request fits the on-die caches, and keeping it out of them measured 3-6 % faster; default 512 MiB; UINT64_MAX = never */
    uint64_t armed_chain_min_bytes;   /* prelaunch mode: a request moving more than this many bytes waits in a one-workgroup gate kernel and copies with a full-grid kernel enqueued behind it, instead of waiting and copying with one capped grid; ignored when armed_blocks is set; default 256 MiB */
} dl_config;

int dl_get_config(dl_config *cfg);
int dl_set_config(const dl_config *cfg);

/* Host-only: apply "name=value,name=value" (names as in dl_config, values as
 * C integer literals) to *cfg.  Unknown names, malformed values and settings
 * that dl_set_config would refuse return DL_ERR_INVALID and leave *cfg as it
 * was.  dl_init() applies the environment variable DL_CONFIG this way on top
 * of the defaults (and fails with DL_ERR_INVALID if it does not parse). */
int dl_parse_config(const char *text, dl_config *cfg);

/* -------------------------------------------------- lowering, for inspection */

/* One lowered copy: read `bytes` at src once, write them to k destinations. */
#define DL_PLAN_FANOUT 8
typedef struct dl_plan_item {
    const void *src;
    size_t bytes;
    uint32_t k;
    uint32_t reserved;
    void *dst[DL_PLAN_FANOUT];
} dl_plan_item;

/*
 * Batch of read-once/write-many copies (paper Sec. IV-B generalised, and the
 * broadcast form of the batched runtime call of Sec. VI): item i reads
 * items[i].bytes bytes at items[i].src once and writes them to its
 * items[i].k destinations, 1 <= k <= DL_PLAN_FANOUT.  Independent and unordered
 * like dl_batch_copy, same hazard rule, one completion.  items: host array.
 */
int dl_batch_fanout(const dl_plan_item *items, size_t n, void *stream);

/*
 * Token dispatch of an expert-parallel mixture-of-experts layer (paper
 * Sec. II-A1: ranks exchange tokens by expert preference; Sec. IV-B: a token
 * sent to several experts is one source with several destinations).
 * in[i] (device) holds tokens[i] rows of row_bytes bytes.  dest (host) has one
 * byte per (token, rank), tokens numbered over all ranks in rank order:
 * dest[g*W + j] != 0 sends token g to rank j.  out[j] (device) receives its
 * rows packed in token order (source rank first, then row index), so it must
 * hold row_bytes times the number of non-zero entries in column j of dest.
 * Lowered to one read-once/write-k copy per token; a token with no destination
 * moves nothing.  tokens: host array of W counts.  1 <= W <= DL_MAX_FANOUT.
 * The lowering runs on the host, or (dl_config.device_lowering, many tokens) on
 * the device from the mask alone; the result is the same.
 */
int dl_token_dispatch(const void *const *in, void *const *out, int W, const uint32_t *tokens, size_t row_bytes,
                      const uint8_t *dest, void *stream);

/*
 * dl_token_dispatch with the routing mask in DEVICE memory, where the router
 * kernel of a mixture-of-experts layer leaves it: same layout (one byte per
 * (token, rank), non-zero = send), same result, but dest_device is a device
 * pointer (8-byte aligned) and nothing of the mask crosses the host link: the
 * device counts, builds the copy list and executes it, three launches on
 * `stream`, ordered behind whatever produced the mask there.  Always executed
 * as in DL_MODE_ONESHOT.  The host does not learn how many rows each rank
 * receives: out[j] must have room for what the mask sends it (at most all
 * tokens).  Rows and buffers may have any length and alignment.  Limits:
 * exactly 8 ranks (DL_ERR_INVALID otherwise); at most
 * DL_DISPATCH_DEVICE_MAX_TOKENS tokens in all (one slot of the library's table
 * memory holds their copy list; more: DL_ERR_CAPACITY, nothing is enqueued).
 */
#define DL_DISPATCH_DEVICE_MAX_TOKENS 10240
int dl_token_dispatch_device(const void *const *in, void *const *out, int W, const uint32_t *tokens, size_t row_bytes,
                             const uint8_t *dest_device, void *stream);

/*
 * Host-only: lower a collective to the list of copies the device executes
 * (the analogue of building the command list, paper Sec. III-B2 "control").
 * Pointers are treated as opaque addresses and never dereferenced, so these
 * work without a GPU.  Writes at most `cap` items to `items` (may be NULL when
 * cap == 0) and returns the number of items the request lowers to, or a
 * negative dl_status.
 */
long dl_plan_allgather(const void *const *in, void *const *out, int W, size_t bytes_per_rank,
                       int fuse_broadcast, dl_plan_item *items, size_t cap);
long dl_plan_alltoall(const void *const *in, void *const *out, int W, const size_t *chunk_bytes,
                      dl_plan_item *items, size_t cap);
long dl_plan_broadcast(const void *src, void *const *dsts, int k, size_t bytes,
                       dl_plan_item *items, size_t cap);
long dl_plan_batch(const dl_copy_desc *desc, size_t n, dl_plan_item *items, size_t cap);
long dl_plan_token_dispatch(const void *const *in, void *const *out, int W, const uint32_t *tokens, size_t row_bytes,
                            const uint8_t *dest, dl_plan_item *items, size_t cap);

/* Host-only: what dl_batch_copy does with a batch when dl_config.infer_broadcast
 * is on (paper Sec. VI: the runtime inspects a batch and turns copies with the
 * same source and the same size into a broadcast): copies that share source
 * address and byte count are merged into read-once/write-k items, up to
 * DL_PLAN_FANOUT destinations each, in order of first appearance. */
long dl_plan_batch_inferred(const dl_copy_desc *desc, size_t n, dl_plan_item *items, size_t cap);

/* Host-only: index of the first item whose destination overlaps another
 * destination or any source (the hazard rule), or -1 if there is none. */
long dl_plan_first_hazard(const dl_plan_item *items, size_t n);

/* Host-only: the swaps an in-place all-to-all lowers to (at most `cap` written;
 * returns their number, or a negative dl_status). */
long dl_plan_alltoall_inplace(void *const *buf, int W, size_t chunk_bytes, dl_swap_desc *swaps, size_t cap);

/* Host-only: index of the first swap one of whose ranges overlaps another range
 * of the batch (its own other range included), or -1 if there is none. */
long dl_plan_swap_first_hazard(const dl_swap_desc *swaps, size_t n);

/* Host-only: number of workgroup tiles the item list is cut into for a given
 * tile size, a multiple of 128 (the grid of the one-shot launch).  Tiles lie on
 * the grid of tile_bytes of each item's first destination: an item whose first
 * destination stands s bytes behind a 128-byte boundary takes
 * ceil((bytes + s) / tile_bytes) tiles. */
uint64_t dl_plan_tiles(const dl_plan_item *items, size_t n, uint32_t tile_bytes);

#ifdef __cplusplus
}
#endif
#endif /* DMALATTE_H */
