// Internal declarations shared by the library's translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "../../include/dmalatte.h"
#include "dl_work.h"

// One lock around the library's host state: every entry point that reads or changes it takes the lock for
// the length of the call (lowering and launch: microseconds), so several host threads may drive the library.
// The waits (dl_wait, dl_wait_armed, dl_complete) look their words up under the lock and spin without it.
// Recursive, because entry points call each other.
extern std::recursive_mutex g_dl_lock;
#define DL_LOCKED std::lock_guard<std::recursive_mutex> dl_lock_guard_(g_dl_lock)

// What "the most recent request" means to a caller: the most recent one of the calling thread.
struct dl_thread_last {
    uint64_t session = 0;  // the prelaunch session the ticket belongs to
    uint64_t ticket = 0;
    int mode = DL_MODE_ONESHOT;
};
extern thread_local dl_thread_last t_dl_last;

// Library state (one device).
struct dl_state {
    bool inited = false;
    int device = -1;
    int num_cu = 0;
    int mode = DL_MODE_ONESHOT;       // as set by the caller
    int validate = 0;
    int last_hip = 0;
    int trace = 0;  // armed kernels record phase stamps
    uint32_t armed_words = 0;  // completion words the armed kernel launched last reports in (see dl_arm::own_word)
    dl_config cfg{};
};
extern dl_state g_dl;

#define DL_HIP(call)                                  \
    do {                                              \
        hipError_t e_ = (call);                       \
        if (e_ != hipSuccess) {                       \
            g_dl.last_hip = (int)e_;                  \
            (void)hipGetLastError();                  \
            return DL_ERR_HIP;                        \
        }                                             \
    } while (0)

// Launch geometry chosen on the host for one request.
struct dl_launch_shape {
    uint32_t tile_bytes;
    uint32_t block_threads;
    uint32_t split;       // sub-groups of a workgroup sharing out the destinations of a fused item: 1, 2 or 4
    uint32_t max_blocks;  // 0 = one workgroup per tile
    int policy;           // cache policy of the copy loop (DL_POL_*)
    bool rows = false;    // the list qualifies for the row path of the list kernels
    bool chain = false;   // prelaunch mode, a large request: a one-workgroup gate kernel waits, the copy kernel follows it on the stream
    uint32_t rows2d_width = 0;  // row path on a two-dimensional grid (item by item), this many tiles wide; 0: one-dimensional
};

// What an armed (prelaunched) kernel needs to wait for its doorbell and to
// report completion.  Passed by value in the kernel arguments.
struct dl_arm {
    const uint64_t *bell;  // bell[0] = doorbell, bell[1] = cancel; both only ever grow.  Host-coherent memory, or device memory that the host writes through the BAR
    uint64_t *done;        // host-coherent: completion word of this ticket's slot
    uint64_t *armed;       // host-coherent: "resident and polling" word of this ticket's slot
    uint64_t *go;          // device: fan-out flags of this ticket's slot, one per group, DL_ARM_STRIDE bytes apart
    uint32_t *arrive;      // device: arrival counters of this slot: one per group, then the top one, same spacing
    // A slot has two sets of counters, used by its requests in turn.  A request leaves its set as counted
    // (no reset on the way to the completion word) and clears the other one before it waits: that set's last
    // user has finished, and its next user is armed only after this request has.
    uint32_t *arrive_clear;
    uint64_t ticket;
    uint64_t limit_ticks;   // give up this long after becoming resident
    uint64_t margin_ticks;  // extra time a non-polling workgroup grants the polling one
    uint32_t direct;        // 1: every workgroup polls the doorbell itself
    uint32_t direct_max;    // grids up to this many workgroups do so (more where the doorbell is in device memory: polls there do not queue up on the host link)
    uint32_t max_spins;     // backstop that does not depend on the clock: give up after this many polls
    uint32_t nowait;        // 1: no doorbell, copy at once (DL_MODE_SIGNAL, and what DL_MODE_STANDBY cannot hand to an executor); the completion side is unchanged
    // 1: a grid of at most DL_DONE_WORDS workgroups, each of which reports in a completion word of its own
    // (done[blockIdx.x]) as soon as its stores have drained: no arrival count on the way to the host, which
    // waits for all of the grid's words.  0: arrivals are counted and the last workgroup writes done[0].
    uint32_t own_word;
    // 1 (with nowait): the kernel runs behind a gate kernel on the same stream, which did the waiting with a single
    // workgroup and left (ticket << 2 | go) in go[0]; this kernel copies only if that says "run" for its ticket.
    uint32_t gated;
    // Phase stamps (device wall-clock ticks), null unless tracing is on: host-coherent, 4 words: doorbell seen,
    // first copy begins (the polling workgroup's), last copy ends (the last arriver's), completion issued
    uint64_t *trace_host;
};
constexpr uint32_t DL_DONE_WORDS = 16;  // completion words per slot (two cache lines of host memory); with 32 or 64 words the host-side wait cost more than the count on the device
constexpr uint32_t DL_ARM_DIRECT_MAX_HOST = 16;    // grids up to this size poll a doorbell in host memory themselves
constexpr uint32_t DL_ARM_DIRECT_MAX_DEVICE = 1024;  // ... and one in device memory
constexpr uint32_t DL_ARM_GROUPS = 16;  // workgroup b belongs to group b % DL_ARM_GROUPS
constexpr uint32_t DL_ARM_FLAT_MAX = 64;  // grids up to this size count their arrivals at one word (0.5 us less than two levels; 256 arrivals at one word: 1.3 us more)
constexpr uint32_t DL_ARM_STRIDE = 4352;  // flags and counters sit 4 KiB + 256 B apart: separate lines and memory channels
constexpr uint64_t DL_DONE_SKIPPED = 1ull << 63;  // set in the completion word when nothing was copied

// dl_exec.hip: execution of a lowered list on a stream.  With arm == nullptr one
// kernel launch per call (more for very long lists).  With arm != nullptr the
// launch is an armed kernel: its workgroups first wait for the doorbell.
// *launched tells whether a kernel was enqueued (empty requests enqueue none).
int dl_exec_plain(const dl_plain_item *items, size_t n, hipStream_t stream, const dl_arm *arm, bool *launched);
int dl_exec_fused(const dl_fused_item *items, size_t n, hipStream_t stream, const dl_arm *arm, bool *launched);
int dl_exec_swap(const dl_swap_item *items, size_t n, hipStream_t stream, const dl_arm *arm, bool *launched);
int dl_exec_init();
int dl_exec_shutdown();
dl_launch_shape dl_choose_shape(uint64_t src_bytes, uint64_t max_item_bytes, uint32_t max_k);

// Shape of the row kernel over a table of read-once/write-k items in device memory: sub-groups per
// 1 KiB row (each stores to DL_FAN / split destinations) and threads per workgroup.
constexpr uint32_t DL_TABLE_ROWS_SPLIT = 2;
constexpr uint32_t DL_TABLE_ROWS_THREADS = 128;

// dl_exec.hip: the staging ring (pinned host slots of DL_RING_SLOT_BYTES, each with a device mirror).
//   dl_ring_acquire  waits until the next slot's previous user has finished on the device
//   dl_ring_stage    enqueues a copy of the first `bytes` (a multiple of 16) of the host slot to its mirror
//   dl_ring_release  marks the slot as in use until everything enqueued on `stream` so far has finished
constexpr size_t DL_RING_SLOT_BYTES = 1u << 20;
int dl_ring_acquire(size_t *slot, char **host, char **dev);
int dl_ring_stage(size_t slot, uint64_t bytes, hipStream_t stream);
int dl_ring_release(size_t slot, hipStream_t stream);
// dl_exec.hip: short tables written by the host straight into device memory (through the BAR).
//   dl_push_acquire  a slot for `bytes` (at most DL_PUSH_PAYLOAD_BYTES) that a kernel launched on `stream` next
//                    will read, or null if that way is not open (no such BAR, switched off, too long);
//                    *rc != DL_OK on an error.  Write only.
//   dl_push_seal     after the last write: fences, writes the slot's stamp behind the payload, fences again, and
//                    returns the stamp.  The kernel gets the stamp as an argument and reads the payload, past the
//                    caches, only once it sees the stamp (dl_pushed_sealed in dl_device.h): writes that cross the
//                    link arrive in order, so the stamp vouches for what was written before it.
//   dl_push_commit   after the launch, with its stream
//   dl_ring_forget_armed  every armed request has finished (their tickets start over with the next session)
//   dl_ring_own_stream  the library's own stream for armed requests exists (or, null, is about to be destroyed):
//                    the one stream besides the default stream that cannot go away between two calls
//   dl_push_kernel_args  what the kernel that reads the slot gets: the stamp, how often to look for it, where to
//                    report that it never came (stamp 0: a kernel whose table did not go this way)
//   dl_device_error_pending  a kernel has reported such a loss and dl_last_device_error() has not been called since
uint64_t dl_push_seal(char *slot);
dl_pushed dl_push_kernel_args(uint64_t stamp);
bool dl_device_error_pending();
void dl_ring_forget_armed();
void dl_ring_own_stream(hipStream_t stream);
char *dl_push_acquire(size_t bytes, hipStream_t stream, int *rc);
int dl_push_commit(hipStream_t stream);

// dl_exec.hip: the row kernel over a table of n equally sized read-once/write-k items that is already in
// device memory, destinations laid out for DL_TABLE_ROWS_SPLIT sub-groups (see slots_by_subgroup).  max_shift: no
// item's first destination lies further than this behind a DL_CUT boundary (0: they all stand on one); every item
// gets the workgroups that the worst position allowed by it needs.  on_grid: every item lies as the on-grid
// instance of the row kernel wants it (see dl_rows_body).
int dl_launch_fused_rows_table(const dl_fused_item *dev_items, uint32_t n, uint64_t item_bytes, uint32_t max_shift,
                               bool on_grid, hipStream_t stream);

// dl_exec.hip: the table kernel over m plain copies of at most entry_bytes (< 2^32) each that are already in device
// memory (entry b is workgroup b's), with the cache policy that suits `moved` bytes read + written.
int dl_launch_plain_table(const dl_plain_item *dev_items, uint32_t m, uint32_t entry_bytes, uint64_t moved, hipStream_t stream);

// dl_static.hip: the address of this device's copy of the static table (dl_batch_copy_static).
int dl_static_init(int device);

// dl_dispatch.hip: token dispatch lowered on the device (the destination mask is scanned into a table of
// read-once/write-k items in device memory, which the row kernel then executes).  *taken says whether the request qualified; if not,
// nothing was enqueued and the caller lowers on the host.
int dl_dispatch_on_device(const void *const *in, void *const *out, int W, const uint32_t *tokens, size_t row_bytes,
                          const uint8_t *dest, hipStream_t stream, bool *taken);

// Standby executors (DL_MODE_STANDBY): armed kernels that wait, not for a request that is known already, but for
// any small request.  The host writes the request's copy list into a record (in device memory, through the BAR,
// where the device has one that covers its memory; else in host-coherent memory) and rings the executor's own
// doorbell, which sits behind the record; the executor reads the record, copies, and reports in the request's completion
// words like a small armed grid does (one word per workgroup).  An executor serves one request and ends; the
// library keeps DL_STANDBY_POOL of them armed, each on a stream of its own.
constexpr int DL_STANDBY_POOL = 2;
constexpr uint32_t DL_STANDBY_GRID = 64;      // workgroups of an executor: the most tiles a request may have
constexpr uint32_t DL_STANDBY_THREADS = 512;
constexpr uint32_t DL_STANDBY_TILE = 8192;     // one 1 KiB row per wavefront
constexpr size_t DL_STANDBY_REC_BYTES = 2048;  // room for the record
constexpr uint32_t DL_STANDBY_IDLE_US = 2000;  // an executor that has waited this long gives up (or the arm limit, if shorter)
// dl_exec.hip: write the record of a request that fits an executor (at most 8 items, or at most 64 that are all
// plain copies, and max_tiles tiles; default tunables) and return the number of completion words it will report in (one per tile up to DL_DONE_WORDS tiles,
// else one, counted at the record, which must then be in device memory); 0 if it does not fit.  Launch an
// executor that will read that record.  arrive_clear: the counter set of the ticket's slot that the request is
// to clear (see dl_arm).
uint32_t dl_standby_fill(void *rec_mem, const dl_plan_item *items, size_t n, uint64_t activation, uint64_t ticket,
                         uint64_t *done, uint32_t *arrive_clear, uint32_t max_tiles);
int dl_standby_launch(void *rec_mem, const dl_arm *a, hipStream_t stream);
// dl_prelaunch.hip: hand the request to a waiting executor if it fits and one is fresh; *taken says whether.
int dl_standby_try(const dl_plan_item *items, size_t n, bool *taken);
int dl_standby_enter();  // arm the pool
int dl_standby_leave();  // cancel what is armed and wait until it has left the device

// dl_exec.hip: `bytes` of zeroed device memory that the host can store into through the BAR (null where the
// device does not expose all of its memory that way); never freed.
void *dl_bar_memory(size_t bytes);

// dl_prelaunch.hip: tickets, doorbell and completion words of armed requests.
bool dl_armed_ready();
bool dl_armed_untriggered(uint64_t ticket);  // armed, neither triggered nor cancelled, and not finished
int dl_armed_begin(dl_arm *arm, hipStream_t *stream);  // next ticket's words; picks the library stream if *stream is null
void dl_armed_commit(uint32_t done_words);             // the ticket of the last dl_armed_begin was launched and reports in that many words
