// Prelaunched ("armed") requests: tickets, the doorbell and the completion
// words (Sec. IV-E: copies pre-enqueued behind a poll, triggered later by a
// plain memory write, so that the launch is off the critical path).
//
// Each request issued in prelaunch mode is its own kernel, enqueued at once on
// the caller's stream (or the library's non-blocking stream).  Its workgroups
// poll the doorbell (in device memory that the host writes through the BAR,
// else in host-coherent memory) until it reaches the request's ticket, copy,
// and report in the request's completion words, in host-coherent memory: each
// workgroup in a word of its own if they are few, else the last one to finish
// in one word.  dl_trigger() is one 8-byte store (two where the doorbell has a
// copy on the device); dl_wait() spins on the completion words.
//
// A wave never lives longer than the arm limit (plus the copy itself): a
// request that is not triggered in time gives up without copying and reports
// that.  Nothing stays resident between requests, except in standby mode, where
// two generic kernels wait for whatever small request comes next (2 ms at most).
#include "dl_internal.h"

#include <immintrin.h>
#include <string.h>
#include <time.h>

namespace {

constexpr uint32_t SLOTS = 64;  // requests that may be armed and not yet completed

struct arm_host {  // pinned, host-coherent
    uint64_t bell;    // host -> device: every ticket <= bell may run
    uint64_t cancel;  // host -> device: every ticket <= cancel gives up
    uint64_t pad[6];
    // device -> host: ticket (| DL_DONE_SKIPPED) of the last request finished in the slot; a request reports
    // in word 0 or, if its grid is small, in one word per workgroup (arm_state::words)
    uint64_t done[SLOTS][DL_DONE_WORDS];
    uint64_t armed[SLOTS];  // device -> host: ticket of the last request seen resident in the slot
    uint64_t trace[SLOTS][4];  // device -> host, when tracing: phase stamps of the slot's last request (device ticks)
    uint64_t ping[2];       // clock calibration: host -> device round number, device -> host its clock at that round
    // standby executors, per pool slot: {doorbell = activation number, cancel} side by side, the "resident" word,
    // and the record the executor reads after its doorbell
    uint64_t sb_bell[DL_STANDBY_POOL][2];
    uint64_t sb_resident[DL_STANDBY_POOL];
    uint64_t sb_pad[8 - (DL_STANDBY_POOL % 8)];
    alignas(16) uint8_t sb_rec[DL_STANDBY_POOL][DL_STANDBY_REC_BYTES];
};
static_assert(offsetof(arm_host, sb_bell) % 16 == 0 && offsetof(arm_host, sb_rec) % 16 == 0, "16-byte loads");

struct arm_dev {  // device memory; every flag and counter in a cache line of its own
    uint8_t go[SLOTS][DL_ARM_GROUPS * DL_ARM_STRIDE];
    uint8_t arrive[SLOTS][2][(DL_ARM_GROUPS + 1) * DL_ARM_STRIDE];  // two sets per slot, see dl_arm
    uint8_t sb_go[DL_STANDBY_POOL][DL_ARM_GROUPS * DL_ARM_STRIDE];  // fan-out flags of the standby executors
};

struct arm_state {
    bool started = false;
    arm_host *host = nullptr;
    arm_dev *dev = nullptr;
    hipStream_t stream = nullptr;
    uint64_t seq = 0;  // last ticket issued
    uint64_t session = 0;  // which prelaunch session this is (tickets start over with each)
    uint32_t words[SLOTS] = {};  // completion words that the slot's current request reports in
    // standby pool: a stream per executor, when the executor armed last was armed, the ticket the slot served
    // last, and the slot that takes the next request
    bool standby = false;
    hipStream_t sb_stream[DL_STANDBY_POOL] = {};
    uint64_t sb_armed_at[DL_STANDBY_POOL] = {};
    uint64_t sb_limit_ns[DL_STANDBY_POOL] = {};  // the arm limit that executor was given
    uint64_t sb_ticket[DL_STANDBY_POOL] = {};
    int sb_next = 0;
    uint64_t clock_khz = 100000;
} g_arm;

uint64_t now_ns()
{
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
}

inline uint64_t load_word(const uint64_t *p) { return __atomic_load_n(p, __ATOMIC_ACQUIRE); }

// Spin until each of the `count` words holds `ticket` or a later one (slots are reused in ticket
// order).  *seen: the ticket, with DL_DONE_SKIPPED if any of the words that hold exactly it says so.
int wait_words(const uint64_t *words, uint32_t count, uint64_t ticket, uint64_t timeout_ns, uint64_t *seen)
{
    const uint64_t t0 = now_ns();
    uint32_t have = 0;  // words 0 .. have-1 have been seen complete
    uint64_t skipped = 0;
    for (uint32_t spins = 1;; ++spins) {
        while (have < count) {
            const uint64_t v = load_word(words + have);
            if ((v & ~DL_DONE_SKIPPED) < ticket) break;
            if ((v & ~DL_DONE_SKIPPED) == ticket) skipped |= v & DL_DONE_SKIPPED;
            ++have;
        }
        if (have == count) {
            if (seen) *seen = ticket | skipped;
            return DL_OK;
        }
        if (timeout_ns == 0) return DL_ERR_TIMEOUT;
        _mm_pause();
        if ((spins & 63u) == 0 && now_ns() - t0 >= timeout_ns) return DL_ERR_TIMEOUT;
    }
}

int wait_word(const uint64_t *word, uint64_t ticket, uint64_t timeout_ns, uint64_t *seen)
{
    return wait_words(word, 1, ticket, timeout_ns, seen);
}

// Completion of request `ticket`, which must be one of the last SLOTS issued.
int wait_done(uint64_t ticket, uint64_t timeout_ns, uint64_t *seen)
{
    const uint32_t slot = (uint32_t)(ticket % SLOTS);
    return wait_words(g_arm.host->done[slot], g_arm.words[slot] ? g_arm.words[slot] : 1u, ticket, timeout_ns, seen);
}

// Upper bound, in ns, on how long an armed kernel can still be on the device
// once it has started: arm limit + margin + slack for the copy.
// limits of a kernel that is armed now
void arm_limits(dl_arm *arm, uint32_t limit_us)
{
    arm->limit_ticks = (uint64_t)limit_us * g_arm.clock_khz / 1000ull;
    arm->margin_ticks = 5000ull * g_arm.clock_khz / 1000ull;  // 5 ms
    // a poll takes well over 100 ns (a host-link round trip, or a sleep plus a device-memory load)
    arm->max_spins = (limit_us + 5000u) * 10u;
}

uint64_t drain_ns() { return ((uint64_t)g_dl.cfg.arm_timeout_us + 5000ull) * 1000ull + 2000000000ull; }

}  // namespace

bool dl_armed_ready() { return g_arm.started; }

bool dl_armed_untriggered(uint64_t ticket)
{
    if (!g_arm.started || ticket == 0 || ticket > g_arm.seq || g_arm.seq - ticket >= SLOTS) return false;
    if (ticket <= load_word(&g_arm.host->bell) || ticket <= load_word(&g_arm.host->cancel)) return false;
    return wait_done(ticket, 0, nullptr) != DL_OK;
}

namespace {

// The doorbell pair {doorbell, cancel} of armed requests in device memory, where the host can store there through
// the BAR (made once per process, never freed; set to zero at the start of every session, before anything is
// armed).  The pair in host memory is kept up to date as well: the host reads its own doorbell there.
uint64_t *g_bell_dev = nullptr;
int g_bell_dev_device = -1;  // the device it was made for (what was made for another device is left behind)

void bell_store(uint64_t *host_word, uint64_t *dev_word, uint64_t v)
{
    __atomic_store_n(host_word, v, __ATOMIC_RELEASE);
    if (dev_word) {
        _mm_sfence();
        *(volatile uint64_t *)dev_word = v;
        _mm_sfence();
    }
}

}  // namespace

int dl_armed_begin(dl_arm *arm, hipStream_t *stream)
{
    if (!g_arm.started) return DL_ERR_STATE;
    const uint64_t ticket = g_arm.seq + 1;
    const uint32_t slot = (uint32_t)(ticket % SLOTS);
    if (ticket > SLOTS) {
        // the slot's previous request must have left the device before its words are reused
        const int rc = wait_done(ticket - SLOTS, drain_ns(), nullptr);
        if (rc != DL_OK) return rc;
    }
    arm->bell = g_bell_dev ? g_bell_dev : &g_arm.host->bell;
    arm->direct_max = g_bell_dev ? DL_ARM_DIRECT_MAX_DEVICE : DL_ARM_DIRECT_MAX_HOST;
    arm->done = g_arm.host->done[slot];
    arm->own_word = 0;
    arm->gated = 0;
    arm->armed = &g_arm.host->armed[slot];
    arm->go = (uint64_t *)g_arm.dev->go[slot];
    const uint32_t set = (uint32_t)(ticket / SLOTS) & 1u;
    arm->arrive = (uint32_t *)g_arm.dev->arrive[slot][set];
    arm->arrive_clear = (uint32_t *)g_arm.dev->arrive[slot][set ^ 1u];
    arm->ticket = ticket;
    arm_limits(arm, g_dl.cfg.arm_timeout_us);
    arm->direct = 0;
    arm->nowait = g_dl.mode == DL_MODE_PRELAUNCH ? 0u : 1u;  // signal mode, and what standby mode launches itself
    arm->trace_host = g_dl.trace ? g_arm.host->trace[slot] : nullptr;
    if (!*stream) *stream = g_arm.stream;
    return DL_OK;
}

namespace {

// Where the records live.  With a large BAR the host can store into device memory: the record is pushed there
// (posted writes, which the link delivers before the completion of the read that shows the executor its
// doorbell), and the executor finds it in device memory instead of fetching it over the link (1 us less).  The
// allocation is made once per process and never freed.  Without a large BAR the records stay in host memory.
uint8_t *g_sb_rec_dev = nullptr;
int g_sb_rec_dev_device = -1;  // the device it was made for
constexpr size_t SB_DEV_STRIDE = 2 * DL_STANDBY_REC_BYTES;  // per pool slot: the record, then {doorbell, cancel}

// Activation number of the executor armed last in each pool slot (0: none yet).  It only ever grows, over the
// whole life of the process, because the doorbells in device memory outlive a prelaunch session.
uint64_t g_sb_act[DL_STANDBY_POOL] = {};

void *standby_rec(int e)
{
    if (g_sb_rec_dev) return g_sb_rec_dev + (size_t)e * SB_DEV_STRIDE;
    return g_arm.host->sb_rec[e];
}

// The executor's {doorbell, cancel} pair.  With the records in device memory the doorbell is there too, behind
// its record: the two are posted writes on one path, so whoever sees the doorbell finds the record.  (A doorbell
// in host memory would be seen through a read completion, which the host's writes to the device need not precede.)
uint64_t *standby_bell(int e)
{
    if (g_sb_rec_dev) return (uint64_t *)(g_sb_rec_dev + (size_t)e * SB_DEV_STRIDE + DL_STANDBY_REC_BYTES);
    return g_arm.host->sb_bell[e];
}

void standby_store(uint64_t *word, uint64_t v)
{
    if (g_sb_rec_dev) {
        _mm_sfence();  // everything written to the device so far leaves first
        *(volatile uint64_t *)word = v;
        _mm_sfence();
    } else {
        __atomic_store_n(word, v, __ATOMIC_RELEASE);
    }
}

void standby_place_records()
{
    if (g_sb_rec_dev_device == g_dl.device) return;
    g_sb_rec_dev_device = g_dl.device;
    g_sb_rec_dev = nullptr;
    for (int e = 0; e < DL_STANDBY_POOL; ++e) g_sb_act[e] = 0;  // fresh doorbells (zero) on this device
    void *p = dl_bar_memory(DL_STANDBY_POOL * SB_DEV_STRIDE);
    if (!p) return;
    g_sb_rec_dev = (uint8_t *)p;
}

// A fresh executor in pool slot e, behind whatever that slot's stream still holds.
int standby_arm(int e)
{
    dl_arm a;
    memset(&a, 0, sizeof a);
    a.bell = standby_bell(e);
    a.armed = &g_arm.host->sb_resident[e];
    a.go = (uint64_t *)g_arm.dev->sb_go[e];
    a.ticket = ++g_sb_act[e];
    // An executor waits for a request that nobody has promised, on a hardware queue that other streams of the
    // process may have been mapped to as well (the runtime multiplexes streams on a few hardware queues): work on
    // such a stream waits behind the executor.  So an executor gives up early, and idle periods longer than this
    // end with no executor on the device; the first request afterwards takes the ordinary launch.
    const uint32_t limit_us = g_dl.cfg.arm_timeout_us < DL_STANDBY_IDLE_US ? g_dl.cfg.arm_timeout_us : DL_STANDBY_IDLE_US;
    arm_limits(&a, limit_us);
    // A doorbell in device memory is polled by every workgroup.  One in host memory is polled by one workgroup
    // per executor, which passes the word on: with every workgroup of both executors polling over the host link
    // the reads queued up there and each doorbell took 2 us longer to be seen.
    a.direct = g_sb_rec_dev ? 1u : 0u;
    a.own_word = 1;
    g_arm.sb_armed_at[e] = now_ns();  // before the launch: the kernel's own clock starts later than this
    g_arm.sb_limit_ns[e] = (uint64_t)limit_us * 1000ull;
    return dl_standby_launch(standby_rec(e), &a, g_arm.sb_stream[e]);
}

// An executor may be handed a request only while it cannot have reached its arm limit: its clock starts when
// it becomes resident, which is not before it was armed.
bool standby_fresh(int e)
{
    const uint64_t limit_ns = g_arm.sb_limit_ns[e];
    const uint64_t margin_ns = limit_ns / 4 < 2000000ull ? limit_ns / 4 : 2000000ull;
    return g_sb_act[e] != 0 && now_ns() - g_arm.sb_armed_at[e] + margin_ns < limit_ns;
}

void standby_cancel(int e)
{
    if (g_sb_act[e]) standby_store(standby_bell(e) + 1, g_sb_act[e]);
}

}  // namespace

int dl_standby_enter()
{
    if (!g_arm.started) return DL_ERR_STATE;
    if (g_arm.standby) return DL_OK;
    standby_place_records();
    for (int e = 0; e < DL_STANDBY_POOL; ++e)
        if (!g_arm.sb_stream[e]) DL_HIP(hipStreamCreateWithFlags(&g_arm.sb_stream[e], hipStreamNonBlocking));
    for (int e = 0; e < DL_STANDBY_POOL; ++e) {
        const int rc = standby_arm(e);
        if (rc != DL_OK) return rc;
    }
    g_arm.sb_next = 0;
    g_arm.standby = true;
    return DL_OK;
}

int dl_standby_leave()
{
    if (!g_arm.started || !g_arm.standby) return DL_OK;
    for (int e = 0; e < DL_STANDBY_POOL; ++e) standby_cancel(e);
    for (int e = 0; e < DL_STANDBY_POOL; ++e) DL_HIP(hipStreamSynchronize(g_arm.sb_stream[e]));
    g_arm.standby = false;
    return DL_OK;
}

int dl_standby_try(const dl_plan_item *items, size_t n, bool *taken)
{
    *taken = false;
    if (!g_arm.started || !g_arm.standby) return DL_OK;
    const int e = g_arm.sb_next;
    if (!standby_fresh(e)) {
        // too old to be trusted with a request (it may be about to give up): replace it and any other that has
        // aged as much, and let this request take the ordinary launch
        for (int k = 0; k < DL_STANDBY_POOL; ++k) {
            if (standby_fresh(k)) continue;
            standby_cancel(k);
            const int rc = standby_arm(k);
            if (rc != DL_OK) return rc;
        }
        return DL_OK;
    }
    const uint64_t ticket = g_arm.seq + 1;
    const uint32_t slot = (uint32_t)(ticket % SLOTS);
    if (ticket > SLOTS) {
        const int rc = wait_done(ticket - SLOTS, drain_ns(), nullptr);
        if (rc != DL_OK) return rc;
    }
    // the record of this pool slot must have been read by the executor that served the slot's last request
    if (g_arm.sb_ticket[e] && g_arm.seq - g_arm.sb_ticket[e] < SLOTS) {
        const int rc = wait_done(g_arm.sb_ticket[e], drain_ns(), nullptr);
        if (rc != DL_OK) return rc;
    }
    // The record is rewritten only once the executor that will read it is on the device: kernels of one stream
    // run one after the other, so by then every workgroup of the executor before it, which read the record's
    // previous contents (also those that had no tile and reported nothing), has ended.  Mostly true already; a
    // caller that comes back faster than the launch gap waits here for what it would have waited for anyway.
    if (wait_word(&g_arm.host->sb_resident[e], g_sb_act[e], 20000ull, nullptr) != DL_OK) return DL_OK;
    // a request of more tiles than completion words counts its workgroups in at the record: device memory only
    const uint32_t set = (uint32_t)(ticket / SLOTS) & 1u;  // as in dl_armed_begin: this ticket's set; it clears the other
    const uint32_t words = dl_standby_fill(standby_rec(e), items, n, g_sb_act[e], ticket, g_arm.host->done[slot],
                                           (uint32_t *)g_arm.dev->arrive[slot][set ^ 1u],
                                           g_sb_rec_dev ? DL_STANDBY_GRID : DL_DONE_WORDS);
    if (words == 0) return DL_OK;
    standby_store(standby_bell(e), g_sb_act[e]);  // the executor's doorbell, behind its record
    const bool in_time = now_ns() - g_arm.sb_armed_at[e] + 100000ull < g_arm.sb_limit_ns[e];
    __atomic_store_n(&g_arm.host->armed[slot], ticket, __ATOMIC_RELAXED);             // it was resident already
    dl_armed_commit(words);
    g_arm.sb_ticket[e] = ticket;
    g_arm.sb_next = (e + 1) % DL_STANDBY_POOL;
    if (in_time) {
        *taken = true;
        return standby_arm(e);  // the replacement, queued behind the executor that is serving this request
    }
    // This thread was held up between the age check and the doorbell, and the executor may have given up in the
    // meantime, all of it or some of its workgroups.  Wait until it has left; if it did not finish the request,
    // close that ticket by hand and let the request run again through the ordinary launch, under the next
    // ticket: it has no swaps, so copying some of its bytes twice gives the same result.
    DL_HIP(hipStreamSynchronize(g_arm.sb_stream[e]));
    const int served = wait_done(ticket, 0, nullptr);
    if (served != DL_OK) {
        // what the executor would have done for the slot besides copying: clear the other set of counters
        DL_HIP(hipMemsetAsync(g_arm.dev->arrive[slot][set ^ 1u], 0, sizeof g_arm.dev->arrive[slot][set ^ 1u],
                              g_arm.sb_stream[e]));
        DL_HIP(hipStreamSynchronize(g_arm.sb_stream[e]));
        for (uint32_t w = 0; w < words; ++w)
            __atomic_store_n(&g_arm.host->done[slot][w], ticket, __ATOMIC_RELEASE);
    }
    *taken = served == DL_OK;
    return standby_arm(e);
}

void dl_armed_commit(uint32_t done_words)
{
    ++g_arm.seq;
    g_arm.words[g_arm.seq % SLOTS] = done_words >= 1 && done_words <= DL_DONE_WORDS ? done_words : 1u;
    t_dl_last.session = g_arm.session;  // the calling thread's most recent request
    t_dl_last.ticket = g_arm.seq;
}

extern "C" {

int dl_prelaunch_start(void)
{
    DL_LOCKED;
    static uint64_t sessions = 0;
    if (!g_dl.inited) return DL_ERR_STATE;
    if (g_arm.started) return DL_ERR_STATE;
    int clock_khz = 0;
    DL_HIP(hipDeviceGetAttribute(&clock_khz, hipDeviceAttributeWallClockRate, g_dl.device));
    g_arm.clock_khz = clock_khz > 0 ? (uint64_t)clock_khz : 100000ull;
    DL_HIP(hipHostMalloc((void **)&g_arm.host, sizeof(arm_host), hipHostMallocCoherent | hipHostMallocMapped));
    memset(g_arm.host, 0, sizeof(arm_host));
    hipError_t e = hipMalloc((void **)&g_arm.dev, sizeof(arm_dev));
    if (e == hipSuccess) e = hipMemset(g_arm.dev, 0, sizeof(arm_dev));
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&g_arm.stream, hipStreamNonBlocking);
    if (e != hipSuccess) {
        g_dl.last_hip = (int)e;
        (void)hipGetLastError();
        if (g_arm.dev) (void)hipFree(g_arm.dev);
        (void)hipHostFree(g_arm.host);
        g_arm = arm_state{};
        return DL_ERR_HIP;
    }
    if (g_bell_dev_device != g_dl.device) {
        g_bell_dev_device = g_dl.device;
        g_bell_dev = (uint64_t *)dl_bar_memory(256);
    }
    if (g_bell_dev) {  // tickets start over: so do doorbell and cancel word (nothing is armed yet)
        bell_store(&g_arm.host->bell, g_bell_dev, 0);
        bell_store(&g_arm.host->cancel, g_bell_dev + 1, 0);
    }
    g_arm.seq = 0;
    g_arm.session = ++sessions;
    g_arm.started = true;
    dl_ring_own_stream(g_arm.stream);
    return DL_OK;
}

int dl_prelaunch_stop(void)
{
    DL_LOCKED;
    if (!g_arm.started) return DL_ERR_STATE;
    {
        const int rc = dl_standby_leave();
        if (rc != DL_OK) return rc;
    }
    // every request still armed gives up; then wait until all of them have left the device
    bell_store(&g_arm.host->cancel, g_bell_dev ? g_bell_dev + 1 : nullptr, g_arm.seq);
    int rc = DL_OK;
    const uint64_t first = g_arm.seq > SLOTS ? g_arm.seq - SLOTS + 1 : 1;
    for (uint64_t t = first; t <= g_arm.seq && rc == DL_OK; ++t)
        rc = wait_done(t, drain_ns(), nullptr);
    if (rc != DL_OK) return rc;  // words stay allocated: a kernel may still use them
    dl_ring_forget_armed();
    dl_ring_own_stream(nullptr);
    (void)hipStreamSynchronize(g_arm.stream);
    (void)hipStreamDestroy(g_arm.stream);
    for (int e = 0; e < DL_STANDBY_POOL; ++e)
        if (g_arm.sb_stream[e]) (void)hipStreamDestroy(g_arm.sb_stream[e]);
    (void)hipFree(g_arm.dev);
    (void)hipHostFree(g_arm.host);
    g_arm = arm_state{};
    if (g_dl.mode != DL_MODE_ONESHOT) g_dl.mode = DL_MODE_ONESHOT;
    return DL_OK;
}

uint64_t dl_last_ticket(void)
{
    DL_LOCKED;
    return g_arm.started && t_dl_last.session == g_arm.session ? t_dl_last.ticket : 0;
}

int dl_set_trace(int on)
{
    DL_LOCKED;
    g_dl.trace = on ? 1 : 0;
    return DL_OK;
}

int dl_get_trace(uint64_t ticket, dl_trace *out)
{
    DL_LOCKED;
    if (!g_arm.started) return DL_ERR_STATE;
    if (!out || ticket == 0 || ticket > g_arm.seq || ticket + SLOTS <= g_arm.seq) return DL_ERR_INVALID;
    const uint64_t *t = g_arm.host->trace[ticket % SLOTS];
    out->doorbell_seen = load_word(&t[0]);
    out->copy_begin = load_word(&t[1]);
    out->copy_end = load_word(&t[2]);
    out->completion_issued = load_word(&t[3]);
    return DL_OK;
}

// Answers `rounds` pings: waits for ping[0] to reach r, then stores the device clock in ping[1].
// Every wait is bounded by limit_ticks.
__global__ void dl_clock_ping_kernel(uint64_t *ping, uint32_t rounds, uint64_t limit_ticks)
{
    const uint64_t t0 = wall_clock64();
    for (uint32_t r = 1; r <= rounds; ++r) {
        for (;;) {
            if (__hip_atomic_load(ping, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) >= r) break;
            if ((uint64_t)wall_clock64() - t0 > limit_ticks) return;
        }
        __hip_atomic_store(ping + 1, (uint64_t)wall_clock64(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

int dl_trace_clock(double *ticks_per_us, double *host_ns_at_tick0)
{
    DL_LOCKED;
    if (!g_arm.started) return DL_ERR_STATE;
    if (!ticks_per_us || !host_ns_at_tick0) return DL_ERR_INVALID;
    constexpr uint32_t ROUNDS = 32;
    uint64_t *ping = g_arm.host->ping;
    __atomic_store_n(&ping[0], 0, __ATOMIC_RELEASE);
    __atomic_store_n(&ping[1], 0, __ATOMIC_RELEASE);
    const uint64_t limit = 200000ull * g_arm.clock_khz / 1000ull;  // 200 ms for all rounds
    hipLaunchKernelGGL(dl_clock_ping_kernel, dim3(1), dim3(1), 0, g_arm.stream, ping, ROUNDS, limit);
    DL_HIP(hipGetLastError());
    double best_rtt = 1e30, best_host = 0;
    uint64_t best_tick = 0, seen = 0;
    for (uint32_t r = 1; r <= ROUNDS; ++r) {
        const uint64_t t0 = now_ns();
        __atomic_store_n(&ping[0], (uint64_t)r, __ATOMIC_RELEASE);
        uint64_t v;
        for (;;) {
            v = load_word(&ping[1]);
            if (v != seen) break;
            if (now_ns() - t0 > 250000000ull) {
                (void)hipStreamSynchronize(g_arm.stream);
                return DL_ERR_TIMEOUT;
            }
        }
        const uint64_t t1 = now_ns();
        seen = v;
        if (r > 4 && (double)(t1 - t0) < best_rtt) {  // the device stamped its clock about half-way through the round trip
            best_rtt = (double)(t1 - t0);
            best_host = (double)t0 + 0.5 * (double)(t1 - t0);
            best_tick = v;
        }
    }
    DL_HIP(hipStreamSynchronize(g_arm.stream));
    *ticks_per_us = (double)g_arm.clock_khz / 1000.0;
    *host_ns_at_tick0 = best_host - (double)best_tick * 1e6 / (double)g_arm.clock_khz;
    return DL_OK;
}

int dl_trigger(uint64_t ticket)
{
    DL_LOCKED;
    if (!g_arm.started) return DL_ERR_STATE;
    if (ticket == 0 || ticket > g_arm.seq) return DL_ERR_INVALID;
    if (ticket > g_arm.host->bell) bell_store(&g_arm.host->bell, g_bell_dev, ticket);  // the doorbell
    return DL_OK;
}

// The two waits look their words up under the lock and spin without it, so that another thread can issue
// and trigger requests meanwhile.  (The words live until dl_prelaunch_stop, which must not run beside a wait.)
int dl_wait_armed(uint64_t ticket, uint64_t timeout_ns)
{
    const uint64_t *word;
    {
        DL_LOCKED;
        if (!g_arm.started) return DL_ERR_STATE;
        if (ticket == 0 || ticket > g_arm.seq) return DL_ERR_INVALID;
        word = &g_arm.host->armed[ticket % SLOTS];
    }
    return wait_word(word, ticket, timeout_ns, nullptr);
}

int dl_wait(uint64_t ticket, uint64_t timeout_ns)
{
    const uint64_t *words;
    uint32_t count;
    {
        DL_LOCKED;
        if (!g_arm.started) return DL_ERR_STATE;
        if (ticket == 0) return DL_OK;
        if (ticket > g_arm.seq) return DL_ERR_INVALID;
        if (g_arm.seq - ticket >= SLOTS) return DL_OK;  // its slot has been reused since, which waited for it
        const uint32_t slot = (uint32_t)(ticket % SLOTS);
        words = g_arm.host->done[slot];
        count = g_arm.words[slot] ? g_arm.words[slot] : 1u;
    }
    uint64_t seen = 0;
    const int rc = wait_words(words, count, ticket, timeout_ns, &seen);
    if (rc != DL_OK) return rc;
    return seen & DL_DONE_SKIPPED ? DL_ERR_EXPIRED : DL_OK;
}

}  // extern "C"
