// Host-thread model of the protocol of the withdrawn "one launch serves many requests" executor (the order of
// operations only; no GPU code runs here, and nothing of that executor is part of the library).
//
//   host   : fills ring slot seq % SLOTS with a command, then release-stores the slot's ready word
//            (seq << 16 | length): the doorbell.  Before it reuses a slot it waits for the completion word to
//            reach the command that used it last.
//   leader : workgroup 0 polls the ready word of the slot it expects next, copies the command into device
//            memory and its own local memory, release-stores go = (seq << 20 | active workgroups).
//   workers: every other workgroup polls go; the first `active` of them copy the command to local memory and
//            stride over its tiles.
//   finish : every active workgroup bumps an arrival counter behind a release fence; the leader waits for
//            `active` arrivals, clears the counter, release-stores seq into the completion word.
//   exit   : quit flag (leader -> go = EXIT), no doorbell for a bounded number of polls, or arrivals that never
//            come within a bounded number of polls; a worker that sees nothing for a bounded number of polls
//            leaves by itself.  Every wait in the model is bounded, as every wait in the kernel was.
//
// A workgroup is one thread here: what its 256 threads did between two barriers, this thread does in turn.
// Command words, the device copy and the outputs are plain memory, so ThreadSanitizer checks that every access
// to them is ordered by the protocol's atomics; every index (ring slot, command word, tile, output) is checked;
// the schedule is perturbed by random yields.  Where the kernel used a relaxed atomic and a fence, the model
// puts the order on the atomic itself (ThreadSanitizer does not follow fences): that is the weaker of the two, so
// what is ordered here was ordered there.
//
// usage: resident_protocol_model [as_built|reset_late] [requests] [workgroups] [seed]
//   as_built   the protocol as it was written
//   reset_late the planted mistake: the leader clears the arrival counter only after it has published the next
//              command, so arrivals for that command can be wiped out
//   exit status 0: every request completed with every tile written exactly once, then quit, then a second run
//   that ends through the no-doorbell limit; 1: anything else (the report says what).
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <thread>
#include <vector>

namespace {

constexpr uint32_t SLOTS = 8;
constexpr uint32_t CMD_WORDS = 384;       // a 3 KiB slot in 8-byte words
constexpr uint32_t HDR_WORDS = 8;         // the 64-byte header
constexpr uint32_t MAX_TILES = CMD_WORDS - HDR_WORDS;
constexpr uint64_t GO_EXIT = ~0ull;
constexpr uint32_t OUT_SETS = 16;         // outputs of the last OUT_SETS requests are kept apart

enum : uint32_t { ST_NONE, ST_RUNNING, ST_EXITED, ST_EXITED_IDLE, ST_EXITED_STUCK };

struct command {  // header, then one word per tile (what the tile has to write)
    uint64_t words[CMD_WORDS];
    uint32_t &tiles() { return reinterpret_cast<uint32_t *>(words)[2]; }
    uint32_t &active() { return reinterpret_cast<uint32_t *>(words)[3]; }
    uint32_t &vecs() { return reinterpret_cast<uint32_t *>(words)[4]; }  // words to copy
    uint32_t &out_set() { return reinterpret_cast<uint32_t *>(words)[5]; }
};

struct host_mem {
    std::atomic<uint64_t> done{0};
    std::atomic<uint32_t> state{ST_NONE};
    std::atomic<uint32_t> quit{0};
    std::atomic<uint64_t> ready[SLOTS];
    command slot[SLOTS];
};

struct dev_mem {
    std::atomic<uint64_t> go{0};
    std::atomic<uint32_t> arrive{0};
    command cmd;
};

struct limits {
    uint64_t idle_polls, hard_polls;
};

int g_failed = 0;
std::atomic<int> g_checks_failed{0};

#define CHECK(cond, ...)                                   \
    do {                                                   \
        if (!(cond)) {                                     \
            if (g_checks_failed.fetch_add(1) < 10) {       \
                std::printf("CHECK failed: " __VA_ARGS__); \
                std::printf("\n");                         \
            }                                              \
        }                                                  \
    } while (0)

struct jitter {
    std::mt19937 rng;
    explicit jitter(uint32_t seed) : rng(seed) {}
    void operator()()
    {
        const uint32_t r = rng();
        if ((r & 7u) == 0) std::this_thread::yield();
        if ((r & 1023u) == 1) std::this_thread::sleep_for(std::chrono::microseconds(50));
    }
};

uint64_t out[OUT_SETS][MAX_TILES];  // plain memory: what the tiles write

// A workgroup's share of the command in its local memory.
void execute(command &local, uint32_t block, uint32_t active, jitter &j)
{
    const uint32_t tiles = local.tiles(), set = local.out_set();
    CHECK(tiles >= 1 && tiles <= MAX_TILES, "tiles %u", tiles);
    CHECK(active >= 1, "active %u", active);
    CHECK(set < OUT_SETS, "output set %u", set);
    if (active == 0 || set >= OUT_SETS) return;
    for (uint32_t t = block; t < tiles && t < MAX_TILES; t += active) {
        out[set][t] += local.words[HDR_WORDS + t];  // += : a tile moved twice shows
        j();
    }
}

void leader(host_mem &h, dev_mem &d, limits lim, bool reset_late, uint32_t seed)
{
    jitter j(seed);
    command local;
    h.state.store(ST_RUNNING, std::memory_order_release);
    bool clear_pending = false;
    for (uint64_t seq = 1;; ++seq) {
        const uint32_t s = (uint32_t)(seq % SLOTS);
        uint64_t word = 0;
        for (uint64_t polls = 0;; ++polls) {
            const uint64_t w = h.ready[s].load(std::memory_order_acquire);  // (a relaxed poll and an acquire fence behind it)
            if ((w >> 16) == seq) {
                word = w & 0xFFFFu;
                break;
            }
            if (h.quit.load(std::memory_order_relaxed)) {
                word = GO_EXIT;
                break;
            }
            if (polls > lim.idle_polls) {
                word = GO_EXIT - 1;
                break;
            }
            j();
        }
        if (word >= GO_EXIT - 1) {
            d.go.store(GO_EXIT, std::memory_order_release);
            h.state.store(word == GO_EXIT ? ST_EXITED : ST_EXITED_IDLE, std::memory_order_release);
            return;
        }
        const uint32_t vecs = (uint32_t)word;  // the command written before the doorbell is visible from here on
        CHECK(vecs >= HDR_WORDS && vecs <= CMD_WORDS, "vecs %u", vecs);
        for (uint32_t i = 0; i < vecs && i < CMD_WORDS; ++i) {
            local.words[i] = h.slot[s].words[i];
            d.cmd.words[i] = local.words[i];
        }
        const uint32_t active = local.active();
        d.go.store((seq << 20) | active, std::memory_order_release);
        if (clear_pending) {  // (the planted mistake's late clear)
            j();
            d.arrive.store(0, std::memory_order_relaxed);
            clear_pending = false;
        }
        execute(local, 0, active, j);
        d.arrive.fetch_add(1, std::memory_order_release);  // (a release fence and a relaxed add)
        bool stuck = false;
        for (uint64_t polls = 0; d.arrive.load(std::memory_order_acquire) != active; ++polls) {  // (relaxed polls, then an acquire fence)
            if (polls > lim.hard_polls) {
                stuck = true;
                break;
            }
            j();
        }
        if (reset_late)
            clear_pending = true;
        else
            d.arrive.store(0, std::memory_order_relaxed);
        if (stuck) {
            d.go.store(GO_EXIT, std::memory_order_release);
            h.state.store(ST_EXITED_STUCK, std::memory_order_release);
            return;
        }
        h.done.store(seq, std::memory_order_release);
    }
}

void worker(dev_mem &d, uint32_t block, limits lim, uint32_t seed)
{
    jitter j(seed);
    command local;
    uint64_t seen = 0;
    for (;;) {
        uint64_t g = 0;
        for (uint64_t polls = 0;; ++polls) {
            g = d.go.load(std::memory_order_acquire);  // (a relaxed poll and an acquire fence behind it)
            if (g == GO_EXIT || (g >> 20) > seen) break;
            if (polls > lim.idle_polls + lim.hard_polls) {
                g = GO_EXIT;  // the leader is gone or stuck
                break;
            }
            j();
        }
        if (g == GO_EXIT) return;
        seen = g >> 20;
        const uint32_t active = (uint32_t)(g & 0xFFFFFu);
        if (block >= active) continue;
        const uint32_t vecs = d.cmd.vecs();  // the command in device memory, written before go
        CHECK(vecs >= HDR_WORDS && vecs <= CMD_WORDS, "worker %u: vecs %u", block, vecs);
        for (uint32_t i = 0; i < vecs && i < CMD_WORDS; ++i) local.words[i] = d.cmd.words[i];
        execute(local, block, active, j);
        d.arrive.fetch_add(1, std::memory_order_release);
    }
}

// Bounded wait for the completion word.  0: reached; else the executor's state when it was given up.
uint32_t wait_done(host_mem &h, uint64_t ticket)
{
    for (uint64_t spins = 0; spins < (1ull << 34); ++spins) {
        if (h.done.load(std::memory_order_acquire) >= ticket) return 0;
        const uint32_t st = h.state.load(std::memory_order_acquire);
        if (st != ST_RUNNING && st != ST_NONE && h.done.load(std::memory_order_acquire) < ticket) return st;
        if ((spins & 63u) == 0) std::this_thread::yield();
    }
    return ST_NONE;
}

// One life of the executor: `requests` commands, then quit (or, with quit_at_end false, silence until the leader
// gives up).  Returns 0 if everything was as it should be.
int run(bool reset_late, uint32_t requests, uint32_t blocks, uint32_t seed, bool quit_at_end)
{
    static host_mem h;
    static dev_mem d;
    h.done = 0, h.state = ST_NONE, h.quit = 0;
    for (auto &r : h.ready) r = 0;
    d.go = 0, d.arrive = 0;
    std::memset(out, 0, sizeof out);
    const limits lim{quit_at_end ? (1ull << 40) : 2000000ull, 8000000ull};
    std::vector<std::thread> th;
    th.emplace_back(leader, std::ref(h), std::ref(d), lim, reset_late, seed * 7919u + 1u);
    for (uint32_t b = 1; b < blocks; ++b) th.emplace_back(worker, std::ref(d), b, lim, seed * 7919u + 1u + b);

    std::mt19937 rng(seed);
    jitter j(seed + 99u);
    int bad = 0;
    std::vector<uint32_t> tiles_of(requests + 1, 0);
    auto check_outputs = [&](uint64_t seq) {  // after the completion word has reached seq
        const uint32_t set = (uint32_t)(seq % OUT_SETS);
        for (uint32_t t = 0; t < tiles_of[seq]; ++t)
            if (out[set][t] != seq * 1000003ull + t) {
                if (bad++ < 5) std::printf("request %llu tile %u: %llu\n", (unsigned long long)seq, t, (unsigned long long)out[set][t]);
            }
        std::memset(out[set], 0, sizeof out[set]);  // the set is free for request seq + OUT_SETS
    };
    uint64_t checked = 0;
    for (uint64_t seq = 1; seq <= requests && !bad; ++seq) {
        // a slot, and an output set, are reused only when the request that had them last is complete (and checked)
        const uint64_t must = seq > SLOTS ? seq - SLOTS : 0;
        while (checked < must) {
            const uint32_t st = wait_done(h, checked + 1);
            if (st) {
                std::printf("request %llu never completed: executor state %u\n", (unsigned long long)(checked + 1), st);
                bad++;
                break;
            }
            check_outputs(++checked);
        }
        if (bad) break;
        const uint32_t s = (uint32_t)(seq % SLOTS);
        command &c = h.slot[s];
        const uint32_t tiles = 1u + rng() % (rng() % 4 == 0 ? MAX_TILES : 24u);
        tiles_of[seq] = tiles;
        c.tiles() = tiles;
        c.active() = tiles < blocks ? tiles : blocks;
        c.out_set() = (uint32_t)(seq % OUT_SETS);
        c.vecs() = HDR_WORDS + tiles;
        for (uint32_t t = 0; t < tiles; ++t) c.words[HDR_WORDS + t] = seq * 1000003ull + t;
        j();
        h.ready[s].store((seq << 16) | c.vecs(), std::memory_order_release);  // the doorbell
        j();
    }
    while (!bad && checked < requests) {
        const uint32_t st = wait_done(h, checked + 1);
        if (st) {
            std::printf("request %llu never completed: executor state %u\n", (unsigned long long)(checked + 1), st);
            bad++;
            break;
        }
        check_outputs(++checked);
    }
    if (quit_at_end || bad) h.quit.store(1, std::memory_order_release);
    for (auto &t : th) t.join();  // every workgroup leaves: by quit, or by its own limit
    const uint32_t st = h.state.load();
    const uint32_t want = bad ? st : quit_at_end ? (uint32_t)ST_EXITED : (uint32_t)ST_EXITED_IDLE;
    if (st != want) {
        std::printf("executor ended in state %u, expected %u\n", st, want);
        bad++;
    }
    std::printf("%s: %llu of %u requests complete and correct, end state %u\n", quit_at_end ? "quit" : "idle",
                (unsigned long long)checked, requests, st);
    return bad;
}

}  // namespace

int main(int argc, char **argv)
{
    const bool reset_late = argc > 1 && !std::strcmp(argv[1], "reset_late");
    const uint32_t requests = argc > 2 ? (uint32_t)std::atoi(argv[2]) : 3000u;
    const uint32_t blocks = argc > 3 ? (uint32_t)std::atoi(argv[3]) : 6u;
    const uint32_t seed = argc > 4 ? (uint32_t)std::atoi(argv[4]) : 1u;
    if (blocks < 1 || blocks > 64 || requests < 1) return 2;
    g_failed += run(reset_late, requests, blocks, seed, true);
    g_failed += run(reset_late, requests / 4 + 1, blocks, seed + 1, false);
    g_failed += g_checks_failed.load();
    std::printf("%s\n", g_failed ? "FAILED" : "ok");
    return g_failed ? 1 : 0;
}
