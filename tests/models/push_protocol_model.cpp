// Host-thread model of how a copy table reaches a kernel through device memory that the host writes directly
// (the order of operations only; no GPU code runs here).
//
//   writer (the host):  payload words of generation g  ->  fence  ->  stamp = g
//   reader (a kernel):  must pair a stamp with payload that is at least as new
//
// The slot is reused: generation g overwrites generation g - 1 in place.  A reader that loads the payload
// first and the stamp afterwards can see payload g - 1 and stamp g, and would execute a stale table under a
// valid stamp; a reader that looks at the stamp first and loads the payload behind it cannot.  The two orders
// are run under the same forced interleaving (the reader's two loads straddle the writer's update), and then
// free-running against a writer that keeps rewriting the slot.
//
// usage: push_protocol_model stamp_first|payload_first   -> exit status 0 if no stale pairing was seen
#include <atomic>
#include <condition_variable>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <thread>

namespace {

constexpr int WORDS = 11;  // an 88-byte table entry

struct slot_t {
    std::atomic<uint64_t> payload[WORDS];
    std::atomic<uint64_t> stamp;
};

void write_generation(slot_t &s, uint64_t g)
{
    for (int w = 0; w < WORDS; ++w) s.payload[w].store(g * 1000 + (uint64_t)w, std::memory_order_relaxed);
    std::atomic_thread_fence(std::memory_order_release);  // the host's store fence between table and stamp
    s.stamp.store(g, std::memory_order_relaxed);
}

// What the reader got: the stamp it saw and the oldest generation among the payload words it loaded.
struct seen_t {
    uint64_t stamp, oldest_payload;
};

template <class Between>
seen_t read_stamp_first(slot_t &s, Between between)
{
    seen_t r;
    r.stamp = s.stamp.load(std::memory_order_relaxed);
    std::atomic_thread_fence(std::memory_order_acquire);  // the payload loads stay behind the stamp load
    between();
    r.oldest_payload = ~0ull;
    for (int w = 0; w < WORDS; ++w) {
        const uint64_t g = s.payload[w].load(std::memory_order_relaxed) / 1000;
        if (g < r.oldest_payload) r.oldest_payload = g;
    }
    return r;
}

template <class Between>
seen_t read_payload_first(slot_t &s, Between between)
{
    seen_t r;
    r.oldest_payload = ~0ull;
    for (int w = 0; w < WORDS; ++w) {
        const uint64_t g = s.payload[w].load(std::memory_order_relaxed) / 1000;
        if (g < r.oldest_payload) r.oldest_payload = g;
    }
    between();
    r.stamp = s.stamp.load(std::memory_order_relaxed);
    return r;
}

// A pairing is stale if the payload is older than the stamp that vouches for it.
bool stale(const seen_t &r) { return r.oldest_payload < r.stamp; }

}  // namespace

int main(int argc, char **argv)
{
    if (argc != 2) return 2;
    const bool stamp_first = !strcmp(argv[1], "stamp_first");
    if (!stamp_first && strcmp(argv[1], "payload_first")) return 2;
    int bad = 0;

    // 1. forced interleaving: the writer's whole update happens between the reader's two loads
    {
        slot_t s;
        write_generation(s, 1);
        auto update = [&] { std::thread([&] { write_generation(s, 2); }).join(); };
        const seen_t r = stamp_first ? read_stamp_first(s, update) : read_payload_first(s, update);
        printf("forced: stamp %llu payload %llu%s\n", (unsigned long long)r.stamp, (unsigned long long)r.oldest_payload,
               stale(r) ? "  STALE" : "");
        bad += stale(r);
    }

    // 2. free-running: the writer rewrites the slot 200000 times while two readers keep reading
    {
        slot_t s;
        write_generation(s, 1);
        std::atomic<bool> stop{false};
        std::atomic<int> stale_seen{0};
        auto reader = [&] {
            auto nothing = [] {};
            while (!stop.load(std::memory_order_relaxed)) {
                const seen_t r = stamp_first ? read_stamp_first(s, nothing) : read_payload_first(s, nothing);
                if (stale(r)) stale_seen.fetch_add(1, std::memory_order_relaxed);
            }
        };
        std::thread a(reader), b(reader);
        for (uint64_t g = 2; g < 200002; ++g) write_generation(s, g);
        stop.store(true);
        a.join();
        b.join();
        printf("free-running: %d stale pairings\n", stale_seen.load());
        if (stamp_first) bad += stale_seen.load();  // (the other order may or may not be caught by chance)
    }
    return bad ? 1 : 0;
}
