// The C boundary: argument checks, lowering of the collectives to copy lists
// (the "control" phase of Sec. III-B2), the optional hazard check of Sec. IV-D,
// and dispatch to the one-shot or the armed (prelaunched) launcher.
#include "dl_internal.h"

#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <vector>

dl_state g_dl;
std::recursive_mutex g_dl_lock;
thread_local dl_thread_last t_dl_last;

static_assert(sizeof(dl_plan_item) == sizeof(dl_fused_item), "public and device item must share a layout");
static_assert(offsetof(dl_plan_item, dst) == offsetof(dl_fused_item, dst), "public and device item must share a layout");
static_assert(DL_PLAN_FANOUT == DL_FAN, "public and device fan-out must agree");

namespace {

// Collects lowered items into caller storage, counting past its capacity.
struct sink {
    dl_plan_item *items;
    size_t cap;
    size_t n = 0;
    void put(const void *src, size_t bytes, void *const *dst, uint32_t k)
    {
        if (n < cap) {
            dl_plan_item &it = items[n];
            it.src = src;
            it.bytes = bytes;
            it.k = k;
            it.reserved = 0;
            for (uint32_t j = 0; j < (uint32_t)DL_PLAN_FANOUT; ++j) it.dst[j] = j < k ? dst[j] : nullptr;
        }
        ++n;
    }
};

// One source to many destinations, in groups of DL_PLAN_FANOUT.
void put_fanout(sink &s, const void *src, size_t bytes, void *const *dst, size_t k)
{
    for (size_t g = 0; g < k; g += DL_PLAN_FANOUT)
        s.put(src, bytes, dst + g, (uint32_t)std::min<size_t>(DL_PLAN_FANOUT, k - g));
}

long lower_allgather(const void *const *in, void *const *out, int W, size_t B, int fuse, sink &s)
{
    if (W < 1 || W > DL_MAX_FANOUT || !in || !out) return DL_ERR_INVALID;
    if (B == 0) return 0;
    for (int r = 0; r < W; ++r)
        if (!in[r] || !out[r]) return DL_ERR_INVALID;
    void *dst[DL_MAX_FANOUT];
    for (int j = 0; j < W; ++j) {  // source rank j goes to slot j of every receive buffer
        size_t k = 0;
        for (int r = 0; r < W; ++r) {
            void *d = (char *)out[r] + (size_t)j * B;
            if (d == in[j]) continue;  // in-place layout: rank j's own slot already holds its data
            dst[k++] = d;
        }
        if (fuse)
            put_fanout(s, in[j], B, dst, k);
        else
            for (size_t q = 0; q < k; ++q) s.put(in[j], B, &dst[q], 1);
    }
    return (long)s.n;
}

long lower_alltoall(const void *const *in, void *const *out, int W, const size_t *C, sink &s)
{
    if (W < 1 || W > DL_MAX_FANOUT || !in || !out || !C) return DL_ERR_INVALID;
    size_t recv_off[DL_MAX_FANOUT] = {0};  // running offset into each receive buffer
    for (int i = 0; i < W; ++i) {
        size_t send_off = 0;
        for (int j = 0; j < W; ++j) {
            const size_t c = C[(size_t)i * W + j];
            if (c) {
                if (!in[i] || !out[j]) return DL_ERR_INVALID;
                void *d = (char *)out[j] + recv_off[j];
                s.put((const char *)in[i] + send_off, c, &d, 1);
            }
            send_off += c;
            recv_off[j] += c;
        }
    }
    return (long)s.n;
}

long lower_broadcast(const void *src, void *const *dsts, int k, size_t bytes, sink &s)
{
    if (k < 1 || k > DL_MAX_FANOUT || !dsts) return DL_ERR_INVALID;
    if (bytes == 0) return 0;
    if (!src) return DL_ERR_INVALID;
    for (int d = 0; d < k; ++d)
        if (!dsts[d]) return DL_ERR_INVALID;
    put_fanout(s, src, bytes, dsts, (size_t)k);
    return (long)s.n;
}

long lower_batch(const dl_copy_desc *desc, size_t n, sink &s)
{
    if (n && !desc) return DL_ERR_INVALID;
    for (size_t i = 0; i < n; ++i) {
        if (desc[i].bytes == 0) continue;
        if (!desc[i].src || !desc[i].dst) return DL_ERR_INVALID;
        if (desc[i].src == desc[i].dst) continue;  // identical range: nothing to move
        void *d = desc[i].dst;
        s.put(desc[i].src, desc[i].bytes, &d, 1);
    }
    return (long)s.n;
}

// dl_batch_copy with broadcast inference (Sec. VI): copies with the same source
// address and the same byte count become one read-once/write-k item, in order of
// first appearance, at most DL_PLAN_FANOUT destinations per item.
long lower_batch_inferred(const dl_copy_desc *desc, size_t n, sink &s)
{
    if (n && !desc) return DL_ERR_INVALID;
    // slots[]: open-addressing table over the distinct (src, bytes), each entry the index (+1, 0 = empty) of the
    // item that still takes destinations for that key
    static std::vector<uint32_t> slots;
    size_t want = 16;
    while (want < 2 * n) want *= 2;
    slots.assign(want, 0);
    // The items are built where they are wanted if there is room for the worst case (no two copies share a
    // source); else in a buffer of our own, from which the sink takes what it has room for and counts the rest.
    static std::vector<dl_plan_item> own;
    dl_plan_item *out = s.items;
    if (s.cap < n) {
        if (own.size() < n) own.resize(n);
        out = own.data();
    }
    size_t m = 0;
    auto open_item = [&](const dl_copy_desc &d) {
        dl_plan_item &it = out[m++];
        it.src = d.src;
        it.bytes = d.bytes;
        it.k = 1;
        it.reserved = 0;
        it.dst[0] = d.dst;
        for (uint32_t j = 1; j < (uint32_t)DL_PLAN_FANOUT; ++j) it.dst[j] = nullptr;
        return (uint32_t)m;
    };
    for (size_t i = 0; i < n; ++i) {
        const dl_copy_desc &d = desc[i];
        if (d.bytes == 0) continue;
        if (!d.src || !d.dst) return DL_ERR_INVALID;
        if (d.src == d.dst) continue;
        const uint64_t h = ((uint64_t)d.src * 0x9E3779B97F4A7C15ull) ^ ((uint64_t)d.bytes * 0xC2B2AE3D27D4EB4Full);
        size_t q = (size_t)(h >> 20) & (want - 1);
        for (;;) {
            const uint32_t g = slots[q];
            if (g == 0) {  // first copy from this (src, bytes)
                slots[q] = open_item(d);
                break;
            }
            dl_plan_item &it = out[g - 1];
            if (it.src == d.src && it.bytes == d.bytes) {
                if (it.k < (uint32_t)DL_PLAN_FANOUT)
                    it.dst[it.k++] = d.dst;
                else  // full: a fresh item takes over this key
                    slots[q] = open_item(d);
                break;
            }
            q = (q + 1) & (want - 1);
        }
    }
    if (out != s.items)
        for (size_t g = 0; g < m && g < s.cap; ++g) s.items[g] = out[g];
    s.n = m;
    return (long)m;
}

// One read-once/write-k item per token that has a destination; receive buffers
// fill up in token order.
long lower_token_dispatch(const void *const *in, void *const *out, int W, const uint32_t *tokens, size_t row,
                          const uint8_t *dest, sink &s)
{
    if (W < 1 || W > DL_MAX_FANOUT || !in || !out || !tokens) return DL_ERR_INVALID;
    size_t placed[DL_MAX_FANOUT] = {0};  // rows already assigned in each receive buffer
    void *dst[DL_MAX_FANOUT + 1];
    if (tokens && !dest)
        for (int i = 0; i < W; ++i)
            if (tokens[i]) return DL_ERR_INVALID;
    size_t g = 0;
    for (int i = 0; i < W; ++i) {
        if (tokens[i] && row && !in[i]) return DL_ERR_INVALID;
        for (uint32_t t = 0; t < tokens[i]; ++t, ++g) {
            // thousands of tokens per call: no data-dependent branch per (token, rank)
            const uint8_t *m = dest + g * (size_t)W;
            size_t k = 0;
            for (int j = 0; j < W; ++j) {
                const size_t go = m[j] != 0;
                dst[k] = (char *)out[j] + placed[j] * row;
                k += go;
                placed[j] += go;
            }
            if (k == 0 || row == 0) continue;
            put_fanout(s, (const char *)in[i] + (size_t)t * row, row, dst, k);
        }
    }
    for (int j = 0; j < W; ++j)
        if (placed[j] && row && !out[j]) return DL_ERR_INVALID;  // rows were placed at a null buffer: nothing is executed
    return (long)s.n;
}

struct interval {
    uint64_t lo, hi;
    size_t item;
};

long first_hazard(const dl_plan_item *items, size_t n)
{
    std::vector<interval> dst;
    for (size_t i = 0; i < n; ++i) {
        if (items[i].bytes == 0) continue;
        for (uint32_t j = 0; j < items[i].k; ++j)
            dst.push_back({(uint64_t)items[i].dst[j], (uint64_t)items[i].dst[j] + items[i].bytes, i});
    }
    std::sort(dst.begin(), dst.end(), [](const interval &a, const interval &b) { return a.lo < b.lo; });
    long worst = -1;
    auto flag = [&](size_t i) {
        if (worst < 0 || (long)i < worst) worst = (long)i;
    };
    // destination against destination: sweep by start, remember the furthest end so far
    size_t owner = 0;
    for (size_t q = 1; q < dst.size(); ++q) {
        if (dst[q].lo < dst[owner].hi) {
            flag(dst[q].item);
            flag(dst[owner].item);
        }
        if (dst[q].hi > dst[owner].hi) owner = q;
    }
    const bool disjoint = worst < 0;
    // destination against source.  With disjoint destinations, sorted by start is sorted by end: binary search
    // the first destination that ends after the source starts, then take every one that starts before it ends.
    // A batch that has failed already (an error path) is searched the plain way, so that the index reported is
    // the smallest over both kinds of overlap.
    for (size_t i = 0; i < n; ++i) {
        if (items[i].bytes == 0) continue;
        const uint64_t lo = (uint64_t)items[i].src, hi = lo + items[i].bytes;
        auto it = disjoint ? std::partition_point(dst.begin(), dst.end(), [&](const interval &d) { return d.hi <= lo; })
                           : dst.begin();
        for (; it != dst.end() && it->lo < hi; ++it)
            if (it->hi > lo) flag(it->item);
    }
    return worst;
}

// Swaps of an in-place all-to-all with equal chunks: rank i's chunk j and rank
// j's chunk i change places, once per pair i < j.
long lower_alltoall_inplace(void *const *buf, int W, size_t c, dl_swap_desc *out, size_t cap)
{
    if (W < 1 || W > DL_MAX_FANOUT || !buf) return DL_ERR_INVALID;
    if (c == 0) return 0;
    for (int i = 0; i < W; ++i)
        if (!buf[i]) return DL_ERR_INVALID;
    size_t n = 0;
    for (int i = 0; i < W; ++i)
        for (int j = i + 1; j < W; ++j) {
            if (n < cap) out[n] = {(char *)buf[i] + (size_t)j * c, (char *)buf[j] + (size_t)i * c, c};
            ++n;
        }
    return (long)n;
}

// First swap with a range that overlaps any other range of the batch.
long swap_first_hazard(const dl_swap_desc *d, size_t n)
{
    std::vector<interval> r;
    for (size_t i = 0; i < n; ++i) {
        if (d[i].bytes == 0) continue;
        r.push_back({(uint64_t)d[i].a, (uint64_t)d[i].a + d[i].bytes, i});
        // a swap of a range with itself changes nothing, but the range still belongs to it
        if (d[i].a != d[i].b) r.push_back({(uint64_t)d[i].b, (uint64_t)d[i].b + d[i].bytes, i});
    }
    std::sort(r.begin(), r.end(), [](const interval &x, const interval &y) { return x.lo < y.lo; });
    long worst = -1;
    size_t owner = 0;  // the range that reaches furthest so far
    for (size_t q = 1; q < r.size(); ++q) {
        if (r[q].lo < r[owner].hi) {
            const long w = (long)std::min(r[q].item, r[owner].item);
            if (worst < 0 || w < worst) worst = w;
        }
        if (r[q].hi > r[owner].hi) owner = q;
    }
    return worst;
}

std::vector<dl_plan_item> g_items;      // reused between calls: no allocation once warm
std::vector<dl_plain_item> g_plain;
std::vector<dl_swap_item> g_swaps;
std::vector<dl_swap_desc> g_swap_descs;

// Runs `launch(stream, arm, &launched)` in the current mode: in prelaunch mode it
// gets the next ticket's words and the ticket is committed if a kernel went out.
template <class Launch>
int run_in_mode(void *stream, Launch launch)
{
    hipStream_t hs = (hipStream_t)stream;
    dl_arm arm;
    const dl_arm *armp = nullptr;
    if (g_dl.mode != DL_MODE_ONESHOT) {
        const int rc = dl_armed_begin(&arm, &hs);
        if (rc != DL_OK) return rc;
        armp = &arm;
    }
    bool launched = false;
    const int rc = launch(hs, armp, &launched);
    if (armp && rc == DL_OK && launched) dl_armed_commit(g_dl.armed_words);
    return rc;
}

// The size -> mode table (see the header).  One place holds the thresholds; dl_plan_mode() and DL_MODE_AUTO
// both come here.
struct mode_limits {
    uint32_t standby_tiles, standby_items_fanout, standby_items_plain;
    uint64_t signal_max_moved, prelaunch_max_moved;
    uint64_t dispatch_device_tokens;  // a token dispatch of this many tokens is lowered on the device, one-shot
};
constexpr mode_limits MODE_LIMITS = {DL_AUTO_STANDBY_TILES, 8u, 64u, DL_AUTO_SIGNAL_MAX_BYTES,
                                     DL_AUTO_PRELAUNCH_MAX_BYTES, 512u};

int plan_mode(int op, size_t items, uint32_t max_fanout, uint64_t moved, uint64_t tiles, int known_ahead)
{
    if (op < DL_OP_BATCH || op > DL_OP_TOKEN_DISPATCH || (known_ahead != 0 && known_ahead != 1)) return DL_ERR_INVALID;
    if (items && (max_fanout < 1 || max_fanout > (uint32_t)DL_PLAN_FANOUT)) return DL_ERR_INVALID;
    const mode_limits &L = MODE_LIMITS;
    if (known_ahead) return moved <= L.prelaunch_max_moved ? DL_MODE_PRELAUNCH : DL_MODE_ONESHOT;
    if (op == DL_OP_TOKEN_DISPATCH && items >= L.dispatch_device_tokens) return DL_MODE_ONESHOT;
    const bool fits_record = op != DL_OP_SWAP && op != DL_OP_TOKEN_DISPATCH && items >= 1 && tiles >= 1 &&
                             tiles <= L.standby_tiles &&
                             items <= (max_fanout <= 1 ? L.standby_items_plain : L.standby_items_fanout);
    if (fits_record) return DL_MODE_STANDBY;
    return moved <= L.signal_max_moved ? DL_MODE_SIGNAL : DL_MODE_ONESHOT;
}

// In DL_MODE_AUTO: the mode the table gives this lowered list, which the request then runs in.
int auto_mode_for(int op, const dl_plan_item *items, size_t n)
{
    uint64_t moved = 0, tiles = 0;
    uint32_t kmax = 1;
    for (size_t i = 0; i < n; ++i) {
        moved += items[i].bytes * (1ull + items[i].k);
        tiles += dl_item_tiles(*reinterpret_cast<const dl_fused_item *>(&items[i]), DL_STANDBY_TILE);
        if (items[i].k > kmax) kmax = items[i].k;
    }
    return plan_mode(op, n, kmax, moved, tiles, 0);
}

// Runs f with g_dl.mode set to `mode` (the launchers read it), then puts the caller's setting back.
template <class F>
int with_mode(int mode, F f)
{
    const int asked = g_dl.mode;
    g_dl.mode = mode;
    const int rc = f();
    g_dl.mode = asked;
    return rc;
}

int execute_in(int mode, const dl_plan_item *items, size_t n, void *stream);

int execute(const dl_plan_item *items, size_t n, void *stream, int op)
{
    if (!g_dl.inited) return DL_ERR_STATE;
    if (dl_device_error_pending()) return DL_ERR_LOST;
    if (n == 0) return DL_OK;
    if (g_dl.validate && first_hazard(items, n) >= 0) return DL_ERR_OVERLAP;
    if (g_dl.mode != DL_MODE_AUTO) return execute_in(g_dl.mode, items, n, stream);
    const int mode = auto_mode_for(op, items, n);
    if (mode < 0) return mode;
    return with_mode(mode, [&] { return execute_in(mode, items, n, stream); });
}

int execute_in(int mode, const dl_plan_item *items, size_t n, void *stream)
{
    t_dl_last.mode = mode;
    if (mode == DL_MODE_STANDBY) {
        bool taken = false;
        const int rc = dl_standby_try(items, n, &taken);
        if (rc != DL_OK || taken) return rc;
        t_dl_last.mode = DL_MODE_SIGNAL;  // no waiting kernel could take it: the ordinary launch
    }
    bool all_plain = true;
    for (size_t i = 0; i < n; ++i) all_plain &= items[i].k == 1;
    return run_in_mode(stream, [&](hipStream_t hs, const dl_arm *armp, bool *launched) {
        if (all_plain) {
            g_plain.resize(n);
            for (size_t i = 0; i < n; ++i)
                g_plain[i] = {(const char *)items[i].src, (char *)items[i].dst[0], items[i].bytes};
            return dl_exec_plain(g_plain.data(), n, hs, armp, launched);
        }
        return dl_exec_fused(reinterpret_cast<const dl_fused_item *>(items), n, hs, armp, launched);
    });
}

int execute_swaps(const dl_swap_desc *d, size_t n, void *stream)
{
    if (!g_dl.inited) return DL_ERR_STATE;
    if (dl_device_error_pending()) return DL_ERR_LOST;
    if (n && !d) return DL_ERR_INVALID;
    g_swaps.clear();
    for (size_t i = 0; i < n; ++i) {
        if (d[i].bytes == 0) continue;
        if (!d[i].a || !d[i].b) return DL_ERR_INVALID;
        if (d[i].a == d[i].b) continue;  // identical range: nothing changes
        dl_swap_item it;
        it.src = (const char *)d[i].a;
        it.dst = (char *)d[i].b;
        it.bytes = d[i].bytes;
        g_swaps.push_back(it);
    }
    if (g_swaps.empty()) return DL_OK;
    if (g_dl.validate && swap_first_hazard(d, n) >= 0) return DL_ERR_OVERLAP;
    int mode = g_dl.mode;
    if (mode == DL_MODE_AUTO) {
        uint64_t moved = 0;
        for (const dl_swap_item &it : g_swaps) moved += 4 * it.bytes;  // both ranges are read and written
        mode = plan_mode(DL_OP_SWAP, g_swaps.size(), 1, moved, 0, 0);
    } else if (mode == DL_MODE_STANDBY) {
        mode = DL_MODE_SIGNAL;  // swaps are never handed to a waiting kernel
    }
    t_dl_last.mode = mode;
    return with_mode(mode, [&] {
        return run_in_mode(stream, [&](hipStream_t hs, const dl_arm *armp, bool *launched) {
            return dl_exec_swap(g_swaps.data(), g_swaps.size(), hs, armp, launched);
        });
    });
}

// Lower with `fn` into the reusable buffer, growing it when the first pass
// reports more items than fit.
template <class Fn>
int lower_and_execute(Fn fn, void *stream, int op)
{
    if (g_items.size() < 64) g_items.resize(64);
    for (int pass = 0; pass < 2; ++pass) {
        sink s{g_items.data(), g_items.size()};
        const long r = fn(s);
        if (r < 0) return (int)r;
        if ((size_t)r <= g_items.size()) return execute(g_items.data(), (size_t)r, stream, op);
        g_items.resize((size_t)r);
    }
    return DL_ERR_INVALID;
}

bool config_valid(const dl_config &cfg)
{
    const uint32_t t = cfg.tile_bytes, b = cfg.block_threads;
    if (t && (t < 1024 || (t & (t - 1)) || t > (1u << 24))) return false;
    if (b && b != 64 && b != 128 && b != 256 && b != 512) return false;
    if (cfg.arm_timeout_us < 1 || cfg.arm_timeout_us > 1000000) return false;
    const uint32_t fs = cfg.fan_split;
    return fs == 0 || fs == 1 || fs == 2 || fs == 4;
}

// The tunables by name, for dl_parse_config (and so for the DL_CONFIG environment variable).
struct config_field {
    const char *name;
    uint32_t dl_config::*p32;
    uint64_t dl_config::*p64;
};
const config_field CONFIG_FIELDS[] = {
    {"tile_bytes", &dl_config::tile_bytes, nullptr},
    {"block_threads", &dl_config::block_threads, nullptr},
    {"nontemporal_min_bytes", nullptr, &dl_config::nontemporal_min_bytes},
    {"armed_blocks", &dl_config::armed_blocks, nullptr},
    {"arm_timeout_us", &dl_config::arm_timeout_us, nullptr},
    {"fuse_broadcast", &dl_config::fuse_broadcast, nullptr},
    {"max_blocks", &dl_config::max_blocks, nullptr},
    {"fan_split", &dl_config::fan_split, nullptr},
    {"infer_broadcast", &dl_config::infer_broadcast, nullptr},
    {"device_lowering", &dl_config::device_lowering, nullptr},
    {"table_push", &dl_config::table_push, nullptr},
    {"write_through_max_bytes", nullptr, &dl_config::write_through_max_bytes},
    {"stream_plain_min_bytes", nullptr, &dl_config::stream_plain_min_bytes},
    {"armed_chain_min_bytes", nullptr, &dl_config::armed_chain_min_bytes},
};

}  // namespace

extern "C" {

int dl_parse_config(const char *text, dl_config *cfg);

int dl_init(int device)
{
    DL_LOCKED;
    if (g_dl.inited) return g_dl.device == device ? DL_OK : DL_ERR_STATE;
    DL_HIP(hipSetDevice(device));
    int cus = 0;
    DL_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device));
    g_dl.device = device;
    g_dl.num_cu = cus;
    g_dl.mode = DL_MODE_ONESHOT;
    g_dl.validate = 0;
    g_dl.cfg = dl_config{};
    g_dl.cfg.nontemporal_min_bytes = ~0ull;  // streaming hints measured slower: off unless asked for
    g_dl.cfg.write_through_max_bytes = 144ull << 20;  // all-gather of 2 MiB per rank over 8 ranks
    g_dl.cfg.armed_chain_min_bytes = 256ull << 20;    // what the Infinity Cache holds; all-gather: from 4 MiB per rank over 8 ranks
    g_dl.cfg.stream_plain_min_bytes = 512ull << 20;   // twice the Infinity Cache: all-to-all of 4 MiB chunks between 8 ranks
    g_dl.cfg.arm_timeout_us = 20000;
    g_dl.cfg.fuse_broadcast = 1;
    g_dl.cfg.infer_broadcast = 1;
    g_dl.cfg.device_lowering = 1;
    g_dl.cfg.table_push = 1;
    // defaults first, then what the environment asks for (DL_CONFIG="fan_split=2,table_push=0")
    if (dl_parse_config(getenv("DL_CONFIG"), &g_dl.cfg) != DL_OK) return DL_ERR_INVALID;
    int rc = dl_exec_init();
    if (rc == DL_OK) rc = dl_static_init(device);
    if (rc != DL_OK) return rc;
    g_dl.inited = true;
    return DL_OK;
}

int dl_shutdown(void)
{
    DL_LOCKED;
    if (!g_dl.inited) return DL_OK;
    int rc = DL_OK;
    if (dl_armed_ready()) rc = dl_prelaunch_stop();
    dl_exec_shutdown();
    g_dl.inited = false;
    g_dl.device = -1;
    g_dl.mode = DL_MODE_ONESHOT;
    return rc;
}

int dl_set_mode(int mode)
{
    DL_LOCKED;
    if (mode < DL_MODE_ONESHOT || mode > DL_MODE_AUTO) return DL_ERR_INVALID;
    if (mode != DL_MODE_ONESHOT && !dl_armed_ready()) return DL_ERR_STATE;
    if (mode == g_dl.mode) return DL_OK;
    // standby and auto mode keep the pool of waiting kernels armed
    const bool had_pool = g_dl.mode == DL_MODE_STANDBY || g_dl.mode == DL_MODE_AUTO;
    const bool wants_pool = mode == DL_MODE_STANDBY || mode == DL_MODE_AUTO;
    if (had_pool && !wants_pool) {
        const int rc = dl_standby_leave();
        if (rc != DL_OK) return rc;
    }
    if (!had_pool && wants_pool) {
        const int rc = dl_standby_enter();
        if (rc != DL_OK) return rc;
    }
    g_dl.mode = mode;
    return DL_OK;
}

int dl_last_mode(void) { return t_dl_last.mode; }  // the calling thread's own

int dl_plan_mode(int op, size_t items, uint32_t max_fanout, uint64_t moved_bytes, uint64_t tiles, int known_ahead)
{
    return plan_mode(op, items, max_fanout, moved_bytes, tiles, known_ahead);
}

int dl_complete(void *stream, uint64_t timeout_ns)
{
    {
        DL_LOCKED;
        if (!g_dl.inited) return DL_ERR_STATE;
    }
    // the waiting itself happens without the lock
    if (t_dl_last.mode == DL_MODE_ONESHOT) {
        DL_HIP(hipStreamSynchronize((hipStream_t)stream));
        return DL_OK;
    }
    return dl_wait(dl_last_ticket(), timeout_ns);
}

int dl_get_mode(void)
{
    DL_LOCKED;
    return g_dl.mode;
}

int dl_set_validate(int on)
{
    DL_LOCKED;
    g_dl.validate = on ? 1 : 0;
    return DL_OK;
}

const char *dl_strerror(int status)
{
    switch (status) {
    case DL_OK: return "ok";
    case DL_ERR_INVALID: return "invalid argument";
    case DL_ERR_OVERLAP: return "a destination overlaps another destination or a source";
    case DL_ERR_HIP: return "HIP call failed";
    case DL_ERR_TIMEOUT: return "timed out";
    case DL_ERR_STATE: return "library or prelaunch mode not in the required state";
    case DL_ERR_EXPIRED: return "armed request cancelled or not triggered in time; nothing or only part was copied";
    case DL_ERR_CAPACITY: return "the request exceeds the stated maximum of this entry point";
    case DL_ERR_LOST: return "a kernel of an earlier request never saw its copy table complete and copied nothing or only part";
    default: return "unknown status";
    }
}

int dl_last_hip_error(void) { return g_dl.last_hip; }

int dl_get_config(dl_config *cfg)
{
    DL_LOCKED;
    if (!cfg) return DL_ERR_INVALID;
    *cfg = g_dl.cfg;
    return DL_OK;
}

int dl_set_config(const dl_config *cfg)
{
    DL_LOCKED;
    if (!cfg || !config_valid(*cfg)) return DL_ERR_INVALID;
    g_dl.cfg = *cfg;
    return DL_OK;
}

int dl_parse_config(const char *text, dl_config *cfg)
{
    if (!cfg) return DL_ERR_INVALID;
    if (!text) return DL_OK;
    dl_config c = *cfg;
    const char *p = text;
    while (*p) {
        while (*p == ',' || *p == ' ') ++p;
        if (!*p) break;
        const char *eq = strchr(p, '=');
        if (!eq || eq == p) return DL_ERR_INVALID;
        char *end = nullptr;
        const unsigned long long v = strtoull(eq + 1, &end, 0);
        if (end == eq + 1 || (*end && *end != ',' && *end != ' ')) return DL_ERR_INVALID;
        const size_t len = (size_t)(eq - p);
        bool known = false;
        for (const config_field &f : CONFIG_FIELDS) {
            if (strlen(f.name) != len || strncmp(f.name, p, len)) continue;
            if (f.p32) {
                if (v > 0xFFFFFFFFull) return DL_ERR_INVALID;
                c.*(f.p32) = (uint32_t)v;
            } else {
                c.*(f.p64) = (uint64_t)v;
            }
            known = true;
        }
        if (!known) return DL_ERR_INVALID;
        p = end;
    }
    if (!config_valid(c)) return DL_ERR_INVALID;
    *cfg = c;
    return DL_OK;
}

int dl_batch_copy(const dl_copy_desc *desc, size_t n, void *stream)
{
    DL_LOCKED;
    if (g_dl.cfg.infer_broadcast && n > 1)
        return lower_and_execute([&](sink &s) { return lower_batch_inferred(desc, n, s); }, stream, DL_OP_BATCH);
    return lower_and_execute([&](sink &s) { return lower_batch(desc, n, s); }, stream, DL_OP_BATCH);
}

int dl_batch_fanout(const dl_plan_item *items, size_t n, void *stream)
{
    DL_LOCKED;
    if (n && !items) return DL_ERR_INVALID;
    return lower_and_execute(
        [&](sink &s) -> long {
            for (size_t i = 0; i < n; ++i) {
                if (items[i].k < 1 || items[i].k > (uint32_t)DL_PLAN_FANOUT) return DL_ERR_INVALID;
                if (items[i].bytes == 0) continue;
                if (!items[i].src) return DL_ERR_INVALID;
                for (uint32_t j = 0; j < items[i].k; ++j)
                    if (!items[i].dst[j]) return DL_ERR_INVALID;
                s.put(items[i].src, items[i].bytes, items[i].dst, items[i].k);
            }
            return (long)s.n;
        },
        stream, DL_OP_BATCH);
}

int dl_token_dispatch(const void *const *in, void *const *out, int W, const uint32_t *tokens, size_t row_bytes,
                      const uint8_t *dest, void *stream)
{
    DL_LOCKED;
    if (g_dl.inited && dl_device_error_pending()) return DL_ERR_LOST;
    if (g_dl.inited && (g_dl.mode == DL_MODE_ONESHOT || g_dl.mode == DL_MODE_AUTO) && !g_dl.validate &&
        g_dl.cfg.device_lowering) {
        // many tokens: only the destination mask goes to the device, which works out the rest itself (one-shot
        // execution; in DL_MODE_AUTO that is what the table gives such a request)
        bool taken = false;
        const int rc = dl_dispatch_on_device(in, out, W, tokens, row_bytes, dest, (hipStream_t)stream, &taken);
        if (taken) t_dl_last.mode = DL_MODE_ONESHOT;
        if (taken || rc != DL_OK) return rc;
    }
    return lower_and_execute([&](sink &s) { return lower_token_dispatch(in, out, W, tokens, row_bytes, dest, s); },
                             stream, DL_OP_TOKEN_DISPATCH);
}

long dl_plan_token_dispatch(const void *const *in, void *const *out, int W, const uint32_t *tokens, size_t row_bytes,
                            const uint8_t *dest, dl_plan_item *items, size_t cap)
{
    sink s{items, items ? cap : 0};
    return lower_token_dispatch(in, out, W, tokens, row_bytes, dest, s);
}

long dl_plan_batch_inferred(const dl_copy_desc *desc, size_t n, dl_plan_item *items, size_t cap)
{
    DL_LOCKED;
    sink s{items, items ? cap : 0};
    return lower_batch_inferred(desc, n, s);
}

int dl_broadcast(const void *src, void *const *dsts, int k, size_t bytes, void *stream)
{
    DL_LOCKED;
    return lower_and_execute([&](sink &s) { return lower_broadcast(src, dsts, k, bytes, s); }, stream, DL_OP_BROADCAST);
}

int dl_allgather(const void *const *in, void *const *out, int W, size_t bytes_per_rank, void *stream)
{
    DL_LOCKED;
    const int fuse = (int)g_dl.cfg.fuse_broadcast;
    return lower_and_execute([&](sink &s) { return lower_allgather(in, out, W, bytes_per_rank, fuse, s); }, stream,
                             DL_OP_ALLGATHER);
}

int dl_alltoall(const void *const *in, void *const *out, int W, const size_t *chunk_bytes, void *stream)
{
    DL_LOCKED;
    return lower_and_execute([&](sink &s) { return lower_alltoall(in, out, W, chunk_bytes, s); }, stream, DL_OP_ALLTOALL);
}

int dl_batch_swap(const dl_swap_desc *desc, size_t n, void *stream)
{
    DL_LOCKED;
    return execute_swaps(desc, n, stream);
}

int dl_alltoall_inplace(void *const *buf, int W, size_t chunk_bytes, void *stream)
{
    DL_LOCKED;
    const long n = lower_alltoall_inplace(buf, W, chunk_bytes, nullptr, 0);
    if (n < 0) return (int)n;
    g_swap_descs.resize((size_t)n);
    lower_alltoall_inplace(buf, W, chunk_bytes, g_swap_descs.data(), g_swap_descs.size());
    return execute_swaps(g_swap_descs.data(), g_swap_descs.size(), stream);
}

long dl_plan_alltoall_inplace(void *const *buf, int W, size_t chunk_bytes, dl_swap_desc *swaps, size_t cap)
{
    return lower_alltoall_inplace(buf, W, chunk_bytes, swaps, swaps ? cap : 0);
}

long dl_plan_swap_first_hazard(const dl_swap_desc *swaps, size_t n)
{
    if (!swaps) return -1;
    return swap_first_hazard(swaps, n);
}

long dl_plan_allgather(const void *const *in, void *const *out, int W, size_t bytes_per_rank, int fuse_broadcast,
                       dl_plan_item *items, size_t cap)
{
    sink s{items, items ? cap : 0};
    return lower_allgather(in, out, W, bytes_per_rank, fuse_broadcast, s);
}

long dl_plan_alltoall(const void *const *in, void *const *out, int W, const size_t *chunk_bytes, dl_plan_item *items,
                      size_t cap)
{
    sink s{items, items ? cap : 0};
    return lower_alltoall(in, out, W, chunk_bytes, s);
}

long dl_plan_broadcast(const void *src, void *const *dsts, int k, size_t bytes, dl_plan_item *items, size_t cap)
{
    sink s{items, items ? cap : 0};
    return lower_broadcast(src, dsts, k, bytes, s);
}

long dl_plan_batch(const dl_copy_desc *desc, size_t n, dl_plan_item *items, size_t cap)
{
    sink s{items, items ? cap : 0};
    return lower_batch(desc, n, s);
}

long dl_plan_first_hazard(const dl_plan_item *items, size_t n)
{
    if (!items) return -1;
    return first_hazard(items, n);
}

uint64_t dl_plan_tiles(const dl_plan_item *items, size_t n, uint32_t tile_bytes)
{
    if (!items || tile_bytes < DL_CUT || tile_bytes % DL_CUT) return 0;
    uint64_t t = 0;
    for (size_t i = 0; i < n; ++i) t += dl_item_tiles(*reinterpret_cast<const dl_fused_item *>(&items[i]), tile_bytes);
    return t;
}

}  // extern "C"
