// Measurement aid, separate from the library: timing loops around the public
// dl_* calls (host-observed latency per call, device time per call from HIP
// events on the launch stream) and the two runtime copy paths timed beside
// them: one hipMemcpyAsync per chunk, and one hipMemcpyBatchAsync.
// Links against libdmalatte.so; moves no bytes itself.
#include <dlfcn.h>
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <time.h>

#include <vector>

#include "../include/dmalatte.h"

extern "C" {

typedef struct dlb_request {
    int op;  // 0 batch, 1 broadcast, 2 all-gather, 3 all-to-all, 4 hipMemcpyAsync per desc, 5 hipMemcpyBatchAsync,
             // 6 batch of swaps (desc as {a, b, bytes}), 7 in-place all-to-all (out = buffers, bytes = chunk),
             // 8 token dispatch (in, out, W, tokens, bytes = row, dest), 9 fan-out batch (desc = dl_plan_item array),
             // 10 token dispatch with the mask in device memory (dest is a device pointer)
    int k;
    int W;
    int pad;
    const dl_copy_desc *desc;
    size_t n;
    const void *src;
    void *const *dsts;
    size_t bytes;
    const void *const *in;
    void *const *out;
    const size_t *C;
    const uint32_t *tokens;
    const uint8_t *dest;
} dlb_request;

static double now_us()
{
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return ts.tv_sec * 1e6 + ts.tv_nsec * 1e-3;
}

// Issue the request once.  Returns a dl_status, or 1000 + hipError_t for the runtime paths.
int dlb_issue(const dlb_request *r, void *stream)
{
    switch (r->op) {
    case 0: return dl_batch_copy(r->desc, r->n, stream);
    case 1: return dl_broadcast(r->src, r->dsts, r->k, r->bytes, stream);
    case 2: return dl_allgather(r->in, r->out, r->W, r->bytes, stream);
    case 3: return dl_alltoall(r->in, r->out, r->W, r->C, stream);
    case 4:
        for (size_t i = 0; i < r->n; ++i) {
            hipError_t e = hipMemcpyAsync(r->desc[i].dst, r->desc[i].src, r->desc[i].bytes, hipMemcpyDeviceToDevice,
                                          (hipStream_t)stream);
            if (e != hipSuccess) return 1000 + (int)e;
        }
        return 0;
    case 5: {
        static std::vector<void *> d, s;
        static std::vector<size_t> z;
        d.resize(r->n), s.resize(r->n), z.resize(r->n);
        for (size_t i = 0; i < r->n; ++i) {
            d[i] = r->desc[i].dst;
            s[i] = (void *)r->desc[i].src;
            z[i] = r->desc[i].bytes;
        }
        // The batched runtime copy exists only in newer HIP runtimes; take whatever the
        // runtime already loaded in this process offers, and report its absence.
        typedef hipError_t (*batch_fn)(void **, void **, size_t *, size_t, hipMemcpyAttributes *, size_t *, size_t,
                                       size_t *, hipStream_t);
        static batch_fn fn = (batch_fn)dlsym(RTLD_DEFAULT, "hipMemcpyBatchAsync");
        if (!fn) return 1000 + (int)hipErrorNotSupported;
        size_t fail = 0;
        hipError_t e = fn(d.data(), s.data(), z.data(), r->n, nullptr, nullptr, 0, &fail, (hipStream_t)stream);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return 1000 + (int)e;
        }
        return 0;
    }
    case 6: return dl_batch_swap((const dl_swap_desc *)r->desc, r->n, stream);
    case 7: return dl_alltoall_inplace(r->out, r->W, r->bytes, stream);
    case 8: return dl_token_dispatch(r->in, r->out, r->W, r->tokens, r->bytes, r->dest, stream);
    case 9: return dl_batch_fanout((const dl_plan_item *)r->desc, r->n, stream);
    case 10: return dl_token_dispatch_device(r->in, r->out, r->W, r->tokens, r->bytes, r->dest, stream);  // dest: device
    default: return DL_ERR_INVALID;
    }
}

// Host-observed latency per call, in microseconds.
// wait_mode 0 (one-shot): clock before the call -> hipStreamSynchronize(stream) returns.
// wait_mode 1 (prelaunch): the request is armed and seen resident first (untimed);
//             clock before dl_trigger() -> dl_wait() returns.
// wait_mode 2 (prelaunch): clock before the arming call -> dl_trigger() -> dl_wait() returns.
// wait_mode 3 (signal): clock before the call -> dl_wait() on its ticket returns (no trigger, no stream sync).
int dlb_time_host(const dlb_request *r, void *stream, int wait_mode, int warmup, int iters, double *us)
{
    for (int i = -warmup; i < iters; ++i) {
        double t0 = now_us();
        int rc = dlb_issue(r, stream);
        if (rc) return rc;
        if (wait_mode == 0) {
            hipError_t e = hipStreamSynchronize((hipStream_t)stream);
            if (e != hipSuccess) return 1000 + (int)e;
        } else if (wait_mode == 3) {
            rc = dl_wait(dl_last_ticket(), 2000000000ull);
            if (rc) return rc;
        } else {
            const uint64_t t = dl_last_ticket();
            if (wait_mode == 1) {
                rc = dl_wait_armed(t, 2000000000ull);
                if (rc) return rc;
                t0 = now_us();
            }
            rc = dl_trigger(t);
            if (rc) return rc;
            rc = dl_wait(t, 2000000000ull);
            if (rc) return rc;
        }
        const double t1 = now_us();
        if (i >= 0) us[i] = t1 - t0;
    }
    return 0;
}

// One-shot mode, per call in microseconds: call_us[i] = how long the dl_* call itself took on the host (lowering
// and the launch: the "control" phase), total_us[i] = clock before the call -> hipStreamSynchronize returns.
int dlb_time_call(const dlb_request *r, void *stream, int warmup, int iters, double *call_us, double *total_us)
{
    for (int i = -warmup; i < iters; ++i) {
        const double t0 = now_us();
        int rc = dlb_issue(r, stream);
        const double t1 = now_us();
        if (rc) return rc;
        if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return 1000;
        const double t2 = now_us();
        if (i >= 0) {
            call_us[i] = t1 - t0;
            total_us[i] = t2 - t0;
        }
    }
    return 0;
}

// Prelaunch mode with phase stamps (dl_set_trace(1) is switched on and off here), six numbers per call in
// microseconds: out[6 i + ..] =
//   0 arming call on the host (lowering and launch; off the critical path)
//   1 doorbell written by the host -> seen by the polling workgroup
//   2 doorbell seen -> first workgroup begins to copy (fan-out over the workgroups)
//   3 first copy begins -> last workgroup's stores have completed
//   4 last copy ends -> completion word issued (arrival counting)
//   5 completion word issued -> dl_wait returns on the host
// The device clock is related to the host clock anew before every call.
int dlb_phases(const dlb_request *r, int warmup, int iters, double *out)
{
    int rc = dl_set_trace(1);
    for (int i = -warmup; i < iters && !rc; ++i) {
        double tpu = 0, h0 = 0;
        rc = dl_trace_clock(&tpu, &h0);
        if (rc) break;
        const double c0 = now_us();
        rc = dlb_issue(r, nullptr);
        const double c1 = now_us();
        if (rc) break;
        const uint64_t t = dl_last_ticket();
        rc = dl_wait_armed(t, 2000000000ull);
        if (rc) break;
        const double t0 = now_us();
        rc = dl_trigger(t);
        if (!rc) rc = dl_wait(t, 2000000000ull);
        const double t1 = now_us();
        if (rc) break;
        dl_trace tr;
        rc = dl_get_trace(t, &tr);
        if (rc) break;
        if (i < 0) continue;
        const double h0_us = h0 * 1e-3;
        double *o = out + 6 * (size_t)i;
        o[0] = c1 - c0;
        o[1] = h0_us + (double)tr.doorbell_seen / tpu - t0;
        o[2] = ((double)tr.copy_begin - (double)tr.doorbell_seen) / tpu;
        o[3] = ((double)tr.copy_end - (double)tr.copy_begin) / tpu;
        o[4] = ((double)tr.completion_issued - (double)tr.copy_end) / tpu;
        o[5] = t1 - (h0_us + (double)tr.completion_issued / tpu);
    }
    (void)dl_set_trace(0);
    return rc;
}

// Host time of the lowering alone (no GPU work): microseconds per dl_plan_token_dispatch call.
int dlb_time_token_lowering(const dlb_request *r, dl_plan_item *items, size_t cap, int iters, double *us_per_call)
{
    long n = 0;
    const double t0 = now_us();
    for (int i = 0; i < iters; ++i) {
        n = dl_plan_token_dispatch(r->in, r->out, r->W, r->tokens, r->bytes, r->dest, items, cap);
        if (n < 0) return (int)n;
    }
    *us_per_call = (now_us() - t0) / iters;
    return 0;
}

// Device time per call: HIP events on `stream` around `calls` back-to-back issues.
int dlb_time_device(const dlb_request *r, void *stream, int warmup, int calls, double *us_per_call)
{
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return 1000;
    int rc = 0;
    for (int i = 0; i < warmup && !rc; ++i) rc = dlb_issue(r, stream);
    if (!rc && hipStreamSynchronize((hipStream_t)stream) != hipSuccess) rc = 1000;
    if (!rc) {
        (void)hipEventRecord(a, (hipStream_t)stream);
        for (int i = 0; i < calls && !rc; ++i) rc = dlb_issue(r, stream);
        (void)hipEventRecord(b, (hipStream_t)stream);
        if (hipEventSynchronize(b) != hipSuccess) rc = rc ? rc : 1000;
        float ms = 0;
        if (!rc && hipEventElapsedTime(&ms, a, b) == hipSuccess) *us_per_call = ms * 1e3 / calls;
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    return rc;
}

// Device time per call with cold caches: `rounds` passes over nreq requests of the same shape, each on buffers of
// its own (the caller sizes nreq so that one pass moves more bytes than the on-die caches hold), issued back to
// back between two HIP events.
int dlb_time_device_rotating(const dlb_request *const *reqs, int nreq, void *stream, int warmup_rounds, int rounds,
                             double *us_per_call)
{
    if (nreq < 1 || rounds < 1) return DL_ERR_INVALID;
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return 1000;
    int rc = 0;
    for (int i = 0; i < warmup_rounds * nreq && !rc; ++i) rc = dlb_issue(reqs[i % nreq], stream);
    if (!rc && hipStreamSynchronize((hipStream_t)stream) != hipSuccess) rc = 1000;
    if (!rc) {
        (void)hipEventRecord(a, (hipStream_t)stream);
        for (int i = 0; i < rounds * nreq && !rc; ++i) rc = dlb_issue(reqs[i % nreq], stream);
        (void)hipEventRecord(b, (hipStream_t)stream);
        if (hipEventSynchronize(b) != hipSuccess) rc = rc ? rc : 1000;
        float ms = 0;
        if (!rc && hipEventElapsedTime(&ms, a, b) == hipSuccess) *us_per_call = ms * 1e3 / (rounds * nreq);
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    return rc;
}

}  // extern "C"
