// Comparison program, not part of the library: the runtime's own batched copy call (the call the
// paper proposes to extend, Sec. VI) timed on the all-gather's 64 block copies, W = 8 ranks in one
// GPU's memory.  It is a program of its own because it links the ROCm installation's HIP runtime,
// which exports hipMemcpyBatchAsync; a process that has PyTorch loaded runs on the runtime bundled
// with PyTorch, which does not.  Prints one JSON line.
//
// usage: dl_runtime_batch [bytes_per_rank ...]
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

namespace {

constexpr int W = 8;

double now_us()
{
    using namespace std::chrono;
    return duration<double, std::micro>(steady_clock::now().time_since_epoch()).count();
}

double pct(std::vector<double> v, double q)
{
    std::sort(v.begin(), v.end());
    return v[(size_t)(q * (double)(v.size() - 1))];
}

struct fail {
    std::string what;
};

void check(hipError_t e, const char *what)
{
    if (e != hipSuccess) throw fail{std::string(what) + ": " + hipGetErrorString(e)};
}

struct list {
    std::vector<void *> dst, src;
    std::vector<size_t> bytes;
};

// One batched call.  The attribute array is documented as unsupported; one stream-ordered
// attribute for all copies is tried first (the form the CUDA call of the same name requires),
// then none.
hipError_t batch(list &l, int form, hipStream_t s)
{
    size_t fail_idx = 0;
    if (form == 0) {
        hipMemcpyAttributes a{};
        a.srcAccessOrder = hipMemcpySrcAccessOrderStream;
        size_t idx = 0;
        return hipMemcpyBatchAsync(l.dst.data(), l.src.data(), l.bytes.data(), l.dst.size(), &a, &idx, 1, &fail_idx, s);
    }
    return hipMemcpyBatchAsync(l.dst.data(), l.src.data(), l.bytes.data(), l.dst.size(), nullptr, nullptr, 0, &fail_idx, s);
}

}  // namespace

int main(int argc, char **argv)
{
    std::vector<size_t> sizes;
    for (int i = 1; i < argc; ++i) sizes.push_back((size_t)strtoull(argv[i], nullptr, 10));
    if (sizes.empty()) sizes = {4096, 65536, 1u << 20, 16u << 20};
    std::string out = "{\"runtime_version\": ";
    try {
        int ver = 0;
        check(hipRuntimeGetVersion(&ver), "hipRuntimeGetVersion");
        out += std::to_string(ver) + ", \"rows\": [";
        check(hipSetDevice(0), "hipSetDevice");
        hipStream_t s;
        check(hipStreamCreate(&s), "hipStreamCreate");
        hipEvent_t e0, e1;
        check(hipEventCreate(&e0), "hipEventCreate");
        check(hipEventCreate(&e1), "hipEventCreate");
        bool first_row = true;
        for (size_t B : sizes) {
            char *in[W], *o[W];
            for (int r = 0; r < W; ++r) {
                check(hipMalloc((void **)&in[r], B), "hipMalloc");
                check(hipMalloc((void **)&o[r], W * B), "hipMalloc");
                check(hipMemset(in[r], r + 1, B), "hipMemset");
                check(hipMemset(o[r], 0, W * B), "hipMemset");
            }
            list l;
            for (int r = 0; r < W; ++r)
                for (int j = 0; j < W; ++j) {
                    l.dst.push_back(o[r] + (size_t)j * B);
                    l.src.push_back(in[j]);
                    l.bytes.push_back(B);
                }
            std::string row = "{\"bytes_per_rank\": " + std::to_string(B);
            int form = 0;
            hipError_t e = batch(l, form, s);
            if (e != hipSuccess) {
                (void)hipGetLastError();
                form = 1;
                e = batch(l, form, s);
            }
            if (e != hipSuccess) {
                (void)hipGetLastError();
                row += std::string(", \"memcpy_batch\": \"") + hipGetErrorString(e) + "\"";
            } else {
                check(hipStreamSynchronize(s), "hipStreamSynchronize");
                // the result, once: rank 5's receive buffer must hold W blocks of bytes 1..W
                std::vector<unsigned char> h(W * B);
                check(hipMemcpy(h.data(), o[5], W * B, hipMemcpyDeviceToHost), "hipMemcpy");
                bool ok = true;
                for (int j = 0; j < W && ok; ++j)
                    ok = h[(size_t)j * B] == j + 1 && h[(size_t)j * B + B - 1] == j + 1;
                const int iters = B <= (1u << 20) ? 100 : 20;
                std::vector<double> lat;
                for (int i = 0; i < 10 + iters; ++i) {
                    const double t0 = now_us();
                    check(batch(l, form, s), "hipMemcpyBatchAsync");
                    check(hipStreamSynchronize(s), "hipStreamSynchronize");
                    if (i >= 10) lat.push_back(now_us() - t0);
                }
                check(hipEventRecord(e0, s), "hipEventRecord");
                for (int i = 0; i < 10; ++i) check(batch(l, form, s), "hipMemcpyBatchAsync");
                check(hipEventRecord(e1, s), "hipEventRecord");
                check(hipEventSynchronize(e1), "hipEventSynchronize");
                float ms = 0;
                check(hipEventElapsedTime(&ms, e0, e1), "hipEventElapsedTime");
                char buf[256];
                snprintf(buf, sizeof buf,
                         ", \"memcpy_batch\": {\"attributes\": %s, \"result_ok\": %s, \"host_us\": {\"p50\": %.2f, \"p10\": %.2f, "
                         "\"p90\": %.2f}, \"device_us\": %.2f}",
                         form == 0 ? "\"one, stream-ordered\"" : "\"none\"", ok ? "true" : "false", pct(lat, .5),
                         pct(lat, .1), pct(lat, .9), ms * 1e3 / 10);
                row += buf;
            }
            // the same list as one hipMemcpyAsync per copy, in this runtime
            {
                const int iters = B <= (1u << 20) ? 50 : 10;
                std::vector<double> lat;
                for (int i = 0; i < 5 + iters; ++i) {
                    const double t0 = now_us();
                    for (size_t c = 0; c < l.dst.size(); ++c)
                        check(hipMemcpyAsync(l.dst[c], l.src[c], l.bytes[c], hipMemcpyDeviceToDevice, s), "hipMemcpyAsync");
                    check(hipStreamSynchronize(s), "hipStreamSynchronize");
                    if (i >= 5) lat.push_back(now_us() - t0);
                }
                char buf[160];
                snprintf(buf, sizeof buf, ", \"memcpy_async_per_chunk_host_us\": {\"p50\": %.2f, \"p10\": %.2f, \"p90\": %.2f}",
                         pct(lat, .5), pct(lat, .1), pct(lat, .9));
                row += buf;
            }
            row += "}";
            out += (first_row ? "" : ", ") + row;
            first_row = false;
            for (int r = 0; r < W; ++r) {
                check(hipFree(in[r]), "hipFree");
                check(hipFree(o[r]), "hipFree");
            }
        }
        out += "]}";
        check(hipStreamDestroy(s), "hipStreamDestroy");
    } catch (const fail &f) {
        printf("{\"error\": \"%s\"}\n", f.what.c_str());
        return 1;
    }
    printf("%s\n", out.c_str());
    return 0;
}
