// Opt-in per-kernel timing with HIP events (off by default; when off, launches are not touched).
// When enabled, every kernel launch of the library is bracketed by two events on the launch stream;
// kfac_kernel_timing_report() waits for them and adds up elapsed time and launch count per kernel name.
// This is a measurement aid for benchmarks: it serialises nothing but adds two event records per launch,
// so it is never enabled inside a throughput measurement.
#include <atomic>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "common.h"

namespace kfac {

struct TimedLaunch {
    const char* name;
    hipEvent_t start, stop;
};

static std::mutex g_mu;
static std::atomic<bool> g_enabled{false};
static std::vector<TimedLaunch> g_launches;

bool timing_enabled() { return g_enabled.load(std::memory_order_relaxed); }

void timing_begin(const char* name, hipStream_t stream, void** token) {
    *token = nullptr;
    if (!timing_enabled()) return;
    TimedLaunch* tl = new TimedLaunch;
    tl->name = name;
    if (hipEventCreate(&tl->start) != hipSuccess || hipEventCreate(&tl->stop) != hipSuccess) {
        delete tl;
        return;
    }
    (void)hipEventRecord(tl->start, stream);
    *token = tl;
}

void timing_end(hipStream_t stream, void* token) {
    if (!token) return;
    TimedLaunch* tl = (TimedLaunch*)token;
    (void)hipEventRecord(tl->stop, stream);
    std::lock_guard<std::mutex> lk(g_mu);
    g_launches.push_back(*tl);
    delete tl;
}

}  // namespace kfac

extern "C" int kfac_kernel_timing_enable(int enable) {
    std::lock_guard<std::mutex> lk(kfac::g_mu);
    kfac::g_enabled.store(enable != 0);
    return KFAC_OK;
}

extern "C" int kfac_kernel_timing_report(char* buf_host, size_t buf_bytes) {
    if (!buf_host || buf_bytes == 0) return KFAC_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(kfac::g_mu);
    struct Row { std::string name; double ms; long n; };
    std::vector<Row> rows;
    for (auto& tl : kfac::g_launches) {
        float ms = 0.f;
        if (hipEventSynchronize(tl.stop) != hipSuccess || hipEventElapsedTime(&ms, tl.start, tl.stop) != hipSuccess)
            ms = 0.f;
        (void)hipEventDestroy(tl.start);
        (void)hipEventDestroy(tl.stop);
        bool found = false;
        for (auto& r : rows)
            if (r.name == tl.name) { r.ms += ms; r.n += 1; found = true; break; }
        if (!found) rows.push_back({tl.name, ms, 1});
    }
    kfac::g_launches.clear();
    std::string out;
    for (auto& r : rows) {
        char line[256];
        snprintf(line, sizeof line, "%s %.6f %ld\n", r.name.c_str(), r.ms, r.n);
        out += line;
    }
    if (out.size() + 1 > buf_bytes) return KFAC_ERR_WORKSPACE;
    memcpy(buf_host, out.c_str(), out.size() + 1);
    return KFAC_OK;
}
