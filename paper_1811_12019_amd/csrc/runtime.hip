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

// ---- probes of the machine's peaks (what a kernel can at best reach on this GPU) ---------------------------------------
// Register-resident matrix-core loops: four independent accumulator blocks per wavefront, operands never reloaded.
template <int KIND>
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ out, int iters) {
    v16f c0 = {}, c1 = {}, c2 = {}, c3 = {};
    if constexpr (KIND == KFAC_F32) {
        const float a = threadIdx.x * 1e-3f, b = 1.0f;
        for (int i = 0; i < iters; ++i) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c3, 0, 0, 0);
        }
    } else if constexpr (KIND == KFAC_BF16) {
        v8bf a, b;
        for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 1e-3f); b[i] = (__bf16)1.0f; }
        for (int i = 0; i < iters; ++i) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
        }
    } else {
        typedef _Float16 v8h_t __attribute__((ext_vector_type(8)));
        v8h_t a, b;
        for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(threadIdx.x * 1e-3f); b[i] = (_Float16)1.0f; }
        for (int i = 0; i < iters; ++i) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
        }
    }
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = c0[0] + c1[1] + c2[2] + c3[3];
}

// Streaming copy / read of 16-byte vectors, grid-stride.
__global__ __launch_bounds__(256) void probe_copy_kernel(const v4f* __restrict__ in, v4f* __restrict__ out, size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) out[i] = in[i];
}
__global__ __launch_bounds__(256) void probe_read_kernel(const v4f* __restrict__ in, float* __restrict__ out, size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    v4f s = {0.f, 0.f, 0.f, 0.f};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) s += in[i];
    if (s.x + s.y + s.z + s.w == 12345.678f) out[0] = 1.f;      // (keeps the loads alive)
}

}  // namespace kfac

extern "C" int kfac_probe_mfma(int32_t dtype, int32_t workgroups, int32_t iters, float* out, void* stream) {
    if (!out || workgroups <= 0 || workgroups > 65536 || iters <= 0) return KFAC_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == KFAC_F32) hipLaunchKernelGGL(kfac::probe_mfma_kernel<KFAC_F32>, dim3(workgroups), dim3(256), 0, st, out, iters);
    else if (dtype == KFAC_BF16) hipLaunchKernelGGL(kfac::probe_mfma_kernel<KFAC_BF16>, dim3(workgroups), dim3(256), 0, st, out, iters);
    else if (dtype == KFAC_F16) hipLaunchKernelGGL(kfac::probe_mfma_kernel<KFAC_F16>, dim3(workgroups), dim3(256), 0, st, out, iters);
    else return KFAC_ERR_INVALID_ARG;
    return hipGetLastError() == hipSuccess ? KFAC_OK : KFAC_ERR_HIP;
}

extern "C" int kfac_probe_copy(const void* src, void* dst, size_t bytes, int32_t workgroups, void* stream) {
    if (!src || bytes == 0 || (bytes & 15) || workgroups <= 0 || workgroups > (1 << 20)) return KFAC_ERR_INVALID_ARG;
    if (((uintptr_t)src | (uintptr_t)dst) & 15) return KFAC_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (dst) hipLaunchKernelGGL(kfac::probe_copy_kernel, dim3(workgroups), dim3(256), 0, st, (const kfac::v4f*)src, (kfac::v4f*)dst, bytes / 16);
    else return KFAC_ERR_INVALID_ARG;
    return hipGetLastError() == hipSuccess ? KFAC_OK : KFAC_ERR_HIP;
}

extern "C" int kfac_probe_read(const void* src, float* sink, size_t bytes, int32_t workgroups, void* stream) {
    if (!src || !sink || bytes == 0 || (bytes & 15) || ((uintptr_t)src & 15) || workgroups <= 0 || workgroups > (1 << 20))
        return KFAC_ERR_INVALID_ARG;
    hipLaunchKernelGGL(kfac::probe_read_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, (const kfac::v4f*)src, sink, bytes / 16);
    return hipGetLastError() == hipSuccess ? KFAC_OK : KFAC_ERR_HIP;
}

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
