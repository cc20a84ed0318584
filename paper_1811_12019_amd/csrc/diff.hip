// Change rate of a statistic between two refreshes,  Diff = ||X - X_prev||_F / ||X_prev||_F  (Sec. 5.4, "Staleness of
// Fisher information"), for many matrices in one call.  HBM bound: 8 bytes per element, each read once.
// Two deterministic passes: every workgroup reduces one 8192-element chunk of one matrix to a (numerator,
// denominator) pair of doubles in the caller's scratch; one workgroup per matrix then adds its pairs in a fixed order.
#include <mutex>

#include "common.h"

namespace kfac {

constexpr int DF_MAX = 128;               // matrices per launch (argument block under 4 KB)
constexpr unsigned DF_CHUNK = 8192;       // elements per workgroup

struct DiffBatch {
    int count;
    unsigned prefix[DF_MAX + 1];          // first chunk of matrix i
    unsigned long long n[DF_MAX];         // elements of matrix i
    const float* x[DF_MAX];
    const float* x_prev[DF_MAX];
};

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

__global__ __launch_bounds__(256) void diff_partial_kernel(DiffBatch b, double* partial_) {
    __shared__ double red[2][4];
    const int t = threadIdx.x;
    const unsigned wg = blockIdx.x;
    const int m = __syncthreads_count(t < b.count - 1 && b.prefix[t + 1] <= wg);
    const size_t n = b.n[m];
    const gfloat* __restrict__ X = as_global(b.x[m]);
    const gfloat* __restrict__ Y = as_global(b.x_prev[m]);
    const size_t base = (size_t)(wg - b.prefix[m]) * DF_CHUNK;
    const bool aligned = (((uintptr_t)b.x[m] | (uintptr_t)b.x_prev[m]) & 15) == 0;
    float num = 0.f, den = 0.f;                       // 32 terms per thread: fp32 is ample, the sums across threads are double
    if (aligned && base + DF_CHUNK <= n) {
        v4f xv[8], yv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const size_t i = base + (size_t)(j * 256 + t) * 4;
            xv[j] = *(const KFAC_AS1 v4f*)(X + i);
            yv[j] = *(const KFAC_AS1 v4f*)(Y + i);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float dlt = xv[j][e] - yv[j][e];
                num = fmaf(dlt, dlt, num);
                den = fmaf(yv[j][e], yv[j][e], den);
            }
    } else {
        for (size_t i = base + t; i < n && i < base + DF_CHUNK; i += 256) {
            const float dlt = X[i] - Y[i];
            num = fmaf(dlt, dlt, num);
            den = fmaf(Y[i], Y[i], den);
        }
    }
    const double wn = wave_sum((double)num), wd = wave_sum((double)den);
    if ((t & 63) == 0) { red[0][t >> 6] = wn; red[1][t >> 6] = wd; }
    __syncthreads();
    if (t == 0) {
        partial_[2 * (size_t)wg] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        partial_[2 * (size_t)wg + 1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
}

__global__ __launch_bounds__(256) void diff_final_kernel(DiffBatch b, const double* partial_, float* out) {
    __shared__ double red[2][256];
    const int m = blockIdx.x, t = threadIdx.x;
    const unsigned first = b.prefix[m], last = b.prefix[m + 1];
    double num = 0.0, den = 0.0;
    for (unsigned c = first + t; c < last; c += 256) { num += partial_[2 * (size_t)c]; den += partial_[2 * (size_t)c + 1]; }
    red[0][t] = num; red[1][t] = den;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (t < s) { red[0][t] += red[0][t + s]; red[1][t] += red[1][t + s]; }
        __syncthreads();
    }
    if (t == 0) out[m] = (float)(sqrt(red[0][0]) / sqrt(red[1][0]));
}

static unsigned chunks_of(int dim) { return (unsigned)(((size_t)dim * dim + DF_CHUNK - 1) / DF_CHUNK); }

// Scratch of the entry point that allocates nothing: room for the chunk pairs of 2^29 matrix elements (2 GiB of fp32
// factors; all 108 factors of ResNet-50 are 0.15 x 2^30 elements), 1 MiB per GPU the library runs on, held until the
// process ends.  In host code the array's name only stands for the symbol: its device address is looked up once per
// device (static_scratch) and that pointer is what the kernels get.
constexpr size_t DF_STATIC_CHUNKS = 65536;
static __device__ __align__(256) double scratch[2 * DF_STATIC_CHUNKS];

constexpr int DF_MAX_DEVICES = 64;
static std::mutex g_scratch_mu;
static double* g_scratch_ptr[DF_MAX_DEVICES] = {};

// Device address of `scratch` on the current device, or nullptr if it cannot be had.
static double* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= DF_MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = (double*)p;
    }
    return g_scratch_ptr[dev];
}

static int diff_check(const kfac_diff_item* items_host, int32_t count, const float* out) {
    if (!items_host || count < 0) return KFAC_ERR_INVALID_ARG;
    if (count == 0) return KFAC_OK;
    if (!out) return KFAC_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i)
        if (!items_host[i].x || !items_host[i].x_prev || items_host[i].dim <= 0 || items_host[i].dim > 32768)
            return KFAC_ERR_INVALID_ARG;
    return KFAC_OK;
}

// Both passes for all matrices; partial: 2 doubles per chunk, device memory.
static int diff_run(const kfac_diff_item* items_host, int32_t count, float* out, double* partial, hipStream_t stream) {
    for (int first = 0; first < count; first += DF_MAX) {
        const int cnt = count - first < DF_MAX ? count - first : DF_MAX;
        DiffBatch b;
        b.count = cnt;
        unsigned chunks = 0;
        for (int i = 0; i < cnt; ++i) {
            const kfac_diff_item& it = items_host[first + i];
            b.prefix[i] = chunks;
            b.n[i] = (unsigned long long)it.dim * it.dim;
            b.x[i] = it.x;
            b.x_prev[i] = it.x_prev;
            chunks += chunks_of(it.dim);
        }
        b.prefix[cnt] = chunks;
        KFAC_LAUNCH(diff_partial_kernel, dim3(chunks), dim3(256), stream, b, partial);
        KFAC_LAUNCH(diff_final_kernel, dim3(cnt), dim3(256), stream, b, (const double*)partial, out + first);
        partial += 2 * (size_t)chunks;
    }
    return KFAC_OK;
}

}  // namespace kfac

using namespace kfac;

extern "C" size_t kfac_factor_diff_workspace_bytes(const kfac_diff_item* items_host, int32_t count) {
    if (!items_host || count <= 0) return 0;
    size_t chunks = 0;
    for (int i = 0; i < count; ++i) {
        if (items_host[i].dim <= 0 || items_host[i].dim > 32768) return 0;
        chunks += chunks_of(items_host[i].dim);
    }
    return align_up(chunks * 2 * sizeof(double), 256);
}

extern "C" int kfac_factor_diff_batched(const kfac_diff_item* items_host, int32_t count, float* out, void* ws,
                                        size_t ws_bytes, void* stream) {
    const int rc = diff_check(items_host, count, out);
    if (rc != KFAC_OK || count == 0) return rc;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < kfac_factor_diff_workspace_bytes(items_host, count)) return KFAC_ERR_WORKSPACE;
    return diff_run(items_host, count, out, (double*)ws, (hipStream_t)stream);
}

extern "C" int kfac_factor_diff_batched_noalloc(const kfac_diff_item* items_host, int32_t count, float* out, void* stream) {
    const int rc = diff_check(items_host, count, out);
    if (rc != KFAC_OK || count == 0) return rc;
    size_t chunks = 0;
    for (int i = 0; i < count; ++i) chunks += chunks_of(items_host[i].dim);
    if (chunks > DF_STATIC_CHUNKS) return KFAC_ERR_TOO_LARGE;
    double* partial = static_scratch();
    if (!partial) return KFAC_ERR_HIP;
    return diff_run(items_host, count, out, partial, (hipStream_t)stream);
}

extern "C" size_t kfac_factor_diff_noalloc_max_elements(void) { return DF_STATIC_CHUNKS * (size_t)DF_CHUNK; }
