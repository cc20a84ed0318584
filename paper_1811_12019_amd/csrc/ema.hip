// Running average of a Kronecker factor: S <- decay * S + (1 - decay) * X, element-wise over dim x dim floats.
// Bandwidth-bound: 12 bytes of HBM traffic per element (read S, read X, write S), one grid-stride pass.
#include "common.h"

namespace kfac {

__global__ __launch_bounds__(256) void ema_kernel(float* __restrict__ running, const float* __restrict__ fresh,
                                                  size_t n, float decay, float one_minus) {
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    const bool aligned = (((uintptr_t)running | (uintptr_t)fresh) & 15) == 0;
    for (; i < n; i += stride) {
        if (aligned && i + 3 < n) {
            v4f s = *(const v4f*)(running + i);
            v4f x = *(const v4f*)(fresh + i);
            v4f o;
            o.x = fmaf(decay, s.x, one_minus * x.x);
            o.y = fmaf(decay, s.y, one_minus * x.y);
            o.z = fmaf(decay, s.z, one_minus * x.z);
            o.w = fmaf(decay, s.w, one_minus * x.w);
            *(v4f*)(running + i) = o;
        } else {
            for (size_t j = i; j < n && j < i + 4; ++j) running[j] = fmaf(decay, running[j], one_minus * fresh[j]);
        }
    }
}

// Many running averages in one launch.  Each workgroup owns one 4096-element chunk of one matrix; the chunk ->
// matrix map is a prefix array carried in the kernel arguments and searched by one ballot-style count.
constexpr int EMA_MAX = 128;            // matrices per launch (the argument block stays under 4 KB)
constexpr unsigned EMA_CHUNK = 4096;    // elements per workgroup

struct EmaBatch {
    int count;
    unsigned prefix[EMA_MAX + 1];       // first chunk of matrix i
    unsigned long long n[EMA_MAX];      // elements of matrix i
    float* running[EMA_MAX];
    const float* fresh[EMA_MAX];
};

__global__ __launch_bounds__(256) void ema_batched_kernel(EmaBatch b, float decay, float one_minus) {
    const int t = threadIdx.x;
    const unsigned wg = blockIdx.x;
    const int m = __syncthreads_count(t < b.count - 1 && b.prefix[t + 1] <= wg);   // matrices that end before this chunk
    const size_t n = b.n[m];
    gfloat* __restrict__ run = as_global(b.running[m]);
    const gfloat* __restrict__ fre = as_global(b.fresh[m]);
    const size_t base = (size_t)(wg - b.prefix[m]) * EMA_CHUNK;
    const bool aligned = (((uintptr_t)b.running[m] | (uintptr_t)b.fresh[m]) & 15) == 0;
    if (aligned && base + EMA_CHUNK <= n) {
        v4f s[4], x[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const size_t i = base + (size_t)(j * 256 + t) * 4;
            s[j] = *(const KFAC_AS1 v4f*)(run + i);
            x[j] = *(const KFAC_AS1 v4f*)(fre + i);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const size_t i = base + (size_t)(j * 256 + t) * 4;
            v4f o;
            o.x = fmaf(decay, s[j].x, one_minus * x[j].x);
            o.y = fmaf(decay, s[j].y, one_minus * x[j].y);
            o.z = fmaf(decay, s[j].z, one_minus * x[j].z);
            o.w = fmaf(decay, s[j].w, one_minus * x[j].w);
            *(KFAC_AS1 v4f*)(run + i) = o;
        }
    } else {
        for (size_t i = base + t; i < n && i < base + EMA_CHUNK; i += 256) run[i] = fmaf(decay, run[i], one_minus * fre[i]);
    }
}

}  // namespace kfac

extern "C" int kfac_ema(float* running, const float* fresh, int32_t dim, float decay, void* stream) {
    if (!running || !fresh || dim <= 0 || dim > 32768) return KFAC_ERR_INVALID_ARG;
    if (!(decay >= 0.f && decay <= 1.f)) return KFAC_ERR_INVALID_ARG;
    const size_t n = (size_t)dim * dim;
    const float* rb = running;
    if (!(fresh + n <= rb || rb + n <= fresh)) return KFAC_ERR_INVALID_ARG;   // overlap
    size_t blocks = (n + 1023) / 1024;
    if (blocks > 256 * 16) blocks = 256 * 16;
    KFAC_LAUNCH(kfac::ema_kernel, dim3((unsigned)blocks), dim3(256), (hipStream_t)stream, running, fresh, n,
                       decay, 1.0f - decay);
    return KFAC_OK;
}

extern "C" int kfac_ema_batched(const kfac_ema_item* items_host, int32_t count, float decay, void* stream) {
    if (!items_host || count < 0) return KFAC_ERR_INVALID_ARG;
    if (!(decay >= 0.f && decay <= 1.f)) return KFAC_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i) {
        const kfac_ema_item& it = items_host[i];
        if (!it.running || !it.fresh || it.dim <= 0 || it.dim > 32768) return KFAC_ERR_INVALID_ARG;
        const size_t n = (size_t)it.dim * it.dim;
        const float* rb = it.running;
        if (!(it.fresh + n <= rb || rb + n <= it.fresh)) return KFAC_ERR_INVALID_ARG;   // overlap
    }
    for (int first = 0; first < count; first += kfac::EMA_MAX) {
        const int cnt = count - first < kfac::EMA_MAX ? count - first : kfac::EMA_MAX;
        kfac::EmaBatch b;
        b.count = cnt;
        unsigned chunks = 0;
        for (int i = 0; i < cnt; ++i) {
            const kfac_ema_item& it = items_host[first + i];
            b.prefix[i] = chunks;
            b.n[i] = (unsigned long long)it.dim * it.dim;
            b.running[i] = it.running;
            b.fresh[i] = it.fresh;
            chunks += (unsigned)((b.n[i] + kfac::EMA_CHUNK - 1) / kfac::EMA_CHUNK);
        }
        b.prefix[cnt] = chunks;
        KFAC_LAUNCH(kfac::ema_batched_kernel, dim3(chunks), dim3(256), (hipStream_t)stream, b, decay, 1.0f - decay);
    }
    return KFAC_OK;
}
