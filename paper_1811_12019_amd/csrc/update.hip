// Optimizer tail: the weight update with momentum (Sec. 4.3) followed by the rescaling of every layer's weights to norm
// sqrt(2 d_out) (Sec. 4.4), for all layers of a network in two launches:
//   pass 1   u = w - eta * P + m * (w - w_prev);  w_prev <- w;  w <- u;  sum of u^2 per 4096-element chunk (double)
//   pass 2   w <- sqrt(2 d_out) / (||u|| + eps) * w, the norm summed from the chunk sums in a fixed order
// HBM bound: 20 + 8 bytes per weight.
#include "common.h"

namespace kfac {

constexpr int WU_MAX = 128;               // layers per launch (a 4.6 KB argument block)
constexpr unsigned WU_CHUNK = 4096;       // elements per workgroup

struct UpdateBatch {
    int count;
    unsigned prefix[WU_MAX + 1];          // first chunk of layer i
    unsigned n[WU_MAX];                   // weights of layer i
    float target[WU_MAX];                 // sqrt(2 d_out)
    float* w[WU_MAX];
    float* w_prev[WU_MAX];
    const float* p[WU_MAX];
};

__device__ __forceinline__ int wu_locate(const UpdateBatch& b) {
    const int t = threadIdx.x;
    return __syncthreads_count(t < b.count - 1 && b.prefix[t + 1] <= blockIdx.x);
}

__global__ __launch_bounds__(256) void weight_update_kernel(UpdateBatch b, float eta, float mom, double* partial) {
    __shared__ double red[4];
    const int t = threadIdx.x;
    const int m = wu_locate(b);
    const unsigned n = b.n[m];
    gfloat* __restrict__ W = as_global(b.w[m]);
    gfloat* __restrict__ Wp = as_global(b.w_prev[m]);
    const gfloat* __restrict__ P = as_global(b.p[m]);
    const unsigned base = (blockIdx.x - b.prefix[m]) * WU_CHUNK;
    const bool aligned = (((uintptr_t)b.w[m] | (uintptr_t)b.w_prev[m] | (uintptr_t)b.p[m]) & 15) == 0;
    float ss = 0.f;
    if (aligned && base + WU_CHUNK <= n) {
        v4f w[4], wp[4], g[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned i = base + (j * 256 + t) * 4;
            w[j] = *(const KFAC_AS1 v4f*)(W + i);
            wp[j] = *(const KFAC_AS1 v4f*)(Wp + i);
            g[j] = *(const KFAC_AS1 v4f*)(P + i);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned i = base + (j * 256 + t) * 4;
            v4f u;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                u[e] = fmaf(mom, w[j][e] - wp[j][e], fmaf(-eta, g[j][e], w[j][e]));
                ss = fmaf(u[e], u[e], ss);
            }
            *(KFAC_AS1 v4f*)(Wp + i) = w[j];
            *(KFAC_AS1 v4f*)(W + i) = u;
        }
    } else {
        for (unsigned i = base + t; i < n && i < base + WU_CHUNK; i += 256) {
            const float w = W[i];
            const float u = fmaf(mom, w - Wp[i], fmaf(-eta, P[i], w));
            ss = fmaf(u, u, ss);
            Wp[i] = w;
            W[i] = u;
        }
    }
    double s = (double)ss;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
    if ((t & 63) == 0) red[t >> 6] = s;
    __syncthreads();
    if (t == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(256) void weight_rescale_kernel(UpdateBatch b, float eps, const double* partial) {
    __shared__ double red[256];
    const int t = threadIdx.x;
    const int m = wu_locate(b);
    // every workgroup of a layer adds the layer's chunk sums in the same order: same norm everywhere
    double s = 0.0;
    for (unsigned c = b.prefix[m] + t; c < b.prefix[m + 1]; c += 256) s += partial[c];
    red[t] = s;
    __syncthreads();
    for (int k = 128; k > 0; k >>= 1) {
        if (t < k) red[t] += red[t + k];
        __syncthreads();
    }
    const float scale = b.target[m] / ((float)sqrt(red[0]) + eps);
    const unsigned n = b.n[m];
    gfloat* __restrict__ W = as_global(b.w[m]);
    const unsigned base = (blockIdx.x - b.prefix[m]) * WU_CHUNK;
    if ((((uintptr_t)b.w[m]) & 15) == 0 && base + WU_CHUNK <= n) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned i = base + (j * 256 + t) * 4;
            v4f w = *(const KFAC_AS1 v4f*)(W + i);
            w *= scale;
            *(KFAC_AS1 v4f*)(W + i) = w;
        }
    } else {
        for (unsigned i = base + t; i < n && i < base + WU_CHUNK; i += 256) W[i] *= scale;
    }
}

static unsigned wu_chunks(unsigned n) { return (n + WU_CHUNK - 1) / WU_CHUNK; }

}  // namespace kfac

using namespace kfac;

static bool wu_item_ok(const kfac_update_item& it) {
    if (!it.w || !it.w_prev || !it.precond || it.n <= 0 || it.d_out <= 0) return false;
    const char *a = (const char*)it.w, *b = (const char*)it.w_prev, *c = (const char*)it.precond;
    const size_t bytes = (size_t)it.n * sizeof(float);
    auto apart = [&](const char* x, const char* y) { return x + bytes <= y || y + bytes <= x; };
    return apart(a, b) && apart(a, c) && apart(b, c);
}

extern "C" size_t kfac_weight_update_workspace_bytes(const kfac_update_item* items_host, int32_t count) {
    if (!items_host || count <= 0) return 0;
    size_t chunks = 0;
    for (int i = 0; i < count; ++i) {
        if (items_host[i].n <= 0) return 0;
        chunks += wu_chunks((unsigned)items_host[i].n);
    }
    return align_up(chunks * sizeof(double), 256);
}

extern "C" int kfac_weight_update_batched(const kfac_update_item* items_host, int32_t count, float eta, float momentum,
                                          float eps, void* ws, size_t ws_bytes, void* stream) {
    if (!items_host || count < 0) return KFAC_ERR_INVALID_ARG;
    if (count == 0) return KFAC_OK;
    if (!(eps >= 0.f)) return KFAC_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i)
        if (!wu_item_ok(items_host[i])) return KFAC_ERR_INVALID_ARG;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < kfac_weight_update_workspace_bytes(items_host, count)) return KFAC_ERR_WORKSPACE;
    double* partial = (double*)ws;
    for (int first = 0; first < count; first += WU_MAX) {
        const int cnt = count - first < WU_MAX ? count - first : WU_MAX;
        UpdateBatch b;
        b.count = cnt;
        unsigned chunks = 0;
        for (int i = 0; i < cnt; ++i) {
            const kfac_update_item& it = items_host[first + i];
            b.prefix[i] = chunks;
            b.n[i] = (unsigned)it.n;
            b.target[i] = sqrtf(2.0f * (float)it.d_out);
            b.w[i] = it.w;
            b.w_prev[i] = it.w_prev;
            b.p[i] = it.precond;
            chunks += wu_chunks((unsigned)it.n);
        }
        b.prefix[cnt] = chunks;
        KFAC_LAUNCH(weight_update_kernel, dim3(chunks), dim3(256), (hipStream_t)stream, b, eta, momentum, partial);
        KFAC_LAUNCH(weight_rescale_kernel, dim3(chunks), dim3(256), (hipStream_t)stream, b, eps, (const double*)partial);
        partial += chunks;
    }
    return KFAC_OK;
}
