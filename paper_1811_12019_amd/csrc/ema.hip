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
