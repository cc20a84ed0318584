// Damping of Sec. 4.2: the warm-up schedule of gamma (host arithmetic on scalars), the refresh intervals of Sec. 5.4
// (host), and the split of a block's damping gamma between its two Kronecker factors in proportion to their scale
//     lambda_A = pi sqrt(gamma),  lambda_G = sqrt(gamma) / pi,  pi = sqrt((tr A / d_A) / (tr G / d_G))
// (the factored Tikhonov damping of Martens & Grosse 2015, which Sec. 4.2 names without a formula), computed on the
// device from the running averages so that the inversions that follow need no host round trip.
#include <cmath>

#include "common.h"

namespace kfac {

constexpr int PI_MAX = 128;               // layers per launch (a 3 KB argument block)

struct PiBatch {
    int count;
    int dA[PI_MAX], dG[PI_MAX];
    const float* A[PI_MAX];
    const float* G[PI_MAX];
};

// sum of the diagonal of a dim x dim row-major matrix over the workgroup, in double, fixed order
__device__ __forceinline__ double block_trace(const gfloat* __restrict__ M, int dim, double* __restrict__ red) {
    double s = 0.0;
    for (int i = threadIdx.x; i < dim; i += 256) s += (double)M[(size_t)i * dim + i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    s = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    return s;
}

// one workgroup per layer: lam[2 i] = lambda_A, lam[2 i + 1] = lambda_G
__global__ __launch_bounds__(256) void pi_damping_kernel(PiBatch b, int first, float root_gamma, float* __restrict__ lam) {
    __shared__ double red[4];
    const int m = blockIdx.x;
    const double ta = block_trace(as_global(b.A[m]), b.dA[m], red) / (double)b.dA[m];
    const double tg = block_trace(as_global(b.G[m]), b.dG[m], red) / (double)b.dG[m];
    if (threadIdx.x == 0) {
        // a factor without a positive trace has no scale to go by: even split
        const double pi = (ta > 0.0 && tg > 0.0) ? sqrt(ta / tg) : 1.0;
        lam[2 * (first + m)] = (float)(pi * (double)root_gamma);
        lam[2 * (first + m) + 1] = (float)((double)root_gamma / pi);
    }
}

}  // namespace kfac

using namespace kfac;

extern "C" int kfac_pi_damping_batched(const kfac_pi_item* items_host, int32_t count, float gamma, float* lam,
                                       void* stream) {
    if (count == 0) return KFAC_OK;
    if (!items_host || count < 0 || !lam || !(gamma >= 0.f)) return KFAC_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i) {
        const kfac_pi_item& it = items_host[i];
        if (!it.A || !it.G || it.dA <= 0 || it.dG <= 0 || it.dA > 32768 || it.dG > 32768) return KFAC_ERR_INVALID_ARG;
    }
    const float root = sqrtf(gamma);
    for (int first = 0; first < count; first += PI_MAX) {
        PiBatch b;
        b.count = count - first < PI_MAX ? count - first : PI_MAX;
        for (int i = 0; i < b.count; ++i) {
            b.A[i] = items_host[first + i].A; b.G[i] = items_host[first + i].G;
            b.dA[i] = items_host[first + i].dA; b.dG[i] = items_host[first + i].dG;
        }
        KFAC_LAUNCH(pi_damping_kernel, dim3(b.count), dim3(256), (hipStream_t)stream, b, first, root, lam);
    }
    return KFAC_OK;
}

extern "C" double kfac_warmup_damping_alpha(double gamma0, double gamma_target, double t_warmup) {
    if (!(gamma0 > 0.0) || !(gamma_target > 0.0) || !(t_warmup > 0.0)) return NAN;
    return 2.0 * log10(gamma0 / gamma_target) / t_warmup;
}

extern "C" double kfac_warmup_damping_next(double gamma, double gamma_target, double alpha) {
    return (1.0 - alpha) * gamma + alpha * gamma_target;
}

extern "C" double kfac_bn_damping(double gamma, double rho_bn) { return rho_bn * gamma; }

extern "C" int32_t kfac_refresh_interval(int32_t epoch, int32_t heuristic) {
    if (epoch < 0) return -1;
    if (heuristic == KFAC_REFRESH_GROWING) {
        const int32_t v = 5 * (epoch / 5) + 1;
        return v < 20 ? v : 20;
    }
    if (heuristic == KFAC_REFRESH_LATE) return epoch < 13 ? 1 : 20;
    return -1;
}
