// Preconditioned gradient P = Ginv . gradW . Ainv  (Eq. 7 written for the d_G x d_A weight-gradient matrix;
// Algorithm 1 stage 5), fp32 on the matrix cores.
//
// Both products run as "NT" tile products (both operands K-contiguous), using the symmetry of the inverses:
//   Yt[dA x dG] = Ainv . gradW^T      Yt[j, i] = sum_k Ainv[j, k] gradW[i, k]
//   P [dG x dA] = Ginv . Yt^T         P [i, j] = sum_k Ginv[i, k] Yt[j, k]
#include "gemm_f32.h"

namespace kfac {

// C[M x N] (ldc) = A[M x K] (lda) . B[N x K]^T (ldb)
__global__ __launch_bounds__(256) void gemm_nt_kernel(const float* __restrict__ A, int lda, const float* __restrict__ B,
                                                      int ldb, float* __restrict__ C, int ldc, int M, int N, int K) {
    __shared__ float lds[GEMM_LDS_FLOATS];
    const int i0 = blockIdx.y * TM, j0 = blockIdx.x * TM;
    const int irows = min(TM, M - i0), jrows = min(TM, N - j0);
    TileAcc acc;
    tile_mma_nt(A + (size_t)i0 * lda, lda, irows, B + (size_t)j0 * ldb, ldb, jrows, K, lds, acc);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = acc_row(wm, mb, r, lane), col = acc_col(wn, nb, lane);
                if (row < irows && col < jrows) C[(size_t)(i0 + row) * ldc + j0 + col] = acc.c[mb][nb][r];
            }
}

static int gemm_nt(const float* A, int lda, const float* B, int ldb, float* C, int ldc, int M, int N, int K,
                   hipStream_t stream) {
    dim3 grid(ceil_div(N, TM), ceil_div(M, TM));
    KFAC_LAUNCH(gemm_nt_kernel, grid, dim3(256), stream, A, lda, B, ldb, C, ldc, M, N, K);
    return KFAC_OK;
}

}  // namespace kfac

using namespace kfac;

extern "C" size_t kfac_precondition_workspace_bytes(int32_t dG, int32_t dA) {
    if (dG <= 0 || dA <= 0 || dG > 32768 || dA > 32768) return 0;
    return align_up((size_t)dG * dA * sizeof(float), 256);
}

extern "C" int kfac_precondition(const float* Ginv, const float* Ainv, const float* gradW, int32_t dG, int32_t dA,
                                 float* out, void* ws, size_t ws_bytes, void* stream) {
    if (!Ginv || !Ainv || !gradW || !out || dG <= 0 || dA <= 0 || dG > 32768 || dA > 32768) return KFAC_ERR_INVALID_ARG;
    if (out == gradW || out == Ginv || out == Ainv) return KFAC_ERR_INVALID_ARG;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < kfac_precondition_workspace_bytes(dG, dA)) return KFAC_ERR_WORKSPACE;
    float* Yt = (float*)ws;
    int rc = gemm_nt(Ainv, dA, gradW, dA, Yt, dG, dA, dG, dA, (hipStream_t)stream);
    if (rc != KFAC_OK) return rc;
    return gemm_nt(Ginv, dG, Yt, dG, out, dA, dG, dA, dG, (hipStream_t)stream);
}

extern "C" const char* kfac_status_string(int status) {
    switch (status) {
        case KFAC_OK: return "ok";
        case KFAC_ERR_INVALID_ARG: return "invalid argument";
        case KFAC_ERR_UNSUPPORTED: return "unsupported";
        case KFAC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case KFAC_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}
