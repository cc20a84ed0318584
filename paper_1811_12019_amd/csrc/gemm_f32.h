// fp32 "NT" tile product on the gfx950 matrix cores: acc[128 x 128] = A[128 x K] . B[128 x K]^T with both
// operands row-major and K contiguous, v_mfma_f32_32x32x2_f32, fp32 accumulate.  Used by the sweep steps of
// the damped inverse and by the two products of the preconditioner.
//
// One workgroup = 256 threads = 4 wavefronts in a 2 x 2 arrangement, each wavefront owning a 64 x 64 quadrant
// as 2 x 2 MFMA blocks (64 accumulator registers per lane).  K advances 16 at a time through LDS; the next
// K-slab is fetched into registers while the current one is multiplied.
#pragma once

#include "common.h"

namespace kfac {

constexpr int TM = 128;          // tile rows (= tile columns)
constexpr int TK = 16;           // K-slab per LDS stage
constexpr int TLD = TK + 4;      // LDS row stride in floats (keeps float4 alignment, spreads banks)
constexpr int GEMM_LDS_FLOATS = 2 * TM * TLD;

struct TileAcc {
    v16f c[2][2];
};

// Row / column (inside the 128 x 128 tile) of accumulator register r of MFMA block (mb, nb) for this lane.
__device__ __forceinline__ int acc_row(int wm, int mb, int r, int lane) {
    return wm * 64 + mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
}
__device__ __forceinline__ int acc_col(int wn, int nb, int lane) { return wn * 64 + nb * 32 + (lane & 31); }

__device__ __forceinline__ v4f load4_guard(const float* p, bool row_ok, int k, int K) {
    v4f v = {0.f, 0.f, 0.f, 0.f};
    if (row_ok) {
        if (k + 3 < K) {
            f4u u = *(const f4u*)(p + k);
            v.x = u.x; v.y = u.y; v.z = u.z; v.w = u.w;
        } else {
            if (k < K) v.x = p[k];
            if (k + 1 < K) v.y = p[k + 1];
            if (k + 2 < K) v.z = p[k + 2];
        }
    }
    return v;
}

// A: first row of the tile's A operand, lda floats between rows, arows (<=128) valid rows; same for B.
// copyA (optional): the A slabs are also written to copyA[row * ldcopy + k] as they stream through.
__device__ __forceinline__ void tile_mma_nt(const float* __restrict__ A, int lda, int arows,
                                            const float* __restrict__ B, int ldb, int brows, int K,
                                            float* __restrict__ lds, TileAcc& acc,
                                            float* __restrict__ copyA = nullptr, int ldcopy = 0) {
    float* As = lds;
    float* Bs = lds + TM * TLD;
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = t >> 2, kq = (t & 3) * 4;
    const int lm = lane & 31, h = lane >> 5;

#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc.c[mb][nb][r] = 0.f;

    v4f ra[2], rb[2];
    const float* pa0 = A + (size_t)lr * lda;
    const float* pa1 = A + (size_t)(lr + 64) * lda;
    const float* pb0 = B + (size_t)lr * ldb;
    const float* pb1 = B + (size_t)(lr + 64) * ldb;
    const bool a0 = lr < arows, a1 = lr + 64 < arows, b0 = lr < brows, b1 = lr + 64 < brows;

    ra[0] = load4_guard(pa0, a0, kq, K);
    ra[1] = load4_guard(pa1, a1, kq, K);
    rb[0] = load4_guard(pb0, b0, kq, K);
    rb[1] = load4_guard(pb1, b1, kq, K);

    for (int k0 = 0; k0 < K; k0 += TK) {
        *(v4f*)&As[lr * TLD + kq] = ra[0];
        *(v4f*)&As[(lr + 64) * TLD + kq] = ra[1];
        *(v4f*)&Bs[lr * TLD + kq] = rb[0];
        *(v4f*)&Bs[(lr + 64) * TLD + kq] = rb[1];
        if (copyA) {
            int k = k0 + kq;
            if (a0 && k < K) *(v4f*)&copyA[(size_t)lr * ldcopy + k] = ra[0];
            if (a1 && k < K) *(v4f*)&copyA[(size_t)(lr + 64) * ldcopy + k] = ra[1];
        }
        __syncthreads();
        if (k0 + TK < K) {
            int k = k0 + TK + kq;
            ra[0] = load4_guard(pa0, a0, k, K);
            ra[1] = load4_guard(pa1, a1, k, K);
            rb[0] = load4_guard(pb0, b0, k, K);
            rb[1] = load4_guard(pb1, b1, k, K);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            v4f a[2], b[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) a[mb] = *(const v4f*)&As[(wm * 64 + mb * 32 + lm) * TLD + 8 * s + 4 * h];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) b[nb] = *(const v4f*)&Bs[(wn * 64 + nb * 32 + lm) * TLD + 8 * s + 4 * h];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                        acc.c[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mb][i], b[nb][i], acc.c[mb][nb], 0, 0, 0);
        }
        __syncthreads();
    }
}

}  // namespace kfac
