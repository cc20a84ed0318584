// fp32 "NT" tile product on the gfx950 matrix cores: acc[128 x 128] = A[128 x K] . B[128 x K]^T with both
// operands row-major and K contiguous, v_mfma_f32_32x32x2_f32, fp32 accumulate.  Used by the sweep steps of
// the damped inverse and by the two products of the preconditioner.
//
// One workgroup = 256 threads = 4 wavefronts in a 2 x 2 arrangement, each wavefront owning a 64 x 64 quadrant
// as 2 x 2 MFMA blocks (64 accumulator registers per lane).  K advances 32 at a time through LDS; the next
// K-slab is fetched into registers while the current one is multiplied.
#pragma once

#include "common.h"

namespace kfac {

constexpr int TM = 128;          // tile rows (= tile columns)
// K-slab per LDS stage is a template parameter (16 or 32); the LDS row stride is slab + 4 floats (keeps float4
// alignment, spreads banks).
constexpr int GEMM_LDS_FLOATS = 2 * TM * (32 + 4);     // 36,864 B: enough for either slab; reused as epilogue staging
constexpr int EPI_LD = 65;       // staging for transposed stores: per wavefront 32 x 64 floats, padded rows

struct TileAcc {
    v16f c[2][2];
};

// Row / column (inside the 128 x 128 tile) of accumulator register r of MFMA block (mb, nb) for this lane.
__device__ __forceinline__ int acc_row(int wm, int mb, int r, int lane) {
    return wm * 64 + mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
}
__device__ __forceinline__ int acc_col(int wn, int nb, int lane) { return wn * 64 + nb * 32 + (lane & 31); }

__device__ __forceinline__ v4f load4_guard(const gfloat* p, bool row_ok, int k, int K) {
    v4f v = {0.f, 0.f, 0.f, 0.f};
    if (row_ok) {
        if (k + 3 < K) {
            v = *(const KFAC_AS1 v4f_a4*)(p + k);
        } else {
            if (k < K) v.x = p[k];
            if (k + 1 < K) v.y = p[k + 1];
            if (k + 2 < K) v.z = p[k + 2];
        }
    }
    return v;
}

// A: first row of the tile's A operand, lda floats between rows, arows (<=128) valid rows; same for B.
// A_TRANS: the A operand is stored transposed in memory, element (m, k) at A[k * lda + m] (used for the part of
//          a symmetric matrix's block column that only exists, transposed, in the lower triangle).
// copyA (optional): the A slabs are also written to copyA[row * ldcopy + k] as they stream through.
// skip_upper_right: the (wm = 0, wn = 1) quadrant is not needed (diagonal tile of a symmetric result).
template <bool A_TRANS = false, int TK = 32>
__device__ __forceinline__ void tile_mma_nt(const gfloat* __restrict__ A, int lda, int arows,
                                            const gfloat* __restrict__ B, int ldb, int brows, int K,
                                            float* __restrict__ lds, TileAcc& acc,
                                            gfloat* __restrict__ copyA = nullptr, int ldcopy = 0,
                                            bool skip_upper_right = false) {
    constexpr int TLD = TK + 4;
    constexpr int QK = TK / 4;                        // float4 per row of a slab
    constexpr int RP = 256 / QK;                      // rows per pass (32 or 64)
    constexpr int NP = TM / RP;                       // passes per operand (4 or 2)
    static_assert(TK == 16 || TK == 32, "slab must be 16 or 32");
    float* As = lds;
    float* Bs = lds + TM * TLD;
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = t / QK, kq = (t % QK) * 4;         // RP rows x QK float4 per pass
    const int tm = (t & 31) * 4, tk = t >> 5;         // transposed A: 8 k x 32 float4 (along m) per pass
    const int lm = lane & 31, h = lane >> 5;
    const bool compute = !(skip_upper_right && wm == 0 && wn == 1);

#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc.c[mb][nb][r] = 0.f;

    v4f ra[NP], rb[NP];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int row = lr + RP * p;
            if constexpr (A_TRANS) {
                const int k = k0 + tk + 8 * p;      // NP passes of 8 k each cover the slab (TK = 8 * NP)
                ra[p] = load4_guard(A + (size_t)k * lda, k < K, tm, arows);
            } else {
                ra[p] = load4_guard(A + (size_t)row * lda, row < arows, k0 + kq, K);
            }
            rb[p] = load4_guard(B + (size_t)row * ldb, row < brows, k0 + kq, K);
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += TK) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int row = lr + RP * p;
            if constexpr (A_TRANS) {
                const int kk = tk + 8 * p;
#pragma unroll
                for (int i = 0; i < 4; ++i) As[(tm + i) * TLD + kk] = ra[p][i];
            } else {
                *(v4f*)&As[row * TLD + kq] = ra[p];
                if (copyA && row < arows && k0 + kq < K) *(KFAC_AS1 v4f*)&copyA[(size_t)row * ldcopy + k0 + kq] = ra[p];
            }
            *(v4f*)&Bs[row * TLD + kq] = rb[p];
        }
        __syncthreads();
        if constexpr (A_TRANS) {
            if (copyA) {
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    const int row = lr + RP * p;
                    if (row < arows && k0 + kq < K)
                        *(KFAC_AS1 v4f*)&copyA[(size_t)row * ldcopy + k0 + kq] = *(const v4f*)&As[row * TLD + kq];
                }
            }
        }
        if (k0 + TK < K) fetch(k0 + TK);
        if (compute) {
#pragma unroll
            for (int s = 0; s < TK / 8; ++s) {
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
        }
        __syncthreads();
    }
}

// Transposed store of this wavefront's 64 x 64 accumulator quadrant: dst[(c0 + col) * ldd + r0 + row] = value,
// staged through a wavefront-private LDS region so that every store instruction writes two contiguous runs of 32
// floats.  `lds` must no longer be in use as operand storage (call after the product's final barrier).
// keep(row, col) decides per element (tile-local quadrant coordinates added by the caller through r0/c0).
template <class Keep>
__device__ __forceinline__ void store_quadrant_transposed(const v16f (&q)[2][2], float* __restrict__ lds,
                                                          gfloat* __restrict__ dst, size_t ldd, int r0, int c0,
                                                          int rows_valid, int cols_valid, Keep keep) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lm = lane & 31, h = lane >> 5;
    float* epi = lds + wave * (32 * EPI_LD);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) epi[((r >> 2) * 8 + h * 4 + (r & 3)) * EPI_LD + nb * 32 + lm] = q[mb][nb][r];
        for (int c2 = 0; c2 < 64; c2 += 2) {
            const int col = c2 + h, row = mb * 32 + lm;
            const float v = epi[lm * EPI_LD + col];
            if (row < rows_valid && col < cols_valid && keep(row, col)) dst[(size_t)(c0 + col) * ldd + r0 + row] = v;
        }
    }
}

}  // namespace kfac
