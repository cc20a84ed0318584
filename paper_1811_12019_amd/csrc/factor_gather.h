// Matrix-core factor builder for narrow 16-bit NHWC layers whose channel count is not a multiple of 8 (the first
// convolution: 3 channels, 7 x 7 taps, 148 columns, 401,408 unfolded rows at batch 32): tall and skinny, so one
// workgroup accumulates the whole (at most 160 x 160) factor for a range of rows.
//
// Per 64 unfolded rows: lane l of every wavefront owns row l (its patch geometry is decoded once), the wavefronts
// share out the columns (column -> tap/channel offsets come from a table built once in LDS) and gather the slab
// element by element into LDS transposed, Ut[column][row]; an MFMA operand (8 consecutive rows of one column) is
// then one 16-byte LDS read.  The 15 lower 32 x 32 blocks are dealt to the four wavefronts.  Partial factors of
// all row ranges are summed by factor_reduce_kernel<32>.
#pragma once

#include "common.h"
#include "factor_dma.h"

namespace kfac {

constexpr int GA_ROWS = 64;          // unfolded rows per slab
constexpr int GA_LD = 72;            // Ut row stride in elements: 144 bytes keeps the 16-byte reads conflict free
constexpr int GA_DMAX = 160;         // columns, padded to a multiple of 32
constexpr int GA_T = 32;             // block edge of the partial-sum layout
constexpr int GA_COLS_PER_WAVE = GA_DMAX / 4;

template <bool F16>
__global__ __launch_bounds__(256) void factor_gather_kernel(Unfold u, const void* x_, float* partial_, int rows_per_split) {
    __shared__ __attribute__((aligned(16))) unsigned short Ut[GA_DMAX * GA_LD];
    __shared__ int col_off[GA_DMAX];     // element offset of the column's tap/channel from the patch origin; -1 zero column, -2 bias
    __shared__ int col_tap[GA_DMAX];     // (ki << 16) | kj
    const KFAC_AS1 unsigned short* __restrict__ x = (const KFAC_AS1 unsigned short*)x_;
    gfloat* __restrict__ partial = as_global(partial_);
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int lm = lane & 31, h = lane >> 5;
    const int nblk = (u.d + GA_T - 1) / GA_T;
    const int ntiles = nblk * (nblk + 1) / 2;
    const int split = blockIdx.x;
    const int r_begin = split * rows_per_split;
    const int r_end = min(u.R, r_begin + rows_per_split);
    const float inv_howo = 1.0f / (float)(u.Ho * u.Wo), inv_wo = 1.0f / (float)u.Wo;

    if (t < GA_DMAX) {
        const int kdata = u.d - u.has_bias;
        int off = -1, tap = 0;
        if (t < kdata) {
            const int tp = t / u.C, ch = t - tp * u.C;
            const int ki = tp / u.kw, kj = tp - ki * u.kw;
            off = (ki * u.W + kj) * u.C + ch;
            tap = (ki << 16) | kj;
        } else if (t == kdata && u.has_bias) {
            off = -2;
        }
        col_off[t] = off;
        col_tap[t] = tap;
    }
    // this wavefront's blocks of the lower triangle: tiles wave, wave + 4, ...
    int bI[4], bJ[4];
    bool bon[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int tile = wave + 4 * b;
        bon[b] = tile < ntiles;
        tri_decode(bon[b] ? tile : 0, bI[b], bJ[b]);
    }
    v16f acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;
    const unsigned short one = F16 ? 0x3C00 : 0x3F80;
    __syncthreads();

    // values of one slab: the 40 columns of this wavefront for this lane's row
    auto fetch = [&](int r0, unsigned short (&v)[GA_COLS_PER_WAVE]) {
        const int R = r0 + lane;
        const bool rvalid = R < r_end;
        const int Rc = rvalid ? R : r_begin;
        const int n = fast_div(Rc, u.Ho * u.Wo, inv_howo);
        const int rem = Rc - n * (u.Ho * u.Wo);
        const int yo = fast_div(rem, u.Wo, inv_wo);
        const int xo = rem - yo * u.Wo;
        const int y0 = yo * u.stride - u.pad, x0 = xo * u.stride - u.pad;
        const int pix = ((n * u.H + y0) * u.W + x0) * u.C;
#pragma unroll
        for (int i = 0; i < GA_COLS_PER_WAVE; ++i) {
            const int c = wave + 4 * i;
            const int off = col_off[c], tap = col_tap[c];                // uniform
            const int y = y0 + (tap >> 16), xx = x0 + (tap & 0xffff);
            const bool ok = rvalid && off >= 0 && (unsigned)y < (unsigned)u.H && (unsigned)xx < (unsigned)u.W;
            // every lane loads (element 0 when the tap is padding or the column is not data) and masks: no branches
            const unsigned val = x[ok ? pix + off : 0];
            const unsigned keep = ok ? 0xffffu : 0u, fill = (rvalid && off == -2) ? (unsigned)one : 0u;
            v[i] = (unsigned short)((val & keep) | fill);
        }
    };
    unsigned short cur[GA_COLS_PER_WAVE], nxt[GA_COLS_PER_WAVE];
    fetch(r_begin, cur);
    for (int r0 = r_begin; r0 < r_end; r0 += GA_ROWS) {
        if (r0 + GA_ROWS < r_end) fetch(r0 + GA_ROWS, nxt);               // in flight during the stores and the product
#pragma unroll
        for (int i = 0; i < GA_COLS_PER_WAVE; ++i) Ut[(wave + 4 * i) * GA_LD + lane] = cur[i];
        __syncthreads();
        // ---- multiply: 4 K-steps of 16 rows ----
#pragma unroll
        for (int ks = 0; ks < GA_ROWS / 16; ++ks)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (!bon[b]) continue;                                   // uniform
                const uint4 a = *(const uint4*)&Ut[(bI[b] * GA_T + lm) * GA_LD + ks * 16 + 8 * h];
                const uint4 bb = *(const uint4*)&Ut[(bJ[b] * GA_T + lm) * GA_LD + ks * 16 + 8 * h];
                acc[b] = mfma16<F16>(a, bb, acc[b]);
            }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < GA_COLS_PER_WAVE; ++i) cur[i] = nxt[i];
    }
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        if (!bon[b]) continue;
        gfloat* dst = partial + ((size_t)split * ntiles + wave + 4 * b) * (GA_T * GA_T);
#pragma unroll
        for (int r = 0; r < 16; ++r) dst[((r >> 2) * 8 + h * 4 + (r & 3)) * GA_T + lm] = acc[b][r];
    }
}

// Sum of the partial factors: one workgroup per (block, row of the block).  32 lanes along the row times 8 groups
// that each add every 8th partial, then a fixed-order sum of the 8 group totals: deterministic, 128-byte reads.
__global__ __launch_bounds__(256) void factor_gather_reduce_kernel(const float* partial_, int nsplit, int ntiles, int d,
                                                                   float scale, OutSpec os) {
    __shared__ float part[8][32];
    const gfloat* __restrict__ partial = as_global(partial_);
    const int tile = blockIdx.x >> 5, trow = blockIdx.x & 31;
    const int col = threadIdx.x & 31, grp = threadIdx.x >> 5;
    int I, J;
    tri_decode(tile, I, J);
    const gfloat* src = partial + (size_t)tile * (GA_T * GA_T) + trow * GA_T + col;
    const size_t stride = (size_t)ntiles * (GA_T * GA_T);
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int sp = grp;
    for (; sp + 24 < nsplit; sp += 32) {
        s0 += src[(size_t)sp * stride];
        s1 += src[(size_t)(sp + 8) * stride];
        s2 += src[(size_t)(sp + 16) * stride];
        s3 += src[(size_t)(sp + 24) * stride];
    }
    for (; sp < nsplit; sp += 8) s0 += src[(size_t)sp * stride];
    part[grp][col] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (grp == 0) {
        float s = 0.f;
#pragma unroll
        for (int g = 0; g < 8; ++g) s += part[g][col];
        s *= scale;
        const int row = I * GA_T + trow, c = J * GA_T + col;
        if (row < d && c < d && (I != J || c <= row)) emit_sym(os, d, row, c, s, row != c);
    }
}

}  // namespace kfac
