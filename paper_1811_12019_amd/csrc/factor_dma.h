// Matrix-core factor builder, LDS-DMA version, for 16-bit NHWC tensors in (kh, kw, c) column order, C % 8 == 0.
//
// One 128 x 128 tile of  Xbar^T Xbar  per workgroup (tiles on or below the diagonal), Xbar the implicitly unfolded
// patch matrix.  The contraction index (unfolded row) is the slow index in memory, and the MFMA wants it
// contiguous per lane; gfx950 has exactly the two instructions that make this cheap:
//   * global_load_lds_dwordx4 copies 16 bytes per lane from global memory straight into LDS (lane i lands at
//     base + 16 i) without passing through registers, so a 3-stage ring of 32-row slabs can be kept in flight
//     with no register cost and a single barrier per slab;
//   * ds_read_b64_tr_b16 reads a 16 x 4 block of 16-bit values transposed: within 16 lanes, lane j receives
//     element (j % 4) of lanes j/4, j/4 + 4, j/4 + 8, j/4 + 12.  With lanes pointed at 4 rows x 4 column groups
//     of a raw slab, lane j gets four consecutive unfolded rows of column j: an MFMA operand half.
// Rows outside a workgroup's range, taps that fall into the zero padding and columns beyond the matrix are
// fetched from a 16-byte block of zeros, the bias column from a constant {1, 0, ..., 0} block, so the slab in LDS
// is always complete and the inner loop has no special cases.
//
// LDS slab layout (per stage and operand panel: 32 rows x 128 columns = 8 blocks of 1 KB): block b holds rows
// 4b..4b+3; inside a block the 16-byte chunk (row r, column chunk q) sits in slot 8 (q / 2) + 2 r + (q % 2), which
// makes every 16-lane transposed read a contiguous 128-byte run (no bank conflicts).
#pragma once

#include "common.h"
#include "factor_mfma.h"

namespace kfac {

constexpr int DK = 32;                       // unfolded rows per stage
constexpr int DNS = 3;                       // stages in the ring (DNS - 1 in flight)
constexpr int DPANEL = 8 * 1024;             // bytes per operand panel per stage
constexpr int DSTAGE = 2 * DPANEL;
constexpr int FACTOR_DMA_LDS = DNS * DSTAGE; // 49,152 B (the epilogue staging aliases it)

static __device__ uint4 g_zero_chunk = {0u, 0u, 0u, 0u};
static __device__ uint4 g_one_chunk_bf16 = {0x3F80u, 0u, 0u, 0u};
static __device__ uint4 g_one_chunk_f16 = {0x3C00u, 0u, 0u, 0u};

typedef unsigned v2u __attribute__((ext_vector_type(2)));

__device__ __forceinline__ int fast_div(int a, int d, float inv) {   // exact for 0 <= a < 2^24
    int q = (int)((float)a * inv);
    int rem = a - q * d;
    if (rem < 0) --q;
    else if (rem >= d) ++q;
    return q;
}

#define KFAC_TR_READ(dst, addr, off) \
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off))

template <bool F16>
__device__ __forceinline__ v16f mfma16_halves(v2u a0, v2u a1, v2u b0, v2u b1, v16f c) {
    uint4 a = make_uint4(a0.x, a0.y, a1.x, a1.y), b = make_uint4(b0.x, b0.y, b1.x, b1.y);
    return mfma16<F16>(a, b, c);
}

// One tile (workgroup `wg` of ntiles * nsplit) of one factor build.  x, out and partial are global-memory pointers.
template <bool PLAIN, bool F16>
__device__ __forceinline__ void factor_dma_tile(const Unfold& u, const KFAC_AS1 unsigned char* x, float scale,
                                                const OutSpec os, gfloat* __restrict__ partial,
                                                int rows_per_split, int ntiles, int nsplit, int wg,
                                                unsigned char* smem) {
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    typedef const __attribute__((address_space(1))) unsigned char gbyte;
    const float inv_howo = 1.0f / (float)(u.Ho * u.Wo), inv_wo = 1.0f / (float)u.Wo;

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const int lm = lane & 31, h = lane >> 5;

    // The caller pads every build's workgroup count to a multiple of 8 and starts it at a multiple of 8, so that
    // wg % 8 is the XCD this workgroup runs on (workgroups are dealt to the 8 XCDs round-robin).  XCD x takes the
    // x-th contiguous eighth of the build's work list (row ranges in order, tiles row-major inside a range): the
    // tiles of a row range, which all read the same rows, share one L2 instead of fetching them eight times.
    int split, tile;
    {
        const int work = ntiles * nsplit;
        const int per_xcd = (work + 7) >> 3;
        const int unit = (wg & 7) * per_xcd + (wg >> 3);
        if ((wg >> 3) >= per_xcd || unit >= work) return;      // padding workgroup (uniform, before any barrier)
        split = unit / ntiles;
        tile = unit - split * ntiles;
    }
    int I, J;
    tri_decode_blocked<4>(ceil_div(u.d, FT), tile, I, J);   // (tiles that share row panels run together: see the function)
    const bool diag = I == J;
    const int r_begin = split * rows_per_split;
    const int r_end = min(u.R, r_begin + rows_per_split);
    const int nst = (r_end - r_begin + DK - 1) / DK;

    // ---- producer side: which chunks this lane fetches ----
    // DMA instruction = one 1 KB block (4 rows x 16 column chunks).  Off-diagonal tiles: wavefronts 0,1 fill panel A
    // (blocks w, w+2, w+4, w+6), wavefronts 2,3 panel B.  Diagonal tiles: one panel, blocks w and w+4.
    const int ninstr = diag ? 2 : 4;
    const int pan = diag ? 0 : (wave >> 1);
    const int blk0 = diag ? wave : (wave & 1), blkstep = diag ? 4 : 2;
    const int dr = (lane & 7) >> 1;                       // row inside the block
    const int dq = 2 * (lane >> 3) + (lane & 1);          // column chunk (8 columns)
    const ColGroup g = decode_group(u, (pan == 0 ? I : J) * FT + dq * 8);
    gbyte* xg = x;
    gbyte* zero_src = (gbyte*)&g_zero_chunk;
    gbyte* one_src = (gbyte*)(F16 ? &g_one_chunk_f16 : &g_one_chunk_bf16);
    lds_byte* lds0 = (lds_byte*)smem;

    // per-stage row geometry, computed by lane k for stage row k and handed out with bpermute
    auto issue_stage = [&](int s, int bufidx) {
        const int rbase = r_begin + s * DK;
        int pix = 0, yx = 0;
        bool rvalid;
        if constexpr (!PLAIN) {
            const int R = rbase + lm;
            rvalid = R < r_end;
            const int Rc = rvalid ? R : 0;
            const int n = fast_div(Rc, u.Ho * u.Wo, inv_howo);
            const int rem = Rc - n * (u.Ho * u.Wo);
            const int yo = fast_div(rem, u.Wo, inv_wo);
            const int xo = rem - yo * u.Wo;
            const int y0 = yo * u.stride - u.pad, x0 = xo * u.stride - u.pad;
            pix = ((n * u.H + y0) * u.W + x0) * u.C;
            yx = rvalid ? (((y0 + 0x4000) << 16) | (x0 + 0x4000)) : -1;      // -1: row outside the range
        }
        // All four sources are worked out first, branch-free (the cross-lane exchanges go out back to back and are
        // waited for once); then the DMA instructions, of which a diagonal tile issues only two.
        gbyte* src[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int b = blk0 + j * blkstep;
            const int k = (4 * b + dr) & (DK - 1);                           // row inside the stage (j >= ninstr: unused)
            // branch-free source selection: data element, the constant one-chunk (bias column), or zeros
            bool row_ok, tap_ok = true;
            size_t eoff;
            if constexpr (PLAIN) {
                const int R = rbase + k;
                row_ok = R < r_end;
                eoff = (size_t)R * u.C + g.off;
            } else {
                const int rp = __builtin_amdgcn_ds_bpermute(4 * k, pix);
                const int ryx = __builtin_amdgcn_ds_bpermute(4 * k, yx);
                row_ok = ryx != -1;
                const int y = (ryx >> 16) - 0x4000 + g.ki, xx = (ryx & 0xffff) - 0x4000 + g.kj;
                tap_ok = (unsigned)y < (unsigned)u.H && (unsigned)xx < (unsigned)u.W;
                eoff = (size_t)(unsigned)(rp + g.off);
            }
            const bool is_data = row_ok && tap_ok && g.kind == 0;
            const bool is_one = row_ok && g.kind == 1;
            src[j] = is_data ? xg + 2 * eoff : (is_one ? one_src : zero_src);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j >= ninstr) break;
            const int b = blk0 + j * blkstep;
            lds_byte* dst = lds0 + bufidx * DSTAGE + pan * DPANEL + b * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src[j],
                                             (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
        }
    };

    // ---- consumer side ----
    // A wavefront whose 64 x 64 quadrant lies entirely beyond the matrix edge skips the arithmetic (it still
    // takes part in the loads and barriers); partly covered quadrants simply multiply zeros.
    const bool wave_on = I * FT + wm * 64 < u.d && J * FT + wn * 64 < u.d;
    // byte address (inside a stage) of this lane's 8-byte piece for operand block q, k-block offset excluded
    unsigned a_addr[2], b_addr[2];
    {
        const int grp = lane >> 4, p = lane & 15, r = p >> 2, cg4 = p & 3;
        const unsigned lane_part = (unsigned)((2 * (grp >> 1)) * 1024 + (2 * r + (cg4 >> 1)) * 16 + (cg4 & 1) * 8);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int ca = wm * 64 + q * 32, cb = wn * 64 + q * 32;
            a_addr[q] = lane_part + (unsigned)(8 * (ca / 16 + (grp & 1)) * 16);
            b_addr[q] = lane_part + (unsigned)(8 * (cb / 16 + (grp & 1)) * 16) + (diag ? 0u : (unsigned)DPANEL);
        }
    }

    v16f acc[2][2];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[p][q][r] = 0.f;

    // prologue: DNS - 1 stages in flight
#pragma unroll
    for (int s = 0; s < DNS - 1; ++s) issue_stage(s, s);

    for (int it = 0; it < nst; it += DNS) {
#pragma unroll
        for (int bi = 0; bi < DNS; ++bi) {
            const int s = it + bi;
            if (s >= nst) break;                                   // uniform
            // this thread's DMA for stage s has landed (two later stages may still be in flight) ...
            if constexpr (DNS == 4) {
                if (diag) asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");   // ... and so has everybody else's
            } else {
                static_assert(DNS == 3 || DNS == 4, "ring depth");
                if (diag) asm volatile("s_waitcnt vmcnt(2)\n\ts_barrier" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");
            }
            issue_stage(s + DNS - 1, (bi + DNS - 1) % DNS);        // refill the buffer stage s-1 just vacated
            if (wave_on) {
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    v2u a[2][2], b[2][2];
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        KFAC_TR_READ(a[q][0], a_addr[q], bi * DSTAGE + (4 * ks + 0) * 1024);
                        KFAC_TR_READ(a[q][1], a_addr[q], bi * DSTAGE + (4 * ks + 1) * 1024);
                        KFAC_TR_READ(b[q][0], b_addr[q], bi * DSTAGE + (4 * ks + 0) * 1024);
                        KFAC_TR_READ(b[q][1], b_addr[q], bi * DSTAGE + (4 * ks + 1) * 1024);
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)"
                                 : "+v"(a[0][0]), "+v"(a[0][1]), "+v"(a[1][0]), "+v"(a[1][1]),
                                   "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[1][0]), "+v"(b[1][1]));
#pragma unroll
                    for (int p = 0; p < 2; ++p)
#pragma unroll
                        for (int q = 0; q < 2; ++q)
                            acc[p][q] = mfma16_halves<F16>(a[p][0], a[p][1], b[q][0], b[q][1], acc[p][q]);
                }
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");               // trailing (all-zero) stages must not land later
    __syncthreads();

    // ---- epilogue (same as the register-transpose kernel) ----
    const int i0 = I * FT + wm * 64, j0 = J * FT + wn * 64;
    // A tile wholly inside the matrix (nearly all of a large factor's) stores without per-element guards: 64 guards
    // are 64 branches, and tiles of the widest layers have few rows to amortise them over.
    const bool whole = (I + 1) * FT <= u.d && (J + 1) * FT <= u.d;
    if (nsplit > 1) {
        gfloat* dst = partial + ((size_t)split * ntiles + tile) * (FT * FT);
        if (whole) {
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int row = wm * 64 + p * 32 + (r >> 2) * 8 + h * 4 + (r & 3), col = wn * 64 + q * 32 + lm;
                        dst[row * FT + col] = acc[p][q][r];
                    }
            return;
        }
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int row = wm * 64 + p * 32 + (r >> 2) * 8 + h * 4 + (r & 3), col = wn * 64 + q * 32 + lm;
                    if (I * FT + row < u.d && J * FT + col < u.d) dst[row * FT + col] = acc[p][q][r];
                }
        return;
    }
    gfloat* __restrict__ out = os.dst;
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < 2; ++q) acc[p][q] *= scale;
    if (os.mode == OUT_EMA) {
        // running average folded in: the old values of this (lower) tile are read, all loads before the first use; the
        // mirror image gets the same new values (the running average is symmetric)
        float old[2][2][16];
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int row = i0 + p * 32 + (r >> 2) * 8 + h * 4 + (r & 3), col = j0 + q * 32 + lm;
                    old[p][q][r] = (whole || (row < u.d && col < u.d)) ? out[(size_t)row * u.d + col] : 0.f;
                }
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[p][q][r] = fmaf(os.decay, old[p][q][r], os.one_minus * acc[p][q][r]);
    }
    const bool packed = os.mode == OUT_PACKED;
    if (!packed) {
        if (whole) {
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int row = i0 + p * 32 + (r >> 2) * 8 + h * 4 + (r & 3), col = j0 + q * 32 + lm;
                        out[(size_t)row * u.d + col] = acc[p][q][r];
                    }
        } else {
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int row = i0 + p * 32 + (r >> 2) * 8 + h * 4 + (r & 3), col = j0 + q * 32 + lm;
                        if (row < u.d && col < u.d) out[(size_t)row * u.d + col] = acc[p][q][r];
                    }
        }
    } else if (diag) {
        // packed upper triangle: of a diagonal tile, the elements on or above the diagonal, row by row
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int row = i0 + p * 32 + (r >> 2) * 8 + h * 4 + (r & 3), col = j0 + q * 32 + lm;
                    if (row < u.d && col < u.d && col >= row) out[packed_row_base(row, u.d) + col] = acc[p][q][r];
                }
    }
    if (diag) return;
    // mirror image (rows of the upper triangle), transposed through LDS so that stores run along rows
    float* epi = (float*)smem + wave * (32 * FEPI_LD);
#pragma unroll
    for (int p = 0; p < 2; ++p) {
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = (r >> 2) * 8 + h * 4 + (r & 3), col = q * 32 + lm;
                epi[row * FEPI_LD + col] = acc[p][q][r];
            }
        if (whole && !packed) {
#pragma unroll 8
            for (int c2 = 0; c2 < 64; c2 += 2) {
                const int c = c2 + h;
                out[(size_t)(j0 + c) * u.d + i0 + p * 32 + lm] = epi[lm * FEPI_LD + c];
            }
        } else {
            for (int c2 = 0; c2 < 64; c2 += 2) {
                int c = c2 + h;
                int col = j0 + c, row = i0 + p * 32 + lm;
                float v = epi[lm * FEPI_LD + c];
                if (col < u.d && row < u.d) out[(packed ? packed_row_base(col, u.d) : (size_t)col * u.d) + row] = v;
            }
        }
    }
}

}  // namespace kfac
