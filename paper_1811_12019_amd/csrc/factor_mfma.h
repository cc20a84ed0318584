// Matrix-core factor builder for 16-bit NHWC tensors, column order (kh, kw, c), C % 8 == 0.
//
// Computes one 128 x 128 tile of  Xbar^T Xbar  per workgroup (only tiles on or below the diagonal), where
// Xbar is the implicitly unfolded patch matrix (R rows) with an optional trailing ones column.  The
// contraction runs over the R unfolded rows, which are the *slow* index of Xbar in memory, while the MFMA
// operands want the contraction index contiguous per lane.  So each thread fetches an 8 rows x 8 columns
// block with eight 16-byte loads (coalesced along the channel axis), transposes it in registers with byte
// permutes, and stores eight 16-byte "one column, eight consecutive rows" chunks into LDS.  An MFMA operand
// is then a single 16-byte LDS read per lane.  Because A and B operands are read with the same chunk index,
// the order of the rows inside a chunk is irrelevant.
//
// LDS panel layout: [128 columns][8 chunks of 8 rows], 144-byte column stride, the chunk position XOR-ed with
// (column / 8) % 8 so that both the transposed stores and the operand reads are bank-conflict free.
//
// 256 threads = 4 wavefronts (2 x 2), each owning a 64 x 64 quadrant = 2 x 2 blocks of
// v_mfma_f32_32x32x16_{bf16,f16}; blocks that lie entirely beyond the matrix edge are skipped.
#pragma once

#include "common.h"

namespace kfac {

constexpr int FT = 128;               // tile edge
constexpr int FK = 64;                // unfolded rows per LDS stage
constexpr int FCOL_BYTES = 144;       // LDS bytes per column: 8 chunks x 16 B + 16 B pad
constexpr int FPANEL_BYTES = FT * FCOL_BYTES;
constexpr int FEPI_LD = 65;           // epilogue staging: per-wavefront 32 x 64 floats, padded rows

struct RowEnt {
    int pix;      // element offset of pixel (n, yo*stride - pad, xo*stride - pad), may lie outside the image
    int y0, x0;   // top-left input coordinate of the patch
    int ok;       // row inside this workgroup's row range
};

typedef _Float16 v8h __attribute__((ext_vector_type(8)));

template <bool F16>
__device__ __forceinline__ v16f mfma16(const uint4& a, const uint4& b, v16f c) {
    if constexpr (F16) {
        v8h av, bv;
        __builtin_memcpy(&av, &a, 16);
        __builtin_memcpy(&bv, &b, 16);
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, c, 0, 0, 0);
    } else {
        v8bf av, bv;
        __builtin_memcpy(&av, &a, 16);
        __builtin_memcpy(&bv, &b, 16);
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, c, 0, 0, 0);
    }
}

// What one thread needs to know about its 8-column group.
struct ColGroup {
    int kind;     // 0 data, 1 bias group (first column is the constant 1), 2 beyond the matrix
    int ki, kj;   // kernel tap
    int off;      // element offset of (ki, kj, c0) relative to the patch's top-left pixel
};

__device__ __forceinline__ ColGroup decode_group(const Unfold& u, int gcol0) {
    ColGroup g;
    g.ki = g.kj = g.off = 0;
    const int kdata = u.d - u.has_bias;
    if (gcol0 < kdata) {
        g.kind = 0;
        int tap = gcol0 / u.C;
        int c0 = gcol0 - tap * u.C;
        g.ki = tap / u.kw;
        g.kj = tap - g.ki * u.kw;
        g.off = (g.ki * u.W + g.kj) * u.C + c0;
    } else if (gcol0 == kdata && u.has_bias) {
        g.kind = 1;
    } else {
        g.kind = 2;
    }
    return g;
}

// PLAIN: 1x1 kernel, stride 1, no padding -> Xbar[r][c] = x[r*C + c], no patch geometry at all.
template <bool PLAIN, bool F16>
__global__ __launch_bounds__(256) void factor_mfma_kernel(Unfold u, const uint16_t* __restrict__ x, float scale,
                                                          float* __restrict__ out, float* __restrict__ partial,
                                                          int rows_per_split, int ntiles, int nsplit) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* panelA = smem;
    unsigned char* panelB = smem + FPANEL_BYTES;
    RowEnt* rowtab = (RowEnt*)(smem + 2 * FPANEL_BYTES);      // [2][FK]

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const int lm = lane & 31, h = lane >> 5;

    // workgroup -> (split, tile).  With a multiple of 8 splits, workgroups that share a row range (and hence
    // re-read the same input rows for different tiles) get ids that are equal mod 8, i.e. the same XCD / L2.
    int split, tile;
    {
        const int id = blockIdx.x;
        if ((nsplit & 7) == 0) {
            const int xcd = id & 7, j = id >> 3;
            split = xcd + 8 * (j / ntiles);
            tile = j % ntiles;
        } else {
            split = id / ntiles;
            tile = id - split * ntiles;
        }
    }
    int I, J;
    tri_decode(tile, I, J);
    const bool diag = I == J;
    const int r_begin = split * rows_per_split;
    const int r_end = min(u.R, r_begin + rows_per_split);

    // this thread's 8x8 block: which panel, which 8-row group of the stage, which 8-column group
    const int pan = t >> 7;                 // 0: columns of tile row I (operand A), 1: tile row J (operand B)
    const int rg = (t >> 4) & 7, cg = t & 15;
    const bool loader = !(diag && pan == 1);
    const ColGroup g = decode_group(u, (pan == 0 ? I : J) * FT + cg * 8);
    unsigned char* my_panel = pan == 0 ? panelA : panelB;
    const int lds_store = (cg * 8) * FCOL_BYTES + ((rg ^ (cg & 7)) << 4);

    auto fill_rowtab = [&](int r0, int buf) {
        if (!PLAIN && t < FK) {
            int r = r0 + t;
            RowEnt e;
            e.ok = r < r_end;
            int rr = e.ok ? r : 0;
            int n = rr / (u.Ho * u.Wo);
            int rem = rr - n * (u.Ho * u.Wo);
            int yo = rem / u.Wo;
            int xo = rem - yo * u.Wo;
            e.y0 = yo * u.stride - u.pad;
            e.x0 = xo * u.stride - u.pad;
            e.pix = ((n * u.H + e.y0) * u.W + e.x0) * u.C;
            rowtab[buf * FK + t] = e;
        }
    };

    uint4 blk[8];
    auto fetch = [&](int r0, int buf) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (loader) {
                const int rl = rg * 8 + i;
                if constexpr (PLAIN) {
                    const int r = r0 + rl;
                    if (r < r_end) {
                        if (g.kind == 0) v = *(const uint4*)(x + (size_t)r * u.C + g.off);
                        else if (g.kind == 1) v.x = F16 ? 0x3C00u : 0x3F80u;
                    }
                } else {
                    const RowEnt e = rowtab[buf * FK + rl];
                    if (e.ok) {
                        if (g.kind == 0) {
                            if ((unsigned)(e.y0 + g.ki) < (unsigned)u.H && (unsigned)(e.x0 + g.kj) < (unsigned)u.W)
                                v = *(const uint4*)(x + (e.pix + g.off));
                        } else if (g.kind == 1) {
                            v.x = F16 ? 0x3C00u : 0x3F80u;
                        }
                    }
                }
            }
            blk[i] = v;
        }
    };

    auto stage = [&]() {
        if (!loader) return;
        // 8 rows x 8 columns of 16-bit values -> for each column the 8 rows packed into 16 bytes
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const unsigned sel = (c & 1) ? 0x07060302u : 0x05040100u;
            uint4 o;
            const int q = c >> 1;
            const unsigned r0 = q == 0 ? blk[0].x : q == 1 ? blk[0].y : q == 2 ? blk[0].z : blk[0].w;
            const unsigned r1 = q == 0 ? blk[1].x : q == 1 ? blk[1].y : q == 2 ? blk[1].z : blk[1].w;
            const unsigned r2 = q == 0 ? blk[2].x : q == 1 ? blk[2].y : q == 2 ? blk[2].z : blk[2].w;
            const unsigned r3 = q == 0 ? blk[3].x : q == 1 ? blk[3].y : q == 2 ? blk[3].z : blk[3].w;
            const unsigned r4 = q == 0 ? blk[4].x : q == 1 ? blk[4].y : q == 2 ? blk[4].z : blk[4].w;
            const unsigned r5 = q == 0 ? blk[5].x : q == 1 ? blk[5].y : q == 2 ? blk[5].z : blk[5].w;
            const unsigned r6 = q == 0 ? blk[6].x : q == 1 ? blk[6].y : q == 2 ? blk[6].z : blk[6].w;
            const unsigned r7 = q == 0 ? blk[7].x : q == 1 ? blk[7].y : q == 2 ? blk[7].z : blk[7].w;
            o.x = __builtin_amdgcn_perm(r1, r0, sel);
            o.y = __builtin_amdgcn_perm(r3, r2, sel);
            o.z = __builtin_amdgcn_perm(r5, r4, sel);
            o.w = __builtin_amdgcn_perm(r7, r6, sel);
            *(uint4*)(my_panel + lds_store + c * FCOL_BYTES) = o;
        }
    };

    // which of this wavefront's 32-wide blocks touch the matrix at all
    bool a_on[2], b_on[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        a_on[q] = I * FT + wm * 64 + q * 32 < u.d;
        b_on[q] = J * FT + wn * 64 + q * 32 < u.d;
    }
    const unsigned char* opA = panelA;
    const unsigned char* opB = diag ? panelA : panelB;
    int a_off[2], b_off[2], a_sw[2], b_sw[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        int ca = wm * 64 + q * 32 + lm, cb = wn * 64 + q * 32 + lm;
        a_off[q] = ca * FCOL_BYTES;
        a_sw[q] = (ca >> 3) & 7;
        b_off[q] = cb * FCOL_BYTES;
        b_sw[q] = (cb >> 3) & 7;
    }

    v16f acc[2][2];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[p][q][r] = 0.f;

    int buf = 0;
    fill_rowtab(r_begin, 0);
    if (!PLAIN) __syncthreads();
    fetch(r_begin, 0);
    for (int r0 = r_begin; r0 < r_end; r0 += FK) {
        stage();
        fill_rowtab(r0 + FK, buf ^ 1);
        __syncthreads();
        if (r0 + FK < r_end) fetch(r0 + FK, buf ^ 1);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int chunk = 2 * s + h;
            uint4 a[2], b[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                if (a_on[q]) a[q] = *(const uint4*)(opA + a_off[q] + ((chunk ^ a_sw[q]) << 4));
                if (b_on[q]) b[q] = *(const uint4*)(opB + b_off[q] + ((chunk ^ b_sw[q]) << 4));
            }
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    if (a_on[p] && b_on[q]) acc[p][q] = mfma16<F16>(a[p], b[q], acc[p][q]);
        }
        __syncthreads();
        buf ^= 1;
    }

    // ---- epilogue ----
    const int i0 = I * FT + wm * 64, j0 = J * FT + wn * 64;
    if (nsplit > 1) {
        // raw partial sums for the second pass: [split][tile][128 x 128]
        float* dst = partial + ((size_t)split * ntiles + tile) * (FT * FT);
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
    // direct: rows of the tile are written from registers (32 consecutive floats per store) ...
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = i0 + p * 32 + (r >> 2) * 8 + h * 4 + (r & 3), col = j0 + q * 32 + lm;
                if (row < u.d && col < u.d) out[(size_t)row * u.d + col] = acc[p][q][r] * scale;
            }
    if (diag) return;
    // ... and the mirrored tile goes through LDS (a region private to this wavefront, 32 tile rows at a time)
    // so that its rows are written as contiguous runs as well.  All panel reads ended at the loop's last barrier.
    float* epi = (float*)smem + wave * (32 * FEPI_LD);
#pragma unroll
    for (int p = 0; p < 2; ++p) {
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = (r >> 2) * 8 + h * 4 + (r & 3), col = q * 32 + lm;
                epi[row * FEPI_LD + col] = acc[p][q][r] * scale;
            }
        for (int c2 = 0; c2 < 64; c2 += 2) {
            int c = c2 + h;
            int col = j0 + c, row = i0 + p * 32 + lm;
            float v = epi[lm * FEPI_LD + c];
            if (col < u.d && row < u.d) out[(size_t)col * u.d + row] = v;
        }
    }
}

constexpr int FACTOR_MFMA_LDS = 2 * FPANEL_BYTES + 2 * FK * (int)sizeof(RowEnt);   // 38,912 B (epilogue staging fits inside)

}  // namespace kfac
