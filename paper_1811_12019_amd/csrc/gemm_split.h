// fp32 "NT" tile product on the bf16 matrix cores: acc[128 x 128] += A[128 x K] . B[128 x K]^T, both operands
// fp32, row-major, K contiguous.  Each fp32 operand value is split on the fly into NS bf16 pieces
//     x = x0 + x1 (+ x2),   x0 = bf16(x), x1 = bf16(x - x0), x2 = bf16(x - x0 - x1)
// (8 significant bits each, so 2 pieces carry 16 bits of x and 3 pieces all 24), and the product is the sum of
// the bf16 x bf16 MFMAs (exact products, fp32 accumulate) of all piece pairs whose combined order is below NS:
//     NS = 2:  a0 b0 + a0 b1 + a1 b0                            relative error of a product ~ 2^-16
//     NS = 3:  a0 b0 + a0 b1 + a1 b0 + a0 b2 + a1 b1 + a2 b0    ~ 2^-23: on a par with fp32 multiply-add
// v_mfma_f32_32x32x16_bf16 runs at 16 times the rate of v_mfma_f32_32x32x2_f32, so 3 (6) products per fp32
// product still leave a factor 5.3 (2.7) over the fp32 matrix-core peak.
//
// (A variant with two fp16 pieces of scaled operands, split ahead of time by the producer, is at the end of this file.)
//
// One workgroup = 4 wavefronts in a 2 x 2 arrangement, each owning a 64 x 64 quadrant as 2 x 2 MFMA blocks.  K
// advances 16 at a time through a double-buffered LDS stage: the next slab is fetched into registers while the
// current one is multiplied, then split and stored to the other buffer; one barrier per slab.
// LDS layout per buffer: operand (A, B) x piece x 128 rows x 32 bytes (16 bf16 = the slab's K); the two 16-byte
// halves of a row swap places from one group of 4 rows to the next and again from one group of 8 to the next, which
// makes the 16-byte MFMA operand reads (served 16 consecutive rows at a time from 64 banks) bank-conflict free.
#pragma once

#include "factor_mfma.h"
#include "gemm_f32.h"

namespace kfac {

constexpr int SPLIT_KS = 16;                           // K per LDS stage
constexpr int SPLIT_PLANE = 128 * 32;                  // bytes of one operand piece per stage
template <int NS> constexpr int split_lds_bytes() { return 2 * 2 * NS * SPLIT_PLANE; }   // 32 KB (NS=2), 48 KB (NS=3)

typedef __bf16 v2bf_t __attribute__((ext_vector_type(2)));
typedef float v2f_t __attribute__((ext_vector_type(2)));

// bf16 pieces of four floats: piece[p] holds 4 bf16 (8 bytes) for p < NS
template <int NS>
__device__ __forceinline__ void split4(const v4f& x, uint2 (&piece)[NS]) {
    v4f rem = x;
#pragma unroll
    for (int p = 0; p < NS; ++p) {
        const v2f_t lo2 = {rem.x, rem.y}, hi2 = {rem.z, rem.w};
        const v2bf_t a = __builtin_convertvector(lo2, v2bf_t), b = __builtin_convertvector(hi2, v2bf_t);
        unsigned ua, ub;
        __builtin_memcpy(&ua, &a, 4);
        __builtin_memcpy(&ub, &b, 4);
        piece[p] = make_uint2(ua, ub);
        if (p + 1 < NS) {
            rem.x -= __uint_as_float(ua << 16);
            rem.y -= __uint_as_float(ua & 0xffff0000u);
            rem.z -= __uint_as_float(ub << 16);
            rem.w -= __uint_as_float(ub & 0xffff0000u);
        }
    }
}

// lds: split_lds_bytes<NS>() bytes, 16-byte aligned.  acc is accumulated into (the caller zeroes it).
// skip_upper_right: the (wm = 0, wn = 1) quadrant is not needed (diagonal tile of a symmetric result).
// NEG_A: the product is subtracted (the A operand is negated before it is split).
// NST > 0: both operands are complete, 16-byte aligned panels (all 128 rows present, K exactly NST * 16): loads are
// unguarded, every wavefront multiplies, and the stage loop is unrolled completely.  With no branches left the
// compiler counts the loads in flight exactly instead of draining them at every join, which is what makes the
// two-stage look-ahead effective.
// ROWS_ALIGN4 (with NST > 0): the panels' rows are only 4-byte aligned (odd leading dimension).
template <int NS, bool NEG_A = false, int NST = 0, bool ROWS_ALIGN4 = false>
__device__ __forceinline__ void tile_mma_nt_split(const gfloat* __restrict__ A, int lda, int arows,
                                                  const gfloat* __restrict__ B, int ldb, int brows, int K,
                                                  unsigned char* __restrict__ lds, TileAcc& acc,
                                                  bool skip_upper_right = false) {
    static_assert(NS == 2 || NS == 3, "two or three bf16 pieces");
    constexpr int BUF = 2 * NS * SPLIT_PLANE;          // bytes per buffer
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const int lm = lane & 31, h = lane >> 5;
    const bool compute = !(skip_upper_right && wm == 0 && wn == 1);
    // producer: rows lr and lr + 64, floats 4 kq .. 4 kq + 3 of the slab
    const int lr = t >> 2, kq = t & 3;
    unsigned w_off[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int row = lr + 64 * p;
        w_off[p] = (unsigned)(row * 32 + (((kq >> 1) ^ ((row >> 2) & 1) ^ ((row >> 3) & 1)) * 16) + (kq & 1) * 8);
    }
    // consumer: byte offsets (inside one piece plane) of this lane's 16 bytes for row blocks 0, 1
    unsigned a_off[2], b_off[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int ra = wm * 64 + q * 32 + lm, rb = wn * 64 + q * 32 + lm;
        a_off[q] = (unsigned)(ra * 32 + ((h ^ ((ra >> 2) & 1) ^ ((ra >> 3) & 1)) * 16));
        b_off[q] = (unsigned)(rb * 32 + ((h ^ ((rb >> 2) & 1) ^ ((rb >> 3) & 1)) * 16) + NS * SPLIT_PLANE);
    }

    // Two register sets: the slab two stages ahead is in flight while the current one is multiplied, so a fetch
    // has two stage times to arrive (the operands of a sweep step were just written by another kernel and come
    // from beyond the L2).
    v4f ra[2][2], rb[2][2];
    auto fetch = [&](int k0, v4f (&xa)[2], v4f (&xb)[2]) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int row = lr + 64 * p;
            if constexpr (NST > 0 && ROWS_ALIGN4) {
                xa[p] = *(const KFAC_AS1 v4f_a4*)(A + (size_t)row * lda + k0 + 4 * kq);
                xb[p] = *(const KFAC_AS1 v4f_a4*)(B + (size_t)row * ldb + k0 + 4 * kq);
            } else if constexpr (NST > 0) {
                xa[p] = *(const KFAC_AS1 v4f*)(A + (size_t)row * lda + k0 + 4 * kq);
                xb[p] = *(const KFAC_AS1 v4f*)(B + (size_t)row * ldb + k0 + 4 * kq);
            } else {
                xa[p] = load4_guard(A + (size_t)row * lda, row < arows, k0 + 4 * kq, K);
                xb[p] = load4_guard(B + (size_t)row * ldb, row < brows, k0 + 4 * kq, K);
            }
        }
    };
    auto stash = [&](int buf, const v4f (&xa)[2], const v4f (&xb)[2]) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            uint2 pa[NS], pb[NS];
            split4<NS>(NEG_A ? -xa[p] : xa[p], pa);     // negated here, not at the fetch: a use would force the wait early
            split4<NS>(xb[p], pb);
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                *(uint2*)(lds + buf * BUF + s * SPLIT_PLANE + w_off[p]) = pa[s];
                *(uint2*)(lds + buf * BUF + (NS + s) * SPLIT_PLANE + w_off[p]) = pb[s];
            }
        }
    };
    auto mma = [&](int buf) {
        if (NST == 0 && !compute) return;
        uint4 a[2][NS], b[2][NS];
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int p = 0; p < NS; ++p) {
                a[q][p] = *(const uint4*)(lds + buf * BUF + p * SPLIT_PLANE + a_off[q]);
                b[q][p] = *(const uint4*)(lds + buf * BUF + p * SPLIT_PLANE + b_off[q]);
            }
        // smallest terms first
#pragma unroll
        for (int order = NS - 1; order >= 0; --order)
#pragma unroll
            for (int pa = 0; pa <= order; ++pa)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                        acc.c[mb][nb] = mfma16<false>(a[mb][pa], b[nb][order - pa], acc.c[mb][nb]);
    };

    if constexpr (NST > 0) {
        fetch(0, ra[0], rb[0]);
        if (NST > 1) fetch(SPLIT_KS, ra[1], rb[1]);
        stash(0, ra[0], rb[0]);
        __syncthreads();
#pragma unroll
        for (int s = 0; s < NST; ++s) {
            if (s + 2 < NST) fetch((s + 2) * SPLIT_KS, ra[s & 1], rb[s & 1]);
            mma(s & 1);
            if (s + 1 < NST) stash((s + 1) & 1, ra[(s + 1) & 1], rb[(s + 1) & 1]);
            __syncthreads();
        }
        return;
    }
    // general K: one slab of look-ahead (a second register set only costs occupancy here: inside a loop the
    // compiler drains all loads at the back edge anyway)
    const int nst = (K + SPLIT_KS - 1) / SPLIT_KS;
    fetch(0, ra[0], rb[0]);
    stash(0, ra[0], rb[0]);
    __syncthreads();
    for (int s = 0; s < nst; ++s) {
        const int buf = s & 1;
        if (s + 1 < nst) fetch((s + 1) * SPLIT_KS, ra[0], rb[0]);
        mma(buf);
        if (s + 1 < nst) stash(buf ^ 1, ra[0], rb[0]);
        __syncthreads();
    }
}

// ---- two fp16 pieces ---------------------------------------------------------------------------------------------
// x = h0 + h1 with h0 = fp16(x), h1 = fp16(x - h0): 11 significant bits each, 22 together, and the three piece
// products h0 h0 + h0 h1 + h1 h0 (exact in the fp32 accumulator) leave a relative error of ~2^-22 per product: on a
// par with fp32 for a sum of 128 terms, at half the matrix-core work and two thirds of the LDS traffic of three bf16
// pieces.  fp16 has a narrow exponent range, so every operand panel comes with a power-of-two scale that brings its
// largest magnitude to about 2^8 (smaller entries then lose bits only below 2^-32 of the largest); the caller scales the accumulators to match (exact) and back afterwards.
typedef _Float16 v2h_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void split4_h2(const v4f& x, uint2 (&piece)[2]) {
    v4f rem = x;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const v2f_t lo2 = {rem.x, rem.y}, hi2 = {rem.z, rem.w};
        const v2h_t a = __builtin_convertvector(lo2, v2h_t), b = __builtin_convertvector(hi2, v2h_t);
        unsigned ua, ub;
        __builtin_memcpy(&ua, &a, 4);
        __builtin_memcpy(&ub, &b, 4);
        piece[p] = make_uint2(ua, ub);
        if (p == 0) {
            const v2f_t la = __builtin_convertvector(a, v2f_t), lb = __builtin_convertvector(b, v2f_t);
            rem.x -= la.x; rem.y -= la.y; rem.z -= lb.x; rem.w -= lb.y;
        }
    }
}

// Scale (a power of two, as a float) that brings a panel whose largest magnitude is `amax` to at most 2^8: fp16 has
// seven binades above that before it overflows, and the further up the values sit, the later their low pieces
// (2^-11 of the value) drop into fp16's subnormal range: entries down to 2^-11 of the largest keep all 22 bits.
// Exponents are kept within +-30 so that products of two scales and their reciprocals stay far from the ends of the
// fp32 range.
constexpr int PANEL_TOP = 8;
__device__ __forceinline__ float panel_scale(float amax) {
    int e = 0;
    if (amax > 0.f) {
        (void)frexpf(amax, &e);                        // amax = m 2^e, 0.5 <= m < 1
        e = max(-30, min(30, e));
    }
    return ldexpf(1.0f, PANEL_TOP - e);
}

// Largest of the 256 threads' values (red: 4 floats of LDS); two barriers.  Must be called by all threads.
__device__ __forceinline__ float block_absmax(float x, float* __restrict__ red) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
    __syncthreads();
    x = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    return x;
}

// ---- operands split ahead of time ----------------------------------------------------------------------------------
// A panel (128-row slabs x 128 columns of the contraction index) that many tile products read is scaled and split
// into its two fp16 pieces once, by the kernel that produces it, instead of by every product that consumes it: the
// consumer then has no conversion work at all and moves the pieces from global memory straight into LDS
// (global_load_lds_dwordx4: lane i's 16 bytes land at base + 16 i, no registers involved).  To make those copies
// whole contiguous kilobytes, a piece plane is stored in the order the product wants it in LDS: slab by slab, and
// inside a slab one 4 KB block per 16-wide slice of the contraction index, holding for every row its two 16-byte
// halves (8 fp16 each) at byte offset split_plane_offset(row, half).  The halves swap places from one group of four rows
// to the next and again from one group of eight to the next: a 16-byte operand read is served 16 lanes (consecutive rows)
// at a time from 64 four-byte banks, and with this order any 16 consecutive rows' halves fall into 16 different
// 16-byte bank groups (so do any 8 rows' in 8 of 32 banks); with rows simply 32 bytes apart, rows r and r + 8 collide.
constexpr int PRE_BLOCK = 128 * SPLIT_KS * 2;          // bytes of one (slab, 16-wide slice) block of one piece plane
constexpr int PRE_SLAB = (128 / SPLIT_KS) * PRE_BLOCK; // bytes of one 128 x 128 slab of one piece plane
constexpr int PRE_STAGE = 4 * PRE_BLOCK;               // LDS per ring stage: A high, A low, B high, B low
constexpr int PRE_NS = 3;                              // ring stages (two in flight)

__host__ __device__ __forceinline__ int split_plane_offset(int row, int half) {
    return row * 32 + ((half ^ ((row >> 2) & 1) ^ ((row >> 3) & 1)) * 16);
}

// Scaled fp16 pieces of four consecutive contraction-index values k4 .. k4 + 3 (k4 a multiple of 4) of one row of a
// slab, written to the planes `hi` / `lo` (pointing at the slab).
__device__ __forceinline__ void store_split4_h2(KFAC_AS1 unsigned char* hi, KFAC_AS1 unsigned char* lo, int row, int k4,
                                                const v4f& x_scaled) {
    uint2 piece[2];
    split4_h2(x_scaled, piece);
    const int off = (k4 >> 4) * PRE_BLOCK + split_plane_offset(row, (k4 >> 3) & 1) + (k4 & 7) * 2;
    typedef unsigned v2u_t __attribute__((ext_vector_type(2)));
    *(KFAC_AS1 v2u_t*)(hi + off) = v2u_t{piece[0].x, piece[0].y};
    *(KFAC_AS1 v2u_t*)(lo + off) = v2u_t{piece[1].x, piece[1].y};
}

// The rank-128 products of a tile.  The operands of consecutive products sit in consecutive buffers of a ring of `nbuf`
// equally laid out buffers `stride` bytes apart: product q reads buffer (first + q) mod nbuf, the
// high pieces of its A slab at a_hi + buffer * stride, the low pieces `plane` bytes further, and likewise b_hi;
// scale[q] = sa * sb is what the product of the stored pieces is scaled by.
template <int MAXN>
struct SplitRun {
    const KFAC_AS1 unsigned char* a_hi;                // in buffer 0
    const KFAC_AS1 unsigned char* b_hi;
    size_t plane;                                      // bytes from a high plane to its low plane
    size_t stride;                                     // bytes from one buffer to the next
    float scale[MAXN];
    int first, nbuf;
    int n;                                             // 1 .. MAXN products
};

// acc[128 x 128] (+)= sum over the products q of A_q B_q^T, A_q / B_q complete 128 x 128 slabs given as piece planes
// (high x high + high x low + low x high on the fp16 matrix cores).  The products may be scaled differently: acc is
// brought to product q's scale before it is added to (acc holds the caller's values, at scale 1, on entry), and the
// returned factor brings it back to scale 1 (the caller multiplies).  lds: PRE_NS * PRE_STAGE bytes, 1 KB aligned.
// All 256 threads must call; ends with the ring drained and a barrier.
template <int MAXN>
__device__ __forceinline__ float tile_mma_presplit(const SplitRun<MAXN>& p, unsigned char* __restrict__ lds, TileAcc& acc) {
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    constexpr int NSL = 128 / SPLIT_KS;                // slices per product
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const int lm = lane & 31, h = lane >> 5;
    lds_byte* l0 = (lds_byte*)lds;
    unsigned a_addr[2], b_addr[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        a_addr[q] = (unsigned)split_plane_offset(wm * 64 + q * 32 + lm, h);
        b_addr[q] = (unsigned)(2 * PRE_BLOCK + split_plane_offset(wn * 64 + q * 32 + lm, h));
    }
    const int nst = p.n * NSL;
    const unsigned lane_off = (unsigned)(wave * 1024 + lane * 16);   // this lane's 16 bytes inside every block
    auto issue = [&](int s, int buf) {
        const int sc = s < nst ? s : nst - 1;          // past the end: re-read the last slice (never consumed)
        const int q = sc / NSL, ks = sc - q * NSL;
        const int bq = p.first + q;                    // (first < nbuf, q < nbuf)
        const size_t boff = (size_t)(bq >= p.nbuf ? bq - p.nbuf : bq) * p.stride;
        const KFAC_AS1 unsigned char* pa = p.a_hi + boff;
        const KFAC_AS1 unsigned char* pb = p.b_hi + boff;
        const KFAC_AS1 unsigned char* src[4] = {pa, pa + p.plane, pb, pb + p.plane};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + ks * PRE_BLOCK + lane_off),
                                             (__attribute__((address_space(3))) void*)(l0 + buf * PRE_STAGE + j * PRE_BLOCK + wave * 1024),
                                             16, 0, 0);
    };
    float back = 1.0f;
#pragma unroll
    for (int s = 0; s < PRE_NS - 1; ++s) issue(s, s);
    for (int it = 0; it < nst; it += PRE_NS) {
#pragma unroll
        for (int bi = 0; bi < PRE_NS; ++bi) {
            const int s = it + bi;
            if (s >= nst) break;                                            // uniform
            static_assert(PRE_NS == 3, "the wait below counts (PRE_NS - 2) * 4 younger copies");
            asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");   // slice s landed (everybody's part)
            issue(s + PRE_NS - 1, (bi + PRE_NS - 1) % PRE_NS);               // refill the slot slice s - 1 vacated
            if (s % NSL == 0) {                                              // uniform: a new product begins
                float sq = p.scale[0];
#pragma unroll
                for (int q = 1; q < MAXN; ++q) sq = s / NSL == q ? p.scale[q] : sq;
                const float f = sq * back;
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb) acc.c[mb][nb] *= f;
                back = 1.0f / sq;
            }
            v4f a[2][2], b[2][2];                                            // (16 bytes = 8 fp16 each)
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int pc = 0; pc < 2; ++pc) {
                    // (the stage's base goes into the address: an instruction offset holds 16 bits only)
                    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(a[q][pc]) : "v"(a_addr[q] + bi * PRE_STAGE), "n"(pc * PRE_BLOCK));
                    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(b[q][pc]) : "v"(b_addr[q] + bi * PRE_STAGE), "n"(pc * PRE_BLOCK));
                }
            asm volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(a[0][0]), "+v"(a[0][1]), "+v"(a[1][0]), "+v"(a[1][1]),
                           "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[1][0]), "+v"(b[1][1]));
            // smallest terms first
#pragma unroll
            for (int term = 0; term < 3; ++term)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                    {
                        v8h av, bv;
                        __builtin_memcpy(&av, &a[mb][term == 0 ? 1 : 0], 16);
                        __builtin_memcpy(&bv, &b[nb][term == 1 ? 1 : 0], 16);
                        acc.c[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc.c[mb][nb], 0, 0, 0);
                    }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");            // ring idle: the LDS may be reused
    return back;
}

// A long contraction: product q reads the q-th consecutive 128 x 128 block of its operands' planes (the blocks of one
// 128-row slab of a matrix stored block by block along the contraction index); scale_lds[q] (LDS, filled and made
// visible by the caller) is the product of the two blocks' scales.
struct SplitSeq {
    const KFAC_AS1 unsigned char* a_hi;                // first block of the A slab's high plane
    const KFAC_AS1 unsigned char* b_hi;
    size_t plane_a, plane_b;                           // bytes from each operand's high plane to its low plane
    const float* scale_lds;
    int n;
    __device__ __forceinline__ const KFAC_AS1 unsigned char* a_blk(int q) const { return a_hi + (size_t)q * PRE_SLAB; }
    __device__ __forceinline__ const KFAC_AS1 unsigned char* b_blk(int q) const { return b_hi + (size_t)q * PRE_SLAB; }
    __device__ __forceinline__ size_t a_plane() const { return plane_a; }
    __device__ __forceinline__ size_t b_plane() const { return plane_b; }
    __device__ __forceinline__ float scale_of(int q) const { return scale_lds[q]; }
};

// The same product loop for a long contraction given as a SplitSeq (kept apart from the SplitRun form, whose register
// allocation inside the sweep's update kernel is tight).
__device__ __forceinline__ float tile_mma_presplit_seq(const SplitSeq& p, unsigned char* __restrict__ lds, TileAcc& acc) {
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    constexpr int NSL = 128 / SPLIT_KS;                // slices per product
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const int lm = lane & 31, h = lane >> 5;
    lds_byte* l0 = (lds_byte*)lds;
    unsigned a_addr[2], b_addr[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        a_addr[q] = (unsigned)split_plane_offset(wm * 64 + q * 32 + lm, h);
        b_addr[q] = (unsigned)(2 * PRE_BLOCK + split_plane_offset(wn * 64 + q * 32 + lm, h));
    }
    const int nst = p.n * NSL;
    const unsigned lane_off = (unsigned)(wave * 1024 + lane * 16);   // this lane's 16 bytes inside every block
    auto issue = [&](int s, int buf) {
        const int sc = s < nst ? s : nst - 1;          // past the end: re-read the last slice (never consumed)
        const int q = sc / NSL, ks = sc - q * NSL;
        const KFAC_AS1 unsigned char* pa = p.a_blk(q);
        const KFAC_AS1 unsigned char* pb = p.b_blk(q);
        const KFAC_AS1 unsigned char* src[4] = {pa, pa + p.a_plane(), pb, pb + p.b_plane()};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + ks * PRE_BLOCK + lane_off),
                                             (__attribute__((address_space(3))) void*)(l0 + buf * PRE_STAGE + j * PRE_BLOCK + wave * 1024),
                                             16, 0, 0);
    };
    float back = 1.0f;
#pragma unroll
    for (int s = 0; s < PRE_NS - 1; ++s) issue(s, s);
    for (int it = 0; it < nst; it += PRE_NS) {
#pragma unroll
        for (int bi = 0; bi < PRE_NS; ++bi) {
            const int s = it + bi;
            if (s >= nst) break;                                            // uniform
            static_assert(PRE_NS == 3, "the wait below counts (PRE_NS - 2) * 4 younger copies");
            asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");   // slice s landed (everybody's part)
            issue(s + PRE_NS - 1, (bi + PRE_NS - 1) % PRE_NS);               // refill the slot slice s - 1 vacated
            if (s % NSL == 0) {                                              // uniform: a new product begins
                const float sq = p.scale_of(s / NSL);
                const float f = sq * back;
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb) acc.c[mb][nb] *= f;
                back = 1.0f / sq;
            }
            v4f a[2][2], b[2][2];                                            // (16 bytes = 8 fp16 each)
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int pc = 0; pc < 2; ++pc) {
                    // (the stage's base goes into the address: an instruction offset holds 16 bits only)
                    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(a[q][pc]) : "v"(a_addr[q] + bi * PRE_STAGE), "n"(pc * PRE_BLOCK));
                    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(b[q][pc]) : "v"(b_addr[q] + bi * PRE_STAGE), "n"(pc * PRE_BLOCK));
                }
            asm volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(a[0][0]), "+v"(a[0][1]), "+v"(a[1][0]), "+v"(a[1][1]),
                           "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[1][0]), "+v"(b[1][1]));
            // smallest terms first
#pragma unroll
            for (int term = 0; term < 3; ++term)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                    {
                        v8h av, bv;
                        __builtin_memcpy(&av, &a[mb][term == 0 ? 1 : 0], 16);
                        __builtin_memcpy(&bv, &b[nb][term == 1 ? 1 : 0], 16);
                        acc.c[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc.c[mb][nb], 0, 0, 0);
                    }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");            // ring idle: the LDS may be reused
    return back;
}

}  // namespace kfac
