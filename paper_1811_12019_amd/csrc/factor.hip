// Kronecker-factor builders: A = scale * Xbar^T Xbar and G = scale * Gamma^T Gamma (Sec. 3.2, Eq. 5;
// Algorithm 1 stages 1 and 2) computed straight from the activation / output-gradient tensor.  The
// unfolded patch matrix is never materialised: tiles of it are gathered on the fly into LDS.
//
// Two kernels:
//   factor_dma_kernel      NHWC bf16/fp16, (kh, kw, c) column order, C % 8 == 0: matrix cores (factor_dma.h); many
//                          builds can share one launch (workgroup -> (build, tile) through a prefix table).
//   factor_generic_kernel  any layout / dtype / column order, fp32 FMA.  The fallback.
// Both enumerate only the lower-triangular tiles of the symmetric output and mirror them, and both
// can split the R unfolded rows over several workgroups (deterministic two-pass reduction through
// the caller's workspace, no float atomics).
#include <cstdlib>
#include <mutex>

#include "common.h"
#include "factor_mfma.h"
#include "factor_dma.h"
#include "factor_gather.h"

namespace kfac {

__device__ __forceinline__ float load_elem(const void* x, int dtype, int idx) {
    if (dtype == KFAC_F32) return ((const float*)x)[idx];
    uint16_t b = ((const uint16_t*)x)[idx];
    return dtype == KFAC_BF16 ? bf16_bits_to_float(b) : half_bits_to_float(b);
}

// Column of the unfolded matrix -> (channel, tap row, tap column); kind: 0 data, 1 bias (constant 1), 2 padding (0)
struct ColInfo {
    int c, i, j, kind;
};

__device__ __forceinline__ ColInfo decode_col(const Unfold& u, int col) {
    ColInfo ci;
    ci.c = ci.i = ci.j = 0;
    if (col >= u.d) {
        ci.kind = 2;
    } else if (u.has_bias && col == u.d - 1) {
        ci.kind = 1;
    } else {
        ci.kind = 0;
        if (u.order == KFAC_ORDER_C_KH_KW) {
            int khw = u.kh * u.kw;
            ci.c = col / khw;
            int rem = col - ci.c * khw;
            ci.i = rem / u.kw;
            ci.j = rem - ci.i * u.kw;
        } else {
            int tap = col / u.C;
            ci.c = col - tap * u.C;
            ci.i = tap / u.kw;
            ci.j = tap - ci.i * u.kw;
        }
    }
    return ci;
}

constexpr int GT = 64;   // generic kernel: output tile edge
constexpr int GK = 16;   // unfolded rows per LDS stage

__global__ __launch_bounds__(256) void factor_generic_kernel(Unfold u, const void* __restrict__ x, float scale,
                                                             OutSpec os, float* __restrict__ partial,
                                                             int rows_per_split) {
    __shared__ float As[GK][GT + 4];
    __shared__ float Bs[GK][GT + 4];
    __shared__ int rowN[GK], rowY[GK], rowX[GK];

    const int t = threadIdx.x;
    int I, J;
    tri_decode(blockIdx.x, I, J);
    const int split = blockIdx.y;
    const int r_begin = split * rows_per_split;
    const int r_end = min(u.R, r_begin + rows_per_split);

    const int m = t & 63, kb = t >> 6;
    const ColInfo ca = decode_col(u, I * GT + m);
    const ColInfo cb = decode_col(u, J * GT + m);
    const int tx = t & 15, ty = t >> 4;

    float acc[4][4] = {};
    for (int r0 = r_begin; r0 < r_end; r0 += GK) {
        if (t < GK) {
            int r = r0 + t;
            if (r < r_end) {
                int n = r / (u.Ho * u.Wo);
                int rem = r - n * (u.Ho * u.Wo);
                int yo = rem / u.Wo;
                int xo = rem - yo * u.Wo;
                rowN[t] = n;
                rowY[t] = yo * u.stride - u.pad;
                rowX[t] = xo * u.stride - u.pad;
            } else {
                rowN[t] = -1;
                rowY[t] = 0;
                rowX[t] = 0;
            }
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int k = kb + 4 * e;
            int n = rowN[k];
            float va = 0.f, vb = 0.f;
            if (n >= 0) {
                {
                    if (ca.kind == 1) va = 1.f;
                    else if (ca.kind == 0) {
                        int y = rowY[k] + ca.i, xx = rowX[k] + ca.j;
                        if (y >= 0 && y < u.H && xx >= 0 && xx < u.W) {
                            int idx = u.layout == KFAC_NHWC ? ((n * u.H + y) * u.W + xx) * u.C + ca.c
                                                            : ((n * u.C + ca.c) * u.H + y) * u.W + xx;
                            va = load_elem(x, u.dtype, idx);
                        }
                    }
                }
                if (I == J) vb = va;
                else {
                    if (cb.kind == 1) vb = 1.f;
                    else if (cb.kind == 0) {
                        int y = rowY[k] + cb.i, xx = rowX[k] + cb.j;
                        if (y >= 0 && y < u.H && xx >= 0 && xx < u.W) {
                            int idx = u.layout == KFAC_NHWC ? ((n * u.H + y) * u.W + xx) * u.C + cb.c
                                                            : ((n * u.C + cb.c) * u.H + y) * u.W + xx;
                            vb = load_elem(x, u.dtype, idx);
                        }
                    }
                }
            }
            As[k][m] = va;
            Bs[k][m] = vb;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < GK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                a[q] = As[k][ty * 4 + q];
                b[q] = Bs[k][tx * 4 + q];
            }
#pragma unroll
            for (int p = 0; p < 4; ++p)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[p][q] = fmaf(a[p], b[q], acc[p][q]);
        }
        __syncthreads();
    }

    if (gridDim.y == 1) {
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int row = I * GT + ty * 4 + p, col = J * GT + tx * 4 + q;
                if (row < u.d && col < u.d) emit_sym(os, u.d, row, col, acc[p][q] * scale, I != J);
            }
    } else {
        float* dst = partial + ((size_t)split * gridDim.x + blockIdx.x) * (GT * GT);
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int q = 0; q < 4; ++q) dst[(ty * 4 + p) * GT + tx * 4 + q] = acc[p][q];
    }
}

// Second pass of a split build: sum the per-split partial tiles in a fixed order, scale, write the tile and its
// mirror.  One workgroup per 32 x 32 sub-block of a tile: every thread owns four consecutive columns of one row, so
// partial reads are 128-byte runs; the mirror goes through an LDS transpose.
template <int T>
__device__ __forceinline__ void factor_reduce_block(const gfloat* __restrict__ partial, int nsplit, int ntiles,
                                                    int tile, int sub, int d, float scale, const OutSpec& os,
                                                    float (*tr)[33]) {
    int I, J;
    if constexpr (T == FT) tri_decode_blocked<4>(ceil_div(d, T), tile, I, J);   // (the matrix-core kernel's tile order)
    else tri_decode(tile, I, J);
    constexpr int SB = T / 32;
    const int si = sub / SB, sj = sub - si * SB;
    const int lr = threadIdx.x >> 3, lc = (threadIdx.x & 7) * 4;
    const int trow = si * 32 + lr, tcol = sj * 32 + lc;              // inside the tile
    const int row = I * T + trow, col = J * T + tcol;
    if (I * T + si * 32 >= d || J * T + sj * 32 >= d) return;       // whole sub-block outside the matrix
    v4f s = {0.f, 0.f, 0.f, 0.f};
    if (row < d && col < d) {
        const gfloat* src = partial + (size_t)tile * (T * T) + trow * T + tcol;
        const size_t stride = (size_t)ntiles * (T * T);
        int sp = 0;
        for (; sp + 4 <= nsplit; sp += 4) {
            v4f a = *(const KFAC_AS1 v4f*)(src + (size_t)sp * stride);
            v4f b = *(const KFAC_AS1 v4f*)(src + (size_t)(sp + 1) * stride);
            v4f c = *(const KFAC_AS1 v4f*)(src + (size_t)(sp + 2) * stride);
            v4f e = *(const KFAC_AS1 v4f*)(src + (size_t)(sp + 3) * stride);
            s += a; s += b; s += c; s += e;
        }
        for (; sp < nsplit; ++sp) s += *(const KFAC_AS1 v4f*)(src + (size_t)sp * stride);
        s *= scale;
        gfloat* __restrict__ out = os.dst;
        if (os.mode == OUT_PACKED) {                                 // only elements on or above the diagonal exist
            if (I == J) {
                const size_t rb = packed_row_base(row, d);
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (col + q < d && col + q >= row) out[rb + col + q] = s[q];
            }
        } else {
            if (os.mode == OUT_EMA) {
                if (col + 3 < d) {
                    const v4f o = *(const KFAC_AS1 v4f_a4*)(out + (size_t)row * d + col);
#pragma unroll
                    for (int q = 0; q < 4; ++q) s[q] = fmaf(os.decay, o[q], os.one_minus * s[q]);
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (col + q < d) s[q] = fmaf(os.decay, out[(size_t)row * d + col + q], os.one_minus * s[q]);
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (col + q < d) out[(size_t)row * d + col + q] = s[q];
        }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) tr[lr][lc + q] = s[q];
    if (I == J) return;                                              // uniform: diagonal tiles hold their own mirror
    __syncthreads();
    // transposed: thread (lr, lc..lc+3) now owns mirrored row (J*T + sj*32 + lr), columns I*T + si*32 + lc..+3
    const int mrow = J * T + sj * 32 + lr, mcol = I * T + si * 32 + lc;
    if (mrow < d) {
        gfloat* __restrict__ mout = os.dst + (os.mode == OUT_PACKED ? packed_row_base(mrow, d) : (size_t)mrow * d);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (mcol + q < d) mout[mcol + q] = tr[lc + q][lr];
    }
}

template <int T>
__global__ __launch_bounds__(256) void factor_reduce_kernel(const float* __restrict__ partial, int nsplit, int d,
                                                            float scale, OutSpec os) {
    __shared__ float tr[32][33];
    factor_reduce_block<T>(as_global(partial), nsplit, gridDim.x, blockIdx.x, blockIdx.y, d, scale, os, tr);
}

struct FactorPlan {
    int tiles_dim;   // tiles per dimension
    int ntiles;      // lower-triangular tiles
    int nsplit;
    int rows_per_split;
    size_t ws_bytes;
};

static FactorPlan plan_generic(const Unfold& u) {
    FactorPlan p;
    p.tiles_dim = ceil_div(u.d, GT);
    p.ntiles = p.tiles_dim * (p.tiles_dim + 1) / 2;
    int want = ceil_div(2048, p.ntiles);
    int max_split = ceil_div(u.R, 4 * GK);
    p.nsplit = want < 1 ? 1 : (want > max_split ? max_split : want);
    if (p.nsplit < 1) p.nsplit = 1;
    p.rows_per_split = ceil_div(ceil_div(u.R, p.nsplit), GK) * GK;
    p.nsplit = ceil_div(u.R, p.rows_per_split);
    p.ws_bytes = p.nsplit > 1 ? (size_t)p.nsplit * p.ntiles * GT * GT * sizeof(float) : 0;
    return p;
}

// The matrix-core kernel needs 16-byte channel vectors in (kh, kw, c) column order, and its row decode is exact
// below 2^24 rows.
static __host__ __device__ bool dma_eligible(const Unfold& u) {
    if (u.dtype != KFAC_BF16 && u.dtype != KFAC_F16) return false;
    if (u.layout != KFAC_NHWC || (u.C & 7)) return false;
    if (u.order != KFAC_ORDER_KH_KW_C && !(u.kh == 1 && u.kw == 1)) return false;
    // the kernel packs a row's patch origin (y0, x0), each offset by 16384, into one 32-bit word
    if (u.H + u.pad >= 16384 || u.W + u.pad >= 16384 || u.pad >= 16384) return false;
    return u.R < (1 << 24);
}

// `target`: workgroups wanted for this build.  A build launched alone wants about two per CU; in a batched launch
// the other builds fill the chip, and fewer, longer row splits mean fewer partial sums through HBM.
constexpr int FTARGET_ALONE = 512;
constexpr int FTARGET_BATCHED_PLAIN = 128;   // measured best on the 54-layer ResNet-50 batch
constexpr int FTARGET_BATCHED_CONV = 64;

static __host__ __device__ FactorPlan plan_dma(const Unfold& u, int target = FTARGET_ALONE) {
    FactorPlan p;
    p.tiles_dim = ceil_div(u.d, FT);
    p.ntiles = p.tiles_dim * (p.tiles_dim + 1) / 2;
    int want = target / p.ntiles;
    int max_split = u.R / (8 * 64);        // at least 512 rows per workgroup
    int ns = want < max_split ? want : max_split;
    if (ns < 1) ns = 1;
    if (ns >= 8) ns = ns / 8 * 8;          // multiples of 8 keep a row range on one XCD
    p.rows_per_split = ceil_div(ceil_div(u.R, ns), 64) * 64;
    p.nsplit = ceil_div(u.R, p.rows_per_split);
    p.ws_bytes = p.nsplit > 1 ? (size_t)p.nsplit * p.ntiles * FT * FT * sizeof(float) : 0;
    return p;
}

// Narrow 16-bit NHWC layers the LDS-DMA kernel cannot take (channels not a multiple of 8) with many rows.
static bool gather_eligible(const Unfold& u) {
    if (u.dtype != KFAC_BF16 && u.dtype != KFAC_F16) return false;
    if (u.layout != KFAC_NHWC || (u.C & 7) == 0) return false;
    if (u.order != KFAC_ORDER_KH_KW_C && !(u.kh == 1 && u.kw == 1)) return false;
    return u.d <= GA_DMAX && u.R >= 4096 && u.R < (1 << 24);
}

static FactorPlan plan_gather(const Unfold& u) {
    FactorPlan p;
    p.tiles_dim = ceil_div(u.d, GA_T);
    p.ntiles = p.tiles_dim * (p.tiles_dim + 1) / 2;
    int ns = u.R / (4 * GA_ROWS);                   // at least 256 rows per workgroup
    if (ns > 512) ns = 512;                         // two workgroups per CU
    if (ns < 1) ns = 1;
    p.rows_per_split = ceil_div(ceil_div(u.R, ns), GA_ROWS) * GA_ROWS;
    p.nsplit = ceil_div(u.R, p.rows_per_split);
    p.ws_bytes = (size_t)p.nsplit * p.ntiles * GA_T * GA_T * sizeof(float);
    return p;
}

// Where an item's result goes.
static __host__ __device__ __forceinline__ OutSpec out_spec(const kfac_factor_item& it) {
    OutSpec o;
    o.decay = it.decay;
    o.one_minus = 1.0f - it.decay;
    if (it.running) { o.dst = (gfloat*)it.running; o.mode = OUT_EMA; }
    else { o.dst = (gfloat*)it.out; o.mode = it.packed ? OUT_PACKED : OUT_PLAIN; }
    return o;
}

// ---- batched launches: many factor builds in one grid -------------------------------------------------------------
constexpr int FMAXB = 120;

struct FBatch {
    const kfac_factor_item* table;   // device table, or nullptr -> `single`
    kfac_factor_item single;
    int count;
    int target;                      // plan_dma's workgroup target for every build of this launch
    int index[FMAXB];                // table index of the i-th build of this launch
    int prefix[FMAXB + 1];           // workgroup prefix sums
};

__device__ __forceinline__ int fbatch_locate(const FBatch& b, int wg, int& local) {
    int lo = 0, hi = b.count;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (b.prefix[mid] <= wg) lo = mid; else hi = mid;
    }
    local = wg - b.prefix[lo];
    return lo;
}

template <bool PLAIN, bool F16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 8))) void factor_dma_kernel(FBatch b) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    int local;
    const int m = fbatch_locate(b, blockIdx.x, local);
    const kfac_factor_item it = b.table ? b.table[b.index[m]] : b.single;
    Unfold u;
    if (it.op == KFAC_OP_FACTOR_A) make_unfold_A(&it.desc, &u); else make_unfold_G(&it.desc, &u);
    const FactorPlan p = plan_dma(u, b.target);
    const float scale = it.scale == 0.f ? 1.0f / (float)u.R : it.scale;
    factor_dma_tile<PLAIN, F16>(u, (const KFAC_AS1 unsigned char*)it.x, scale, out_spec(it),
                                as_global((float*)it.ws), p.rows_per_split, p.ntiles, p.nsplit, local, smem);
}

__global__ __launch_bounds__(256) void factor_reduce_batched_kernel(FBatch b) {
    __shared__ float tr[32][33];
    int local;
    const int m = fbatch_locate(b, blockIdx.x, local);
    const kfac_factor_item it = b.table ? b.table[b.index[m]] : b.single;
    Unfold u;
    if (it.op == KFAC_OP_FACTOR_A) make_unfold_A(&it.desc, &u); else make_unfold_G(&it.desc, &u);
    const FactorPlan p = plan_dma(u, b.target);
    const float scale = it.scale == 0.f ? 1.0f / (float)u.R : it.scale;
    constexpr int SUBS = (FT / 32) * (FT / 32);
    factor_reduce_block<FT>(as_global((const float*)it.ws), p.nsplit, p.ntiles, local / SUBS, local % SUBS, u.d, scale,
                            out_spec(it), tr);
}

static bool item_unfold(const kfac_factor_item& it, Unfold* u) {
    if (it.op == KFAC_OP_FACTOR_A) return make_unfold_A(&it.desc, u);
    if (it.op == KFAC_OP_FACTOR_G) return make_unfold_G(&it.desc, u);
    return false;
}

static size_t item_ws_bytes(const Unfold& u) {
    size_t a = plan_generic(u).ws_bytes;                       // either kernel may serve the build
    size_t b = dma_eligible(u) ? plan_dma(u).ws_bytes : 0;
    size_t c = gather_eligible(u) ? plan_gather(u).ws_bytes : 0;
    if (b > a) a = b;
    if (c > a) a = c;
    return align_up(a, 256);
}

static int check_item(const kfac_factor_item& it, Unfold* u) {
    if (!item_unfold(it, u)) return KFAC_ERR_INVALID_ARG;
    if (!it.x) return KFAC_ERR_INVALID_ARG;
    // exactly one destination: the fresh factor (square or packed) or the running average it is folded into
    if (it.running ? (it.out != nullptr || it.packed != 0 || !(it.decay >= 0.f && it.decay <= 1.f)) : !it.out) return KFAC_ERR_INVALID_ARG;
    if (it.packed != 0 && it.packed != 1) return KFAC_ERR_INVALID_ARG;
    const size_t need = item_ws_bytes(*u);
    if (need > 0 && (!it.ws || ((uintptr_t)it.ws & 255) || it.ws_bytes < need)) return KFAC_ERR_WORKSPACE;
    return KFAC_OK;
}

template <bool PLAIN, bool F16>
static int launch_dma_group(const FBatch& b, hipStream_t stream) {
    static std::once_flag attr_once;                 // (one per kernel variant; safe from any number of host threads)
    std::call_once(attr_once, [] {
        (void)hipFuncSetAttribute((const void*)factor_dma_kernel<PLAIN, F16>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, FACTOR_DMA_LDS);
    });
    void* tok = nullptr;
    if (timing_enabled()) timing_begin(PLAIN ? "factor_dma_kernel<plain>" : "factor_dma_kernel<conv>", stream, &tok);
    hipLaunchKernelGGL((factor_dma_kernel<PLAIN, F16>), dim3(b.prefix[b.count]), dim3(256), FACTOR_DMA_LDS, stream, b);
    if (tok) timing_end(stream, tok);
    if (hipGetLastError() != hipSuccess) return KFAC_ERR_HIP;
    return KFAC_OK;
}

static int run_gather(const Unfold& u, const kfac_factor_item& it, hipStream_t stream) {
    const float scale = it.scale == 0.f ? 1.0f / (float)u.R : it.scale;
    const FactorPlan p = plan_gather(u);
    if (u.dtype == KFAC_F16) {
        KFAC_LAUNCH(factor_gather_kernel<true>, dim3(p.nsplit), dim3(256), stream, u, it.x, (float*)it.ws, p.rows_per_split);
    } else {
        KFAC_LAUNCH(factor_gather_kernel<false>, dim3(p.nsplit), dim3(256), stream, u, it.x, (float*)it.ws, p.rows_per_split);
    }
    KFAC_LAUNCH(factor_gather_reduce_kernel, dim3(p.ntiles * GA_T), dim3(256), stream, (const float*)it.ws, p.nsplit, p.ntiles,
                u.d, scale, out_spec(it));
    return KFAC_OK;
}

static int run_generic(const Unfold& u, const kfac_factor_item& it, hipStream_t stream) {
    if (gather_eligible(u) && ((uintptr_t)it.x & 1) == 0) return run_gather(u, it, stream);
    const float scale = it.scale == 0.f ? 1.0f / (float)u.R : it.scale;
    FactorPlan p = plan_generic(u);
    dim3 grid(p.ntiles, p.nsplit);
    KFAC_LAUNCH(factor_generic_kernel, grid, dim3(256), stream, u, it.x, scale, out_spec(it), (float*)it.ws, p.rows_per_split);
    if (p.nsplit > 1) {
        KFAC_LAUNCH(factor_reduce_kernel<GT>, dim3(p.ntiles, (GT / 32) * (GT / 32)), dim3(256), stream,
                    (const float*)it.ws, p.nsplit, u.d, scale, out_spec(it));
    }
    return KFAC_OK;
}

// All builds of items[0..count): matrix-core builds grouped by kernel variant into batched launches, the rest one
// by one through the generic kernel.  `dev` may be nullptr only when count == 1.
static int run_factor_items(const kfac_factor_item* host, const kfac_factor_item* dev, int count, hipStream_t stream) {
    for (int i = 0; i < count; ++i) {
        Unfold u;
        int rc = check_item(host[i], &u);
        if (rc != KFAC_OK) return rc;
    }
    // variants: 0 plain bf16, 1 plain f16, 2 conv bf16, 3 conv f16
    int n_dma = 0;
    for (int i = 0; i < count; ++i) {
        Unfold u;
        item_unfold(host[i], &u);
        if (dma_eligible(u) && ((uintptr_t)host[i].x & 15) == 0) ++n_dma;
    }
    for (int variant = 0; variant < 4; ++variant) {
        const int target = n_dma < 16 ? FTARGET_ALONE : variant < 2 ? FTARGET_BATCHED_PLAIN : FTARGET_BATCHED_CONV;
        int next = 0;
        while (next < count) {
            FBatch b, r;
            b.table = r.table = dev;
            b.count = r.count = 0;
            b.target = r.target = target;
            b.prefix[0] = r.prefix[0] = 0;
            for (; next < count && b.count < FMAXB; ++next) {
                Unfold u;
                item_unfold(host[next], &u);
                if (!dma_eligible(u) || ((uintptr_t)host[next].x & 15)) continue;
                const bool plain = u.kh == 1 && u.kw == 1 && u.stride == 1 && u.pad == 0;
                const bool f16 = u.dtype == KFAC_F16;
                if ((plain ? 0 : 2) + (f16 ? 1 : 0) != variant) continue;
                const FactorPlan p = plan_dma(u, target);
                b.index[b.count] = next;
                b.prefix[b.count + 1] = b.prefix[b.count] + align_up(p.ntiles * p.nsplit, 8);   // see factor_dma_tile
                if (!dev) b.single = host[next];
                ++b.count;
                if (p.nsplit > 1) {
                    r.index[r.count] = next;
                    r.prefix[r.count + 1] = r.prefix[r.count] + p.ntiles * (FT / 32) * (FT / 32);
                    if (!dev) r.single = host[next];
                    ++r.count;
                }
            }
            if (b.count == 0) continue;
            int rc = variant == 0 ? launch_dma_group<true, false>(b, stream)
                   : variant == 1 ? launch_dma_group<true, true>(b, stream)
                   : variant == 2 ? launch_dma_group<false, false>(b, stream)
                                  : launch_dma_group<false, true>(b, stream);
            if (rc != KFAC_OK) return rc;
            if (r.count > 0) {
                KFAC_LAUNCH(factor_reduce_batched_kernel, dim3(r.prefix[r.count]), dim3(256), stream, r);
            }
        }
    }
    for (int i = 0; i < count; ++i) {
        Unfold u;
        item_unfold(host[i], &u);
        if (dma_eligible(u) && ((uintptr_t)host[i].x & 15) == 0) continue;
        int rc = run_generic(u, host[i], stream);
        if (rc != KFAC_OK) return rc;
    }
    return KFAC_OK;
}

}  // namespace kfac

using namespace kfac;

extern "C" size_t kfac_factor_workspace_bytes(int op, const kfac_layer_desc* desc) {
    Unfold u;
    bool ok = op == KFAC_OP_FACTOR_A ? make_unfold_A(desc, &u) : op == KFAC_OP_FACTOR_G ? make_unfold_G(desc, &u) : false;
    if (!ok) return 0;
    return item_ws_bytes(u);
}

static int factor_single(int op, const kfac_layer_desc* desc, const void* x, float scale, float* out, void* ws,
                         size_t ws_bytes, void* stream) {
    if (!desc) return KFAC_ERR_INVALID_ARG;
    kfac_factor_item it;
    it.desc = *desc; it.x = x; it.out = out; it.ws = ws; it.ws_bytes = ws_bytes; it.scale = scale; it.op = op;
    it.running = nullptr; it.decay = 0.f; it.packed = 0;
    return run_factor_items(&it, nullptr, 1, (hipStream_t)stream);
}

extern "C" int kfac_factor_A(const kfac_layer_desc* desc, const void* act, float scale, float* A, void* ws,
                             size_t ws_bytes, void* stream) {
    return factor_single(KFAC_OP_FACTOR_A, desc, act, scale, A, ws, ws_bytes, stream);
}

extern "C" int kfac_factor_G(const kfac_layer_desc* desc, const void* gout, float scale, float* G, void* ws,
                             size_t ws_bytes, void* stream) {
    return factor_single(KFAC_OP_FACTOR_G, desc, gout, scale, G, ws, ws_bytes, stream);
}

extern "C" int kfac_factor_batched(const kfac_factor_item* items_host, const kfac_factor_item* items_dev, int32_t count,
                                   void* stream) {
    if (count == 0) return KFAC_OK;                       // nothing to do, no launch
    if (!items_host || !items_dev || count < 0) return KFAC_ERR_INVALID_ARG;
    return run_factor_items(items_host, items_dev, count, (hipStream_t)stream);
}
