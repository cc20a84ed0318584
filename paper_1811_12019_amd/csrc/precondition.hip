// Preconditioned gradient P = Ginv . gradW . Ainv  (Eq. 7 written for the d_G x d_A weight-gradient matrix;
// Algorithm 1 stage 5), fp32 results from the fp16 matrix cores.
//
// Both products run as "NT" tile products (both operands contiguous along the contraction index), using the symmetry
// of the inverses:
//   Yt[dA x dG] = Ainv . gradW^T      Yt[j, i] = sum_k Ainv[j, k] gradW[i, k]
//   P [dG x dA] = Ginv . Yt^T         P [i, j] = sum_k Ginv[i, k] Yt[j, k]
// Every fp32 operand is first cut into 128 x 128 blocks, each scaled by a power of two of its own (largest magnitude
// -> about 1) and split into two fp16 pieces (22 significant bits together), stored as planes in the order the tile
// product wants them in LDS (gemm_split.h): one pass over the inverses and the gradient (pre_split_kernel), and the
// first product's epilogue writes Yt in the same form.  The tile products then do no conversion work at all: operand
// slices go from global memory to LDS by DMA, and each 128-long piece of the contraction is three fp16 MFMAs per
// 32 x 32 block (high x high + high x low + low x high), the accumulators following the blocks' scales exactly.
// Splitting inside the product instead (three bf16 pieces of every operand, by every tile that reads it) kept the
// vector ALUs and LDS busier than the matrix cores.
// A batch of layers runs as three launches (split, product 1, product 2) over the blocks / tiles of all layers
// together, so that the many small layers fill the machine; the workgroup -> (layer, tile) map is a prefix table in
// the kernel arguments.
#include <algorithm>

#include "gemm_split.h"

namespace kfac {

constexpr int PMAXB = 120;       // layers per launch group

struct PBatch {
    const kfac_precond_item* table;   // device table, or nullptr -> `single`
    kfac_precond_item single;
    int first, count;
    int prefix[PMAXB + 1];            // workgroup prefix sums over the items of this launch
    short order[PMAXB];               // launch position -> item (relative to first): longest contraction first
};

// A matrix of r x k elements as planes: ceil(r / 128) slabs of ceil(k / 128) blocks of 128 x 128 (zero padded), block
// (s, c) at ((s * chunks + c) * PRE_SLAB) bytes in the plane of high pieces and in the plane of low pieces that
// follows it, then one float per block: its scale.  The four plane sets of a layer (Ainv, Ginv, gradW: dG x dA, Yt:
// dA x dG) live one after the other in its scratch; the inverses' may instead be the ones the inversion wrote.
struct PlaneSet {
    KFAC_AS1 unsigned char* hi;
    size_t plane;                     // bytes of one plane
    __device__ __forceinline__ gfloat* scales() const { return (gfloat*)(hi + 2 * plane); }
};
struct PlaneLayout {
    int nA, nG;                       // 128-blocks along d_A, d_G
    size_t a_plane, g_plane, w_plane; // bytes of one plane of Ainv, Ginv, gradW (= Yt)
    size_t a_off, g_off, w_off, y_off;
    size_t bytes;
};
static inline __host__ __device__ size_t plane_set_bytes(size_t plane, int blocks) {
    return (2 * plane + sizeof(float) * blocks + 255) & ~(size_t)255;
}
static inline __host__ __device__ PlaneLayout plane_layout(int dG, int dA) {
    PlaneLayout L;
    L.nA = (dA + TM - 1) / TM; L.nG = (dG + TM - 1) / TM;
    L.a_plane = (size_t)L.nA * L.nA * PRE_SLAB;
    L.g_plane = (size_t)L.nG * L.nG * PRE_SLAB;
    L.w_plane = (size_t)L.nG * L.nA * PRE_SLAB;
    L.a_off = 0;
    L.g_off = L.a_off + plane_set_bytes(L.a_plane, L.nA * L.nA);
    L.w_off = L.g_off + plane_set_bytes(L.g_plane, L.nG * L.nG);
    L.y_off = L.w_off + plane_set_bytes(L.w_plane, L.nG * L.nA);
    L.bytes = L.y_off + plane_set_bytes(L.w_plane, L.nG * L.nA);
    return L;
}
struct LayerPlanes { PlaneSet a, g, w, y; };
__device__ __forceinline__ LayerPlanes layer_planes(const kfac_precond_item& it, const PlaneLayout& L) {
    KFAC_AS1 unsigned char* ws = (KFAC_AS1 unsigned char*)as_global((float*)it.ws);
    LayerPlanes P;
    P.a.hi = it.Ainv_planes ? (KFAC_AS1 unsigned char*)as_global((float*)it.Ainv_planes) : ws + L.a_off; P.a.plane = L.a_plane;
    P.g.hi = it.Ginv_planes ? (KFAC_AS1 unsigned char*)as_global((float*)it.Ginv_planes) : ws + L.g_off; P.g.plane = L.g_plane;
    P.w.hi = ws + L.w_off; P.w.plane = L.w_plane;
    P.y.hi = ws + L.y_off; P.y.plane = L.w_plane;
    return P;
}
// 128 x 128 blocks the call has to split itself
static inline __host__ __device__ int split_blocks_A(const kfac_precond_item& it, int nA) { return it.Ainv_planes ? 0 : nA * nA; }
static inline __host__ __device__ int split_blocks_G(const kfac_precond_item& it, int nG) { return it.Ginv_planes ? 0 : nG * nG; }

__device__ __forceinline__ kfac_precond_item locate_item(const PBatch& b, int wg, int& local) {
    int lo = 0, hi = b.count;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (b.prefix[mid] <= wg) lo = mid; else hi = mid;
    }
    local = wg - b.prefix[lo];
    return b.table ? b.table[b.first + b.order[lo]] : b.single;
}

// 128 rows (row0 ..) x 128 columns of fp32 values held one float4 per thread and pass (thread t: columns 4 (t % 32) ..,
// rows t / 32 + 8 p) -> the block's scale and its two piece planes.
__device__ __forceinline__ void emit_block(const v4f (&v)[16], KFAC_AS1 unsigned char* hi, size_t plane, gfloat* scale,
                                           float* red) {
    const int t = threadIdx.x, c4 = (t & 31) * 4, rr = t >> 5;
    float m = 0.f;
#pragma unroll
    for (int p = 0; p < 16; ++p)
#pragma unroll
        for (int i = 0; i < 4; ++i) m = fmaxf(m, fabsf(v[p][i]));
    const float sc = panel_scale(block_absmax(m, red));
    if (t == 0) *scale = sc;
#pragma unroll
    for (int p = 0; p < 16; ++p) store_split4_h2(hi, hi + plane, rr + 8 * p, c4, v[p] * sc);
}

// One 128 x 128 block of Ainv, Ginv (unless their planes came with the call) or gradW per workgroup.
__global__ __launch_bounds__(256) void pre_split_kernel(PBatch b) {
    __shared__ float red[4];
    int local;
    const kfac_precond_item it = locate_item(b, blockIdx.x, local);
    const PlaneLayout L = plane_layout(it.dG, it.dA);
    const LayerPlanes P = layer_planes(it, L);
    const gfloat* X;
    int rows, cols, chunks;
    PlaneSet set;
    const int na = split_blocks_A(it, L.nA), ng = split_blocks_G(it, L.nG);
    if (local < na) {
        X = as_global(it.Ainv); rows = cols = it.dA; chunks = L.nA; set = P.a;
    } else if ((local -= na) < ng) {
        X = as_global(it.Ginv); rows = cols = it.dG; chunks = L.nG; set = P.g;
    } else {
        local -= ng;
        X = as_global(it.gradW); rows = it.dG; cols = it.dA; chunks = L.nA; set = P.w;
    }
    const int s = local / chunks, c = local - s * chunks;
    const int r0 = s * TM, k0 = c * TM;
    const int t = threadIdx.x, c4 = (t & 31) * 4, rr = t >> 5;
    v4f v[16];
    if (r0 + TM <= rows && k0 + TM <= cols) {            // all loads go out together (a guard per load would serialise them)
#pragma unroll
        for (int p = 0; p < 16; ++p) v[p] = *(const KFAC_AS1 v4f_a4*)(X + (size_t)(r0 + rr + 8 * p) * cols + k0 + c4);
    } else {
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = r0 + rr + 8 * p;
            v[p] = load4_guard(X + (size_t)(row < rows ? row : 0) * cols, row < rows, k0 + c4, cols);
        }
    }
    emit_block(v, set.hi + (size_t)local * PRE_SLAB, set.plane, set.scales() + local, red);
}

// phase 1: Yt[dA x dG] = Ainv . gradW^T (written as planes)      phase 2: out[dG x dA] = Ginv . Yt^T
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 8))) void gemm_nt_kernel(PBatch b, int phase) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[PRE_NS * PRE_STAGE];
    __shared__ float sc[256];
    __shared__ float red[4];
    int local;
    const kfac_precond_item it = locate_item(b, blockIdx.x, local);
    const PlaneLayout L = plane_layout(it.dG, it.dA);
    const LayerPlanes P = layer_planes(it, L);
    // Workgroups go to the 8 XCDs round-robin, each with an L2 of its own.  Inside a block of 8 tile rows, the eight
    // XCDs take one tile row each and walk along it: the tiles that share an A slab (128 rows of the inverse, the
    // large operand when the contraction is long) run on one L2, side by side, instead of on all eight.
    const int tm = phase == 1 ? L.nA : L.nG, tn = phase == 1 ? L.nG : L.nA;
    const int blk = local / (8 * tn), within = local - blk * 8 * tn;
    const int rb = min(8, tm - 8 * blk);
    const int ti = 8 * blk + within % rb, tj = within / rb;
    SplitSeq run;
    const gfloat *sa, *sb;
    if (phase == 1) {
        run.n = L.nA;
        run.a_hi = P.a.hi + (size_t)ti * L.nA * PRE_SLAB; run.plane_a = P.a.plane;
        run.b_hi = P.w.hi + (size_t)tj * L.nA * PRE_SLAB; run.plane_b = P.w.plane;
        sa = P.a.scales() + ti * L.nA; sb = P.w.scales() + tj * L.nA;
    } else {
        run.n = L.nG;
        run.a_hi = P.g.hi + (size_t)ti * L.nG * PRE_SLAB; run.plane_a = P.g.plane;
        run.b_hi = P.y.hi + (size_t)tj * L.nG * PRE_SLAB; run.plane_b = P.y.plane;
        sa = P.g.scales() + ti * L.nG; sb = P.y.scales() + tj * L.nG;
    }
    run.scale_lds = sc;
    const int t = threadIdx.x;
    if (t < run.n) sc[t] = sa[t] * sb[t];                // (at most 256 blocks along a contraction: dimensions end at 32768)
    TileAcc acc;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc.c[mb][nb][r] = 0.f;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // (the product counts its own copies in flight)
    __syncthreads();
    const float back = tile_mma_presplit_seq(run, lds, acc);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) acc.c[mb][nb] *= back;
    const int lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    if (phase == 2) {
        gfloat* C = as_global(it.out);
        const int i0 = ti * TM, j0 = tj * TM;
        const int irows = min(TM, it.dG - i0), jrows = min(TM, it.dA - j0);
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int row = acc_row(wm, mb, r, lane), col = acc_col(wn, nb, lane);
                    if (row < irows && col < jrows) C[(size_t)(i0 + row) * it.dA + j0 + col] = acc.c[mb][nb][r];
                }
        return;
    }
    // Yt block (slab ti, chunk tj) leaves as scaled fp16 pieces: through LDS, 64 rows at a time, so that a thread holds
    // four consecutive values of a row (rows and columns beyond the matrix are exact zeros: their operands were).
    float m = 0.f;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) m = fmaxf(m, fabsf(acc.c[mb][nb][r]));
    const float sy = panel_scale(block_absmax(m, red));
    const int blkidx = ti * L.nG + tj;
    if (t == 0) P.y.scales()[blkidx] = sy;
    KFAC_AS1 unsigned char* yh = P.y.hi + (size_t)blkidx * PRE_SLAB;
    constexpr int RLD = TM + 4;
    float* stage = (float*)lds;
    static_assert(64 * RLD * 4 <= PRE_NS * PRE_STAGE, "half a tile fits the ring's memory");
    const int c4 = (t & 31) * 4, rr = t >> 5;
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        if (half == 1) __syncthreads();
        if (wm == half) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        stage[(acc_row(0, mb, r, lane)) * RLD + acc_col(wn, nb, lane)] = acc.c[mb][nb][r];
        }
        __syncthreads();
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int row = rr + 8 * p;
            const v4f x = *(const v4f*)&stage[row * RLD + c4];
            store_split4_h2(yh, yh + P.y.plane, half * 64 + row, c4, x * sy);
        }
    }
}

static inline int tiles_of(int M, int N) { return ceil_div(M, TM) * ceil_div(N, TM); }

static int run_group(const kfac_precond_item* host, const kfac_precond_item* dev, int first, int count,
                     hipStream_t stream) {
    PBatch b;
    b.table = dev;
    b.first = first;
    b.count = count;
    if (!dev) b.single = host[first];
    // the operands' piece planes: one workgroup per 128 x 128 block of Ainv, Ginv and gradW
    b.prefix[0] = 0;
    for (int i = 0; i < count; ++i) {
        b.order[i] = (short)i;
        const kfac_precond_item& it = host[first + i];
        const int nA = ceil_div(it.dA, TM), nG = ceil_div(it.dG, TM);
        b.prefix[i + 1] = b.prefix[i] + split_blocks_A(it, nA) + split_blocks_G(it, nG) + nG * nA;
    }
    KFAC_LAUNCH(pre_split_kernel, dim3(b.prefix[count]), dim3(256), stream, b);
    for (int phase = 1; phase <= 2; ++phase) {
        // tiles with the longest contraction (K = dA in phase 1, dG in phase 2) go first: workgroups are dispatched in
        // order, so the long ones start early and the short ones fill the tail
        for (int i = 0; i < count; ++i) b.order[i] = (short)i;
        std::stable_sort(b.order, b.order + count, [&](short x, short y) {
            const kfac_precond_item &a = host[first + x], &c = host[first + y];
            return (phase == 1 ? a.dA : a.dG) > (phase == 1 ? c.dA : c.dG);
        });
        b.prefix[0] = 0;
        for (int i = 0; i < count; ++i) {
            const kfac_precond_item& it = host[first + b.order[i]];
            b.prefix[i + 1] = b.prefix[i] + (phase == 1 ? tiles_of(it.dA, it.dG) : tiles_of(it.dG, it.dA));
        }
        KFAC_LAUNCH(gemm_nt_kernel, dim3(b.prefix[count]), dim3(256), stream, b, phase);
    }
    return KFAC_OK;
}

static bool item_ok(const kfac_precond_item& it) {
    if (!it.Ginv || !it.Ainv || !it.gradW || !it.out || !it.ws) return false;
    if (it.dG <= 0 || it.dA <= 0 || it.dG > 32768 || it.dA > 32768) return false;
    if (it.out == it.gradW || it.out == it.Ginv || it.out == it.Ainv) return false;
    if (((uintptr_t)it.ws | (uintptr_t)it.Ginv_planes | (uintptr_t)it.Ainv_planes) & 255) return false;
    return true;
}

}  // namespace kfac

using namespace kfac;

extern "C" size_t kfac_precondition_workspace_bytes(int32_t dG, int32_t dA) {
    if (dG <= 0 || dA <= 0 || dG > 32768 || dA > 32768) return 0;
    return align_up(plane_layout(dG, dA).bytes, 256);
}

extern "C" int kfac_precondition(const float* Ginv, const float* Ainv, const float* gradW, int32_t dG, int32_t dA,
                                 float* out, void* ws, size_t ws_bytes, void* stream) {
    if (!Ginv || !Ainv || !gradW || !out || dG <= 0 || dA <= 0 || dG > 32768 || dA > 32768) return KFAC_ERR_INVALID_ARG;
    if (out == gradW || out == Ginv || out == Ainv) return KFAC_ERR_INVALID_ARG;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < kfac_precondition_workspace_bytes(dG, dA)) return KFAC_ERR_WORKSPACE;
    kfac_precond_item it;
    it.Ginv = Ginv; it.Ainv = Ainv; it.gradW = gradW; it.out = out; it.ws = ws; it.dG = dG; it.dA = dA;
    it.Ginv_planes = it.Ainv_planes = nullptr;
    return run_group(&it, nullptr, 0, 1, (hipStream_t)stream);
}

extern "C" int kfac_precondition_batched(const kfac_precond_item* items_host, const kfac_precond_item* items_dev,
                                         int32_t count, void* stream) {
    if (count == 0) return KFAC_OK;                       // nothing to do, no launch
    if (!items_host || !items_dev || count < 0) return KFAC_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i)
        if (!item_ok(items_host[i])) return KFAC_ERR_INVALID_ARG;
    for (int first = 0; first < count; first += PMAXB) {
        int n = count - first < PMAXB ? count - first : PMAXB;
        int rc = run_group(items_host, items_dev, first, n, (hipStream_t)stream);
        if (rc != KFAC_OK) return rc;
    }
    return KFAC_OK;
}

extern "C" const char* kfac_status_string(int status) {
    switch (status) {
        case KFAC_OK: return "ok";
        case KFAC_ERR_INVALID_ARG: return "invalid argument";
        case KFAC_ERR_UNSUPPORTED: return "unsupported";
        case KFAC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case KFAC_ERR_HIP: return "HIP runtime error";
        case KFAC_ERR_TOO_LARGE: return "request exceeds the fixed scratch of the no-allocation entry point";
        default: return "unknown status";
    }
}
