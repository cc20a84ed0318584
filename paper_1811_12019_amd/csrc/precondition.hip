// Preconditioned gradient P = Ginv . gradW . Ainv  (Eq. 7 written for the d_G x d_A weight-gradient matrix;
// Algorithm 1 stage 5), fp32 on the matrix cores.
//
// Both products run as "NT" tile products (both operands K-contiguous), using the symmetry of the inverses:
//   Yt[dA x dG] = Ainv . gradW^T      Yt[j, i] = sum_k Ainv[j, k] gradW[i, k]
//   P [dG x dA] = Ginv . Yt^T         P [i, j] = sum_k Ginv[i, k] Yt[j, k]
// A batch of layers runs as two launches (one per product) over the tiles of all layers together, so that the
// many small layers fill the machine; the workgroup -> (layer, tile) map is a prefix table in the kernel arguments.
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

// phase 1: Yt[dA x dG] = Ainv . gradW^T      phase 2: out[dG x dA] = Ginv . Yt^T
__global__ __launch_bounds__(256) void gemm_nt_kernel(PBatch b, int phase) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[split_lds_bytes<3>()];
    int lo = 0, hi = b.count;
    const int wg = blockIdx.x;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (b.prefix[mid] <= wg) lo = mid; else hi = mid;
    }
    const kfac_precond_item it = b.table ? b.table[b.first + b.order[lo]] : b.single;
    const int local = wg - b.prefix[lo];
    const gfloat *A, *B;
    gfloat* C;
    int M, N, K;
    if (phase == 1) { A = as_global(it.Ainv); B = as_global(it.gradW); C = as_global((float*)it.ws); M = it.dA; N = it.dG; K = it.dA; }
    else            { A = as_global(it.Ginv); B = as_global((const float*)it.ws); C = as_global(it.out); M = it.dG; N = it.dA; K = it.dG; }
    // Workgroups go to the 8 XCDs round-robin, each with an L2 of its own.  Inside a block of 8 tile rows, the eight
    // XCDs take one tile row each and walk along it: the tiles that share an A panel (128 rows of the inverse, the
    // large operand when K is long) run on one L2, side by side, instead of on all eight (a third less traffic
    // beyond L2).
    const int tm = (M + TM - 1) / TM, tn = (N + TM - 1) / TM;
    const int blk = local / (8 * tn), within = local - blk * 8 * tn;
    const int rb = min(8, tm - 8 * blk);
    const int ti = 8 * blk + within % rb, tj = within / rb;
    const int i0 = ti * TM, j0 = tj * TM;
    const int irows = min(TM, M - i0), jrows = min(TM, N - j0);
    TileAcc acc;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc.c[mb][nb][r] = 0.f;
    // Interior tiles take the contraction 128 columns at a time through the unrolled, branch-free pipeline (two slabs
    // of look-ahead with exact wait counts; the general loop has one slab of look-ahead and pays a memory round trip
    // per slab, which a long contraction with few tiles cannot hide); the rest of K, and edge tiles, go the general way.
    const gfloat* At = A + (size_t)i0 * K;
    const gfloat* Bt = B + (size_t)j0 * K;
    int kdone = 0;
    if (irows == TM && jrows == TM) {
        for (; kdone + 128 <= K; kdone += 128)
            tile_mma_nt_split<3, false, 128 / SPLIT_KS, true>(At + kdone, K, TM, Bt + kdone, K, TM, 128, lds, acc);
    }
    if (kdone < K) tile_mma_nt_split<3>(At + kdone, K, irows, Bt + kdone, K, jrows, K - kdone, lds, acc);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = acc_row(wm, mb, r, lane), col = acc_col(wn, nb, lane);
                if (row < irows && col < jrows) C[(size_t)(i0 + row) * N + j0 + col] = acc.c[mb][nb][r];
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
    if ((uintptr_t)it.ws & 255) return false;
    return true;
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
    kfac_precond_item it;
    it.Ginv = Ginv; it.Ainv = Ainv; it.gradW = gradW; it.out = out; it.ws = ws; it.dG = dG; it.dA = dA;
    return run_group(&it, nullptr, 0, 1, (hipStream_t)stream);
}

extern "C" int kfac_precondition_batched(const kfac_precond_item* items_host, const kfac_precond_item* items_dev,
                                         int32_t count, void* stream) {
    if (!items_host || !items_dev || count <= 0) return KFAC_ERR_INVALID_ARG;
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
