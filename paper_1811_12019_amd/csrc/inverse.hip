// Damped inverse of symmetric positive definite factors: Minv = (S + lambda I)^-1  (Sec. 4.2 damping, Eq. 6;
// Algorithm 1 stage 4), fp32.
//
// Method: blocked symmetric sweep (block Gauss-Jordan without pivoting, which is safe for SPD matrices).
// With the matrix cut into 128-wide blocks, eliminating block k does
//     P        = W_kk^-1                       (one workgroup, register/LDS resident)
//     T        = W_:k P                        (panel, MFMA)
//     W_ij    -= T_i W_jk^T   for i, j != k    (rank-128 update of the whole matrix, MFMA)
//     W_:k = T, W_k: = T^T, W_kk = -P
// and after all blocks W = -M^-1; the sign flip is folded into the last step.  Only tiles on or below the
// diagonal are computed; each is mirrored, so W stays exactly symmetric.  Every step touches the full matrix,
// so all steps expose the same, large amount of parallelism, and a batch of matrices of different sizes
// advances together: one launch per stage per step for the whole batch (the workgroup -> (matrix, tile) map is a
// prefix table passed in the kernel arguments).
#include "gemm_f32.h"

namespace kfac {

constexpr int NB = 128;          // elimination block = tile edge
constexpr int MAXB = 120;        // matrices per launch group

struct Batch {
    const kfac_inverse_item* table;   // device table, or nullptr -> `single`
    kfac_inverse_item single;
    int first;                        // index of the first matrix of this group in `table`
    int count;                        // active matrices in this launch
    int prefix[MAXB + 1];             // workgroup prefix sums over the active matrices
};

__device__ __forceinline__ kfac_inverse_item get_item(const Batch& b, int m) {
    return b.table ? b.table[b.first + m] : b.single;
}

__device__ __forceinline__ void locate(const Batch& b, int wg, int& m, int& local) {
    int lo = 0, hi = b.count;   // find m with prefix[m] <= wg < prefix[m+1]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (b.prefix[mid] <= wg) lo = mid; else hi = mid;
    }
    m = lo;
    local = wg - b.prefix[lo];
}

struct WsView {
    float* U;   // d_pad x NB : copy of the pivot block column before the step
    float* T;   // d_pad x NB : U . P
    float* P;   // NB x NB    : inverse of the pivot block
};

__host__ __device__ inline WsView ws_view(void* ws, int dim) {
    int d_pad = (dim + NB - 1) / NB * NB;
    WsView v;
    v.U = (float*)ws;
    v.T = v.U + (size_t)d_pad * NB;
    v.P = v.T + (size_t)d_pad * NB;
    return v;
}

// W = S + lambda I from S's lower triangle, written to both triangles; info = 0.
__global__ __launch_bounds__(256) void inv_init_kernel(Batch b) {
    int m, tile;
    locate(b, blockIdx.x, m, tile);
    const kfac_inverse_item it = get_item(b, m);
    const int d = it.dim;
    int I, J;
    tri_decode(tile, I, J);
    if (tile == 0 && threadIdx.x == 0 && it.info) *it.info = 0;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int r = ty; r < NB; r += 8) {
        int row = I * NB + r;
        if (row >= d) break;
        for (int c = tx; c < NB; c += 32) {
            int col = J * NB + c;
            if (col >= d || col > row) continue;
            float v = it.S[(size_t)row * d + col];
            if (row == col) v += it.damping;
            it.Minv[(size_t)row * d + col] = v;
            if (row != col) it.Minv[(size_t)col * d + row] = v;
        }
    }
}

// Inverse of the (at most 128 x 128) pivot block by an unblocked symmetric sweep held in registers:
// thread (ti, tj) of a 16 x 16 grid owns entries (ti + 16a, tj + 16b), a, b = 0..7.
__global__ __launch_bounds__(256) void inv_pivot_kernel(Batch b, int step, int write_from_S) {
    __shared__ float v[2][NB];
    __shared__ float sD[NB][NB + 1];
    __shared__ int bad;
    const int m = blockIdx.x;
    const kfac_inverse_item it = get_item(b, m);
    const int d = it.dim;
    const int k0 = step * NB;
    const int nb = min(NB, d - k0);
    const bool last = k0 + NB >= d;
    const int t = threadIdx.x, ti = t >> 4, tj = t & 15;
    float* W = it.Minv;
    WsView ws = ws_view(it.ws, d);
    if (t == 0) bad = 0;

    float D[8][8];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            int r = ti + 16 * a, q = tj + 16 * c;
            float x = (r == q) ? 1.f : 0.f;
            if (r < nb && q < nb) {
                int hi = max(r, q), lo = min(r, q);
                if (write_from_S) {
                    x = it.S[(size_t)(k0 + hi) * d + k0 + lo];
                    if (r == q) x += it.damping;
                } else {
                    x = W[(size_t)(k0 + hi) * d + k0 + lo];
                }
            }
            D[a][c] = x;
        }
    __syncthreads();

    int buf = 0;
#pragma unroll
    for (int q8 = 0; q8 < 8; ++q8) {
        for (int jj = 0; jj < 16; ++jj) {
            const int j = q8 * 16 + jj;
            if (j >= nb) break;
            if (tj == jj) {
#pragma unroll
                for (int a = 0; a < 8; ++a) v[buf][ti + 16 * a] = D[a][q8];
            }
            __syncthreads();
            const float p = v[buf][j];
            if (!(p > 0.f) && t == 0 && bad == 0) bad = k0 + j + 1;
            const float ip = 1.0f / p;
            float wi[8], vj[8];
#pragma unroll
            for (int a = 0; a < 8; ++a) wi[a] = v[buf][ti + 16 * a] * ip;
#pragma unroll
            for (int c = 0; c < 8; ++c) vj[c] = v[buf][tj + 16 * c];
#pragma unroll
            for (int a = 0; a < 8; ++a)
#pragma unroll
                for (int c = 0; c < 8; ++c) D[a][c] = fmaf(-wi[a], vj[c], D[a][c]);
            if (tj == jj) {
#pragma unroll
                for (int a = 0; a < 8; ++a) D[a][q8] = wi[a];
            }
            if (ti == jj) {
#pragma unroll
                for (int c = 0; c < 8; ++c) D[q8][c] = vj[c] * ip;
                if (tj == jj) D[q8][q8] = -ip;
            }
            buf ^= 1;
        }
    }
    __syncthreads();
    if (t == 0 && it.info) {
        if (write_from_S) *it.info = bad;                       // single-block matrix: this is its only kernel
        else if (bad != 0) atomicCAS((int*)it.info, 0, bad);    // keep the first failing minor
    }

    // D now holds -P up to rounding asymmetry; take the lower triangle as the truth so that P is exactly
    // symmetric.  The matrix gets -P (or +P on the last step, which folds in the final sign flip); the
    // workspace gets +P for the panel product.
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            int r = ti + 16 * a, q = tj + 16 * c;
            if (r >= q) sD[r][q] = D[a][c];
        }
    __syncthreads();
    const float sgn = last ? -1.f : 1.f;
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            int r = ti + 16 * a, q = tj + 16 * c;
            if (r < nb && q < nb) {
                float x = sD[max(r, q)][min(r, q)];
                W[(size_t)(k0 + r) * d + k0 + q] = sgn * x;
                if (!write_from_S) ws.P[r * NB + q] = -x;
            }
        }
}

// T = U . P for every 128-row slab of the pivot block column; U is copied aside for the update.
__global__ __launch_bounds__(256) void inv_panel_kernel(Batch b, int step) {
    __shared__ float lds[GEMM_LDS_FLOATS];
    int m, slab;
    locate(b, blockIdx.x, m, slab);
    const kfac_inverse_item it = get_item(b, m);
    const int d = it.dim;
    const int k0 = step * NB;
    const int nb = min(NB, d - k0);
    if (slab == step) return;                 // the pivot block's own rows are not needed
    const int r0 = slab * NB;
    const int rows = min(NB, d - r0);
    WsView ws = ws_view(it.ws, d);
    TileAcc acc;
    tile_mma_nt(it.Minv + (size_t)r0 * d + k0, d, rows, ws.P, NB, nb, nb, lds, acc, ws.U + (size_t)r0 * NB, NB);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = acc_row(wm, mb, r, lane), col = acc_col(wn, nbk, lane);
                if (row < rows && col < nb) ws.T[(size_t)(r0 + row) * NB + col] = acc.c[mb][nbk][r];
            }
}

// Rank-nb update of every tile on or below the diagonal, mirrored; the pivot block row/column receive T.
__global__ __launch_bounds__(256) void inv_update_kernel(Batch b, int step) {
    __shared__ float lds[GEMM_LDS_FLOATS];
    int m, tile;
    locate(b, blockIdx.x, m, tile);
    const kfac_inverse_item it = get_item(b, m);
    const int d = it.dim;
    int I, J;
    tri_decode(tile, I, J);
    const int kb = step;
    if (I == kb && J == kb) return;
    const int k0 = step * NB;
    const int nb = min(NB, d - k0);
    const bool last = k0 + NB >= d;
    const float sgn = last ? -1.f : 1.f;
    float* W = it.Minv;
    WsView ws = ws_view(it.ws, d);

    if (I == kb || J == kb) {
        // rows X0.. of the pivot column and their mirror in the pivot row
        const int X = (I == kb) ? J : I;
        const int x0 = X * NB;
        const int rows = min(NB, d - x0);
        const int c = threadIdx.x & 127, rh = threadIdx.x >> 7;
        if (c < nb) {
            for (int r = rh; r < rows; r += 2) {
                float v = sgn * ws.T[(size_t)(x0 + r) * NB + c];
                W[(size_t)(x0 + r) * d + k0 + c] = v;
                W[(size_t)(k0 + c) * d + x0 + r] = v;
            }
        }
        return;
    }

    const int i0 = I * NB, j0 = J * NB;
    const int irows = min(NB, d - i0), jrows = min(NB, d - j0);
    TileAcc acc;
    tile_mma_nt(ws.T + (size_t)i0 * NB, NB, irows, ws.U + (size_t)j0 * NB, NB, jrows, nb, lds, acc);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = acc_row(wm, mb, r, lane), col = acc_col(wn, nbk, lane);
                if (row >= irows || col >= jrows) continue;
                if (I == J && col > row) continue;
                size_t idx = (size_t)(i0 + row) * d + j0 + col;
                float v = sgn * (W[idx] - acc.c[mb][nbk][r]);
                W[idx] = v;
                if (!(I == J && col == row)) W[(size_t)(j0 + col) * d + i0 + row] = v;
            }
}

static inline int nblk_of(int dim) { return (dim + NB - 1) / NB; }
static inline int tri_tiles(int dim) { int n = nblk_of(dim); return n * (n + 1) / 2; }

// items must be sorted by non-increasing dim (checked by the caller of this function).
static int run_group(const kfac_inverse_item* host, const kfac_inverse_item* dev, int first, int count,
                     hipStream_t stream) {
    Batch b;
    b.table = dev;
    b.first = first;
    if (!dev) b.single = host[first];
    const kfac_inverse_item* h = host + first;
    const int max_steps = nblk_of(h[0].dim);

    // matrices needing the blocked path (more than one block) come first in the sorted order
    int n_multi = 0;
    while (n_multi < count && nblk_of(h[n_multi].dim) > 1) ++n_multi;

    if (n_multi > 0) {
        b.count = n_multi;
        b.prefix[0] = 0;
        for (int i = 0; i < n_multi; ++i) b.prefix[i + 1] = b.prefix[i] + tri_tiles(h[i].dim);
        KFAC_LAUNCH(inv_init_kernel, dim3(b.prefix[n_multi]), dim3(256), stream, b);
    }
    for (int step = 0; step < max_steps; ++step) {
        int active = 0;   // multi-block matrices that still have a block `step`
        while (active < n_multi && nblk_of(h[active].dim) > step) ++active;
        if (step == 0) {
            // single-block matrices: damp, invert and write in one kernel, straight from S
            if (count > n_multi) {
                Batch s = b;
                s.first = first + n_multi;
                if (!dev) s.single = host[first + n_multi];
                s.count = count - n_multi;
                KFAC_LAUNCH(inv_pivot_kernel, dim3(s.count), dim3(256), stream, s, 0, 1);
            }
        }
        if (active == 0) continue;
        b.count = active;
        KFAC_LAUNCH(inv_pivot_kernel, dim3(active), dim3(256), stream, b, step, 0);
        b.prefix[0] = 0;
        for (int i = 0; i < active; ++i) b.prefix[i + 1] = b.prefix[i] + nblk_of(h[i].dim);
        KFAC_LAUNCH(inv_panel_kernel, dim3(b.prefix[active]), dim3(256), stream, b, step);
        for (int i = 0; i < active; ++i) b.prefix[i + 1] = b.prefix[i] + tri_tiles(h[i].dim);
        KFAC_LAUNCH(inv_update_kernel, dim3(b.prefix[active]), dim3(256), stream, b, step);
    }
    return KFAC_OK;
}

static bool item_ok(const kfac_inverse_item& it) {
    if (!it.S || !it.Minv || it.dim <= 0 || it.dim > 32768) return false;
    if (it.S == it.Minv) return false;
    if (nblk_of(it.dim) > 1 && (!it.ws || ((uintptr_t)it.ws & 255))) return false;
    return true;
}

}  // namespace kfac

using namespace kfac;

extern "C" size_t kfac_inverse_workspace_bytes(int32_t dim) {
    if (dim <= 0 || dim > 32768) return 0;
    if (nblk_of(dim) == 1) return 256;
    size_t d_pad = (size_t)nblk_of(dim) * NB;
    return align_up((2 * d_pad * NB + (size_t)NB * NB) * sizeof(float), 256);
}

extern "C" int kfac_damped_inverse(const float* S, int32_t dim, float damping, float* Minv, int32_t* info,
                                   void* ws, size_t ws_bytes, void* stream) {
    kfac_inverse_item it;
    it.S = S; it.Minv = Minv; it.ws = ws; it.info = info; it.dim = dim; it.damping = damping;
    if (dim <= 0 || dim > 32768 || !S || !Minv || S == Minv) return KFAC_ERR_INVALID_ARG;
    if (nblk_of(dim) > 1) {
        if (!ws || ((uintptr_t)ws & 255) || ws_bytes < kfac_inverse_workspace_bytes(dim)) return KFAC_ERR_WORKSPACE;
    }
    return run_group(&it, nullptr, 0, 1, (hipStream_t)stream);
}

extern "C" int kfac_damped_inverse_batched(const kfac_inverse_item* items_host, const kfac_inverse_item* items_dev,
                                           int32_t count, void* stream) {
    if (!items_host || !items_dev || count <= 0) return KFAC_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i) {
        if (!item_ok(items_host[i])) return KFAC_ERR_INVALID_ARG;
        if (i > 0 && items_host[i].dim > items_host[i - 1].dim) return KFAC_ERR_INVALID_ARG;   // sorted, largest first
    }
    for (int first = 0; first < count; first += MAXB) {
        int n = count - first < MAXB ? count - first : MAXB;
        int rc = run_group(items_host, items_dev, first, n, (hipStream_t)stream);
        if (rc != KFAC_OK) return rc;
    }
    return KFAC_OK;
}
