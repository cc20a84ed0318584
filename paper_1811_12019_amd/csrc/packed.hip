// Packed upper triangles of the symmetric Kronecker factors (Sec. 3.4, symmetry-aware communication: only the upper
// triangular part of a factor travels), and the running average fed from a packed factor.
//
// Packed layout: row i of the upper triangle contributes S[i][i], S[i][i+1], ..., S[i][n-1], rows in order; row i
// starts at i n - i (i - 1) / 2 and the whole has n (n + 1) / 2 elements.
// All matrices of a call go in one launch (workgroup -> matrix through prefix sums in the kernel arguments).  Packing
// walks the packed array linearly (aligned 16-byte stores; the sources are runs of matrix rows).  The packed running
// average works on 128 x 128 tiles (I <= J), one workgroup per tile: a tile row is a contiguous run both in the full
// matrix and in the packed array, and the mirrored tile is written row-wise after a transpose through LDS.  HBM bound.
#include "common.h"

namespace kfac {

constexpr int PK_T = 128;             // tile edge
constexpr int PK_MAX = 128;           // matrices per launch (keeps the argument block under 4 KB)

struct PackBatch {
    int count;
    unsigned prefix[PK_MAX + 1];      // first workgroup of matrix i
    int dim[PK_MAX];
    float* full[PK_MAX];              // dim x dim
    float* packed[PK_MAX];            // dim (dim + 1) / 2
};

static inline __host__ __device__ int pk_tiles(int dim) { const int t = (dim + PK_T - 1) / PK_T; return t * (t + 1) / 2; }

__device__ __forceinline__ size_t pk_row_start(int i, int n) { return (size_t)i * n - (size_t)i * (i - 1) / 2; }

__device__ __forceinline__ void pk_locate(const PackBatch& b, int& m, int& I, int& J) {
    const unsigned wg = blockIdx.x;
    const int t = threadIdx.x;
    m = __syncthreads_count(t < b.count - 1 && b.prefix[t + 1] <= wg);     // matrices that end before this workgroup
    // consecutive workgroups walk along a tile row (neighbouring tiles are neighbours in memory, in the full matrix
    // and in the packed array): pairs (a >= b) with b fastest, read as (tile row, tile column) = (T-1-a, T-1-b)
    int a, bb;
    tri_decode((int)(wg - b.prefix[m]), a, bb);
    const int T = (b.dim[m] + PK_T - 1) / PK_T;
    I = T - 1 - a; J = T - 1 - bb;                                           // tile row <= tile column
}

// Thread = 4 consecutive columns of one tile row (16-byte accesses at 4-byte alignment: rows of an odd-sized matrix
// and rows of the packed array start anywhere); 8 tile rows per pass, 16 passes, the loads of 8 passes in flight.
__device__ __forceinline__ v4f pk_load4(const gfloat* p, int valid_from, int valid_to) {     // elements [from, to) of 4
    if (valid_from == 0 && valid_to == 4) return *(const KFAC_AS1 v4f_a4*)p;
    v4f v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (e >= valid_from && e < valid_to) v[e] = p[e];
    return v;
}

__device__ __forceinline__ void pk_store4(gfloat* p, const v4f& v, int valid_from, int valid_to) {
    if (valid_from == 0 && valid_to == 4) { *(KFAC_AS1 v4f_a4*)p = v; return; }
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (e >= valid_from && e < valid_to) p[e] = v[e];
}

// Row of the upper triangle that holds packed element p: the largest i with i n - i (i - 1) / 2 <= p.
__device__ __forceinline__ int pk_row_of(size_t p, int n) {
    const double t = 2.0 * n + 1.0;
    int i = (int)((t - sqrt(t * t - 8.0 * (double)p)) * 0.5);
    i = max(0, min(i, n - 1));
    while (i > 0 && pk_row_start(i, n) > p) --i;
    while (i + 1 < n && pk_row_start(i + 1, n) <= p) ++i;
    return i;
}

// packed <- upper triangle of full.  The packed array is walked linearly, four elements (one aligned 16-byte store)
// per thread; their sources are consecutive in a row of the matrix except where a row ends.
constexpr unsigned PK_CHUNK = 4096;       // packed elements per workgroup
__global__ __launch_bounds__(256) void pack_upper_kernel(PackBatch b) {
    const unsigned wg = blockIdx.x;
    const int t = threadIdx.x;
    const int m = __syncthreads_count(t < b.count - 1 && b.prefix[t + 1] <= wg);
    const int n = b.dim[m];
    const size_t total = (size_t)n * (n + 1) / 2;
    const gfloat* __restrict__ S = as_global(b.full[m]);
    gfloat* __restrict__ P = as_global(b.packed[m]);
    const bool aligned = ((uintptr_t)b.packed[m] & 15) == 0;
    const size_t base = (size_t)(wg - b.prefix[m]) * PK_CHUNK;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const size_t p = base + (size_t)(k * 256 + t) * 4;
        if (p >= total) continue;
        int i = pk_row_of(p, n);
        int j = i + (int)(p - pk_row_start(i, n));
        if (aligned && p + 3 < total && j + 3 < n) {
            *(KFAC_AS1 v4f*)(P + p) = *(const KFAC_AS1 v4f_a4*)(S + (size_t)i * n + j);
        } else {
            for (int e = 0; e < 4 && p + e < total; ++e) {
                P[p + e] = S[(size_t)i * n + j];
                if (++j == n) { ++i; j = i; }
            }
        }
    }
}

// running <- decay * running + (1 - decay) * unpack(packed), both triangles of running written, exactly symmetric
constexpr int PK_TPR = PK_T / 4;            // threads per tile row
constexpr int PK_RPP = 256 / PK_TPR;        // tile rows per pass
constexpr int PK_NP = PK_T / PK_RPP;        // passes
constexpr int PK_GROUP = 8;                 // passes whose loads are in flight together
__global__ __launch_bounds__(256) void ema_packed_kernel(PackBatch b, float decay, float one_minus) {
    __shared__ float tile[PK_T][PK_T + 1];
    int m, I, J;
    pk_locate(b, m, I, J);
    const int n = b.dim[m];
    gfloat* __restrict__ R = as_global(b.full[m]);
    const gfloat* __restrict__ P = as_global(b.packed[m]);
    const int c4 = (threadIdx.x % PK_TPR) * 4, r0 = threadIdx.x / PK_TPR;
    const int j = J * PK_T + c4;
#pragma unroll
    for (int g = 0; g < PK_NP; g += PK_GROUP) {
        v4f run[PK_GROUP], fresh[PK_GROUP];
        int from[PK_GROUP], to[PK_GROUP];
#pragma unroll
        for (int q = 0; q < PK_GROUP; ++q) {
            const int i = I * PK_T + r0 + PK_RPP * (g + q);
            from[q] = min(4, max(0, i - j));
            to[q] = i < n ? min(4, max(0, n - j)) : 0;
            if (from[q] >= to[q]) { from[q] = to[q] = 0; continue; }
            run[q] = pk_load4(R + (size_t)i * n + j, from[q], to[q]);
            fresh[q] = pk_load4(P + pk_row_start(i, n) + (j - i), from[q], to[q]);
        }
#pragma unroll
        for (int q = 0; q < PK_GROUP; ++q) {
            const int r = r0 + PK_RPP * (g + q), i = I * PK_T + r;
            v4f v = {0.f, 0.f, 0.f, 0.f};
            if (from[q] < to[q]) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = fmaf(decay, run[q][e], one_minus * fresh[q][e]);
                pk_store4(R + (size_t)i * n + j, v, from[q], to[q]);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) tile[r][c4 + e] = v[e];
        }
    }
    __syncthreads();
    // mirror image: row J*T + r', columns I*T + c' <- tile[c'][r'], strictly below the diagonal only
    const int i2 = I * PK_T + c4;
#pragma unroll
    for (int p = 0; p < PK_NP; ++p) {
        const int r = r0 + PK_RPP * p, j2 = J * PK_T + r;
        if (j2 >= n) continue;
        const int hi = min(4, min(n - i2, j2 - i2));             // columns i2 + e < min(n, j2)
        if (hi <= 0) continue;
        v4f v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = tile[c4 + e][r];
        pk_store4(R + (size_t)j2 * n + i2, v, 0, hi);
    }
}

static int fill_pack(PackBatch& b, const int* dims, float* const* full, float* const* packed, int cnt, bool tiles) {
    b.count = cnt;
    unsigned wgs = 0;
    for (int i = 0; i < cnt; ++i) {
        b.prefix[i] = wgs;
        b.dim[i] = dims[i];
        b.full[i] = full[i];
        b.packed[i] = packed[i];
        wgs += tiles ? (unsigned)pk_tiles(dims[i])
                     : (unsigned)(((size_t)dims[i] * (dims[i] + 1) / 2 + PK_CHUNK - 1) / PK_CHUNK);
    }
    b.prefix[cnt] = wgs;
    return (int)wgs;
}

}  // namespace kfac

using namespace kfac;

static bool tri_args_ok(const void* full, const void* packed, int dim) {
    if (!full || !packed || dim <= 0 || dim > 32768) return false;
    const size_t nf = (size_t)dim * dim * sizeof(float), np = (size_t)dim * (dim + 1) / 2 * sizeof(float);
    const char *f = (const char*)full, *p = (const char*)packed;
    return f + nf <= p || p + np <= f;                                       // no overlap
}

extern "C" int kfac_pack_upper_batched(const kfac_pack_item* items_host, int32_t count, void* stream) {
    if (!items_host || count < 0) return KFAC_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i)
        if (!tri_args_ok(items_host[i].full, items_host[i].packed, items_host[i].dim)) return KFAC_ERR_INVALID_ARG;
    for (int first = 0; first < count; first += PK_MAX) {
        const int cnt = count - first < PK_MAX ? count - first : PK_MAX;
        int dims[PK_MAX];
        float *full[PK_MAX], *packed[PK_MAX];
        for (int i = 0; i < cnt; ++i) {
            dims[i] = items_host[first + i].dim;
            full[i] = const_cast<float*>(items_host[first + i].full);
            packed[i] = items_host[first + i].packed;
        }
        PackBatch b;
        const int wgs = fill_pack(b, dims, full, packed, cnt, false);
        KFAC_LAUNCH(pack_upper_kernel, dim3(wgs), dim3(256), (hipStream_t)stream, b);
    }
    return KFAC_OK;
}

extern "C" int kfac_ema_packed_batched(const kfac_ema_packed_item* items_host, int32_t count, float decay, void* stream) {
    if (!items_host || count < 0) return KFAC_ERR_INVALID_ARG;
    if (!(decay >= 0.f && decay <= 1.f)) return KFAC_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i)
        if (!tri_args_ok(items_host[i].running, items_host[i].packed_fresh, items_host[i].dim)) return KFAC_ERR_INVALID_ARG;
    for (int first = 0; first < count; first += PK_MAX) {
        const int cnt = count - first < PK_MAX ? count - first : PK_MAX;
        int dims[PK_MAX];
        float *full[PK_MAX], *packed[PK_MAX];
        for (int i = 0; i < cnt; ++i) {
            dims[i] = items_host[first + i].dim;
            full[i] = items_host[first + i].running;
            packed[i] = const_cast<float*>(items_host[first + i].packed_fresh);
        }
        PackBatch b;
        const int wgs = fill_pack(b, dims, full, packed, cnt, true);
        KFAC_LAUNCH(ema_packed_kernel, dim3(wgs), dim3(256), (hipStream_t)stream, b, decay, 1.0f - decay);
    }
    return KFAC_OK;
}
