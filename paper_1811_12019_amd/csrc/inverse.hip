// Damped inverse of symmetric positive definite factors: Minv = (S + lambda I)^-1  (Sec. 4.2 damping, Eq. 6;
// Algorithm 1 stage 4), fp32.
//
// Method: blocked symmetric sweep (block Gauss-Jordan without pivoting, which is safe for SPD matrices).
// With the matrix cut into 128-wide blocks, eliminating block k does
//     P        = W_kk^-1                       (one workgroup, register resident)
//     T        = W_:k P                        (panel, MFMA)
//     W_ij    -= T_i W_jk^T   for i, j != k    (rank-128 update of the whole matrix, MFMA)
//     W_:k = T, W_k: = T^T, W_kk = -P
// and after all blocks W = -M^-1; the sign flip is folded into the last step.  Every step touches the whole
// matrix, so all steps expose the same, large amount of parallelism, and a batch of matrices of different sizes
// advances together: one launch per stage per step for the whole batch (the workgroup -> (matrix, tile) map is a
// prefix table passed in the kernel arguments).
//
// Launch structure.  Pivot -> panel -> update -> next pivot is a chain of dependent launches, 37 links long for a
// 4609-wide factor, so the launches are arranged to keep the chain short and the bulk of the flops off it:
//   * the update launch of step k gives the tile that is pivot block k + 1 to a workgroup of its own, which updates
//     it, keeps it in registers and inverts it at once: a step is two launches (panel, update), and the pivot runs
//     beside the tile updates (inv_pivot_kernel only serves a matrix's first block and single-block matrices);
//   * steps are taken in groups of GM; inside a group only the next panel's block column / row and the diagonal
//     tiles of the blocks still to come are brought up to date, every other tile receives a whole group as one
//     rank-(GM * 128) update during the next group's launches (see Plan below);
//   * every matrix of a batch carries its own step number, so that matrices with fewer blocks spread their steps
//     over the launches of the largest one.
// Products: the panel on the bf16 matrix cores with operands split three ways; the updates on the fp16 matrix cores
// from operands that the panel launch has already scaled per 128-row slab and split two ways, stored as planes that
// go to LDS by DMA (gemm_split.h); both to fp32 accuracy.
//
// Storage.  The sweep works on a copy W of the matrix in the caller's workspace whose rows are padded to a
// multiple of 32 floats, so that every 128-wide tile row is a run of whole 128-byte lines, and it keeps only the
// lower triangle (tiles on or below the diagonal) up to date: the part of block column k that lies above the
// pivot block is read, transposed, from block row k.  Only the last step writes the caller's dense output, both
// triangles, exactly symmetric (the upper one is a copy of the lower one).
#include "gemm_split.h"

namespace kfac {

constexpr int NB = 128;          // elimination block = tile edge
constexpr int MAXB = 64;         // matrices per launch of the kernels that read S (bounded by the 4 KB of kernel arguments)
constexpr int CMAXB = 112;       // matrices per launch of the sweep's per-step kernels, whose argument block is leaner
constexpr int UPD_WAVES = 3;     // wavefronts per SIMD the update kernel is compiled for (register budget)
constexpr int SLD = 132;         // epilogue staging stride (floats) for row-wise float4 access
constexpr int SLD_T = 129;       // epilogue staging stride when the stage is also read column-wise

// Everything a launch needs to know about its matrices travels in the kernel arguments (scalar loads, no dependent
// memory round trip at the start of every workgroup).
struct Batch {
    int count;                        // matrices in this launch
    int prefix[MAXB + 1];             // workgroup prefix sums over them
    int dim[MAXB];
    int step[MAXB];                   // the elimination step this launch takes for the matrix, or -1: none
    float damping[MAXB];
    const float* damping_dev[MAXB];   // NULL, or where the damping is to be read from instead
    const float* S[MAXB];
    float* Minv[MAXB];
    void* ws[MAXB];
    int32_t* info[MAXB];
};

static_assert(sizeof(Batch) <= 4096, "the batch travels in the kernel arguments");

// The same for the panel and update launches of the sweep, which no longer need the input matrix or the damping: more
// matrices per launch, i.e. fewer, fuller launches for a batch of many small matrices.
struct ChainBatch {
    int count;
    int prefix[CMAXB + 1];
    int dim[CMAXB];
    int step[CMAXB];                  // the elimination step this launch takes for the matrix, or -1: none
    float* Minv[CMAXB];
    void* ws[CMAXB];
    int32_t* info[CMAXB];
};
static_assert(sizeof(ChainBatch) <= 4096, "the batch travels in the kernel arguments");

// One matrix of the batch as the kernels see it: pointers typed as global memory.
struct Item {
    const gfloat* S;
    gfloat* Minv;
    gfloat* ws;
    gint* info;
    int dim;
    float damping;
};

__device__ __forceinline__ Item get_item(const Batch& b, int m) {
    Item it;
    it.S = as_global(b.S[m]);
    it.Minv = as_global(b.Minv[m]);
    it.ws = as_global((float*)b.ws[m]);
    it.info = as_global((int*)b.info[m]);
    it.dim = b.dim[m];
    it.damping = b.damping_dev[m] ? *as_global(b.damping_dev[m]) : b.damping[m];
    return it;
}

__device__ __forceinline__ Item get_item(const ChainBatch& b, int m) {
    Item it;
    it.S = nullptr;
    it.Minv = as_global(b.Minv[m]);
    it.ws = as_global((float*)b.ws[m]);
    it.info = as_global((int*)b.info[m]);
    it.dim = b.dim[m];
    it.damping = 0.f;
    return it;
}

// Which matrix workgroup `wg` of a launch belongs to (prefix[m] <= wg < prefix[m + 1]) and its index inside it.
// Every thread compares one prefix entry and the workgroup counts the matrices that end at or before wg: one vector
// load and one barrier instead of a binary search of dependent scalar loads (2 us at the start of every workgroup).
// Must be called by all threads of the workgroup.
template <class B>
__device__ __forceinline__ void locate(const B& b, int wg, int& m, int& local) {
    const int t = threadIdx.x;
    m = __syncthreads_count(t < b.count - 1 && b.prefix[t + 1] <= wg);
    local = wg - b.prefix[m];
}

static inline __host__ __device__ int nblk_of(int dim) { return (dim + NB - 1) / NB; }
static inline __host__ __device__ int ldw_of(int dim) { return (dim + 31) / 32 * 32; }

// Optional second form of the result, for the products that consume the inverse (preconditioning): the matrix cut
// into 128 x 128 blocks (zero padded), every element scaled by one power of two and split into two fp16 pieces, as two
// planes of n x n blocks in the layout of gemm_split.h (block (s, c) at (s n + c) PRE_SLAB bytes) followed by n x n
// floats that all hold the scale.  The scale: the damped matrix is S + lambda I with S positive semidefinite, so no
// entry of the inverse exceeds 1 / lambda in magnitude; 2^(8 + floor(log2 lambda)) maps that bound to at most 2^8, which
// leaves fp16's range seven more binades before overflow and keeps all 22 bits of entries down to 2^-11 of the bound
// (smaller ones lose bits only below 2^-33 of it).
static inline __host__ __device__ size_t inverse_plane_bytes(int dim) { return (size_t)nblk_of(dim) * nblk_of(dim) * PRE_SLAB; }
static inline __host__ __device__ size_t inverse_planes_bytes(int dim) {
    return 2 * inverse_plane_bytes(dim) + sizeof(float) * nblk_of(dim) * nblk_of(dim);
}
__device__ __forceinline__ float inverse_plane_scale(float damping) {
    return damping > 0.f ? ldexpf(1.0f, 8 + ilogbf(damping)) : 1.0f;
}
// Steps are taken in groups of up to GM consecutive blocks, none of them the matrix's last.  Inside a group only the
// tiles that the group's remaining pivots and panels need are kept up to date step by step (block rows / columns of
// the blocks still to come, all of them short lists: "narrow" launches); every other tile receives the group's
// rank-128 updates together, in one pass over the matrix, in the launch of the group's last step ("wide"), which
// cuts the traffic of the working copy by the group size.  The arithmetic per tile is the same sequence of fp32
// operations as step-by-step updating.
constexpr int GM = 4;
struct Group {
    int g0;      // first step of the group that `step` belongs to
    int m;       // its size (1 .. GM); 0: `step` is the matrix's last step, which is never part of a group
    int j;       // step - g0
};
static inline __host__ __device__ Group group_of(int dim, int step) {
    const int n = nblk_of(dim);
    Group g;
    g.g0 = step / GM * GM;
    g.j = step - g.g0;
    g.m = min(GM, n - 1 - g.g0);
    if (g.m < 0 || g.j >= g.m) g.m = 0;
    return g;
}
// Tiles of the update launch of `step` = k, per matrix: "chain" tiles, which the next step needs at once, and "lag"
// tiles.
//   * Chain launch (every step but the two kinds below).  Inside a group, and from one group to the next, a tile is
//     brought up to date only when the next step needs it:
//       - the tiles of block column / row k + 1 (all of them but the diagonal one, which the look-ahead pivot workgroup
//         takes): each sees, in one visit, every step it still owes, up to k -- at most the whole group before its own
//         and its own group's steps so far (chain_tile);
//       - the diagonal tiles of the blocks still to come in the group and of the first block after it, which are
//         kept up to date step by step so that a look-ahead pivot never owes more than one product; in a group's last
//         step these are the diagonal tiles of the next group's blocks and of the first block after those, which see
//         the whole group.
//     In a group's last step the off-diagonal tiles of the next group's other block columns / rows also see the whole
//     group ("early" tiles: not needed by the next step, but their chain visits then owe only their own group's steps).
//     Every other tile owes the group's steps: the rest of the matrix is dealt, as lag tiles, to the next group's
//     chain launches (all but its last), where it runs beside the pivot workgroups that set those launches' duration.
//   * Whole: the last step of a group that is not followed by a group of two or more steps; all tiles of the triangle
//     are brought up to date.
//   * Last: the matrix's last step, which writes the output.
// The panels of two consecutive groups coexist in the NBUF buffers, so lag tiles read the previous group's.
struct Plan {
    Group g;
    int kind;            // PLAN_CHAIN, PLAN_WHOLE, PLAN_LAST
    int d_begin, d_end;  // chain: diagonal tiles of blocks d_begin .. d_end - 1
    int chain;           // number of chain tiles
    int lag;             // number of lag tiles in this launch
    int lag_off;         // index of the first one in the lag list
    int early;           // number of early tiles (a group's last step; no lag tiles then): see plan_of
    int next_m;          // size of the next group (early tiles)
};
constexpr int PLAN_CHAIN = 0, PLAN_WHOLE = 2, PLAN_LAST = 3;

static inline __host__ __device__ Plan plan_of(int dim, int step) {
    const int n = nblk_of(dim);
    Plan p;
    p.g = group_of(dim, step);
    p.lag = p.lag_off = 0;
    p.early = p.next_m = 0;
    p.d_begin = p.d_end = 0;
    if (p.g.m == 0) { p.kind = PLAN_LAST; p.chain = n * (n + 1) / 2; return p; }
    const int E = p.g.g0 + p.g.m;
    if (p.g.j < p.g.m - 1) {
        p.kind = PLAN_CHAIN;
        p.d_begin = step + 2; p.d_end = E + 1;
        p.chain = n - 1 + p.d_end - p.d_begin;
        if (p.g.g0 > 0) {                                   // the previous group left its update of the bulk to this one
            const int nc = n - p.g.m;                       // (the tiles with no index inside this group)
            const int total = nc * (nc + 1) / 2, per = (total + p.g.m - 2) / (p.g.m - 1);
            p.lag_off = p.g.j * per;
            p.lag = max(0, min(per, total - p.lag_off));
        }
        return p;
    }
    const Group next = group_of(dim, E);
    if (next.m >= 2) {
        p.kind = PLAN_CHAIN;
        p.d_begin = E + 1; p.d_end = E + next.m + 1;
        p.chain = n - 1 + p.d_end - p.d_begin;
        // Early tiles: the off-diagonal tiles of the next group's other block columns / rows c = E + 1 .. E + next.m - 1
        // (row part J < E, column part I > c) receive this group's steps now, beside the chain tiles and off the chain,
        // so that their own chain visits inside the next group owe only that group's steps (1 .. 3 products instead of
        // 5 .. 7 on the chain's critical path).
        p.next_m = next.m;
        for (int c = E + 1; c < E + next.m; ++c) p.early += E + n - 1 - c;
    } else {
        p.kind = PLAN_WHOLE;
        p.chain = n * (n + 1) / 2;
    }
    return p;
}
static inline __host__ __device__ int update_tiles(int dim, int step) {
    const Plan p = plan_of(dim, step);
    return p.chain + p.lag + p.early;
}
// Tile index of a chain list -> (I, J): block row c = step + 1 left of the diagonal, block column c below it, then
// the diagonal tiles d_begin ..
__device__ __forceinline__ void chain_decode(int n, int c, int d_begin, int t, int& I, int& J) {
    if (t < c) { I = c; J = t; }
    else if (t < n - 1) { I = t + 1; J = c; }
    else { I = J = d_begin + (t - (n - 1)); }
}
// index in the early list of a launch (E: first block of the next group, nm its size) -> (I, J)
__device__ __forceinline__ void early_decode(int n, int E, int nm, int t, int& I, int& J) {
    for (int c = E + 1; c < E + nm; ++c) {
        const int cnt = E + n - 1 - c;
        if (t < cnt) {
            if (t < E) { I = c; J = t; }
            else { I = c + 1 + (t - E); J = c; }
            return;
        }
        t -= cnt;
    }
    I = J = 0;                                           // (not reached)
}
// index in the lag list of a group [E, E + m) -> (I, J): the lower triangle over the blocks outside the group
__device__ __forceinline__ void lag_decode(int n, int E, int m, int t, int& I, int& J) {
    tri_decode_blocked(n - m, t, I, J);
    if (I >= E) I += m;
    if (J >= E) J += m;
}

// Panels of one step, kept in buffer (step % NBUF): the fp32 copy U of block column k as it was before the step (all
// rows, assembled from both triangles), the fp32 product T = U P, and the scaled fp16 pieces of both (the negated T and
// U, each as a plane of high and a plane of low pieces in the layout of gemm_split.h), which the tile updates multiply.
constexpr int NBUF = 2 * GM;
struct WsView {
    gfloat* W;      // dim x ldw : working copy, lower triangle maintained
    int ldw;
    gfloat* buf0;   // NBUF panel buffers, `stride` floats each: U | T | -T high | -T low | U high | U low
    size_t stride;
    size_t plane;   // bytes of one piece plane (d_pad x NB fp16)
    gfloat* P;      // NB x NB    : inverse of the pivot block
    gfloat* SC;     // 2 NBUF x nblk: power-of-two scales of the 128-row slabs of T and U of every buffer (gemm_split.h)
    int nblk;
    __device__ __forceinline__ gfloat* U(int q) const { return buf0 + q * stride; }
    __device__ __forceinline__ gfloat* T(int q) const { return buf0 + q * stride + plane / 2; }
    __device__ __forceinline__ KFAC_AS1 unsigned char* TH(int q) const { return (KFAC_AS1 unsigned char*)(buf0 + q * stride + plane); }
    __device__ __forceinline__ KFAC_AS1 unsigned char* UH(int q) const { return TH(q) + 2 * plane; }
    __device__ __forceinline__ gfloat& scaleT(int q, int slab) const { return SC[(q * 2 + 0) * nblk + slab]; }
    __device__ __forceinline__ gfloat& scaleU(int q, int slab) const { return SC[(q * 2 + 1) * nblk + slab]; }
};

static inline __host__ __device__ size_t panel_buffer_floats(int dim) { return (size_t)nblk_of(dim) * NB * NB * 4; }

__device__ inline WsView ws_view(gfloat* ws, int dim) {
    const size_t d_pad = (size_t)nblk_of(dim) * NB;
    WsView v;
    v.ldw = ldw_of(dim);
    v.nblk = nblk_of(dim);
    v.W = ws;
    v.buf0 = v.W + d_pad * v.ldw;
    v.stride = panel_buffer_floats(dim);                 // 2 fp32 panels + 4 fp16 planes = 4 d_pad NB floats
    v.plane = d_pad * NB * 2;
    v.P = v.buf0 + NBUF * v.stride;
    v.SC = v.P + (size_t)NB * NB;
    return v;
}

// W(lower) = S(lower) + lambda I; info = 0.
__global__ __launch_bounds__(256) void inv_init_kernel(Batch b) {
    int m, tile;
    locate(b, blockIdx.x, m, tile);
    const Item it = get_item(b, m);
    const int d = it.dim;
    int I, J;
    tri_decode(tile, I, J);
    if (tile == 0 && threadIdx.x == 0 && it.info) *it.info = 0;
    const WsView ws = ws_view(it.ws, d);
    const gfloat* __restrict__ S = it.S;
    const float lam = it.damping;
    const int c = threadIdx.x & 127, rh = threadIdx.x >> 7;
    const int col = J * NB + c;
#pragma unroll 1
    for (int r8 = 0; r8 < NB; r8 += 16) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {                    // loads only: arithmetic on a guarded load would make the
            const int row = I * NB + r8 + 2 * i + rh;    // compiler wait for each load in turn
            v[i] = (row < d && col <= row) ? S[(size_t)row * d + col] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = I * NB + r8 + 2 * i + rh;
            if (row < d && col < ws.ldw) ws.W[(size_t)row * ws.ldw + col] = v[i] + (row == col ? lam : 0.f);
        }
    }
}

// ---- pivot block -----------------------------------------------------------------------------------------------
// Inverse of the (at most 128 x 128) pivot block by a symmetric sweep in 16-wide sub-blocks.  The block D lives in
// registers in MFMA accumulator layout (4 wavefronts x 64 x 64 quadrants); per sub-block j:
//   1. the owners of D's columns j copy them to LDS (U16, 128 x 16);
//   2. wavefront 0 inverts the 16 x 16 diagonal sub-block with a register sweep (quad broadcasts + bpermute);
//   3. every thread computes its part of T16 = U16 . P16; the rows of the sub-block itself are set to -P16;
//   4. D -= T16 . U16^T on the matrix cores (K = 16), then rows / columns j of D are overwritten with T16.
// Padding with the identity makes ragged blocks (fewer than 128 rows) need no special cases.
constexpr int PSB = 16;          // sub-block
constexpr int PLD = 20;          // LDS row stride of the 16-wide panels (float4 aligned)

__device__ __forceinline__ float quad_bcast(float x, int k) {   // value of lane (4*(lane/4) + k)
    const int v = __float_as_int(x);
    int r;
    switch (k) {
        case 0: r = __builtin_amdgcn_update_dpp(v, v, 0x00, 0xf, 0xf, false); break;
        case 1: r = __builtin_amdgcn_update_dpp(v, v, 0x55, 0xf, 0xf, false); break;
        case 2: r = __builtin_amdgcn_update_dpp(v, v, 0xAA, 0xf, 0xf, false); break;
        default: r = __builtin_amdgcn_update_dpp(v, v, 0xFF, 0xf, 0xf, false); break;
    }
    return __int_as_float(r);
}

// One wavefront: Ps = inverse of the symmetric positive definite 16 x 16 block D16 (rows of Us), lower triangle
// taken as the truth.  Lane (i = lane/4, g = lane%4) holds E[i][4g..4g+3].  Returns the 1-based index of the first
// non-positive pivot, or 0.
__device__ __forceinline__ int invert16_wave(const float* __restrict__ D16, int ld, float* __restrict__ Ps) {
    const int lane = threadIdx.x & 63, i = lane >> 2, g = lane & 3;
    float E[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int c = 4 * g + q;
        E[q] = D16[max(i, c) * ld + min(i, c)];
    }
    int bad = 0;
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        const float vi = quad_bcast(E[s & 3], s >> 2);                                    // E(i, s)
        const float p = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(vi), 4 * s));   // E(s, s)
        if (!(p > 0.f) && bad == 0) bad = s + 1;
        float ip = __builtin_amdgcn_rcpf(p);              // 1 ulp estimate + one Newton step: ample for a pivot
        ip = ip * fmaf(-p, ip, 2.0f);
        float vc[4];                                                                      // E(4g+q, s) = E(s, 4g+q)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            vc[q] = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (4 * (4 * g + q)), __float_as_int(vi)));
        const float wi = vi * ip;
        // (selects, not branches: the pivot row's lanes would otherwise run a path of their own after everybody else's)
        const bool prow = i == s, pcol = g == (s >> 2);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float upd = fmaf(-wi, vc[q], E[q]), piv = vc[q] * ip;
            E[q] = prow ? piv : upd;
        }
        E[s & 3] = pcol ? (prow ? -ip : wi) : E[s & 3];
    }
    // E = -P16 up to rounding asymmetry: publish, then re-read the lower triangle so that P16 is exactly symmetric
#pragma unroll
    for (int q = 0; q < 4; ++q) Ps[i * PLD + 4 * g + q] = -E[q];
    float sym[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int c = 4 * g + q;
        sym[q] = Ps[max(i, c) * PLD + min(i, c)];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) Ps[i * PLD + 4 * g + q] = sym[q];
    return bad;
}

// LDS of the pivot code: the block's packed lower triangle (row r holds columns 0..r) while it is brought into or
// out of the registers, and the sweep's panels in between, in the same memory.
constexpr int TRI_FLOATS = NB * (NB + 1) / 2;                        // 33,024 bytes
constexpr int PIV_US = 0, PIV_TS = NB * PLD, PIV_PS = 2 * NB * PLD, PIV_BAD = PIV_PS + PSB * PLD;
constexpr int PIV_LDS_FLOATS = TRI_FLOATS;
static_assert(PIV_BAD + 1 <= PIV_LDS_FLOATS, "the sweep's panels must fit the triangle's memory");

__device__ __forceinline__ int tri_at(int r, int c) { return ((r * (r + 1)) >> 1) + c; }          // r >= c
__device__ __forceinline__ int tri_sym(int r, int c) { return r >= c ? tri_at(r, c) : tri_at(c, r); }

// D (accumulator layout, all four quadrants) <- the symmetric block whose lower triangle is in tri, bordered by the
// identity beyond nb.  HAVE_LOWER: the registers already hold the lower triangle, only the rest is fetched.
// Ends with a barrier: tri may be overwritten afterwards.
template <bool HAVE_LOWER = false>
__device__ __forceinline__ void pivot_fill(v16f (&acc)[2][2], const float* __restrict__ tri, int nb) {
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = acc_row(wm, mb, r, lane), col = acc_col(wn, nbk, lane);
                if (!(row < nb && col < nb)) acc[mb][nbk][r] = row == col ? 1.f : 0.f;
                else if (!HAVE_LOWER || row < col) acc[mb][nbk][r] = tri[tri_sym(row, col)];
            }
    __syncthreads();
}

// D (accumulator layout) holds a symmetric block's lower triangle; the rest is filled in from it, bordered by the
// identity beyond nb.  Three 64 x 64 transposes through LDS (3 x 4096 floats): the quadrant below the diagonal goes,
// transposed, to the wavefront that owns the quadrant above it, and each diagonal quadrant to itself.  Element (a, b)
// of a quadrant is kept at b * 64 + (a ^ b): writes (lanes along b) and reads (lanes along a) both touch 32 different
// banks.  Ends with a barrier: lds may be overwritten afterwards.
__device__ __forceinline__ void pivot_symmetrize(v16f (&acc)[2][2], float* __restrict__ lds, int nb) {
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const int lm = lane & 31, h = lane >> 5;
    // writers: wavefronts (0,0), (1,0), (1,1) -> squares 0, 1, 2
    if (!(wm == 0 && wn == 1)) {
        float* sq = lds + (wm + wn) * 4096;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int a = mb * 32 + (r >> 2) * 8 + h * 4 + (r & 3), b = nbk * 32 + lm;
                    sq[b * 64 + (a ^ b)] = acc[mb][nbk][r];
                }
    }
    __syncthreads();
    // readers: target (a, b) of a quadrant takes source (b, a) of square (0,0) -> 0, (0,1) -> 1, (1,1) -> 2
    if (!(wm == 1 && wn == 0)) {
        const float* sq = lds + (wm + wn) * 4096;
        const bool whole = wm != wn;                     // the quadrant above the diagonal: every element
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int a = mb * 32 + (r >> 2) * 8 + h * 4 + (r & 3), b = nbk * 32 + lm;
                    const float v = sq[a * 64 + (b ^ a)];
                    acc[mb][nbk][r] = (whole || a < b) ? v : acc[mb][nbk][r];
                }
    }
    if (nb < NB) {                                       // (uniform) ragged block: identity beyond nb
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = acc_row(wm, mb, r, lane), col = acc_col(wn, nbk, lane);
                    if (!(row < nb && col < nb)) acc[mb][nbk][r] = row == col ? 1.f : 0.f;
                }
    }
    __syncthreads();
}

// The symmetric sweep of D in 16-wide sub-blocks (see above); lds: PIV_LDS_FLOATS floats.  Returns (to every thread)
// the 1-based index inside the block of the first non-positive pivot, or 0.  Ends with a barrier.
__device__ __forceinline__ int pivot_sweep(v16f (&acc)[2][2], int nb, float* __restrict__ lds) {
    float* __restrict__ Us = lds + PIV_US;
    float* __restrict__ Ts = lds + PIV_TS;
    float* __restrict__ Ps = lds + PIV_PS;
    int* bad = (int*)(lds + PIV_BAD);
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const int lm = lane & 31, h = lane >> 5;
    if (t == 0) *bad = 0;
#pragma unroll
    for (int jb = 0; jb < NB / PSB; ++jb) {
        const int j0 = jb * PSB;
        if (j0 >= nb) break;                         // uniform
        const int own_w = jb >> 2;                   // wn (for columns) / wm (for rows) that owns sub-block jb
        const int own_b = (jb >> 1) & 1;             // nbk / mb inside the quadrant
        const int own_h = jb & 1;                    // which 16 of the block's 32
        __syncthreads();                             // previous sub-step's readers of Us / Ts are done
        // 1. U16 = D[:, j0 : j0+16]
        if (wn == own_w && (lm >> 4) == own_h) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    Us[acc_row(wm, mb, r, lane) * PLD + (lm & 15)] = acc[mb][own_b][r];
        }
        __syncthreads();
        // 2. P16
        if (wave == 0) {
            const int f = invert16_wave(Us + j0 * PLD, PLD, Ps);
            if (f != 0 && lane == 0 && *bad == 0) *bad = j0 + f;
        }
        __syncthreads();
        // 3. T16 = U16 . P16 on the matrix cores (v_mfma_f32_16x16x4_f32: lane l supplies A[l % 16][l / 16] and
        //    B[l / 16][l % 16] and receives C[4 (l / 16) + i][l % 16], i < 4); a wavefront takes 32 of the 128 rows.
        //    The rows of the sub-block itself are replaced by -P16.
        {
            const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
            for (int rbi = 0; rbi < 2; ++rbi) {
                const int rb0 = (2 * wave + rbi) * PSB;          // first row of this 16-row block
                v4f c4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    c4 = __builtin_amdgcn_mfma_f32_16x16x4f32(Us[(rb0 + l16) * PLD + 4 * kk + lq], Ps[(4 * kk + lq) * PLD + l16],
                                                               c4, 0, 0, 0);
                const bool own = rb0 == j0;                      // (uniform)
#pragma unroll
                for (int i2 = 0; i2 < 4; ++i2) {
                    const int rl = 4 * lq + i2;
                    Ts[(rb0 + rl) * PLD + l16] = own ? -Ps[rl * PLD + l16] : c4[i2];
                }
            }
        }
        __syncthreads();
        // 4. D -= T16 . U16^T  (lane (lm, h) takes k = 8s + 4h .. +3 of both operands), then the fix-ups
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            v4f a[2], bb[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) a[mb] = *(const v4f*)&Ts[(wm * 64 + mb * 32 + lm) * PLD + 8 * s2 + 4 * h];
#pragma unroll
            for (int nbk = 0; nbk < 2; ++nbk) bb[nbk] = *(const v4f*)&Us[(wn * 64 + nbk * 32 + lm) * PLD + 8 * s2 + 4 * h];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int nbk = 0; nbk < 2; ++nbk)
                        acc[mb][nbk] = __builtin_amdgcn_mfma_f32_32x32x2f32(-a[mb][i], bb[nbk][i], acc[mb][nbk], 0, 0, 0);
        }
        // columns j of D <- T16 (and -P16 on the sub-block's own rows)
        if (wn == own_w && (lm >> 4) == own_h) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[mb][own_b][r] = Ts[acc_row(wm, mb, r, lane) * PLD + (lm & 15)];
        }
        // rows j of D <- T16^T
        if (wm == own_w) {
#pragma unroll
            for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                for (int r8 = 0; r8 < 8; ++r8) {
                    const int r = own_h * 8 + r8;                    // registers holding rows 16*own_h .. +15 of block own_b
                    const int rloc = (r8 >> 2) * 8 + h * 4 + (r8 & 3);   // row inside the sub-block
                    acc[own_b][nbk][r] = Ts[acc_col(wn, nbk, lane) * PLD + rloc];
                }
        }
    }
    __syncthreads();
    const int f = *bad;
    __syncthreads();                                 // everybody has read the flag: the memory may be reused
    return f;
}

// D holds -P up to rounding asymmetry; its lower triangle is taken as the truth so that P is exactly symmetric.
// The working copy gets -P; on the matrix's last step the caller's output gets +P (the final sign flip) instead.
// The workspace gets +P for the panel product.
__device__ __forceinline__ void pivot_write(const v16f (&acc)[2][2], float* __restrict__ tri, const Item& it,
                                            const WsView& ws, int k0, int nb, bool last, bool from_S) {
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const int d = it.dim;
    if (!last && !from_S && nb == NB) {
        // A full block inside the sweep (the look-ahead pivot's usual case): the registers hold the whole symmetric block,
        // and a half-wave's 32 lanes hold 32 consecutive floats of a row, so it goes out as it is.
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = acc_row(wm, mb, r, lane), col = acc_col(wn, nbk, lane);
                    const float x = acc[mb][nbk][r];
                    ws.W[(size_t)(k0 + row) * ws.ldw + k0 + col] = x;
                    ws.P[row * NB + col] = -x;
                }
        return;
    }
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = acc_row(wm, mb, r, lane), col = acc_col(wn, nbk, lane);
                if (row >= col) tri[tri_at(row, col)] = acc[mb][nbk][r];
            }
    __syncthreads();
    // thread = four consecutive columns of one row, 8 rows per pass: 16-byte stores (the working copy and the P
    // buffer are 16-byte aligned; the caller's output need not be)
    const int c4 = (t & 31) * 4, r0 = t >> 5;
#pragma unroll 4
    for (int p = 0; p < 16; ++p) {
        const int row = r0 + 8 * p;
        if (row >= nb || c4 >= nb) continue;
        v4f x;
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = tri[tri_sym(row, min(c4 + i, nb - 1))];
        if (last) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (c4 + i < nb) it.Minv[(size_t)(k0 + row) * d + k0 + c4 + i] = -x[i];
        } else {
            *(KFAC_AS1 v4f*)&ws.W[(size_t)(k0 + row) * ws.ldw + k0 + c4] = x;      // a block that is not last is full
        }
        if (!from_S) *(KFAC_AS1 v4f*)&ws.P[row * NB + c4] = -x;    // (columns beyond a ragged block are never read)
    }
}

// Pivot block `step` of every matrix of the batch, read from the working copy.
// from_S: single-block matrices: read S + lambda I and write the caller's output directly.
__global__ __launch_bounds__(256) void inv_pivot_kernel(Batch b, int step, int from_S) {
    __shared__ __attribute__((aligned(16))) float lds[PIV_LDS_FLOATS];
    __builtin_amdgcn_s_setprio(3);
    const int m = blockIdx.x;
    const Item it = get_item(b, m);
    const int d = it.dim;
    const int k0 = step * NB;
    const int nb = min(NB, d - k0);
    const bool last = k0 + NB >= d;
    const int t = threadIdx.x;
    const WsView ws = ws_view(it.ws, d);

    // ---- load: lower triangle, row-wise.  All loads are issued before the first LDS store so that the block costs
    //      one memory round trip, not one per row group ----
    {
        const int c4 = (t & 31) * 4, r0 = t >> 5;        // 8 rows x 32 float4 per pass, 16 passes
        const bool vec_ok = !from_S;                     // the padded working copy is 16-byte aligned, S need not be
        v4f v[16];
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = r0 + 8 * p;
            v4f x = {0.f, 0.f, 0.f, 0.f};
            if (row < nb && c4 <= row) {
                if (vec_ok) {
                    x = *(const KFAC_AS1 v4f*)&ws.W[(size_t)(k0 + row) * ws.ldw + k0 + c4];
                } else {
                    const gfloat* src = it.S + (size_t)(k0 + row) * d + k0 + c4;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (c4 + i <= row) x[i] = src[i];            // (the damping is added at the LDS store below)
                }
            }
            v[p] = x;
        }
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = r0 + 8 * p;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (row < nb && c4 + i <= row) lds[tri_at(row, c4 + i)] = v[p][i] + ((from_S && c4 + i == row) ? it.damping : 0.f);
        }
    }
    __syncthreads();
    v16f acc[2][2];
    pivot_fill(acc, lds, nb);
    const int f = pivot_sweep(acc, nb, lds);
    if (t == 0 && it.info) {
        if (from_S) *it.info = f;                                       // single-block matrix: this is its only kernel
        else if (f != 0) atomicCAS((int*)it.info, 0, k0 + f);           // keep the first failing minor
    }
    pivot_write(acc, lds, it, ws, k0, nb, last, from_S != 0);
}

// T = U . P for every 128-row slab of block column k; U is copied aside for the update.  Slabs below the pivot
// block read the column block itself; slabs above it read block row k transposed.
// Full pivot block (every step but a matrix's last): the slab is first copied to U (through an LDS transpose for the
// slabs above the pivot), all 64 KB in flight at once, and the product then runs on the bf16 matrix cores with both
// operands split three ways, reading the copy.  Ragged pivot block: fp32 matrix cores, operands guarded.
// The transpose and the way out of T pass through LDS 64 rows at a time, so that the workgroup needs no more LDS than
// the product (48 KB): a panel workgroup then fits into the room one finished update (or factor) workgroup leaves on
// a CU.  With a full 128-row stage (66 KB) it had to wait until two of them had finished on the same CU, and the
// panel launches, links of the chain, lasted 47 us instead of 21 us while other streams kept the CUs full.
constexpr int PANEL_TLD = NB + 1;          // LDS row stride of the transpose stage
constexpr int PANEL_RLD = NB + 4;          // LDS row stride when the stage is read back four columns at a time
constexpr int PANEL_LDS_FLOATS = split_lds_bytes<3>() / 4;
static_assert(PANEL_LDS_FLOATS >= GEMM_LDS_FLOATS && PANEL_LDS_FLOATS >= (NB / 2) * PANEL_RLD, "one buffer serves all uses");

__global__ __launch_bounds__(256) void inv_panel_kernel(ChainBatch b) {
    __shared__ __attribute__((aligned(16))) float lds[PANEL_LDS_FLOATS];
    __shared__ float red[4];
    __builtin_amdgcn_s_setprio(3);                       // a link of the chain: ahead of whatever shares its SIMDs
    int m, slab;
    locate(b, blockIdx.x, m, slab);
    const Item it = get_item(b, m);
    const int d = it.dim;
    const int step = b.step[m];
    const int k0 = step * NB;
    const int nb = min(NB, d - k0);
    if (slab == step) return;                 // the pivot block's own rows are not needed
    const int r0 = slab * NB;
    const int rows = min(NB, d - r0);
    const WsView ws = ws_view(it.ws, d);
    const int q = step % NBUF;
    gfloat* __restrict__ Uc = ws.U(q) + (size_t)r0 * NB;
    gfloat* __restrict__ Tc = ws.T(q) + (size_t)r0 * NB;
    const int t = threadIdx.x;
    TileAcc acc;
    if (nb == NB) {
        const int c4 = (t & 31) * 4, rr = t >> 5;            // 8 rows x 32 float4 per pass, 16 passes
        v4f v[16];
        if (slab > step) {
#pragma unroll
            for (int p = 0; p < 16; ++p) {
                const int row = rr + 8 * p;
                v4f x = {0.f, 0.f, 0.f, 0.f};
                if (row < rows) x = *(const KFAC_AS1 v4f*)&ws.W[(size_t)(r0 + row) * ws.ldw + k0 + c4];
                v[p] = x;
            }
#pragma unroll
            for (int p = 0; p < 16; ++p) *(KFAC_AS1 v4f*)&Uc[(size_t)(rr + 8 * p) * NB + c4] = v[p];   // rows past the end: zero
        } else {
            // element (a, k) of the slab is W[k0 + k][r0 + a]; a slab above the pivot has all its 128 rows
#pragma unroll
            for (int p = 0; p < 16; ++p)
                v[p] = *(const KFAC_AS1 v4f*)&ws.W[(size_t)(k0 + rr + 8 * p) * ws.ldw + r0 + c4];
        }
        float um = 0.f;                        // the slab's scale for the update's fp16 pieces
#pragma unroll
        for (int p = 0; p < 16; ++p)
#pragma unroll
            for (int i = 0; i < 4; ++i) um = fmaxf(um, fabsf(v[p][i]));
        um = block_absmax(um, red);
        const float su = panel_scale(um);
        if (t == 0) ws.scaleU(q, slab) = su;
        // the copy (slabs above the pivot) and the slab's scaled fp16 pieces
        KFAC_AS1 unsigned char* uh = ws.UH(q) + (size_t)slab * PRE_SLAB;
        if (slab > step) {
#pragma unroll
            for (int p = 0; p < 16; ++p) store_split4_h2(uh, uh + ws.plane, rr + 8 * p, c4, v[p] * su);
        } else {
            // transposed through LDS, 64 rows of the slab at a time: the threads holding columns c4 .. c4 + 3 of that
            // half write them, then every thread reads four consecutive elements of eight rows
#pragma unroll 1
            for (int half = 0; half < 2; ++half) {
                if (half == 1) __syncthreads();
                if ((c4 >> 6) == half) {
#pragma unroll
                    for (int p = 0; p < 16; ++p)
#pragma unroll
                        for (int i = 0; i < 4; ++i) lds[(c4 + i - 64 * half) * PANEL_TLD + rr + 8 * p] = v[p][i];
                }
                __syncthreads();
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    const int a = 64 * half + rr + 8 * p;
                    const float* src = &lds[(rr + 8 * p) * PANEL_TLD + c4];
                    const v4f x = {src[0], src[1], src[2], src[3]};
                    *(KFAC_AS1 v4f*)&Uc[(size_t)a * NB + c4] = x;
                    store_split4_h2(uh, uh + ws.plane, a, c4, x * su);
                }
            }
        }
        __threadfence_block();
        __syncthreads();                       // the copy is visible to the whole workgroup; the LDS stage is free
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc.c[mb][nbk][r] = 0.f;
        tile_mma_nt_split<3, false, NB / SPLIT_KS>(Uc, NB, NB, ws.P, NB, NB, NB, (unsigned char*)lds, acc);
    } else if (slab > step) {
        tile_mma_nt<false>(ws.W + (size_t)r0 * ws.ldw + k0, ws.ldw, rows, ws.P, NB, nb, nb, lds, acc, Uc, NB);
    } else {
        tile_mma_nt<true>(ws.W + (size_t)k0 * ws.ldw + r0, ws.ldw, rows, ws.P, NB, nb, nb, lds, acc, Uc, NB);
    }
    const int lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    if (nb == NB) {
        // T leaves through LDS, row-wise: the fp32 panel in 16-byte stores and its scaled, negated fp16 pieces
        float tm = 0.f;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                for (int r = 0; r < 16; ++r) tm = fmaxf(tm, fabsf(acc.c[mb][nbk][r]));
        tm = block_absmax(tm, red);                       // (its barriers also separate the product's LDS use from this one)
        const float st = panel_scale(tm);
        if (t == 0) ws.scaleT(q, slab) = st;
        const int c4 = (t & 31) * 4, rr = t >> 5;
        KFAC_AS1 unsigned char* th = ws.TH(q) + (size_t)slab * PRE_SLAB;
#pragma unroll 1
        for (int half = 0; half < 2; ++half) {
            if (half == 1) __syncthreads();
            if (wm == half) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            lds[(acc_row(wm, mb, r, lane) - 64 * half) * PANEL_RLD + acc_col(wn, nbk, lane)] = acc.c[mb][nbk][r];
            }
            __syncthreads();
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int row = 64 * half + rr + 8 * p;
                const v4f x = *(const v4f*)&lds[(rr + 8 * p) * PANEL_RLD + c4];
                if (row < rows) *(KFAC_AS1 v4f*)&Tc[(size_t)row * NB + c4] = x;
                store_split4_h2(th, th + ws.plane, row, c4, x * -st);
            }
        }
        return;
    }
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = acc_row(wm, mb, r, lane), col = acc_col(wn, nbk, lane);
                if (row < rows) Tc[(size_t)row * NB + col] = col < nb ? acc.c[mb][nbk][r] : 0.f;
            }
    // the update streams whole 16-float slabs of T and U: keep the columns beyond a ragged block at zero
    if (nb < NB) {
        for (int e = t; e < rows * NB; e += 256) {
            const int row = e >> 7, col = e & (NB - 1);
            if (col >= nb) Uc[(size_t)row * NB + col] = 0.f;
        }
    }
}

// One tile (I >= J) of one elimination step.  Tile kinds:
//   regular      new = old - T_I U_J^T
//   column       J == k, I > k:  new[a][c] = T[I*128 + a][c]          (block column k below the pivot)
//   row          I == k, J < k:  new[a][c] = T[J*128 + c][a]          (block row k left of the pivot)
// LAST = false: the tile goes back into the padded working copy (whole 512-byte rows).
// LAST = true (the matrix's final step): the tile, negated, goes to the caller's output, and so does its mirror image.
// Column / row tiles and all tiles of a final step pass through an LDS stage, 64 tile rows at a time, so that global
// accesses are row-wise; regular tiles of the other steps go from and to registers (upd_regular_mid_split).
struct UpdCtx {
    gfloat* W; int ldw; const gfloat* T; gfloat* out;
    int d, i0, j0, irows, jrows, nb;
    bool diag;
};

// stage (64 x sld floats) holds rows h0..h0+63 of the tile's new values (or of the product, for regular tiles
// when COMBINE: new = old - stage, old prefetched in oldv).
template <bool LAST, bool COMBINE>
__device__ __forceinline__ void upd_flush(const UpdCtx& c, float* __restrict__ stage, int h0, const v4f (&oldv)[8]) {
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int pr = t >> 5, pc = (t & 31) * 4;
    constexpr int sld = LAST ? SLD_T : SLD;
    if constexpr (!LAST) {
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int rl = pr + 8 * p, row = h0 + rl;
            if (row < c.irows && c.j0 + pc < c.ldw) {
                v4f s = *(const v4f*)&stage[rl * sld + pc];
                if constexpr (COMBINE) s = oldv[p] - s;
                *(KFAC_AS1 v4f*)&c.W[(size_t)(c.i0 + row) * c.ldw + c.j0 + pc] = s;
            }
        }
    } else {
        // final values (sign flipped) back into the stage, then out: rows of the tile and rows of its mirror
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int rl = pr + 8 * p;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float x = stage[rl * sld + pc + i];
                stage[rl * sld + pc + i] = COMBINE ? x - oldv[p][i] : -x;
            }
        }
        __syncthreads();
        // direct: wavefront w writes tile rows h0 + 16w .. +15, two 64-float runs per row
        for (int rr = 0; rr < 16; ++rr) {
            const int rl = wave * 16 + rr, row = h0 + rl;
            if (row >= c.irows) break;
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                const int col = cc * 64 + lane;
                if (col < c.jrows && !(c.diag && col > row))
                    c.out[(size_t)(c.i0 + row) * c.d + c.j0 + col] = stage[rl * sld + col];
            }
        }
        // mirror: wavefront w writes output rows j0 + 32w .. +31, one 64-float run (tile rows h0..h0+63) each
        for (int cc = 0; cc < 32; ++cc) {
            const int col = wave * 32 + cc, row = h0 + lane;
            if (col >= c.jrows) break;
            if (row < c.irows && !(c.diag && col >= row))
                c.out[(size_t)(c.j0 + col) * c.d + c.i0 + row] = stage[lane * sld + col];
        }
    }
}

// Regular tile: acc = T_I . U_J^T with both operand panels (128 rows x nb floats, row stride 128, zero beyond nb)
// streamed through a 3-stage LDS ring by global_load_lds_dwordx4 (lane i's 16 bytes land at block base + 16 i), so
// no registers are spent on staging and one barrier per 16-wide K-slab suffices.  Inside a 1 KB block (16 rows x 4
// chunks of 4 floats) chunk c of row r sits in slot 4 r + (c ^ ((r >> 1) & 3)): the MFMA operand reads (one float4
// per lane, 32 consecutive rows per half-wave) are then bank-conflict free.
constexpr int UK = 16;                    // K-slab
constexpr int UNS = 3;                    // ring stages
constexpr int UPANEL = 8 * 1024;          // bytes per operand panel per stage
constexpr int USTAGE = 2 * UPANEL;
static_assert(UNS * USTAGE <= GEMM_LDS_FLOATS * 4 + 12288, "ring must fit the kernel's LDS");
static_assert(UNS * USTAGE >= PRE_NS * PRE_STAGE, "the tile products' ring shares the kernel's LDS");

#define KFAC_LDS_READ128(dst, addr, off) \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off))

template <bool LAST>
__device__ __forceinline__ void upd_regular(const UpdCtx& c, const gfloat* __restrict__ U, float* __restrict__ lds) {
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const int lm = lane & 31, h = lane >> 5;
    const int pr = t >> 5, pc = (t & 31) * 4;
    constexpr int sld = LAST ? SLD_T : SLD;
    const bool dead = c.diag && wm == 0 && wn == 1;      // strictly above the diagonal, never used
    lds_byte* l0 = (lds_byte*)lds;

    // LAST: old values are fetched row-wise (the epilogue transposes through LDS for the mirror image).
    v4f oldv[8];
    if constexpr (LAST) {
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int row = pr + 8 * p;
            v4f o = {0.f, 0.f, 0.f, 0.f};
            if (row < c.irows && c.j0 + pc < c.ldw) o = *(const KFAC_AS1 v4f*)&c.W[(size_t)(c.i0 + row) * c.ldw + c.j0 + pc];
            oldv[p] = o;
        }
    }

    // ---- producer: wavefronts 0,1 stream T_I, wavefronts 2,3 stream U_J; four 1 KB blocks each per stage ----
    const int pan = wave >> 1;
    const int drow = lane >> 2, dchunk = (lane & 3) ^ ((lane >> 3) & 3);
    const gfloat* src0 = (pan == 0 ? c.T + (size_t)c.i0 * NB : U + (size_t)c.j0 * NB) + (size_t)drow * NB + 4 * dchunk;
    const int nst = (c.nb + UK - 1) / UK;
    auto issue = [&](int s, int buf) {
        const int sc = s < nst ? s : nst - 1;              // past the end: re-read the last slab (never consumed)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int b = (wave & 1) + 2 * j;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src0 + (size_t)(16 * b) * NB + sc * UK),
                                             (__attribute__((address_space(3))) void*)(l0 + buf * USTAGE + pan * UPANEL + b * 1024),
                                             16, 0, 0);
        }
    };

    // ---- consumer: per-lane LDS byte addresses of the float4 holding k = 8 s2 + 4 h .. +3 of its row ----
    unsigned a_addr[2][2], b_addr[2][2];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const int ma = wm * 64 + q * 32 + lm, mb_ = wn * 64 + q * 32 + lm;
            const int ch = 2 * s2 + h;
            a_addr[q][s2] = (unsigned)((ma >> 4) * 1024 + (4 * (ma & 15) + (ch ^ (((ma & 15) >> 1) & 3))) * 16);
            b_addr[q][s2] = (unsigned)(UPANEL + (mb_ >> 4) * 1024 + (4 * (mb_ & 15) + (ch ^ (((mb_ & 15) >> 1) & 3))) * 16);
        }

    TileAcc acc;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc.c[mb][nbk][r] = 0.f;
    issue(0, 0);
    issue(1, 1);
    for (int it = 0; it < nst; it += UNS) {
#pragma unroll
        for (int bi = 0; bi < UNS; ++bi) {
            const int s = it + bi;
            if (s >= nst) break;                                            // uniform
            asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");   // slab s landed (everybody's part)
            issue(s + 2, (bi + 2) % UNS);                                    // refill the slot slab s-1 vacated
            if (!dead) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    v4f a[2], bb[2];
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        KFAC_LDS_READ128(a[q], a_addr[q][s2], bi * USTAGE);
                        KFAC_LDS_READ128(bb[q], b_addr[q][s2], bi * USTAGE);
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]), "+v"(bb[0]), "+v"(bb[1]));
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                            for (int nbk = 0; nbk < 2; ++nbk)
                                acc.c[mb][nbk] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mb][i], bb[nbk][i], acc.c[mb][nbk], 0, 0, 0);
                }
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");            // ring idle: LDS becomes the epilogue stage
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        const int h0 = half * 64;
        if (h0 >= c.irows) break;                          // uniform
        if (half == 1) {
            __syncthreads();                               // everyone is done with the first half's stage
            // old values of the second half, all fetched before anything more is stored
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int row = h0 + pr + 8 * p;
                v4f o = {0.f, 0.f, 0.f, 0.f};
                if (row < c.irows && c.j0 + pc < c.ldw) o = *(const KFAC_AS1 v4f*)&c.W[(size_t)(c.i0 + row) * c.ldw + c.j0 + pc];
                oldv[p] = o;
            }
        }
        if (wm == half) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int rl = mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                        lds[rl * sld + acc_col(wn, nbk, lane)] = dead ? 0.f : acc.c[mb][nbk][r];
                    }
        }
        __syncthreads();
        upd_flush<LAST, true>(c, lds, h0, oldv);
    }
}

// Where a tile's old values come from: element (a, c) of the tile is base[a * rs + c * cs].
struct OldSrc {
    const gfloat* base;
    int rs, cs;
};

// Regular tile of a step that is not the matrix's last one: new = old - A0 B0^T - A1 B1^T - ... (one product per pending
// step, in step order) goes back into the working copy.  Only a matrix's last block can be ragged and the step that eliminates it is its last, so here the pivot
// blocks are full (K = 128 per product).  The products run on the fp16 matrix cores with both operands scaled per
// slab and split two ways (gemm_split.h): the accumulators start as the tile's old values (fetched straight into MFMA register layout:
// register r of a 32 x 32 block is 32 consecutive floats of one row per half-wave), the negated products are added,
// and the result is stored from the registers: nothing is staged in LDS.
// STORE = false: the new values stay in acc (valid where the tile has rows and columns;
// the quadrant above the diagonal of a diagonal tile is not computed) and nothing is written.
constexpr int MAXRUN = GM;               // a tile owes at most one whole group (the group before, or its own so far)
typedef SplitRun<MAXRUN> PanelRun;

// The products of tile (I, J) with the panels of the n consecutive steps first_step .. first_step + n - 1 (buffer =
// step mod NBUF).
__device__ __forceinline__ PanelRun panel_run(const WsView& ws, int first_step, int n, int I, int J) {
    PanelRun r;
    r.a_hi = ws.TH(0) + (size_t)I * PRE_SLAB;
    r.b_hi = ws.UH(0) + (size_t)J * PRE_SLAB;
    r.plane = ws.plane;
    r.stride = ws.stride * sizeof(float);
    r.first = first_step % NBUF;
    r.nbuf = NBUF;
    r.n = n;
#pragma unroll
    for (int q = 0; q < MAXRUN; ++q) {
        const int b = (first_step + q) % NBUF;
        r.scale[q] = ws.scaleT(b, I) * ws.scaleU(b, J);
    }
    return r;
}

template <bool STORE = true>
__device__ __forceinline__ void upd_regular_mid_split(const UpdCtx& c, const OldSrc& o, const PanelRun& pl,
                                                      unsigned char* __restrict__ lds, TileAcc& acc) {
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
    const int lm = lane & 31, h = lane >> 5;
    const bool dead = c.diag && wm == 0 && wn == 1;      // strictly above the diagonal, never used
    gfloat* wtile = c.W + (size_t)c.i0 * c.ldw + c.j0;
    const int rows_left = c.irows - wm * 64 - 4 * h;     // tile rows from the lane's first row on
    bool colok[2];
    gfloat* wq[2];
    const gfloat* oq[2];
#pragma unroll
    for (int nbk = 0; nbk < 2; ++nbk) {
        colok[nbk] = !dead && c.j0 + wn * 64 + nbk * 32 < c.ldw;
        wq[nbk] = wtile + (size_t)(wm * 64 + 4 * h) * c.ldw + wn * 64 + nbk * 32 + lm;
        oq[nbk] = o.base + (wm * 64 + 4 * h) * o.rs + (wn * 64 + nbk * 32 + lm) * o.cs;
    }
    // the products run on operands scaled by sa, sb (powers of two): the accumulators follow, exactly
    // a tile with all its rows and columns, off the diagonal (nearly all of them): no guards, no branches
    const bool whole = !c.diag && c.irows == NB && c.j0 + NB <= c.ldw;
    if (whole) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc.c[mb][nbk][r] = oq[nbk][(mb * 32 + (r >> 2) * 8 + (r & 3)) * o.rs];
    } else {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = mb * 32 + (r >> 2) * 8 + (r & 3);
                    acc.c[mb][nbk][r] = (colok[nbk] && dr < rows_left) ? oq[nbk][dr * o.rs] : 0.f;
                }
    }
    const float back = tile_mma_presplit(pl, lds, acc);  // (what brings acc back to the scale of the tile)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nbk = 0; nbk < 2; ++nbk) acc.c[mb][nbk] *= back;
    if constexpr (STORE) {
        if (whole) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        wq[nbk][(size_t)(mb * 32 + (r >> 2) * 8 + (r & 3)) * c.ldw] = acc.c[mb][nbk][r];
        } else {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nbk = 0; nbk < 2; ++nbk)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int dr = mb * 32 + (r >> 2) * 8 + (r & 3);
                        if (colok[nbk] && dr < rows_left) wq[nbk][(size_t)dr * c.ldw] = acc.c[mb][nbk][r];
                    }
        }
    }
}

// Look-ahead: the diagonal tile that is the next step's pivot block is updated by a workgroup of its own, which
// keeps the new values in registers and inverts the block at once (the pivot sweep is the longest link of the chain
// pivot -> panel -> update; here it runs beside the update of all other tiles instead of after it).
__device__ __forceinline__ void upd_next_pivot(const Item& it, int step, float* __restrict__ lds) {
    const int d = it.dim, kn = step + 1;
    const WsView ws = ws_view(it.ws, d);
    const int k0 = kn * NB, nb = min(NB, d - k0);
    UpdCtx c;
    const int cur = step % NBUF;                         // (the block is kept up to date through the step before)
    c.W = ws.W; c.ldw = ws.ldw; c.T = ws.T(cur); c.out = it.Minv;
    c.d = d;
    c.i0 = c.j0 = k0;
    c.irows = c.jrows = nb;
    c.nb = NB;
    c.diag = true;
    TileAcc acc;
    const OldSrc o = {ws.W + (size_t)k0 * ws.ldw + k0, ws.ldw, 1};
    const PanelRun pl = panel_run(ws, step, 1, kn, kn);
    upd_regular_mid_split<false>(c, o, pl, (unsigned char*)lds, acc);
    __syncthreads();                                     // the product's LDS stages are free
    const int t = threadIdx.x;
    pivot_symmetrize(acc.c, lds, nb);
    const int f = pivot_sweep(acc.c, nb, lds);
    if (t == 0 && it.info && f != 0) atomicCAS((int*)it.info, 0, k0 + f);
    pivot_write(acc.c, lds, it, ws, k0, nb, k0 + NB >= d, false);
}

// column tile (from_rows = true): new[a][c] = T[(i0 + a)][c];  row tile: new[a][c] = T[(j0 + c)][a]
template <bool LAST>
__device__ __forceinline__ void upd_panel(const UpdCtx& c, bool column, float* __restrict__ lds) {
    const int t = threadIdx.x;
    const int pr = t >> 5, pc = (t & 31) * 4;
    constexpr int sld = LAST ? SLD_T : SLD;
    const v4f none[8] = {};
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        const int h0 = half * 64;
        if (h0 >= c.irows) break;
        if (half == 1) __syncthreads();
        // all eight loads go out before the first value is used (a use inside the guarded block would make the
        // compiler wait for every load in turn)
        v4f x[8];
        if (column) {
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int row = h0 + pr + 8 * p;
                x[p] = v4f{0.f, 0.f, 0.f, 0.f};
                if (row < c.irows) x[p] = *(const KFAC_AS1 v4f*)&c.T[(size_t)(c.i0 + row) * NB + pc];
            }
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int rl = pr + 8 * p;
#pragma unroll
                for (int i = 0; i < 4; ++i) lds[rl * sld + pc + i] = pc + i < c.nb ? x[p][i] : 0.f;
            }
        } else {
            const int ta = (t & 15) * 4, tc = t >> 4;     // 16 float4 along a (64 a's), 16 c's per pass
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int cc = tc + 16 * p;
                x[p] = v4f{0.f, 0.f, 0.f, 0.f};
                if (cc < c.jrows) x[p] = *(const KFAC_AS1 v4f*)&c.T[(size_t)(c.j0 + cc) * NB + h0 + ta];
            }
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int cc = tc + 16 * p;
#pragma unroll
                for (int i = 0; i < 4; ++i) lds[(ta + i) * sld + cc] = h0 + ta + i < c.nb ? x[p][i] : 0.f;
            }
        }
        __syncthreads();
        upd_flush<LAST, false>(c, lds, h0, none);
    }
}

// Tile (I, J) of a step that is not the matrix's last: brings it up to date through step kq = g.g0 + g.j of group g.
// single: the tile has been kept up to date step by step (a narrow launch): it sees step kq only, and its old value
// is in the working copy.  Otherwise it sees all of the group's steps up to kq that it has not seen yet: all of them
// for a tile with no index inside the group.  A tile with an index inside the group was kept up to date until its
// later such index c was eliminated (when it became part of panel c: T_I for a tile of block column c, T_J transposed
// for a tile of block row c, neither written to the working copy then), and sees the steps after c; the diagonal tile
// (c, c) is -P_c, which the pivot code did write.
__device__ __forceinline__ void group_tile(const Item& it, const WsView& ws, int I, int J, const Group& g, bool single,
                                           float* __restrict__ lds) {
    const int kq = g.g0 + g.j;
    const int gbuf = g.g0 % NBUF;                        // buffer of the group's first step
    UpdCtx c;
    c.W = ws.W; c.ldw = ws.ldw; c.T = ws.T(gbuf + g.j); c.out = it.Minv;
    c.d = it.dim;
    c.i0 = I * NB; c.j0 = J * NB;
    c.irows = min(NB, c.d - c.i0); c.jrows = min(NB, c.d - c.j0);
    c.nb = NB;                                           // (only a matrix's last block can be ragged)
    c.diag = I == J;
    if (J == kq || I == kq) {                            // block column / row kq becomes the panel
        upd_panel<false>(c, J == kq, lds);
        return;
    }
    OldSrc o = {ws.W + (size_t)c.i0 * ws.ldw + c.j0, ws.ldw, 1};
    int first = g.j;                                     // steps first .. g.j of the group, in order
    if (!single) {
        const bool inI = I >= g.g0 && I < kq, inJ = J >= g.g0 && J < kq;
        first = 0;
        if (inI) {                                       // I is the later index (I >= J)
            first = I - g.g0 + 1;
            if (I != J) o = OldSrc{ws.T(gbuf + I - g.g0) + (size_t)c.j0 * NB, 1, NB};
        } else if (inJ) {                                // I lies beyond the group
            first = J - g.g0 + 1;
            o = OldSrc{ws.T(gbuf + J - g.g0) + (size_t)c.i0 * NB, NB, 1};
        }
    }
    TileAcc acc;
    const PanelRun run = panel_run(ws, g.g0 + first, g.j - first + 1, I, J);
    upd_regular_mid_split(c, o, run, (unsigned char*)lds, acc);
}

// Tile of block column / row c = k + 1 (not the diagonal one) in the chain launch of step k: brought up to date
// through step k, whatever it owes.  With `other` its second index:
//   other == k              it becomes part of panel k: T_I of this step (block column k)
//   lo <= other < k         block column `other` was eliminated at a step inside the window the tile can owe: the tile
//                           then became T_I of that step (not written to the working copy), and owes the steps after it
//   otherwise               its value in the working copy is up to date through step lo - 1 and it owes lo .. k.  For the
//                           first block of a group, lo is the first step of the group before (whose bulk update ran
//                           while that group was under way and skipped the tiles with an index inside it); for the other
//                           blocks of a group it is the group's own first step (the last launch of the group before
//                           brought their tiles up to date: the early tiles of plan_of).
__device__ __forceinline__ void chain_tile(const Item& it, const WsView& ws, int I, int J, int k, float* __restrict__ lds) {
    const int c1 = k + 1;
    UpdCtx c;
    c.W = ws.W; c.ldw = ws.ldw; c.T = ws.T(k % NBUF); c.out = it.Minv;
    c.d = it.dim;
    c.i0 = I * NB; c.j0 = J * NB;
    c.irows = min(NB, c.d - c.i0); c.jrows = min(NB, c.d - c.j0);
    c.nb = NB;
    c.diag = false;
    if (J == k) {                                        // (I == c1: the tile below the pivot block)
        upd_panel<false>(c, true, lds);
        return;
    }
    const int lo = c1 % GM == 0 ? max(0, c1 - GM) : c1 / GM * GM;
    OldSrc o = {ws.W + (size_t)c.i0 * ws.ldw + c.j0, ws.ldw, 1};
    int first = lo;
    if (I == c1 && J >= lo) {                            // (J < k here)
        first = J + 1;
        o = OldSrc{ws.T(J % NBUF) + (size_t)c.i0 * NB, NB, 1};
    }
    TileAcc acc;
    const PanelRun run = panel_run(ws, first, k - first + 1, I, J);
    upd_regular_mid_split(c, o, run, (unsigned char*)lds, acc);
}

// One launch per step for all matrices of the batch that still have a block `step`; a matrix whose last block this
// is takes the output-writing paths (LAST), the others update their working copies.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(UPD_WAVES, 8))) void inv_update_kernel(ChainBatch b) {
    __shared__ __attribute__((aligned(1024))) float lds[UNS * USTAGE / 4];
    // Workgroups go to the 8 XCDs round-robin (id % 8) and each XCD has an L2 of its own.  XCD x therefore takes the
    // x-th contiguous eighth of the tile list (matrix by matrix, row-major over the lower triangle): tiles that
    // share a T panel (same block row) and mostly the same U panels run on the same L2 instead of all eight.
    // The first workgroups (one per matrix, padded to a multiple of 8 so that the others keep their XCD) take the
    // next step's pivot block; they are dispatched first and run the longest.
    const int npiv = (b.count + 7) & ~7;
    if ((int)blockIdx.x < npiv) {
        if ((int)blockIdx.x >= b.count) return;
        __builtin_amdgcn_s_setprio(3);                   // the chain's longest link: ahead of whatever shares its SIMDs
        const Item it = get_item(b, blockIdx.x);
        const int step = b.step[blockIdx.x];
        if (step >= 0 && nblk_of(it.dim) > step + 1) upd_next_pivot(it, step, lds);
        return;
    }
    const unsigned bx = blockIdx.x - npiv;
    const int total = b.prefix[b.count];
    const int per_xcd = (total + 7) >> 3;
    const int lin = (int)(bx & 7) * per_xcd + (int)(bx >> 3);
    if ((int)(bx >> 3) >= per_xcd || lin >= total) return;
    int m, tile;
    locate(b, lin, m, tile);
    const Item it = get_item(b, m);
    const int nblk = nblk_of(it.dim);
    const int step = b.step[m];
    const Plan pl = plan_of(it.dim, step);
    const WsView ws = ws_view(it.ws, it.dim);
    int I, J;
    if (tile >= pl.chain && pl.early > 0) {
        // early tile: this group's steps, all of them (the launch is the group's last)
        early_decode(nblk, pl.g.g0 + pl.g.m, pl.next_m, tile - pl.chain, I, J);
        group_tile(it, ws, I, J, pl.g, false, lds);
        return;
    }
    if (tile >= pl.chain) {
        // lag tile: the whole update of the previous group (steps g0 - GM .. g0 - 1, all GM of them)
        lag_decode(nblk, pl.g.g0, pl.g.m, pl.lag_off + tile - pl.chain, I, J);
        const int E = pl.g.g0 + pl.g.m;
        if (I == J && (I == pl.g.g0 - 1 || I == E)) return;   // -P of the group's last step; a chain tile of this group
        Group pg;
        pg.g0 = pl.g.g0 - GM; pg.m = GM; pg.j = GM - 1;
        group_tile(it, ws, I, J, pg, false, lds);
        return;
    }
    if (pl.kind == PLAN_CHAIN) {
        __builtin_amdgcn_s_setprio(2);                   // the next panel waits for these; lag tiles do not hurry
        chain_decode(nblk, step + 1, pl.d_begin, tile, I, J);
        if (I != J) chain_tile(it, ws, I, J, step, lds);
        else group_tile(it, ws, I, J, pl.g, pl.g.j < pl.g.m - 1, lds);   // kept up to date step by step inside a group
        return;
    }
    tri_decode_blocked(nblk, tile, I, J);
    if (I == J && (I == step || I == step + 1)) return;  // this step's pivot block and the next one's are written elsewhere
    if (pl.kind == PLAN_WHOLE) {
        group_tile(it, ws, I, J, pl.g, false, lds);
        return;
    }
    const int cur = step % NBUF;
    UpdCtx c;
    c.W = ws.W; c.ldw = ws.ldw; c.T = ws.T(cur); c.out = it.Minv;
    c.d = it.dim;
    c.i0 = I * NB; c.j0 = J * NB;
    c.irows = min(NB, c.d - c.i0); c.jrows = min(NB, c.d - c.j0);
    c.nb = min(NB, c.d - step * NB);
    c.diag = I == J;
    if (J == step || I == step) upd_panel<true>(c, J == step, lds);
    else upd_regular<true>(c, ws.U(cur), lds);
}

// The piece planes of finished inverses: one workgroup per 128 x 128 block, read from the caller's output after the
// matrix's last step.  (Written by the last step's tiles themselves the planes cost the update kernel registers that
// its hot paths miss, and more time than this pass over the output.)
constexpr int PLMAXB = 100;
struct PlanesBatch {
    int count;
    int prefix[PLMAXB + 1];           // block prefix sums
    int dim[PLMAXB];
    float damping[PLMAXB];
    const float* damping_dev[PLMAXB];
    const float* Minv[PLMAXB];
    void* planes[PLMAXB];
};
static_assert(sizeof(PlanesBatch) <= 4096, "the batch travels in the kernel arguments");

__global__ __launch_bounds__(256) void inv_planes_kernel(PlanesBatch b) {
    const int t = threadIdx.x;
    const int m = __syncthreads_count(t < b.count - 1 && b.prefix[t + 1] <= (int)blockIdx.x);
    const int blk = blockIdx.x - b.prefix[m];
    const int d = b.dim[m], n = nblk_of(d);
    const int s = blk / n, c = blk - s * n;
    const int r0 = s * NB, k0 = c * NB;
    const float lam = b.damping_dev[m] ? *as_global(b.damping_dev[m]) : b.damping[m];
    const float sc = inverse_plane_scale(lam);
    const gfloat* X = as_global(b.Minv[m]);
    KFAC_AS1 unsigned char* planes = (KFAC_AS1 unsigned char*)as_global((float*)b.planes[m]);
    const size_t plane = inverse_plane_bytes(d);
    if (t == 0) ((gfloat*)(planes + 2 * plane))[blk] = sc;
    const int c4 = (t & 31) * 4, rr = t >> 5;
    v4f v[16];
    if (r0 + NB <= d && k0 + NB <= d) {                 // all loads go out together (a guard per load would serialise them)
#pragma unroll
        for (int p = 0; p < 16; ++p) v[p] = *(const KFAC_AS1 v4f_a4*)(X + (size_t)(r0 + rr + 8 * p) * d + k0 + c4);
    } else {
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = r0 + rr + 8 * p;
            v[p] = load4_guard(X + (size_t)(row < d ? row : 0) * d, row < d, k0 + c4, d);
        }
    }
    KFAC_AS1 unsigned char* dst = planes + (size_t)blk * PRE_SLAB;
#pragma unroll
    for (int p = 0; p < 16; ++p) store_split4_h2(dst, dst + plane, rr + 8 * p, c4, v[p] * sc);
}

// Planes for the matrices of a call that asked for them (after all their steps have been enqueued on `stream`).
static int write_planes(const kfac_inverse_item* h, int count, hipStream_t stream) {
    PlanesBatch b;
    b.count = 0;
    b.prefix[0] = 0;
    for (int i = 0; i <= count; ++i) {
        if (i < count && h[i].planes) {
            const int k = b.count++;
            b.dim[k] = h[i].dim; b.damping[k] = h[i].damping; b.damping_dev[k] = h[i].damping_dev;
            b.Minv[k] = h[i].Minv; b.planes[k] = h[i].planes;
            b.prefix[k + 1] = b.prefix[k] + nblk_of(h[i].dim) * nblk_of(h[i].dim);
        }
        if (b.count == PLMAXB || (i == count && b.count > 0)) {
            KFAC_LAUNCH(inv_planes_kernel, dim3(b.prefix[b.count]), dim3(256), stream, b);
            b.count = 0;
        }
    }
    return KFAC_OK;
}

static inline int tri_tiles(int dim) { int n = nblk_of(dim); return n * (n + 1) / 2; }

static void fill_batch(Batch& b, const kfac_inverse_item* items, int count) {
    b.count = count;
    for (int i = 0; i < count; ++i) {
        b.dim[i] = items[i].dim;
        b.damping[i] = items[i].damping;
        b.damping_dev[i] = items[i].damping_dev;
        b.S[i] = items[i].S;
        b.Minv[i] = items[i].Minv;
        b.ws[i] = items[i].ws;
        b.info[i] = items[i].info;
    }
}

// items must be sorted by non-increasing dim (checked by the caller of this function).
static inline int xcd_grid(int tiles) { return 8 * ((tiles + 7) / 8); }   // eight equal shares, the last one padded

static int run_group(const kfac_inverse_item* h, int count, hipStream_t stream) {
    Batch b;
    const int max_steps = nblk_of(h[0].dim);

    // matrices needing the blocked path (more than one block) come first in the sorted order
    int n_multi = 0;
    while (n_multi < count && nblk_of(h[n_multi].dim) > 1) ++n_multi;

    // single-block matrices: damp, invert and write in one kernel, straight from S
    for (int first = n_multi; first < count; first += MAXB) {
        fill_batch(b, h + first, min(MAXB, count - first));
        KFAC_LAUNCH(inv_pivot_kernel, dim3(b.count), dim3(256), stream, b, 0, 1);
    }
    if (n_multi == 0) return KFAC_OK;
    // damped working copies, then the first pivot blocks (later ones: by the update launches)
    for (int first = 0; first < n_multi; first += MAXB) {
        const int n = min(MAXB, n_multi - first);
        fill_batch(b, h + first, n);
        b.prefix[0] = 0;
        for (int i = 0; i < n; ++i) b.prefix[i + 1] = b.prefix[i] + tri_tiles(h[first + i].dim);
        KFAC_LAUNCH(inv_init_kernel, dim3(b.prefix[n]), dim3(256), stream, b);
    }
    for (int first = 0; first < n_multi; first += MAXB) {
        fill_batch(b, h + first, min(MAXB, n_multi - first));
        KFAC_LAUNCH(inv_pivot_kernel, dim3(b.count), dim3(256), stream, b, 0, 0);
    }
    // One panel and one update launch per step of the matrix with the most blocks.  A matrix with fewer blocks takes
    // its steps at evenly spread launches rather than in the first ones: the tile updates of the whole batch are then
    // spread over all launches, each of which lasts at least as long as a pivot workgroup anyway.
    ChainBatch c;
    c.count = n_multi;
    c.prefix[0] = 0;
    for (int i = 0; i < n_multi; ++i) {
        c.dim[i] = h[i].dim; c.Minv[i] = h[i].Minv; c.ws[i] = h[i].ws; c.info[i] = h[i].info;
    }
    int done[CMAXB] = {};                               // steps taken so far
    for (int l = 0; l < max_steps; ++l) {
        for (int i = 0; i < n_multi; ++i) {
            // (a matrix's last two steps touch all of its tiles, the last one on a slow path: matrices with fewer blocks
            // than the largest finish at different launches, none with the largest ones)
            const int n = nblk_of(h[i].dim);
            const int span = n == max_steps ? n : max(n, max_steps - 2 - 2 * (i % 6));
            const bool run = l < span && (int)(((long long)(l + 1) * n) / span) > (int)(((long long)l * n) / span);
            c.step[i] = run ? done[i] : -1;
        }
        for (int i = 0; i < n_multi; ++i) c.prefix[i + 1] = c.prefix[i] + (c.step[i] >= 0 ? nblk_of(h[i].dim) : 0);
        KFAC_LAUNCH(inv_panel_kernel, dim3(c.prefix[n_multi]), dim3(256), stream, c);
        for (int i = 0; i < n_multi; ++i)
            c.prefix[i + 1] = c.prefix[i] + (c.step[i] >= 0 ? update_tiles(h[i].dim, c.step[i]) : 0);
        KFAC_LAUNCH(inv_update_kernel, dim3(xcd_grid(n_multi) + xcd_grid(c.prefix[n_multi])), dim3(256), stream, c);
        for (int i = 0; i < n_multi; ++i) done[i] += c.step[i] >= 0;
    }
    return KFAC_OK;
}

static size_t ws_bytes_of(int dim) {
    if (nblk_of(dim) == 1) return 256;
    const size_t d_pad = (size_t)nblk_of(dim) * NB;
    return align_up((d_pad * ldw_of(dim) + NBUF * panel_buffer_floats(dim) + (size_t)NB * NB + 2 * NBUF * (size_t)nblk_of(dim)) * sizeof(float), 256);
}

static bool item_ok(const kfac_inverse_item& it) {
    if (!it.S || !it.Minv || it.dim <= 0 || it.dim > 32768) return false;
    if (it.S == it.Minv) return false;
    if (nblk_of(it.dim) > 1 && (!it.ws || ((uintptr_t)it.ws & 255))) return false;
    if (it.planes && (((uintptr_t)it.planes & 255) || (!it.damping_dev && !(it.damping > 0.f)))) return false;
    return true;
}

}  // namespace kfac

using namespace kfac;

extern "C" size_t kfac_inverse_workspace_bytes(int32_t dim) {
    if (dim <= 0 || dim > 32768) return 0;
    return ws_bytes_of(dim);
}

extern "C" size_t kfac_inverse_planes_bytes(int32_t dim) {
    if (dim <= 0 || dim > 32768) return 0;
    return align_up(inverse_planes_bytes(dim), 256);
}

extern "C" int kfac_damped_inverse(const float* S, int32_t dim, float damping, float* Minv, int32_t* info,
                                   void* ws, size_t ws_bytes, void* stream) {
    kfac_inverse_item it;
    it.S = S; it.Minv = Minv; it.ws = ws; it.info = info; it.dim = dim; it.damping = damping; it.damping_dev = nullptr;
    it.planes = nullptr;
    if (dim <= 0 || dim > 32768 || !S || !Minv || S == Minv) return KFAC_ERR_INVALID_ARG;
    if (nblk_of(dim) > 1) {
        if (!ws || ((uintptr_t)ws & 255) || ws_bytes < ws_bytes_of(dim)) return KFAC_ERR_WORKSPACE;
    }
    return run_group(&it, 1, (hipStream_t)stream);
}

extern "C" int kfac_damped_inverse_batched(const kfac_inverse_item* items_host, int32_t count, void* stream) {
    if (count == 0) return KFAC_OK;                       // nothing to do, no launch
    if (!items_host || count < 0) return KFAC_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i) {
        if (!item_ok(items_host[i])) return KFAC_ERR_INVALID_ARG;
        if (i > 0 && items_host[i].dim > items_host[i - 1].dim) return KFAC_ERR_INVALID_ARG;   // sorted, largest first
    }
    // Matrices beyond what one launch's argument block can describe go into further groups.  Dealing them round
    // robin keeps every group's size mix (and hence its step count and load) similar.
    const int ngroups = (count + CMAXB - 1) / CMAXB;
    for (int g = 0; g < ngroups; ++g) {
        kfac_inverse_item sel[CMAXB];
        int n = 0;
        for (int i = g; i < count; i += ngroups) sel[n++] = items_host[i];
        int rc = run_group(sel, n, (hipStream_t)stream);
        if (rc != KFAC_OK) return rc;
    }
    return write_planes(items_host, count, (hipStream_t)stream);
}
