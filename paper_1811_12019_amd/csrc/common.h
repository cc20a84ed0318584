// Internal helpers shared by the gfx950 K-FAC kernels.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/kfac.h"

#define KFAC_HIP_TRY(expr)                         \
    do {                                           \
        hipError_t e__ = (expr);                   \
        if (e__ != hipSuccess) return KFAC_ERR_HIP; \
    } while (0)

#define KFAC_LAUNCH_CHECK()                                     \
    do {                                                        \
        if (hipGetLastError() != hipSuccess) return KFAC_ERR_HIP; \
    } while (0)

// Launch `kernel` and return KFAC_ERR_HIP from the enclosing function if the launch is rejected.
#define KFAC_LAUNCH(kernel, grid, block, stream, ...)                              \
    do {                                                                           \
        void* tok__ = nullptr;                                                     \
        if (kfac::timing_enabled()) kfac::timing_begin(#kernel, stream, &tok__);   \
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);           \
        if (tok__) kfac::timing_end(stream, tok__);                                \
        if (hipGetLastError() != hipSuccess) return KFAC_ERR_HIP;                  \
    } while (0)

// Same, with `lds` bytes of dynamic LDS.
#define KFAC_LAUNCH_LDS(kernel, grid, block, lds, stream, ...)                     \
    do {                                                                           \
        void* tok__ = nullptr;                                                     \
        if (kfac::timing_enabled()) kfac::timing_begin(#kernel, stream, &tok__);   \
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);         \
        if (tok__) kfac::timing_end(stream, tok__);                                \
        if (hipGetLastError() != hipSuccess) return KFAC_ERR_HIP;                  \
    } while (0)

namespace kfac {

// Opt-in per-kernel event timing (runtime.hip).
bool timing_enabled();
void timing_begin(const char* name, hipStream_t stream, void** token);
void timing_end(hipStream_t stream, void* token);

constexpr int WAVE = 64;

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef short v8s __attribute__((ext_vector_type(8)));

// Four floats that are only guaranteed dword alignment (rows of an odd-sized matrix).
typedef v4f v4f_a4 __attribute__((aligned(4)));

static inline __host__ __device__ int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Pointers that kernels load from a descriptor table in memory have no known address space, and the compiler
// would access them with flat instructions (slower, and they tie up the LDS wait counter as well).  Device code
// that handles such pointers therefore uses pointers explicitly typed as global memory.
#define KFAC_AS1 __attribute__((address_space(1)))
typedef KFAC_AS1 float gfloat;
typedef KFAC_AS1 int gint;
template <class T>
__device__ __forceinline__ KFAC_AS1 T* as_global(T* p) {
    return (KFAC_AS1 T*)p;
}

// Where a symmetric d x d result goes (the factor builders' epilogues):
//   plain    dst = the d x d square, both triangles written
//   ema      dst = the running average S, updated in place: S <- decay S + (1 - decay) value   (both triangles)
//   packed   dst = the packed upper triangle (row r contributes columns r .. d-1), d (d + 1) / 2 floats
struct OutSpec {
    gfloat* dst;
    float decay, one_minus;
    int mode;                       // OUT_PLAIN, OUT_EMA, OUT_PACKED
};
constexpr int OUT_PLAIN = 0, OUT_EMA = 1, OUT_PACKED = 2;

// first element of packed row r, minus r (so that adding a column index c >= r gives the element's place)
__device__ __forceinline__ size_t packed_row_base(int r, int d) {
    return (size_t)r * d - ((size_t)r * (r - 1)) / 2 - r;
}

// One element (row, col) of the result, row >= col or inside a diagonal tile that holds both triangles; `mirror`: the
// element (col, row) is this call's to write too.  The slow, general form (the matrix-core epilogues have their own).
__device__ __forceinline__ void emit_sym(const OutSpec& o, int d, int row, int col, float v, bool mirror) {
    if (o.mode == OUT_PACKED) {
        if (mirror || col >= row) {
            const int r = min(row, col), c = max(row, col);
            o.dst[packed_row_base(r, d) + c] = v;
        }
        return;
    }
    const size_t idx = (size_t)row * d + col;
    if (o.mode == OUT_EMA) v = fmaf(o.decay, o.dst[idx], o.one_minus * v);
    o.dst[idx] = v;
    if (mirror) o.dst[(size_t)col * d + row] = v;
}

// lower-triangular tile index -> (I, J), I >= J, tiles numbered row by row
__device__ __forceinline__ void tri_decode(int t, int& I, int& J) {
    int i = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
    while ((i + 1) * (i + 2) / 2 <= t) ++i;
    while (i * (i + 1) / 2 > t) --i;
    I = i;
    J = t - i * (i + 1) / 2;
}

// Index in the list of all lower tiles of an n x n tile triangle -> (I, J), in an order that keeps tiles sharing rows
// and columns together: the triangle is cut into SB x SB super-blocks (row-major over the super-blocks, row-major
// inside one), so that a contiguous range of the list, which is what one XCD (one L2) gets, reads about as many
// different row panels as column panels instead of one or two of the former and all of the latter.
template <int SB = 8>
__device__ __forceinline__ void tri_decode_blocked(int n, int t, int& I, int& J) {
    int r0 = 0;
    for (;;) {                                           // super-row with rows r0 .. r0 + h - 1
        const int h = min(SB, n - r0);
        const int cnt = h * r0 + h * (h + 1) / 2;        // full super-blocks to the left, then the triangular one
        if (t < cnt || r0 + SB >= n) break;
        t -= cnt;
        r0 += SB;
    }
    const int h = min(SB, n - r0);
    if (t < h * r0) {
        const int sj = t / (h * SB), in = t - sj * (h * SB);
        I = r0 + in / SB;
        J = sj * SB + in % SB;
    } else {
        tri_decode(t - h * r0, I, J);
        I += r0;
        J += r0;
    }
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

__device__ __forceinline__ float half_bits_to_float(uint16_t b) {
    _Float16 h;
    __builtin_memcpy(&h, &b, 2);
    return (float)h;
}

// Geometry of an implicit unfold: which input element feeds column `col` of unfolded row `r`.
// factor_G uses the same structure with a 1x1 / stride 1 / no-bias geometry over the output tensor.
struct Unfold {
    int N, C, H, W;      // tensor being read (for G: C = C_out, H = H_o, W = W_o)
    int Ho, Wo;          // rows: r = (n*Ho + yo)*Wo + xo
    int kh, kw, stride, pad;
    int has_bias;
    int layout, dtype, order;
    int R;               // N*Ho*Wo
    int d;               // columns incl. the bias column
};

static inline __host__ __device__ bool make_unfold_A(const kfac_layer_desc* L, Unfold* u) {
    if (!L) return false;
    if (L->N <= 0 || L->C_in <= 0 || L->H <= 0 || L->W <= 0 || L->C_out <= 0 || L->kh <= 0 || L->kw <= 0 ||
        L->stride <= 0 || L->pad < 0)
        return false;
    if (L->layout != KFAC_NCHW && L->layout != KFAC_NHWC) return false;
    if (L->dtype != KFAC_F32 && L->dtype != KFAC_BF16 && L->dtype != KFAC_F16) return false;
    if (L->order != KFAC_ORDER_C_KH_KW && L->order != KFAC_ORDER_KH_KW_C) return false;
    if (L->has_bias != 0 && L->has_bias != 1) return false;
    if (L->H + 2 * L->pad < L->kh || L->W + 2 * L->pad < L->kw) return false;
    long long Ho = (L->H + 2 * L->pad - L->kh) / L->stride + 1;
    long long Wo = (L->W + 2 * L->pad - L->kw) / L->stride + 1;
    long long R = (long long)L->N * Ho * Wo;
    long long d = (long long)L->C_in * L->kh * L->kw + L->has_bias;
    long long in_elems = (long long)L->N * L->C_in * L->H * L->W;
    long long out_elems = R * L->C_out;
    if (R <= 0 || R > 0x7fffffffLL || d > 32768 || L->C_out > 32768) return false;
    if (in_elems > 0x7fffffffLL || out_elems > 0x7fffffffLL) return false;   // 32-bit element offsets
    u->N = L->N; u->C = L->C_in; u->H = L->H; u->W = L->W;
    u->Ho = (int)Ho; u->Wo = (int)Wo;
    u->kh = L->kh; u->kw = L->kw; u->stride = L->stride; u->pad = L->pad;
    u->has_bias = L->has_bias;
    u->layout = L->layout; u->dtype = L->dtype; u->order = L->order;
    u->R = (int)R; u->d = (int)d;
    return true;
}

static inline __host__ __device__ bool make_unfold_G(const kfac_layer_desc* L, Unfold* u) {
    Unfold a;
    if (!make_unfold_A(L, &a)) return false;
    u->N = L->N; u->C = L->C_out; u->H = a.Ho; u->W = a.Wo;
    u->Ho = a.Ho; u->Wo = a.Wo;
    u->kh = 1; u->kw = 1; u->stride = 1; u->pad = 0;
    u->has_bias = 0;
    u->layout = L->layout; u->dtype = L->dtype; u->order = KFAC_ORDER_KH_KW_C;
    u->R = a.R; u->d = L->C_out;
    return true;
}

}  // namespace kfac
