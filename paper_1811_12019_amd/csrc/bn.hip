// Batch Normalization layers (Sec. 5.4): their Fisher matrix is not Kronecker-factorised.  With theta = (scale_1..C,
// shift_1..C), the gradient of sample n is
//     g_n[c] = sum_s gout[n,s,c] * xhat[n,s,c],     g_n[C + c] = sum_s gout[n,s,c]        (s = spatial position)
// and F = (1/N) sum_n g_n g_n^T (2C x 2C), or its diagonal.  This file builds the per-sample gradients from NHWC
// tensors, for all BN layers of a network in one launch per 16-bit dtype plus one for the sums over chunks (HBM bound:
// both tensors are read once), and applies the diagonal form; the full form is the generic factor build + damped
// inverse + product on the (N x 2C) gradient matrix.
#include <algorithm>

#include "common.h"

namespace kfac {

constexpr int BN_MAX = 64;            // layers per launch (argument block under 4 KB)
constexpr int BN_UNIT = 32768;        // elements of each tensor per workgroup of the 16-bit kernel
constexpr int BN_CVW = 64;            // 16-byte vectors (8 channels each) side by side in a workgroup, at most
constexpr int BN_SP_GENERIC = 512;    // positions per workgroup of the general kernel
typedef unsigned v4u __attribute__((ext_vector_type(4)));

// How one layer is cut into workgroups.  16-bit layers: a workgroup owns `cvw` vectors of `sp` consecutive positions of
// one sample; its 256 threads are cvw vectors x (256 / cvw) position lanes.  General layers: all channels of `sp` positions.
struct BnPlan {
    int cvw, ncb, sp, nchunk;
};

static BnPlan bn_plan(int C, int HW, bool vec) {
    BnPlan p;
    if (!vec) {
        p.cvw = 0; p.ncb = 1;
        p.nchunk = (HW + BN_SP_GENERIC - 1) / BN_SP_GENERIC;
        p.sp = BN_SP_GENERIC;
        return p;
    }
    const int cv = C >> 3;
    p.cvw = cv < BN_CVW ? cv : BN_CVW;
    p.ncb = (cv + p.cvw - 1) / p.cvw;
    const int lanes = 256 / p.cvw;
    int sp = BN_UNIT / (p.cvw * 8);
    if (sp < 4 * lanes) sp = 4 * lanes;
    p.nchunk = (HW + sp - 1) / sp;
    p.sp = (HW + p.nchunk - 1) / p.nchunk;            // even chunks, no short tail
    return p;
}

struct BnBatch {
    int count;
    unsigned prefix[BN_MAX + 1];      // first workgroup of layer i
    int C[BN_MAX], HW[BN_MAX], sp[BN_MAX], nchunk[BN_MAX];
    const void* x[BN_MAX];
    const void* gout[BN_MAX];
    float* dst[BN_MAX];               // nchunk == 1: g itself; else the layer's partial sums [n][chunk][2C]
};

struct BnReduceBatch {
    int count;
    unsigned prefix[BN_MAX + 1];      // first workgroup of layer i; one workgroup = 256 columns of one sample
    int C2[BN_MAX], nchunk[BN_MAX];
    const float* partial[BN_MAX];
    float* g[BN_MAX];
};

// 16-bit NHWC, C % 8 == 0.  Both tensors are read once, 16 bytes per thread and load, eight loads in flight.
template <bool F16>
__global__ __launch_bounds__(256) void bn_partial_kernel(BnBatch b) {
    __shared__ float red[256 * 16];                      // [position lane][half][vector][8]
    const int t = threadIdx.x;
    const int m = __syncthreads_count(t < b.count - 1 && b.prefix[t + 1] <= blockIdx.x);
    const int C = b.C[m], HW = b.HW[m], sp = b.sp[m], nchunk = b.nchunk[m];
    const int cv = C >> 3;
    const int cvw = cv < BN_CVW ? cv : BN_CVW;
    const int ncb = (cv + cvw - 1) / cvw;
    const int lanes = 256 / cvw;
    unsigned local = blockIdx.x - b.prefix[m];
    const int cb = local % ncb; local /= ncb;
    const int chunk = local % nchunk;
    const int n = local / nchunk;
    const KFAC_AS1 v4u* __restrict__ X = (const KFAC_AS1 v4u*)b.x[m];
    const KFAC_AS1 v4u* __restrict__ G = (const KFAC_AS1 v4u*)b.gout[m];
    const int vec0 = t % cvw, pl = t / cvw;
    const int vec = cb * cvw + vec0;
    const int s0 = chunk * sp, s1 = min(HW, s0 + sp);
    float ds[8] = {}, db[8] = {};
    if (pl < lanes && vec < cv) {
        const size_t row0 = (size_t)n * HW;
        for (int s = s0 + pl; s < s1; s += 4 * lanes) {
            v4u xv[4], gv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {                // masked, branch free: a position past the end re-reads s
                const int su = s + u * lanes;
                const bool ok = su < s1;
                const size_t at = (row0 + (ok ? su : s)) * cv + vec;
                xv[u] = X[at];
                gv[u] = G[at];
                if (!ok) gv[u] = v4u{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const unsigned xw = xv[u][k], gw = gv[u][k];
                    float x0, x1, g0, g1;
                    if constexpr (F16) {
                        x0 = half_bits_to_float((uint16_t)(xw & 0xffff)); x1 = half_bits_to_float((uint16_t)(xw >> 16));
                        g0 = half_bits_to_float((uint16_t)(gw & 0xffff)); g1 = half_bits_to_float((uint16_t)(gw >> 16));
                    } else {
                        x0 = __uint_as_float(xw << 16); x1 = __uint_as_float(xw & 0xffff0000u);
                        g0 = __uint_as_float(gw << 16); g1 = __uint_as_float(gw & 0xffff0000u);
                    }
                    ds[2 * k] = fmaf(g0, x0, ds[2 * k]);         db[2 * k] += g0;
                    ds[2 * k + 1] = fmaf(g1, x1, ds[2 * k + 1]); db[2 * k + 1] += g1;
                }
        }
    }
    // sum over the position lanes in a fixed order; every thread takes part
    const int w8 = cvw * 8;                              // channels of this workgroup
    if (pl < lanes) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            red[pl * 2 * w8 + vec0 * 8 + e] = ds[e];
            red[pl * 2 * w8 + w8 + vec0 * 8 + e] = db[e];
        }
    }
    __syncthreads();
    gfloat* dst = as_global(b.dst[m]) + ((size_t)n * nchunk + chunk) * (2 * C);
    for (int e = t; e < 2 * w8; e += 256) {
        float a = red[e];
        for (int q = 1; q < lanes; ++q) a += red[q * 2 * w8 + e];
        const int half = e >= w8, c = cb * w8 + (e - half * w8);
        if (c < C) dst[half * C + c] = a;
    }
}

// any dtype / channel count: thread = one channel, slow but general
__global__ __launch_bounds__(256) void bn_partial_generic_kernel(const void* xhat_, const void* gout_, int dtype, int C,
                                                                 int HW, int nchunk, float* partial_) {
    gfloat* __restrict__ partial = as_global(partial_);
    const int n = blockIdx.y, chunk = blockIdx.x;
    const int s0 = chunk * BN_SP_GENERIC, s1 = min(HW, s0 + BN_SP_GENERIC);
    auto at = [&](const void* p, size_t i) -> float {
        if (dtype == KFAC_F32) return ((const KFAC_AS1 float*)p)[i];
        const uint16_t b = ((const KFAC_AS1 uint16_t*)p)[i];
        return dtype == KFAC_BF16 ? bf16_bits_to_float(b) : half_bits_to_float(b);
    };
    for (int c = threadIdx.x; c < C; c += 256) {
        float ds = 0.f, db = 0.f;
        for (int s = s0; s < s1; ++s) {
            const size_t i = ((size_t)n * HW + s) * C + c;
            const float g = at(gout_, i);
            ds = fmaf(g, at(xhat_, i), ds);
            db += g;
        }
        gfloat* dst = partial + ((size_t)n * nchunk + chunk) * (2 * C);
        dst[c] = ds;
        dst[C + c] = db;
    }
}

// g[n][j] = sum over chunks, fixed order
__global__ __launch_bounds__(256) void bn_reduce_kernel(BnReduceBatch b) {
    const int t = threadIdx.x;
    const int m = __syncthreads_count(t < b.count - 1 && b.prefix[t + 1] <= blockIdx.x);
    const int C2 = b.C2[m], nchunk = b.nchunk[m];
    const int cblocks = (C2 + 255) >> 8;
    const unsigned local = blockIdx.x - b.prefix[m];
    const int n = local / cblocks, j = (local % cblocks) * 256 + t;
    if (j >= C2) return;
    const gfloat* __restrict__ partial = as_global(b.partial[m]);
    float s = 0.f;
    for (int q = 0; q < nchunk; ++q) s += partial[((size_t)n * nchunk + q) * C2 + j];
    as_global(b.g[m])[(size_t)n * C2 + j] = s;
}

// diag(F)[j] = (1/N) sum_n g[n][j]^2 ;  out[j] = grad[j] / (diag(F)[j] + damping)
__global__ __launch_bounds__(256) void bn_diag_kernel(const float* g_, int N, int C2, const float* grad, float damping,
                                                      float* fisher_diag, float* out) {
    const gfloat* __restrict__ g = as_global(g_);
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= C2) return;
    float s = 0.f;
    for (int n = 0; n < N; ++n) { const float v = g[(size_t)n * C2 + j]; s = fmaf(v, v, s); }
    s /= (float)N;
    if (fisher_diag) fisher_diag[j] = s;
    if (out) out[j] = grad[j] / (s + damping);
}

}  // namespace kfac

using namespace kfac;

static bool bn_item_ok(const kfac_bn_item& it) {
    if (!it.xhat || !it.gout || !it.g) return false;
    if (it.N <= 0 || it.C <= 0 || it.HW <= 0 || it.N > 65535 || it.C > 16384) return false;
    if (it.dtype != KFAC_F32 && it.dtype != KFAC_BF16 && it.dtype != KFAC_F16) return false;
    return (long long)it.N * it.C * it.HW <= 0x7fffffffLL;
}

static bool bn_item_vec(const kfac_bn_item& it) {
    return it.dtype != KFAC_F32 && (it.C & 7) == 0 && (((uintptr_t)it.xhat | (uintptr_t)it.gout) & 15) == 0;
}

// bytes of partial sums one layer needs (none when a single chunk covers all positions).  The 16-byte alignment of the
// tensors is not known when only the shape is: both cuttings are covered.
static size_t bn_item_ws(int N, int C, int HW, int dtype) {
    int nchunk = bn_plan(C, HW, false).nchunk;
    if (dtype != KFAC_F32 && (C & 7) == 0) nchunk = std::max(nchunk, bn_plan(C, HW, true).nchunk);
    return nchunk > 1 ? align_up((size_t)N * nchunk * 2 * C * sizeof(float), 256) : 0;
}

extern "C" size_t kfac_bn_sample_grads_batched_workspace_bytes(const kfac_bn_item* items_host, int32_t count) {
    if (!items_host || count <= 0) return 0;
    size_t total = 0;
    for (int i = 0; i < count; ++i) {
        const kfac_bn_item& it = items_host[i];
        if (it.N <= 0 || it.C <= 0 || it.HW <= 0) return 0;
        total += bn_item_ws(it.N, it.C, it.HW, it.dtype);
    }
    return total;
}

extern "C" int kfac_bn_sample_grads_batched(const kfac_bn_item* items_host, int32_t count, void* ws, size_t ws_bytes,
                                            void* stream) {
    if (!items_host || count < 0) return KFAC_ERR_INVALID_ARG;
    if (count == 0) return KFAC_OK;
    for (int i = 0; i < count; ++i)
        if (!bn_item_ok(items_host[i])) return KFAC_ERR_INVALID_ARG;
    const size_t need = kfac_bn_sample_grads_batched_workspace_bytes(items_host, count);
    if (need && (!ws || ((uintptr_t)ws & 255) || ws_bytes < need)) return KFAC_ERR_WORKSPACE;
    char* wsp = (char*)ws;
    for (int first = 0; first < count; first += BN_MAX) {
        const int cnt = count - first < BN_MAX ? count - first : BN_MAX;
        BnBatch b16, f16;                                 // bf16 and fp16 layers of this group
        BnReduceBatch rb;
        b16.count = f16.count = rb.count = 0;
        unsigned n16 = 0, nf16 = 0, nred = 0;
        for (int i = 0; i < cnt; ++i) {
            const kfac_bn_item& it = items_host[first + i];
            const bool vec = bn_item_vec(it);
            const BnPlan p = bn_plan(it.C, it.HW, vec);
            float* dst = it.g;
            if (p.nchunk > 1) {
                dst = (float*)wsp;
                const int k = rb.count++;
                rb.prefix[k] = nred;
                rb.C2[k] = 2 * it.C; rb.nchunk[k] = p.nchunk; rb.partial[k] = dst; rb.g[k] = it.g;
                nred += (unsigned)it.N * ((2 * it.C + 255) / 256);
            }
            wsp += bn_item_ws(it.N, it.C, it.HW, it.dtype);
            if (vec) {
                BnBatch& b = it.dtype == KFAC_F16 ? f16 : b16;
                unsigned& units = it.dtype == KFAC_F16 ? nf16 : n16;
                const int k = b.count++;
                b.prefix[k] = units;
                b.C[k] = it.C; b.HW[k] = it.HW; b.sp[k] = p.sp; b.nchunk[k] = p.nchunk;
                b.x[k] = it.xhat; b.gout[k] = it.gout; b.dst[k] = dst;
                units += (unsigned)it.N * p.nchunk * p.ncb;
            } else {
                KFAC_LAUNCH(bn_partial_generic_kernel, dim3(p.nchunk, it.N), dim3(256), (hipStream_t)stream, it.xhat, it.gout,
                            (int)it.dtype, (int)it.C, (int)it.HW, p.nchunk, dst);
            }
        }
        if (b16.count) {
            b16.prefix[b16.count] = n16;
            KFAC_LAUNCH(bn_partial_kernel<false>, dim3(n16), dim3(256), (hipStream_t)stream, b16);
        }
        if (f16.count) {
            f16.prefix[f16.count] = nf16;
            KFAC_LAUNCH(bn_partial_kernel<true>, dim3(nf16), dim3(256), (hipStream_t)stream, f16);
        }
        if (rb.count) {
            rb.prefix[rb.count] = nred;
            KFAC_LAUNCH(bn_reduce_kernel, dim3(nred), dim3(256), (hipStream_t)stream, rb);
        }
    }
    return KFAC_OK;
}

extern "C" size_t kfac_bn_sample_grads_workspace_bytes(int32_t N, int32_t C, int32_t HW) {
    if (N <= 0 || C <= 0 || HW <= 0) return 0;
    return std::max(bn_item_ws(N, C, HW, KFAC_BF16), bn_item_ws(N, C, HW, KFAC_F32));
}

extern "C" int kfac_bn_sample_grads(const void* xhat, const void* gout, int32_t N, int32_t C, int32_t HW, int32_t dtype,
                                    float* g, void* ws, size_t ws_bytes, void* stream) {
    const kfac_bn_item it = {xhat, gout, g, N, C, HW, dtype};
    return kfac_bn_sample_grads_batched(&it, 1, ws, ws_bytes, stream);
}

extern "C" int kfac_bn_diag_precondition(const float* g, int32_t N, int32_t C2, const float* grad, float damping,
                                         float* fisher_diag, float* out, void* stream) {
    if (!g || N <= 0 || C2 <= 0 || (!fisher_diag && !out) || (out && !grad)) return KFAC_ERR_INVALID_ARG;
    if (!(damping >= 0.f)) return KFAC_ERR_INVALID_ARG;
    KFAC_LAUNCH(bn_diag_kernel, dim3((C2 + 255) / 256), dim3(256), (hipStream_t)stream, g, N, C2, grad, damping, fisher_diag, out);
    return KFAC_OK;
}
