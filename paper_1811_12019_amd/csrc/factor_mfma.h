// Helpers of the matrix-core factor builder: the 16-bit MFMA wrapper and the decoding of an 8-column group of the
// unfolded matrix into (kernel tap, channel offset).
#pragma once

#include "common.h"

namespace kfac {

constexpr int FT = 128;               // tile edge
constexpr int FEPI_LD = 65;           // epilogue staging: per-wavefront 32 x 64 floats, padded rows

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

}  // namespace kfac
