// Row classes of the data gradient: input pixels grouped by their residue modulo the stride.
// Shared by the host planner and the weight re-packing kernel so that both agree on the
// order and size of the per-class weight matrices.
#pragma once

#include <hip/hip_runtime.h>

namespace sol {

// Taps kh of a KH-tap filter that can reach input rows hi with hi % stride == phase
// (ho = (hi + pad - kh) / stride must be integral): kh = *first + stride * j, j < return value.
__host__ __device__ inline int class_taps(int KH, int stride, int pad, int phase, int* first) {
    const int f = (phase + pad) % stride;
    *first = f;
    return f < KH ? (KH - f + stride - 1) / stride : 0;
}

// Element offset of class (ph, pw)'s matrix [C_in][Th*Tw*C_out] inside the packed buffer.
__host__ __device__ inline long long class_weight_offset(int C_in, int C_out, int KH, int KW, int stride, int pad,
                                                         int ph, int pw) {
    long long off = 0;
    for (int c = 0; c < ph * stride + pw; ++c) {
        int f;
        off += (long long)C_in * C_out * class_taps(KH, stride, pad, c / stride, &f) *
               class_taps(KW, stride, pad, c % stride, &f);
    }
    return off;
}

}  // namespace sol
