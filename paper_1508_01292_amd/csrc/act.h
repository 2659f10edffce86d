// Activation functions of the cascade networks (paper, Section 3.1, eq. (1)).
#pragma once
#include <hip/hip_runtime.h>

#include "cnnc.h"

namespace cnnc {

// f(x) = 1.7159 * t(2x/3); t is the paper's rational stand-in for tanh,
// t(y) = sgn(y) * (1 - 1/(1 + |y| + y^2 + 1.41645 y^4)), evaluated as N / (1 + N) with
// N = |y| + y^2 + 1.41645 y^4 so that small arguments lose no digits.
// All three forms are non-decreasing, so they commute with max-pooling.
template <int ACT>
__device__ __forceinline__ float act_f(float x)
{
    if (ACT == CNNC_ACT_RATIONAL) {
        const float y = x * 0.66666667f;
        const float a = fabsf(y), y2 = y * y;
        const float n = a + fmaf(1.41645f, y2 * y2, y2);
        const float t = n * __builtin_amdgcn_rcpf(1.0f + n);
        return copysignf(1.7159f * t, y);
    } else if (ACT == CNNC_ACT_SCALED_TANH) {
        return 1.7159f * tanhf(x * 0.66666667f);
    } else if (ACT == CNNC_ACT_TANH) {
        return tanhf(x);
    }
    return x;
}

// Pixel value (possibly a blend, 0..255) to network input.
__device__ __forceinline__ float normalise(float p) { return (p - 128.0f) * 0.0078125f; }

}  // namespace cnnc
