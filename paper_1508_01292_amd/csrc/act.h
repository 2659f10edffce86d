// Activation functions of the cascade networks (paper, Section 3.1, eq. (1)).
#pragma once
#include <hip/hip_runtime.h>

#include "cnnc.h"

namespace cnnc {

// f(x) = 1.7159 * t(2x/3); t is the paper's rational stand-in for tanh,
// t(y) = sgn(y) * (1 - 1/(1 + |y| + y^2 + 1.41645 y^4)).  With y = 2x/3 folded into the coefficients the
// denominator is d = 1 + |x| (2/3 + |x| (4/9 + (1.41645 * 16/81) x^2)), three fused multiply-adds after x^2, and
// f = sgn(x) (1.7159 - 1.7159 / d): seven instructions, one of them the reciprocal.  Absolute error about 2e-7
// (rounding of the final subtraction and of v_rcp_f32), far inside what the later layers need.
// All three forms are non-decreasing, so they commute with max-pooling.
template <int ACT>
__device__ __forceinline__ float act_f(float x)
{
    if (ACT == CNNC_ACT_RATIONAL) {
        const float a = fabsf(x);
        const float d = fmaf(fmaf(fmaf(1.41645f * 16.0f / 81.0f, x * x, 4.0f / 9.0f), a, 2.0f / 3.0f), a, 1.0f);
        return copysignf(fmaf(-1.7159f, __builtin_amdgcn_rcpf(d), 1.7159f), x);
    } else if (ACT == CNNC_ACT_SCALED_TANH) {
        return 1.7159f * tanhf(x * 0.66666667f);
    } else if (ACT == CNNC_ACT_TANH) {
        return tanhf(x);
    }
    return x;
}

// The value that the neighbouring lane (lane ^ 1) holds: a DPP move inside the quad, on the vector ALU, instead of the
// trip through the LDS crossbar that a general shuffle takes.
__device__ __forceinline__ float lane_xor1(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1 /* quad_perm [1, 0, 3, 2] */, 0xF, 0xF, true));
}

// Pixel value (possibly a blend, 0..255) to network input.
__device__ __forceinline__ float normalise(float p) { return (p - 128.0f) * 0.0078125f; }

}  // namespace cnnc
