// Exponential used by every softmax in the library (row softmax and the GEMM's softmax
// epilogue): exp(scale * t) for t <= 0 with a relative error near 2^-23 whatever the size
// of the exponent.
#pragma once
#include <cfloat>
#include <cmath>
#include "device_utils.h"

namespace perf {

// exp(s * t) for t <= 0 as exp2 of a compensated product: p = t*c_hi rounded, the
// rounding residual and the low part of the constant are applied as a first-order
// correction, so the relative error stays near 2^-23 for any exponent magnitude.
// Results below 2^-160 (far under the smallest fp32 subnormal) are returned as 0.
__device__ __forceinline__ float exp_scaled(float t, float c_hi, float c_lo)
{
    t = __builtin_fmaxf(t, -FLT_MAX);  // -inf * 0 would be NaN when scale == 0
    float p = t * c_hi;
    float r = __builtin_fmaf(t, c_hi, -p) + t * c_lo;
    float e = __builtin_amdgcn_exp2f(p);
    float v = __builtin_fmaf(e, r * 0.69314718056f, e);
    return p < -160.f ? 0.f : v;       // also discards the NaN residual of an overflowed p
}

struct ExpConst {
    float sign, c_hi, c_lo;
};

static inline ExpConst make_exp_const(float scale)
{
    // |scale| * log2(e) split into an fp32 head and tail.
    double c = std::fabs((double)scale) * 1.4426950408889634074;
    ExpConst k;
    k.sign = scale < 0.f ? -1.f : 1.f;
    k.c_hi = (float)c;
    k.c_lo = (float)(c - (double)k.c_hi);
    return k;
}

}  // namespace perf
