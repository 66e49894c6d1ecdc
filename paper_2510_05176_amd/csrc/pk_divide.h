// The two divisions of the quantization parameters (Sec. 2.1 Eq. 1: s = (max - z) / (2^b - 1), and 1/s for the
// codes), each correctly rounded like the IEEE binary32 operation but in three instructions.
#pragma once

#include <hip/hip_runtime.h>

namespace pk {

// 1/s for a positive fp16-representable s: a reciprocal estimate and one Newton correction.
// Checked against IEEE division for every positive fp16 value (tests, through pk_probe_divisions).
__device__ __forceinline__ float recip_of_scale(float s)
{
    const float r = __builtin_amdgcn_rcpf(s);
    const float e = fmaf(-s, r, 1.f);
    const float q = fmaf(e, r, r);
    return s < INFINITY ? q : 0.f;   // a scale that overflowed fp16: 1/inf
}

// x / (2^bits - 1) for finite x >= 0: a multiply by the rounded reciprocal of the constant and one residual
// correction.  Checked against IEEE division over all 2^23 mantissas of several binades, divisors 3 and 15.
__device__ __forceinline__ float div_by_levels(float x, int bits)
{
    const float L = (float)((1 << bits) - 1), c = 1.0f / L;   // c: compile-time rounded reciprocal
    const float q = x * c;
    const float r = fmaf(-L, q, x);
    return fmaf(r, c, q);
}

}  // namespace pk
