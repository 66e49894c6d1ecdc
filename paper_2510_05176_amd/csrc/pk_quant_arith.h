// The stored parameters of a quantization group and the code of one residual (Sec. 2.1 Eq. 1 with this build's
// rounding rules: z = group minimum rounded to fp16 towards -inf, s = (max - z) / (2^b - 1) rounded to fp16 towards
// +inf, code = clamp(rint((r - z) * (1/s)), 0, 2^b - 1) in binary32, ties to even; s == 0 gives code 0).  Shared by
// the tuned quantizers (head dimension 128) and the generic ones; files that use it switch FMA contraction off.
#pragma once

#include "pk_divide.h"
#include "pk_internal.h"

namespace pk {

struct GroupParams {
    unsigned short s16, z16;
    float s, z, inv;
};

__device__ __forceinline__ GroupParams group_params(float mn, float mx, int bits)
{
    GroupParams g;
    g.z16 = f2h_down(mn);
    g.z = hbits2f(g.z16);
    const float s32 = div_by_levels(mx - g.z, bits);
    g.s16 = f2h_up(s32);
    g.s = hbits2f(g.s16);
    g.inv = g.s == 0.f ? 0.f : recip_of_scale(g.s);
    return g;
}

__device__ __forceinline__ int quantize_one(float r, const GroupParams &g, int bits)
{
    if (g.s == 0.f) return 0;
    float q = rintf((r - g.z) * g.inv);
    const float qmax = (float)((1 << bits) - 1);
    q = fminf(fmaxf(q, 0.f), qmax);
    return (int)q;
}

}  // namespace pk
