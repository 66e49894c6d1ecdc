// Reconstruction of packed tokens, X^ = M[k*] + (s*code + z) (the rule below Eq. 6 of
// Sec. 3.2), in binary32 and in exactly that order: multiply, add, add.  Used by the
// parity tests and for debugging; the decode path never reconstructs vectors in memory.
#pragma clang fp contract(off)

#include "pk_internal.h"

namespace pk {

namespace {

template <int BITS>
__global__ __launch_bounds__(128) void dequant_kernel(DequantArgs a)
{
    const int t = a.t0 + blockIdx.x, n = blockIdx.y, c = threadIdx.x;
    const int set = a.sets.set_of(n);
    const int G = a.G, Gc = G < kD ? G : kD, ng = kD / Gc;
    const int64_t tok = a.c.map.pos(n, t);   // where token t of the stream is stored
    const int64_t orow = ((int64_t)n * (a.t1 - a.t0) + (t - a.t0)) * kD + c;
    if (a.k_out) {
        int code = 0;
#pragma unroll
        for (int j = 0; j < BITS; ++j)
            code |= (int)((a.c.k_codes[(tok * 4 + (c >> 5)) * BITS + j] >> (c & 31)) & 1u) << j;
        const int64_t prow = (tok / G) * kD + c;
        const float s = h2f(a.c.k_scale[prow]), z = h2f(a.c.k_zero[prow]);
        const float res = s * (float)code + z;
        a.k_out[orow] = h2f(a.patterns_k[((int64_t)set * a.P + a.c.k_idx[tok]) * kD + c]) + res;
    }
    if (a.v_out) {
        const uint32_t *vbase = reinterpret_cast<const uint32_t *>(a.c.v_codes);
        const int64_t word = (((tok >> 4) * 16 + (c & 15)) * (kD / 16) + (c >> 4)) * (BITS / 2);
        int code = 0;
#pragma unroll
        for (int j = 0; j < BITS; ++j) code |= (int)((vbase[word + j / 2] >> (16 * (j % 2) + (t & 15))) & 1u) << j;
        const int64_t prow = ((tok >> 4) * ng + c / Gc) * 16 + (t & 15);
        const float s = h2f(a.c.v_scale[prow]), z = h2f(a.c.v_zero[prow]);
        const float res = s * (float)code + z;
        const int vi = a.c.v_idx[tok];
        if (a.v_thresholded && vi == PK_NO_PATTERN)
            a.v_out[orow] = res;   // quantized without a pattern (adaptive threshold, Sec. 3.3)
        else
            a.v_out[orow] = h2f(a.patterns_v[((int64_t)set * a.P + vi) * kD + c]) + res;
    }
}

}  // namespace

hipError_t launch_dequant(const DequantArgs &a, hipStream_t s)
{
    if (a.d != kD) return launch_generic_dequant(a, s);
    if (a.t1 <= a.t0) return hipSuccess;
    const dim3 grid(a.t1 - a.t0, a.n_streams), block(128);
    if (a.bits == 2)
        hipLaunchKernelGGL((dequant_kernel<2>), grid, block, 0, s, a);
    else
        hipLaunchKernelGGL((dequant_kernel<4>), grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace pk
