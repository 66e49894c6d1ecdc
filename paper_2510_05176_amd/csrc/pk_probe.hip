// Machine-peak probes (include/patternkv_probe.h): streaming read, streaming copy, an fp32 FMA loop and an
// fp16 MFMA loop.  Measurement aids for the benchmark; the hot path does not use them.
#pragma clang fp contract(off)   // as in the quantizer: the division sequences below run exactly as written

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "patternkv_probe.h"
#include "pk_divide.h"

namespace {

constexpr int kGroups = 2048;

typedef _Float16 half8p __attribute__((ext_vector_type(8)));
typedef float floatx4p __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void probe_read_kernel(const uint4 *src, size_t n16, uint4 *sink)
{
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    // four loads in flight per thread and round
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc.x ^= a.x ^ b.x ^ c.x ^ d.x;
        acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
        acc.z ^= a.z ^ b.z ^ c.z ^ d.z;
        acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = src[i];
        acc.x ^= a.x;
        acc.y ^= a.y;
        acc.z ^= a.z;
        acc.w ^= a.w;
    }
    // one lane per workgroup whose checksum words differ writes (in practice: thread 0 of most groups); the
    // value depends on every load, so none can be dropped
    for (int off = 32; off > 0; off >>= 1) {
        acc.x ^= __shfl_xor((int)acc.x, off);
        acc.y ^= __shfl_xor((int)acc.y, off);
        acc.z ^= __shfl_xor((int)acc.z, off);
        acc.w ^= __shfl_xor((int)acc.w, off);
    }
    if (threadIdx.x == 0) sink[blockIdx.x] = acc;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(uint4 *dst, const uint4 *src, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a;
        dst[i + stride] = b;
        dst[i + 2 * stride] = c;
        dst[i + 3 * stride] = d;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void probe_fma_kernel(float *sink, int iters)
{
    float a[16];
    const float x = 1.0f + 1e-7f * (float)threadIdx.x, y = 1e-9f * (float)blockIdx.x;
#pragma unroll
    for (int k = 0; k < 16; ++k) a[k] = (float)k;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 16; ++k) a[k] = __builtin_fmaf(a[k], x, y);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) s += a[k];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void probe_mfma_kernel(float *sink, int iters)
{
    half8p a, b;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        a[k] = (_Float16)(0.001f * (float)((threadIdx.x + k) & 7));
        b[k] = (_Float16)(0.002f * (float)((threadIdx.x + 3 * k) & 7));
    }
    floatx4p acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = floatx4p{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[k], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) s += acc[k][0] + acc[k][1] + acc[k][2] + acc[k][3];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// the quantizer's two division sequences, evaluated on plain arrays
__global__ __launch_bounds__(256) void probe_divisions_kernel(const float *x, size_t n, float *recip, float *by3, float *by15)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const float v = x[i];
        recip[i] = pk::recip_of_scale(v);
        by3[i] = pk::div_by_levels(v, 2);
        by15[i] = pk::div_by_levels(v, 4);
    }
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

int pk_probe_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink || bytes == 0 || bytes % 16 != 0 || !aligned16(src) || !aligned16(sink)) return 1;
    hipLaunchKernelGGL(probe_read_kernel, dim3(kGroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), bytes / 16, static_cast<uint4 *>(sink));
    return hipGetLastError() == hipSuccess ? 0 : 8;
}

int pk_probe_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!src || !dst || bytes == 0 || bytes % 16 != 0 || !aligned16(src) || !aligned16(dst)) return 1;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(kGroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 8;
}

int pk_probe_fma_f32(float *sink, int32_t iters, void *stream)
{
    if (!sink || iters < 1 || !aligned16(sink)) return 1;
    hipLaunchKernelGGL(probe_fma_kernel, dim3(kGroups), dim3(256), 0, static_cast<hipStream_t>(stream), sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : 8;
}

int pk_probe_mfma_f16(float *sink, int32_t iters, void *stream)
{
    if (!sink || iters < 1 || !aligned16(sink)) return 1;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(kGroups), dim3(256), 0, static_cast<hipStream_t>(stream), sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : 8;
}

int pk_probe_divisions(const float *x, size_t n, float *recip, float *by3, float *by15, void *stream)
{
    if (!x || !recip || !by3 || !by15 || n == 0) return 1;
    hipLaunchKernelGGL(probe_divisions_kernel, dim3(kGroups), dim3(256), 0, static_cast<hipStream_t>(stream), x, n, recip, by3, by15);
    return hipGetLastError() == hipSuccess ? 0 : 8;
}

}  // extern "C"
