// Quantize-append kernels: pattern selection (Sec. 3.2 Eq. 6), residual, group
// min/max -> stored (s, z), asymmetric n-bit quantization (Sec. 2.1 Eq. 1), bit-plane
// packing.  K is quantized per channel over groups of G tokens, V per token over
// groups of Gc channels (Sec. 4.1 "Quantization Settings").
//
// The arithmetic that decides a code is a fixed sequence of binary32 operations
// (subtract, one division per group for s, one for 1/s, subtract, multiply, round
// half to even, clamp); contraction into FMAs is switched off for this file so
// that the sequence is exactly what is written.
#pragma clang fp contract(off)

#include "pk_assign.h"
#include "pk_internal.h"

namespace pk {

namespace {

struct GroupParams {
    unsigned short s16, z16;
    float s, z, inv;
};

__device__ __forceinline__ GroupParams group_params(float mn, float mx, int bits)
{
    GroupParams g;
    g.z16 = f2h_down(mn);
    g.z = hbits2f(g.z16);
    const float s32 = (mx - g.z) / (float)((1 << bits) - 1);
    g.s16 = f2h_up(s32);
    g.s = hbits2f(g.s16);
    g.inv = g.s == 0.f ? 0.f : 1.0f / g.s;
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

// ---------------------------------------------------------------------------
// K: one workgroup (128 threads) per (group of G tokens, stream).
// ---------------------------------------------------------------------------
template <int G, int BITS>
__global__ __launch_bounds__(128) void quantize_k_kernel(QuantArgs a)
{
    __shared__ __align__(16) __half xs[G * kXsStride];
    __shared__ AssignScratch sc;
    __shared__ int idx_s[G];
    __shared__ __align__(16) uint32_t pack_s[G * 4 * BITS];

    const int g = blockIdx.x, n = blockIdx.y, tid = threadIdx.x;
    const __half *Mg = a.patterns + (int64_t)a.sets.set_of(n) * a.P * kD;

    stage_rows(xs, G, [&](int r) { return a.src.row(n, g * G + r); });
    // assign_tile starts with a barrier that also publishes xs
    assign_tile<G>(xs, G, Mg, a.P, a.metric, sc, idx_s, nullptr);

    const int64_t tq = (int64_t)a.t0 + (int64_t)g * G;   // first packed position of this group
    if (tid < G) a.idx[(int64_t)n * a.t_capacity + tq + tid] = (uint8_t)idx_s[tid];

    // thread <-> channel
    const int c = tid;
    float mn = INFINITY, mx = -INFINITY;
    for (int t = 0; t < G; ++t) {
        const float r = h2f(xs[t * kXsStride + c]) - h2f(Mg[(int64_t)idx_s[t] * kD + c]);
        mn = fminf(mn, r);
        mx = fmaxf(mx, r);
    }
    const GroupParams gp = group_params(mn, mx, BITS);
    const int64_t grow = ((int64_t)n * (a.t_capacity / G) + tq / G) * kD + c;
    a.scale[grow] = __ushort_as_half(gp.s16);
    a.zero[grow] = __ushort_as_half(gp.z16);

    const int wave = tid >> 6, lane = tid & 63;
    for (int t = 0; t < G; ++t) {
        const float r = h2f(xs[t * kXsStride + c]) - h2f(Mg[(int64_t)idx_s[t] * kD + c]);
        const int code = quantize_one(r, gp, BITS);
#pragma unroll
        for (int j = 0; j < BITS; ++j) {
            const unsigned long long m = __ballot((code >> j) & 1);
            if (lane == 0) {
                pack_s[(t * 4 + 2 * wave) * BITS + j] = (uint32_t)m;
                pack_s[(t * 4 + 2 * wave + 1) * BITS + j] = (uint32_t)(m >> 32);
            }
        }
    }
    __syncthreads();
    uint4 *dst = reinterpret_cast<uint4 *>(a.codes_k + ((int64_t)n * a.t_capacity + tq) * 4 * BITS);
    const uint4 *srcp = reinterpret_cast<const uint4 *>(pack_s);
    for (int i = tid; i < G * BITS; i += 128) dst[i] = srcp[i];
}

// ---------------------------------------------------------------------------
// V: one workgroup (128 threads) per (block of 64 tokens, stream).
// ---------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(128) void quantize_v_kernel(QuantArgs a)
{
    constexpr int TV = 64;
    constexpr int WPU = BITS / 2;   // 32-bit words per (channel, 16-token unit)
    __shared__ __align__(16) __half xs[TV * kXsStride];
    __shared__ AssignScratch sc;
    __shared__ int idx_s[TV];
    __shared__ float red_mn[TV][4], red_mx[TV][4];
    __shared__ __align__(16) uint32_t out_s[TV * kD * BITS / 32];
    __shared__ __align__(16) unsigned short par_s[2][4 * 4 * 16];   // scale / zero slices: [unit][group][16]

    const int tile = blockIdx.x, n = blockIdx.y, tid = threadIdx.x;
    const __half *Mg = a.patterns + (int64_t)a.sets.set_of(n) * a.P * kD;

    stage_rows(xs, TV, [&](int r) { return a.src.row(n, tile * TV + r); });
    assign_tile<TV>(xs, TV, Mg, a.P, a.metric, sc, idx_s, nullptr);

    const int64_t tq = (int64_t)a.t0 + (int64_t)tile * TV;
    if (tid < TV) a.idx[(int64_t)n * a.t_capacity + tq + tid] = (uint8_t)idx_s[tid];

    const int c = tid, lane = tid & 63, quarter = tid >> 5;
    // phase A: min / max of every 32-channel quarter of every token
    for (int t = 0; t < TV; ++t) {
        const float r = h2f(xs[t * kXsStride + c]) - h2f(Mg[(int64_t)idx_s[t] * kD + c]);
        float mn = r, mx = r;
#pragma unroll
        for (int off = 1; off < 32; off <<= 1) {
            mn = fminf(mn, __shfl_xor(mn, off));
            mx = fmaxf(mx, __shfl_xor(mx, off));
        }
        if ((lane & 31) == 0) {
            red_mn[t][quarter] = mn;
            red_mx[t][quarter] = mx;
        }
    }
    __syncthreads();
    // phase B: stored parameters, codes, bit planes along the tokens (16 tokens per word)
    const int Gc = a.G < kD ? a.G : kD;
    const int ng = kD / Gc, qpg = Gc / 32;   // channel groups per token, quarters per group
    const int grp = c / Gc;
    uint32_t acc[BITS];
#pragma unroll
    for (int j = 0; j < BITS; ++j) acc[j] = 0;
    for (int t = 0; t < TV; ++t) {
        float mn = red_mn[t][grp * qpg], mx = red_mx[t][grp * qpg];
        for (int k = 1; k < qpg; ++k) {
            mn = fminf(mn, red_mn[t][grp * qpg + k]);
            mx = fmaxf(mx, red_mx[t][grp * qpg + k]);
        }
        const GroupParams gp = group_params(mn, mx, BITS);
        if (c % Gc == 0) {
            par_s[0][((t >> 4) * ng + grp) * 16 + (t & 15)] = gp.s16;
            par_s[1][((t >> 4) * ng + grp) * 16 + (t & 15)] = gp.z16;
        }
        const float r = h2f(xs[t * kXsStride + c]) - h2f(Mg[(int64_t)idx_s[t] * kD + c]);
        const int code = quantize_one(r, gp, BITS);
#pragma unroll
        for (int j = 0; j < BITS; ++j) acc[j] |= (uint32_t)((code >> j) & 1) << (t & 15);
        if ((t & 15) == 15) {
            const int unit = t >> 4;   // 16-token unit inside the block
#pragma unroll
            for (int w = 0; w < WPU; ++w) {
                out_s[((unit * 16 + (c & 15)) * (kD / 16) + (c >> 4)) * WPU + w] = acc[2 * w] | (acc[2 * w + 1] << 16);
                acc[2 * w] = acc[2 * w + 1] = 0;
            }
        }
    }
    __syncthreads();
    uint4 *dst = reinterpret_cast<uint4 *>(a.codes_v + ((int64_t)n * a.t_capacity + tq) * (kD * BITS / 8));
    const uint4 *srcp = reinterpret_cast<const uint4 *>(out_s);
    for (int i = tid; i < TV * kD * BITS / 8 / 16; i += 128) dst[i] = srcp[i];
    // parameters of the block: 4 units x ng groups x 16 tokens, contiguous in memory
    const int npar = 4 * ng * 16;
    const int64_t pbase = ((int64_t)n * a.t_capacity + tq) * ng;
    for (int i = tid; i < npar; i += 128) {
        a.scale[pbase + i] = __ushort_as_half(par_s[0][i]);
        a.zero[pbase + i] = __ushort_as_half(par_s[1][i]);
    }
}

// ---------------------------------------------------------------------------
// Tail ring: place logical vectors [i0, i1) of an append into their ring slots.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void tail_copy_kernel(TailCopyArgs a)
{
    const int n = blockIdx.y, side = blockIdx.z;
    const int64_t work = (int64_t)(a.i1 - a.i0) * kRowChunks;
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (w >= work) return;
    const int i = a.i0 + (int)(w >> 4), ch = (int)(w & 15);
    const __half *fresh = side == 0 ? a.fresh_k : a.fresh_v;
    __half *ring = side == 0 ? a.ring_k : a.ring_v;
    const uint4 v = *reinterpret_cast<const uint4 *>(fresh + (int64_t)n * a.fresh_stride +
                                                     (int64_t)(i - a.n_ring) * kD + ch * 8);
    const int slot = (int)(((int64_t)a.ring_start + i) % a.ring_len);
    *reinterpret_cast<uint4 *>(ring + ((int64_t)n * a.ring_len + slot) * kD + ch * 8) = v;
}

}  // namespace

hipError_t launch_quantize_k(const QuantArgs &a, hipStream_t s)
{
    const dim3 grid(a.nq / a.G, a.n_streams), block(128);
#define PK_LAUNCH_K(GG, BB)                                                        \
    if (a.G == GG && a.bits == BB) {                                               \
        hipLaunchKernelGGL((quantize_k_kernel<GG, BB>), grid, block, 0, s, a);     \
        return hipGetLastError();                                                  \
    }
    PK_LAUNCH_K(32, 2) PK_LAUNCH_K(64, 2) PK_LAUNCH_K(128, 2)
    PK_LAUNCH_K(32, 4) PK_LAUNCH_K(64, 4) PK_LAUNCH_K(128, 4)
#undef PK_LAUNCH_K
    return hipErrorInvalidValue;
}

hipError_t launch_quantize_v(const QuantArgs &a, hipStream_t s)
{
    const dim3 grid(a.nq / 64, a.n_streams), block(128);
    if (a.bits == 2)
        hipLaunchKernelGGL((quantize_v_kernel<2>), grid, block, 0, s, a);
    else if (a.bits == 4)
        hipLaunchKernelGGL((quantize_v_kernel<4>), grid, block, 0, s, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_tail_copy(const TailCopyArgs &a, hipStream_t s)
{
    const int64_t work = (int64_t)(a.i1 - a.i0) * kRowChunks;
    if (work <= 0) return hipSuccess;
    const dim3 grid((unsigned)((work + 255) / 256), a.n_streams, 2), block(256);
    hipLaunchKernelGGL(tail_copy_kernel, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace pk
