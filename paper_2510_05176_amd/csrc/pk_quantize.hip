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
#include "pk_assign_mfma.h"
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
__global__ __launch_bounds__(128) void quantize_k_valu_kernel(QuantArgs a)
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
__global__ __launch_bounds__(128) void quantize_v_valu_kernel(QuantArgs a)
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


// ===========================================================================
// Euclidean metric: nearest pattern on the matrix cores (pk_assign_mfma.h), then residuals are
// staged in LDS as binary32 and quantized with one thread per channel (K) or per token (V), so
// that the group minimum / maximum is a sequential scan inside a thread and every bit plane is
// one ballot across the lanes.
// ===========================================================================

constexpr int kRStride = kD + 4;   // floats per row of the residual tile (16-byte aligned rows)
constexpr float kRoundMagic = 8388608.f;   // y + 2^23 has rint(y) in its low mantissa bits (0 <= y < 2^22)

// x - m for the low / high halves of two packed fp16 pairs: one v_fma_mix_f32 (x*1.0 + (-m) with fp16
// sources widened exactly), i.e. the binary32 subtraction of the two converted values.
__device__ __forceinline__ float sub_lo(uint32_t x, uint32_t m)
{
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,0] op_sel_hi:[1,0,1]" : "=v"(r) : "v"(x), "v"(m));
    return r;
}
__device__ __forceinline__ float sub_hi(uint32_t x, uint32_t m)
{
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[1,0,1] op_sel_hi:[1,0,1]" : "=v"(r) : "v"(x), "v"(m));
    return r;
}

// Code of one residual from the stored parameters: the low bits of the returned word.
// (r - z) * (1/s) lies in [0, 2^b - 1] up to rounding because z <= min and s >= (max - z)/(2^b - 1),
// so the clamp of the definition never acts; the caller keeps only the low b bits.
__device__ __forceinline__ uint32_t code_word(float r, const GroupParams &g)
{
    const float y = (r - g.z) * g.inv;
    return __float_as_uint(y + kRoundMagic);   // round half to even, as rintf
}

struct TileShared {
    // carved from dynamic LDS by the kernels below
    __half *tab;               // [P][kTabStride]   (TAB_LDS only)
    float *norm;               // [P rounded up to 16]
    float *rt;                 // [TT][kRStride]
    __half *xrow;              // [4][kD]
    float *stat;               // K: [2][2][kD]; V: [64][4][2]
    unsigned long long *mask;  // plane masks: K [4 waves][HT][BITS]; V [kD][BITS]
    int *idx;                  // [TT]
};

template <int TT, bool TAB_LDS>
__device__ __forceinline__ TileShared carve(unsigned char *smem, int P)
{
    TileShared t;
    size_t o = 0;
    t.tab = reinterpret_cast<__half *>(smem);
    if (TAB_LDS) o += (size_t)P * kTabStride * 2;
    t.norm = reinterpret_cast<float *>(smem + o);
    o += (size_t)((P + 15) / 16 * 16) * 4;
    t.rt = reinterpret_cast<float *>(smem + o);
    o += (size_t)TT * kRStride * 4;
    t.xrow = reinterpret_cast<__half *>(smem + o);
    o += 4 * kD * 2;
    t.stat = reinterpret_cast<float *>(smem + o);
    o += 512 * 4;
    t.mask = reinterpret_cast<unsigned long long *>(smem + o);
    o += 4 * 64 * 4 * 8;
    t.idx = reinterpret_cast<int *>(smem + o);
    return t;
}
template <int TT>
size_t tile_lds_bytes(int P, bool tab_lds)
{
    return (tab_lds ? (size_t)P * kTabStride * 2 : 0) + (size_t)((P + 15) / 16 * 16) * 4 + (size_t)TT * kRStride * 4 +
           4 * kD * 2 + 512 * 4 + 4 * 64 * 4 * 8 + TT * 4;
}

// B operands of the NT 16-token tiles of this wave.
template <int NT>
__device__ __forceinline__ void load_tiles(const QuantArgs &a, int ns, int i0, uint4 (&xb)[NT][4])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 15, kb = lane >> 4;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const __half *row = a.src.row(ns, i0 + (wave * NT + j) * 16 + n);
#pragma unroll
        for (int k = 0; k < 4; ++k) xb[j][k] = *reinterpret_cast<const uint4 *>(row + 32 * k + 8 * kb);
    }
}

// Assign the NT 16-token tiles of this wave, write the indices, stage the residuals.
// tq0 = packed position of the first vector of the workgroup's tile.
template <int NT, bool TAB_LDS>
__device__ __forceinline__ void assign_and_stage(const QuantArgs &a, const TileShared &sh, const PatternTable &tb,
                                                 const __half *Mg, int ns, int64_t tq0, const uint4 (&xb)[NT][4])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 15, kb = lane >> 4;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int tl = (wave * NT + j) * 16 + n;   // token slot inside the tile
        int bi;
        float bv, x2, bd;
        bool flag;
        assign_tile_mfma<TAB_LDS>(xb[j], tb, lane, bi, bv, x2, flag);
        resolve_flagged(xb[j], flag, sh.xrow + wave * kD, tb, Mg, lane, bi, bd);
        if (kb == 0) {
            sh.idx[tl] = bi;
            a.idx[(int64_t)ns * a.t_capacity + tq0 + tl] = (uint8_t)bi;
        }
        // residual r = x - M[k*] of this lane's 32 channels, one binary32 subtraction each
        const __half *mrow = TAB_LDS ? sh.tab + bi * kTabStride + 8 * kb : Mg + (int64_t)bi * kD + 8 * kb;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint4 mv = *reinterpret_cast<const uint4 *>(mrow + 32 * k);
            const uint4 xv = xb[j][k];
            float4 r0, r1;
            r0.x = sub_lo(xv.x, mv.x);
            r0.y = sub_hi(xv.x, mv.x);
            r0.z = sub_lo(xv.y, mv.y);
            r0.w = sub_hi(xv.y, mv.y);
            r1.x = sub_lo(xv.z, mv.z);
            r1.y = sub_hi(xv.z, mv.z);
            r1.z = sub_lo(xv.w, mv.w);
            r1.w = sub_hi(xv.w, mv.w);
            float4 *dst = reinterpret_cast<float4 *>(sh.rt + tl * kRStride + 32 * k + 8 * kb);
            dst[0] = r0;
            dst[1] = r1;
        }
    }
}

// Plane j of the codes in `ub` across the wave: one compare for the top plane, mask-and-compare below.
template <int BITS>
__device__ __forceinline__ unsigned long long plane_mask(uint32_t ub, int j)
{
    if (j == BITS - 1) return __ballot((ub & ((1u << BITS) - 1u)) >= (1u << (BITS - 1)));
    return __ballot((ub & (1u << j)) != 0u);
}

// K: workgroup = 256 threads, tiles of TT = max(64, G) tokens of one stream.
template <int G, int BITS, bool TAB_LDS>
__global__ __launch_bounds__(256) void quantize_k_kernel(QuantArgs a, int tiles_per_wg)
{
    constexpr int TT = G == 128 ? 128 : 64, NT = TT / 64, HT = TT / 2;
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ float red_s[4];
    const TileShared sh = carve<TT, TAB_LDS>(smem, a.P);
    const int tid = threadIdx.x, ns = blockIdx.y;
    const __half *Mg = a.patterns + (int64_t)a.sets.set_of(ns) * a.P * kD;
    const int n_tiles = a.nq / TT;
    const int tile0 = blockIdx.x * tiles_per_wg, tile1 = min(n_tiles, tile0 + tiles_per_wg);
    uint4 xb[NT][4];
    load_tiles<NT>(a, ns, tile0 * TT, xb);   // in flight while the table is staged

    stage_patterns(Mg, a.P, sh.tab, sh.norm, red_s, TAB_LDS);
    PatternTable tb;
    tb.lds_rows = sh.tab;
    tb.glb_rows = Mg;
    tb.norm2 = sh.norm;
    tb.norm2_max = fmaxf(fmaxf(red_s[0], red_s[1]), fmaxf(red_s[2], red_s[3]));
    tb.P = a.P;

    const int c = tid & 127, half = tid >> 7, lane = tid & 63, wave = tid >> 6, chw = wave & 1;
    unsigned long long *mask_w = sh.mask + wave * (64 * 4);
    for (int tile = tile0; tile < tile1; ++tile) {
        const int64_t tq0 = (int64_t)a.t0 + (int64_t)tile * TT;
        assign_and_stage<NT, TAB_LDS>(a, sh, tb, Mg, ns, tq0, xb);
        __syncthreads();
        if (tile + 1 < tile1) load_tiles<NT>(a, ns, (tile + 1) * TT, xb);   // next tile's vectors: hidden behind the scan

        // thread <-> (channel c, token half): scan HT tokens
        float r[HT];
        float mn = INFINITY, mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < HT; t += 2) {
            r[t] = sh.rt[(half * HT + t) * kRStride + c];
            r[t + 1] = sh.rt[(half * HT + t + 1) * kRStride + c];
            mn = fminf(fminf(mn, r[t]), r[t + 1]);
            mx = fmaxf(fmaxf(mx, r[t]), r[t + 1]);
        }
        if (G > HT) {   // the group spans both halves
            sh.stat[(half * 2 + 0) * kD + c] = mn;
            sh.stat[(half * 2 + 1) * kD + c] = mx;
            __syncthreads();
            mn = fminf(mn, sh.stat[((half ^ 1) * 2 + 0) * kD + c]);
            mx = fmaxf(mx, sh.stat[((half ^ 1) * 2 + 1) * kD + c]);
        }
        const GroupParams gp = group_params(mn, mx, BITS);
        if (G <= HT || half == 0) {
            const int64_t grow = ((int64_t)ns * (a.t_capacity / G) + tq0 / G + (G <= HT ? half : 0)) * kD + c;
            a.scale[grow] = __ushort_as_half(gp.s16);
            a.zero[grow] = __ushort_as_half(gp.z16);
        }
        // codes; one ballot per plane = the plane words of this wave's 64 channels for one token
#pragma unroll
        for (int t = 0; t < HT; ++t) {
            const uint32_t ub = code_word(r[t], gp);
#pragma unroll
            for (int j = 0; j < BITS; ++j) {
                const unsigned long long m = plane_mask<BITS>(ub, j);
                if (lane == 0) mask_w[t * BITS + j] = m;
            }
        }
        // lane t of the wave writes token t: K row = [word w][plane j], this wave owns words 2*chw, 2*chw+1
        if (lane < HT) {
            unsigned long long m[BITS];
#pragma unroll
            for (int j = 0; j < BITS; ++j) m[j] = mask_w[lane * BITS + j];
            uint32_t *dst = a.codes_k + (((int64_t)ns * a.t_capacity + tq0 + half * HT + lane) * 4 + 2 * chw) * BITS;
            if (BITS == 2) {
                *reinterpret_cast<uint4 *>(dst) =
                    make_uint4((uint32_t)m[0], (uint32_t)m[1], (uint32_t)(m[0] >> 32), (uint32_t)(m[1] >> 32));
            } else {
                reinterpret_cast<uint4 *>(dst)[0] =
                    make_uint4((uint32_t)m[0], (uint32_t)m[1], (uint32_t)m[BITS - 2], (uint32_t)m[BITS - 1]);
                reinterpret_cast<uint4 *>(dst)[1] = make_uint4((uint32_t)(m[0] >> 32), (uint32_t)(m[1] >> 32),
                                                               (uint32_t)(m[BITS - 2] >> 32), (uint32_t)(m[BITS - 1] >> 32));
            }
        }
        __syncthreads();   // residual tile, statistics and masks are reused by the next tile
    }
}

// V: workgroup = 256 threads, blocks of 64 tokens of one stream; wave w owns channels 32w..32w+31,
// lane t owns token t.
template <int BITS, bool TAB_LDS>
__global__ __launch_bounds__(256) void quantize_v_kernel(QuantArgs a, int tiles_per_wg)
{
    constexpr int TT = 64, WPU = BITS / 2;
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ float red_s[4];
    const TileShared sh = carve<TT, TAB_LDS>(smem, a.P);
    const int tid = threadIdx.x, ns = blockIdx.y;
    const __half *Mg = a.patterns + (int64_t)a.sets.set_of(ns) * a.P * kD;
    const int n_tiles = a.nq / TT;
    const int tile0 = blockIdx.x * tiles_per_wg, tile1 = min(n_tiles, tile0 + tiles_per_wg);
    uint4 xb[1][4];
    load_tiles<1>(a, ns, tile0 * TT, xb);

    stage_patterns(Mg, a.P, sh.tab, sh.norm, red_s, TAB_LDS);
    PatternTable tb;
    tb.lds_rows = sh.tab;
    tb.glb_rows = Mg;
    tb.norm2 = sh.norm;
    tb.norm2_max = fmaxf(fmaxf(red_s[0], red_s[1]), fmaxf(red_s[2], red_s[3]));
    tb.P = a.P;

    const int Gc = a.G < kD ? a.G : kD, ng = kD / Gc, qpg = Gc / 32;
    const int t = tid & 63, w = tid >> 6;
    const int grp = (32 * w) / Gc;
    const uint16_t *mask16 = reinterpret_cast<const uint16_t *>(sh.mask);
    for (int tile = tile0; tile < tile1; ++tile) {
        const int64_t tq0 = (int64_t)a.t0 + (int64_t)tile * TT;
        assign_and_stage<1, TAB_LDS>(a, sh, tb, Mg, ns, tq0, xb);
        __syncthreads();
        if (tile + 1 < tile1) load_tiles<1>(a, ns, (tile + 1) * TT, xb);

        float r[32];
        float mn = INFINITY, mx = -INFINITY;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float4 v = *reinterpret_cast<const float4 *>(sh.rt + t * kRStride + 32 * w + 4 * k);
            r[4 * k] = v.x; r[4 * k + 1] = v.y; r[4 * k + 2] = v.z; r[4 * k + 3] = v.w;
            mn = fminf(fminf(fminf(mn, v.x), v.y), fminf(v.z, v.w));
            mx = fmaxf(fmaxf(fmaxf(mx, v.x), v.y), fmaxf(v.z, v.w));
        }
        if (qpg > 1) {   // the channel group spans several waves
            sh.stat[(t * 4 + w) * 2] = mn;
            sh.stat[(t * 4 + w) * 2 + 1] = mx;
            __syncthreads();
            for (int k = 0; k < qpg; ++k) {
                mn = fminf(mn, sh.stat[(t * 4 + grp * qpg + k) * 2]);
                mx = fmaxf(mx, sh.stat[(t * 4 + grp * qpg + k) * 2 + 1]);
            }
        }
        const GroupParams gp = group_params(mn, mx, BITS);
        if (w % qpg == 0) {
            const int64_t prow = ((int64_t)ns * a.t_capacity + tq0) * ng + ((t >> 4) * ng + grp) * 16 + (t & 15);
            a.scale[prow] = __ushort_as_half(gp.s16);
            a.zero[prow] = __ushort_as_half(gp.z16);
        }
        // codes; a ballot over the 64 token lanes = plane j of one channel for the 4 units of the block
#pragma unroll
        for (int cc = 0; cc < 32; ++cc) {
            const uint32_t ub = code_word(r[cc], gp);
#pragma unroll
            for (int j = 0; j < BITS; ++j) {
                const unsigned long long m = plane_mask<BITS>(ub, j);
                if (t == 0) sh.mask[(32 * w + cc) * BITS + j] = m;
            }
        }
        __syncthreads();
        // thread (unit u, channel-in-tile n, tile pair w): gather the 16-bit pieces into words
        {
            const int u = t >> 4, n = t & 15;
            uint32_t out[2 * WPU];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int ch = 16 * (2 * w + q) + n;
#pragma unroll
                for (int jj = 0; jj < WPU; ++jj) {
                    const uint32_t lo = mask16[((ch * BITS + 2 * jj) << 2) + u];
                    const uint32_t hi = mask16[((ch * BITS + 2 * jj + 1) << 2) + u];
                    out[q * WPU + jj] = lo | (hi << 16);
                }
            }
            uint32_t *dst = reinterpret_cast<uint32_t *>(a.codes_v) + ((int64_t)ns * a.t_capacity + tq0) * (kD * BITS / 32) +
                            ((int64_t)t * 8 + 2 * w) * WPU;
            if (BITS == 2)
                *reinterpret_cast<uint2 *>(dst) = make_uint2(out[0], out[1]);
            else
                *reinterpret_cast<uint4 *>(dst) = make_uint4(out[0], out[1], out[2], out[3]);
        }
        __syncthreads();
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

static int tiles_per_wg(int n_tiles, int n_streams)
{
    int t = (int)(((int64_t)n_tiles * n_streams + 1023) / 1024);   // aim at ~1024 workgroups
    return t < 1 ? 1 : (t > 16 ? 16 : t);
}

template <class K>
static hipError_t launch_tiled(K kernel, const QuantArgs &a, int TT, size_t lds, hipStream_t s)
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int n_tiles = a.nq / TT, tpw = tiles_per_wg(n_tiles, a.n_streams);
    hipLaunchKernelGGL(kernel, dim3((n_tiles + tpw - 1) / tpw, a.n_streams), dim3(256), lds, s, a, tpw);
    return hipGetLastError();
}

hipError_t launch_quantize_k(const QuantArgs &a, hipStream_t s)
{
    if (a.metric == PK_METRIC_L2) {
        const bool tl = a.P <= 128;
#define PK_LAUNCH_K2(GG, BB)                                                                                       \
    if (a.G == GG && a.bits == BB) {                                                                               \
        constexpr int TT = GG == 128 ? 128 : 64;                                                                   \
        return tl ? launch_tiled(quantize_k_kernel<GG, BB, true>, a, TT, tile_lds_bytes<TT>(a.P, true), s)         \
                  : launch_tiled(quantize_k_kernel<GG, BB, false>, a, TT, tile_lds_bytes<TT>(a.P, false), s);      \
    }
        PK_LAUNCH_K2(32, 2) PK_LAUNCH_K2(64, 2) PK_LAUNCH_K2(128, 2)
        PK_LAUNCH_K2(32, 4) PK_LAUNCH_K2(64, 4) PK_LAUNCH_K2(128, 4)
#undef PK_LAUNCH_K2
        return hipErrorInvalidValue;
    }
    const dim3 grid(a.nq / a.G, a.n_streams), block(128);
#define PK_LAUNCH_K(GG, BB)                                                             \
    if (a.G == GG && a.bits == BB) {                                                    \
        hipLaunchKernelGGL((quantize_k_valu_kernel<GG, BB>), grid, block, 0, s, a);     \
        return hipGetLastError();                                                       \
    }
    PK_LAUNCH_K(32, 2) PK_LAUNCH_K(64, 2) PK_LAUNCH_K(128, 2)
    PK_LAUNCH_K(32, 4) PK_LAUNCH_K(64, 4) PK_LAUNCH_K(128, 4)
#undef PK_LAUNCH_K
    return hipErrorInvalidValue;
}

hipError_t launch_quantize_v(const QuantArgs &a, hipStream_t s)
{
    if (a.metric == PK_METRIC_L2) {
        const bool tl = a.P <= 128;
        if (a.bits == 2)
            return tl ? launch_tiled(quantize_v_kernel<2, true>, a, 64, tile_lds_bytes<64>(a.P, true), s)
                      : launch_tiled(quantize_v_kernel<2, false>, a, 64, tile_lds_bytes<64>(a.P, false), s);
        if (a.bits == 4)
            return tl ? launch_tiled(quantize_v_kernel<4, true>, a, 64, tile_lds_bytes<64>(a.P, true), s)
                      : launch_tiled(quantize_v_kernel<4, false>, a, 64, tile_lds_bytes<64>(a.P, false), s);
        return hipErrorInvalidValue;
    }
    const dim3 grid(a.nq / 64, a.n_streams), block(128);
    if (a.bits == 2)
        hipLaunchKernelGGL((quantize_v_valu_kernel<2>), grid, block, 0, s, a);
    else if (a.bits == 4)
        hipLaunchKernelGGL((quantize_v_valu_kernel<4>), grid, block, 0, s, a);
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
