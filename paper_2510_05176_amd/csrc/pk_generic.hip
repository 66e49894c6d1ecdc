// The hot path for head dimensions other than 128 (96 and 256, the other two that Sec. 3.3 names): plain kernels,
// thread <-> channel or thread <-> token (vector), with the Euclidean pattern search on the matrix cores.  They
// compute the same definitions with the same arithmetic where it decides an integer (the quantizer's parameters and
// codes come from the shared pk_quant_arith.h; pattern selection gives the exact argmin of the metric in binary32,
// lowest index on ties) and store the same cache format (head_dim enters the layout formulas), so they meet the
// same parity bars; they are kept simple rather than tuned, and the tuned kernels of the other files keep their
// fixed head dimension.  The decode kernels here also serve head dimension 128 for head counts that the matrix-core
// decode does not take.
// Uniform and ragged appends, decode (with shared prefix and with per-sequence fill states), mining, the window
// pattern and dequantize are covered, on contiguous and on paged caches.
#pragma clang fp contract(off)

#include "pk_assign_mfma.h"
#include "pk_quant_arith.h"

namespace pk {

namespace {

constexpr int kGenThreads = 256;   // >= the largest head dimension

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

// Nearest pattern of one vector per thread (lane <-> vector): the vector's D channels stay in registers as loaded,
// the pattern rows pass through LDS in chunks of kTabRows and are read by all lanes at once (one broadcast read per
// 8 channels), four patterns at a time.  Per pattern the metric is evaluated in binary32 - the squared differences
// added in channel order into one accumulator, or d_mm = max - min of the differences (Sec. 3.2) - and patterns are compared in increasing order with a strict <, so the lowest index wins ties.  All threads of the
// workgroup call this together (it has workgroup barriers).
constexpr int kTabRows = 32;
template <int D, int METRIC>
__device__ __forceinline__ void nearest_pattern(const uint4 (&x)[D / 8], const __half *M, int P, __half *tab, int tid,
                                                int &best_i, float &best_d)
{
    float bd = INFINITY;
    int bi = 0;
    for (int p0 = 0; p0 < P; p0 += kTabRows) {
        const int np = min(kTabRows, P - p0);
        __syncthreads();   // the previous chunk has been read
        for (int k = tid; k < np * (D / 8); k += kGenThreads)
            reinterpret_cast<uint4 *>(tab)[k] = reinterpret_cast<const uint4 *>(M + (int64_t)p0 * D)[k];
        __syncthreads();
        for (int p = 0; p < np; p += 4) {
            const __half *m[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) m[j] = tab + min(p + j, np - 1) * D;   // rows past the chunk repeat its last one
            float acc[4], mn[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[j] = METRIC == PK_METRIC_MINMAX ? -INFINITY : 0.f;   // the running maximum under the min-max rule
                mn[j] = INFINITY;
            }
#pragma unroll
            for (int k = 0; k < D / 8; ++k) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint4 mv = *reinterpret_cast<const uint4 *>(m[j] + 8 * k);
                    const uint32_t xw[4] = {x[k].x, x[k].y, x[k].z, x[k].w}, mw[4] = {mv.x, mv.y, mv.z, mv.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float r0 = sub_lo(xw[e], mw[e]), r1 = sub_hi(xw[e], mw[e]);   // binary32 differences
                        if (METRIC == PK_METRIC_MINMAX) {
                            acc[j] = fmaxf(fmaxf(acc[j], r0), r1);
                            mn[j] = fminf(fminf(mn[j], r0), r1);
                        } else {
                            acc[j] = fmaf(r0, r0, acc[j]);
                            acc[j] = fmaf(r1, r1, acc[j]);
                        }
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float dist = METRIC == PK_METRIC_MINMAX ? acc[j] - mn[j] : acc[j];
                if (p + j < np && dist < bd) {
                    bd = dist;
                    bi = p0 + p + j;
                }
            }
        }
    }
    best_i = bi;
    best_d = bd;
}

// ---------------------------------------------------------------------------------------------- Euclidean search
// Nearest pattern under the Euclidean rule on the matrix cores at head dimension D (96 or 256), the scheme of the
// tuned search with D / 32 operand steps: a wave ranks a 16-vector tile against 16 patterns per round,
// e = x.m - (|m|^2 + |x|^2) / 2 = -|x - m|^2 / 2 from v_mfma_f32_16x16x32_f16 (fp16 products are exact in binary32,
// only the accumulation rounds); the binary32 patterns of e, read as unsigned integers with the pattern index in
// the low byte, order like the distances; best and second best are tracked, and a vector whose gap between the
// two is inside the rounding band of that form is evaluated again exactly by the whole wave - the squared binary32
// differences over all patterns, lowest index on ties - so every index equals the exact argmin.  The table lives
// in LDS (rows of D + 16 halves: 16-byte reads of 16 rows x 4 column groups fall on distinct banks), the whole of it
// or, when it would not fit beside a second workgroup, one workgroup per CU.
template <int D>
struct GenSearchLds {
    static constexpr int kStride = D + 16;   // halves per table row
    __half *tab;      // [pad16(P)][kStride], rows past P zero
    float *nh;        // [pad16(P)]  -|m|^2 / 2, -inf past P
    float *red;       // [4]
    __half *xrow;     // [4 waves][D]: the vector under exact evaluation
    __device__ GenSearchLds(unsigned char *base, int P)
    {
        tab = reinterpret_cast<__half *>(base);
        nh = reinterpret_cast<float *>(tab + (size_t)pad16(P) * kStride);
        red = nh + pad16(P);
        xrow = reinterpret_cast<__half *>(red + 4);
    }
    static size_t bytes(int P) { return (size_t)pad16(P) * kStride * 2 + (size_t)pad16(P) * 4 + 16 + (size_t)4 * D * 2; }
};

// Stage the table of one pattern set and the row norms; returns max_p |m_p|^2.  All 256 threads; ends with a barrier.
template <int D>
__device__ __forceinline__ float gen_search_stage(const __half *Mg, int P, const GenSearchLds<D> &sh)
{
    constexpr int kStride = GenSearchLds<D>::kStride;
    const int tid = threadIdx.x, Pp = pad16(P);
    for (int i = tid; i < Pp * (D / 8); i += 256) {
        const int r = i / (D / 8), ch = i - r * (D / 8);
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (r < P) v = *reinterpret_cast<const uint4 *>(Mg + (int64_t)r * D + 8 * ch);
        *reinterpret_cast<uint4 *>(sh.tab + r * kStride + 8 * ch) = v;
    }
    __syncthreads();
    float mx = 0.f;
    for (int r = tid; r < Pp; r += 256) {
        float acc = 0.f;
        for (int ch = 0; ch < D / 8; ++ch) {
            const uint4 v = *reinterpret_cast<const uint4 *>(sh.tab + r * kStride + 8 * ch);
            const half2_t *h = reinterpret_cast<const half2_t *>(&v);
#pragma unroll
            for (int k = 0; k < 4; ++k) acc = __builtin_amdgcn_fdot2(h[k], h[k], acc, false);
        }
        sh.nh[r] = r < P ? -0.5f * acc : -INFINITY;
        mx = fmaxf(mx, acc);
    }
    mx = wave_max(mx);
    if ((tid & 63) == 0) sh.red[tid >> 6] = mx;
    __syncthreads();
    return fmaxf(fmaxf(sh.red[0], sh.red[1]), fmaxf(sh.red[2], sh.red[3]));
}

// One 16-vector tile by one wave: row = the lane's vector (token n = lane % 16 of the tile).  Every lane of column n
// returns the nearest pattern of token n and its squared distance (from the expanded form, 8 mantissa bits dropped,
// or the exact one where the vector was evaluated again).
template <int D>
__device__ __forceinline__ void gen_search_tile(const __half *row, const GenSearchLds<D> &sh, float norm2_max, int P, __half *xrow,
                                                int lane, int &best, float &best_d)
{
    constexpr int KS = D / 32;   // operand steps of 32 channels
    constexpr int kStride = GenSearchLds<D>::kStride;
    const int n = lane & 15, kb = lane >> 4, Pp = pad16(P);
    uint4 xb[KS];   // B operand: token n, channels 32 s + 8 kb + j
#pragma unroll
    for (int s = 0; s < KS; ++s) xb[s] = *reinterpret_cast<const uint4 *>(row + 32 * s + 8 * kb);
    float xx = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        const half2_t *h = reinterpret_cast<const half2_t *>(&xb[s]);
#pragma unroll
        for (int k = 0; k < 4; ++k) xx = __builtin_amdgcn_fdot2(h[k], h[k], xx, false);
    }
    xx += __shfl_xor(xx, 16);
    xx += __shfl_xor(xx, 32);
    const float hx = 0.5f * xx;
    uint32_t k1 = 0xffffffffu, k2 = 0xffffffffu;
    for (int p0 = 0; p0 < Pp; p0 += 16) {
        const __half *arow = sh.tab + (p0 + n) * kStride + 8 * kb;
        const float4 nh = *reinterpret_cast<const float4 *>(sh.nh + p0 + 4 * kb);
        floatx4_t e = {nh.x - hx, nh.y - hx, nh.z - hx, nh.w - hx};
#pragma unroll
        for (int s = 0; s < KS; ++s) e = mfma_f16(*reinterpret_cast<const uint4 *>(arow + 32 * s), xb[s], e);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t key = __builtin_amdgcn_perm(__float_as_uint(e[i]), (uint32_t)(p0 + 4 * kb + i), 0x07060500u);
            k2 = max(min(k1, k2), min(max(k1, k2), key));   // second smallest so far
            k1 = min(k1, key);
        }
    }
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {   // the four lane groups of the column
        const uint32_t o1 = (uint32_t)__shfl_xor((int)k1, off), o2 = (uint32_t)__shfl_xor((int)k2, off);
        k2 = min(min(k2, o2), max(k1, o1));
        k1 = min(k1, o1);
    }
    best = (int)(k1 & 0xffu);
    const float bv = -2.f * __uint_as_float(k1 & 0xffffff00u), second = -2.f * __uint_as_float(k2 & 0xffffff00u);
    best_d = fmaxf(bv, 0.f);
    // rounding band: the accumulation over KS matrix instructions (far below 2^-21 (|x|^2 + |m|^2) each) and the 8
    // mantissa bits the keys drop, with a wide margin
    const float band = (KS > 4 ? 1.52587890625e-05f : 7.62939453125e-06f) * (xx + norm2_max) + 6.103515625e-05f * second;
    const bool flag = P > 1 && !(second - bv > band);
    unsigned long long todo = __ballot(flag) & 0xffffull;   // one bit per column
    while (todo) {
        const int col = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        if (n == col) {
#pragma unroll
            for (int s = 0; s < KS; ++s) *reinterpret_cast<uint4 *>(xrow + 32 * s + 8 * kb) = xb[s];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        float bd = INFINITY;
        int bi = 0x7fffffff;
        for (int p = lane; p < P; p += 64) {
            const __half *m = sh.tab + p * kStride;
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll 4
            for (int ch = 0; ch < D / 8; ++ch) {
                const uint4 mv = *reinterpret_cast<const uint4 *>(m + 8 * ch);
                const uint4 xv = *reinterpret_cast<const uint4 *>(xrow + 8 * ch);
                const float d0 = sub_lo(xv.x, mv.x), d1 = sub_hi(xv.x, mv.x), d2 = sub_lo(xv.y, mv.y), d3 = sub_hi(xv.y, mv.y);
                const float d4 = sub_lo(xv.z, mv.z), d5 = sub_hi(xv.z, mv.z), d6 = sub_lo(xv.w, mv.w), d7 = sub_hi(xv.w, mv.w);
                a0 = fmaf(d0, d0, a0); a1 = fmaf(d1, d1, a1); a2 = fmaf(d2, d2, a2); a3 = fmaf(d3, d3, a3);
                a0 = fmaf(d4, d4, a0); a1 = fmaf(d5, d5, a1); a2 = fmaf(d6, d6, a2); a3 = fmaf(d7, d7, a3);
            }
            const float dist = (a0 + a1) + (a2 + a3);
            if (dist < bd) {
                bd = dist;
                bi = p;
            }
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float od = __shfl_xor(bd, off);
            const int oi = __shfl_xor(bi, off);
            if (od < bd || (od == bd && oi < bi)) {
                bd = od;
                bi = oi;
            }
        }
        if (n == col) {
            best = bi;
            best_d = bd;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// Pattern index of every vector to quantize under the Euclidean rule: a workgroup stages its stream's table once and
// takes tiles_per_wg tiles of 16 vectors, a wave per tile.
template <int D>
__global__ __launch_bounds__(256) void gen_assign_mfma_kernel(QuantArgs a, int tiles_per_wg)
{
    extern __shared__ __align__(16) unsigned char gen_search_smem[];
    const GenSearchLds<D> sh(gen_search_smem, a.P);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ns = blockIdx.y;
    take_sequence_entry(a, ns);
    const int n_tiles = a.nq / 16;   // nq is a multiple of the group size
    const int tile0 = blockIdx.x * tiles_per_wg, tile1 = min(n_tiles, tile0 + tiles_per_wg);
    if (tile0 >= n_tiles) return;    // a ragged append: sized for the longest sequence
    const float norm2_max = gen_search_stage<D>(a.patterns + (int64_t)a.sets.set_of(ns) * a.P * D, a.P, sh);
    for (int tile = tile0 + wave; tile < tile1; tile += 4) {
        int best;
        float bd;
        gen_search_tile<D>(a.src.row_d(ns, tile * 16 + (lane & 15), D), sh, norm2_max, a.P, sh.xrow + wave * D, lane, best, bd);
        if (lane < 16) a.idx[a.map.pos(ns, a.t0 + tile * 16) + lane] = (uint8_t)best;
    }
}

// The assignment step of mining (Sec. 3.1 Eq. 4), the same search over the vectors of a set.
template <int D>
__global__ __launch_bounds__(256) void gen_mine_assign_mfma_kernel(MineArgs a, int last, int tiles_per_wg)
{
    extern __shared__ __align__(16) unsigned char gen_search_smem[];
    const GenSearchLds<D> sh(gen_search_smem, a.P);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, s = blockIdx.y;
    const int n_tiles = (a.T + 15) / 16;
    const int tile0 = blockIdx.x * tiles_per_wg, tile1 = min(n_tiles, tile0 + tiles_per_wg);
    if (tile0 >= n_tiles) return;
    const float norm2_max = gen_search_stage<D>(a.patterns + (int64_t)s * a.P * D, a.P, sh);
    for (int tile = tile0 + wave; tile < tile1; tile += 4) {
        const int t = tile * 16 + (lane & 15);   // a vector past the set's end repeats the last one; nothing is stored for it
        int best;
        float bd;
        gen_search_tile<D>(a.x + (int64_t)s * a.set_stride + (int64_t)min(t, a.T - 1) * D, sh, norm2_max, a.P, sh.xrow + wave * D, lane,
                           best, bd);
        if (lane < 16 && t < a.T) {
            a.assign_ws[(int64_t)s * a.T + t] = best;
            if (last && a.assign) a.assign[(int64_t)s * a.T + t] = best;
            a.best[(int64_t)s * a.T + t] = bd;
        }
    }
}

// ---------------------------------------------------------------------------------------------- quantize-append
// Pattern index of every vector to quantize: a workgroup takes 256 consecutive vectors of a stream.
template <int D, int METRIC>
__global__ __launch_bounds__(kGenThreads) void gen_assign_kernel(QuantArgs a)
{
    __shared__ __align__(16) __half tab[kTabRows * D];
    const int tid = threadIdx.x, ns = blockIdx.y, i = blockIdx.x * kGenThreads + tid;
    take_sequence_entry(a, ns);
    if ((int)(blockIdx.x * kGenThreads) >= a.nq) return;   // a ragged append: sized for the longest sequence
    const bool live = i < a.nq;
    uint4 x[D / 8];
    const uint4 *row = reinterpret_cast<const uint4 *>(a.src.row_d(ns, live ? i : a.nq - 1, D));
#pragma unroll
    for (int k = 0; k < D / 8; ++k) x[k] = row[k];
    int bi;
    float bd;
    nearest_pattern<D, METRIC>(x, a.patterns + (int64_t)a.sets.set_of(ns) * a.P * D, a.P, tab, tid, bi, bd);
    if (live) a.idx[a.map.pos(ns, a.t0 + i)] = (uint8_t)bi;
}

// K: one workgroup per (group of G tokens, stream), thread <-> channel.  Two passes over the group's residuals (the
// second recomputes them): minimum / maximum -> parameters, then codes; a plane word of 32 channels is a wave ballot.
// The group's indices are staged in LDS and the vectors and pattern rows are requested 16 tokens at a time, without
// branches (threads past the head dimension read its last channel and store nothing).
__global__ __launch_bounds__(kGenThreads) void gen_quantize_k_kernel(QuantArgs a)
{
    __shared__ uint8_t idx_s[128];   // G <= 128
    const int c = threadIdx.x, lane = c & 63, ns = blockIdx.y, g = blockIdx.x, d = a.d, G = a.G;
    take_sequence_entry(a, ns);
    if (g * G >= a.nq) return;   // a ragged append: sized for the longest sequence
    const bool on = c < d;
    const int cc = on ? c : d - 1;
    const __half *M = a.patterns + (int64_t)a.sets.set_of(ns) * a.P * d + cc;
    const int64_t p0 = a.map.pos(ns, a.t0 + g * G);   // a group never straddles a page
    if (c < G) idx_s[c] = a.idx[p0 + c];
    __syncthreads();
    float mn = INFINITY, mx = -INFINITY;
    for (int t0 = 0; t0 < G; t0 += 16) {
        float xr[16], mr[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            xr[k] = h2f(a.src.row_d(ns, g * G + t0 + k, d)[cc]);
            mr[k] = h2f(M[(int64_t)idx_s[t0 + k] * d]);
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const float r = xr[k] - mr[k];
            mn = fminf(mn, r);
            mx = fmaxf(mx, r);
        }
    }
    const GroupParams gp = group_params(mn, mx, a.bits);
    if (on) {
        a.scale[(p0 / G) * d + c] = __ushort_as_half(gp.s16);
        a.zero[(p0 / G) * d + c] = __ushort_as_half(gp.z16);
    }
    const int words = d / 32;
    const int w = (c >> 6) * 2 + (lane >> 5);
    const bool writer = (lane & 31) == 0 && w < words;
    for (int t0 = 0; t0 < G; t0 += 16) {
        float xr[16], mr[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            xr[k] = h2f(a.src.row_d(ns, g * G + t0 + k, d)[cc]);
            mr[k] = h2f(M[(int64_t)idx_s[t0 + k] * d]);
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int code = on ? quantize_one(xr[k] - mr[k], gp, a.bits) : 0;
            for (int j = 0; j < a.bits; ++j) {
                const unsigned long long m = __ballot((code >> j) & 1);   // bit l <-> channel 64 * wave + l
                if (writer) a.codes_k[((p0 + t0 + k) * words + w) * a.bits + j] = (uint32_t)(m >> (lane & 32));
            }
        }
    }
}

// Minimum or maximum over each half (32 lanes) of a wave with data-parallel-primitive moves, no LDS traffic: an
// inclusive scan over the rows of 16 lanes (row_shr 1, 2, 4, 8; a lane without a source keeps its own value), then
// lane 15 of rows 0 and 2 is broadcast into rows 1 and 3 (row_bcast15).  The result is in lanes 31 and 63.
template <bool MAX>
__device__ __forceinline__ float half_wave_reduce_to_last(float v)
{
#define PK_DPP_STEP(CTRL, ROWS)                                                                                               \
    {                                                                                                                         \
        const float o = __builtin_bit_cast(                                                                                   \
            float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, v), __builtin_bit_cast(int, v), CTRL, ROWS, 0xf, false)); \
        v = MAX ? fmaxf(v, o) : fminf(v, o);                                                                                  \
    }
    PK_DPP_STEP(0x111, 0xf)
    PK_DPP_STEP(0x112, 0xf)
    PK_DPP_STEP(0x114, 0xf)
    PK_DPP_STEP(0x118, 0xf)
    PK_DPP_STEP(0x142, 0xa)
#undef PK_DPP_STEP
    return v;
}

// V: one workgroup per (16-token unit, stream) in three phases.  (1) thread <-> channel: residuals of the 16 tokens;
// minimum and maximum of the residuals (and, for the adaptive threshold, of the vector) over every 32 channels by
// data-parallel-primitive moves inside half a wave, left in LDS.  (2) thread <-> (token, channel group): the
// threshold's decision of Sec. 3.3 for the whole vector, the group's minimum and maximum from the halves, the stored
// parameters - all 16 tokens of a group in one pass - to LDS and, 16 tokens side by side, to memory.  (3) thread <->
// channel again: codes against the parameters of its group, the bits of the channel's 16 tokens collected in the
// words it stores.
__global__ __launch_bounds__(kGenThreads) void gen_quantize_v_kernel(QuantArgs a)
{
    constexpr int kHalves = kGenThreads / 32;
    __shared__ float4 half_mm[16][kHalves];     // per token and 32 channels: min r, max r, min x, max x
    __shared__ float4 par[16][kHalves];         // per token and channel group: z, 1/s, s, raw flag
    const int c = threadIdx.x, ns = blockIdx.y, u = blockIdx.x, d = a.d;
    take_sequence_entry(a, ns);
    if (u * 16 >= a.nq) return;   // a ragged append: sized for the longest sequence
    const bool on = c < d;
    const int cc = on ? c : d - 1;   // threads past the head dimension read its last channel and store nothing
    const int Gc = a.G < d ? a.G : d, NG = d / Gc, g = cc / Gc;
    const __half *M = a.patterns + (int64_t)a.sets.set_of(ns) * a.P * d + cc;
    const int64_t p0 = a.map.pos(ns, a.t0 + u * 16);   // a multiple of 16: the unit's 16 index bytes are one aligned piece
    const uint4 iw = *reinterpret_cast<const uint4 *>(a.idx + p0);
    const uint32_t iws[4] = {iw.x, iw.y, iw.z, iw.w};
    const bool thresholded = a.v_rho > 0.f;
    float xs[16], rs[16];   // the unit's vectors and residuals
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        xs[i] = h2f(a.src.row_d(ns, u * 16 + i, d)[cc]);
        rs[i] = h2f(M[(int64_t)((iws[i >> 2] >> (8 * (i & 3))) & 255) * d]);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        rs[i] = xs[i] - rs[i];
        const float rmn = half_wave_reduce_to_last<false>(on ? rs[i] : INFINITY);
        const float rmx = half_wave_reduce_to_last<true>(on ? rs[i] : -INFINITY);
        float xmn = 0.f, xmx = 0.f;
        if (thresholded) {   // the vector's own range is needed for the threshold only
            xmn = half_wave_reduce_to_last<false>(on ? xs[i] : INFINITY);
            xmx = half_wave_reduce_to_last<true>(on ? xs[i] : -INFINITY);
        }
        if ((c & 31) == 31) half_mm[i][c >> 5] = make_float4(rmn, rmx, xmn, xmx);
    }
    __syncthreads();
    if (c < 16 * NG) {   // token i, channel group gg
        const int i = c & 15, gg = c >> 4;
        bool raw = false;   // the vector itself is quantized, stored under the index that says so
        if (thresholded) {
            float4 row = half_mm[i][0];
            for (int k = 1; k < d / 32; ++k) {
                const float4 o = half_mm[i][k];
                row = make_float4(fminf(row.x, o.x), fmaxf(row.y, o.y), fminf(row.z, o.z), fmaxf(row.w, o.w));
            }
            raw = !((row.y - row.x) <= a.v_rho * (row.w - row.z));
        }
        float mn = INFINITY, mx = -INFINITY;
        for (int k = gg * (Gc / 32); k < (gg + 1) * (Gc / 32); ++k) {
            const float4 o = half_mm[i][k];
            mn = fminf(mn, raw ? o.z : o.x);
            mx = fmaxf(mx, raw ? o.w : o.y);
        }
        const GroupParams gp = group_params(mn, mx, a.bits);
        par[i][gg] = make_float4(gp.z, gp.inv, gp.s, raw ? 1.f : 0.f);
        a.scale[((p0 >> 4) * NG + gg) * 16 + i] = __ushort_as_half(gp.s16);
        a.zero[((p0 >> 4) * NG + gg) * 16 + i] = __ushort_as_half(gp.z16);
        if (gg == 0 && raw) a.idx[p0 + i] = (uint8_t)PK_NO_PATTERN;
    }
    __syncthreads();
    uint32_t word[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const float4 pr = par[i][g];
        GroupParams gp;
        gp.z = pr.x;
        gp.inv = pr.y;
        gp.s = pr.z;
        const int code = quantize_one(pr.w != 0.f ? xs[i] : rs[i], gp, a.bits);
        for (int j = 0; j < a.bits; ++j) word[j >> 1] |= (uint32_t)((code >> j) & 1) << (16 * (j & 1) + i);
    }
    if (on) {
        uint32_t *codes = reinterpret_cast<uint32_t *>(a.codes_v);
        const int64_t w0 = (((p0 >> 4) * 16 + (c & 15)) * (d / 16) + (c >> 4)) * (a.bits / 2);
        for (int k = 0; k < a.bits / 2; ++k) codes[w0 + k] = word[k];
    }
}

__global__ __launch_bounds__(256) void gen_tail_copy_kernel(TailCopyArgs a)
{
    const int n = blockIdx.y, side = blockIdx.z, chunks = a.d / 8;
    if (a.seq_table) {   // a ragged append: the ring state and the range of the stream's own sequence
        const int32_t *e = a.seq_table + (int64_t)(n / a.n_kv_heads) * kSeqEntry;
        a.ring_start = e[kSeqRingStart];
        a.n_ring = e[kSeqNRing];
        a.i0 = e[kSeqI0];
        a.i1 = e[kSeqI1];
    }
    const int64_t work = (int64_t)(a.i1 - a.i0) * chunks;
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (w >= work) return;
    const int i = a.i0 + (int)(w / chunks), ch = (int)(w % chunks);
    const __half *fresh = side == 0 ? a.fresh_k : a.fresh_v;
    __half *ring = side == 0 ? a.ring_k : a.ring_v;
    const uint4 v = *reinterpret_cast<const uint4 *>(fresh + (int64_t)n * a.fresh_stride + (int64_t)(i - a.n_ring) * a.d + ch * 8);
    const int slot = (int)(((int64_t)a.ring_start + i) % a.ring_len);
    *reinterpret_cast<uint4 *>(ring + ((int64_t)n * a.ring_len + slot) * a.d + ch * 8) = v;
}

// ---------------------------------------------------------------------------------------------- mining
__global__ __launch_bounds__(256) void gen_mine_init_kernel(MineArgs a)
{
    const int s = blockIdx.y;
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (w >= (int64_t)a.P * a.d) return;
    a.patterns[(int64_t)s * a.P * a.d + w] = a.x[(int64_t)s * a.set_stride + w];   // the first P vectors
}

// cluster sums of one chunk of one set for a block of patterns (blockIdx.z).  The chunk is cut into
// pieces of 1024 vectors whose assignments are staged in LDS, and every piece into kGenThreads / d consecutive slices
// (two at d = 96, one at d = 256); thread <-> (slice, channel) adds the slice's vectors in order into the slice's
// [patterns][d] accumulators in LDS (only this thread ever touches its column), the slices are added in order at the
// end: the order of all additions is fixed.  The members are counted by all threads with integer atomics.
// At the end the block goes to the chunk's own [P][d] part of the workspace.  A workgroup reads the assignment of
// every vector of the chunk and the vectors of its own patterns only.
constexpr int kSumsLdsFloats = 12288;   // accumulators per workgroup: floor(12288 / (slices * d)) - 1 patterns per block
__global__ __launch_bounds__(kGenThreads) void gen_mine_sums_kernel(MineArgs a, int chunk, int pblock)
{
    constexpr int kAsg = 1024;             // assignments staged in LDS at a time
    __shared__ float acc[kSumsLdsFloats];
    __shared__ int32_t cnt[kGenThreads];   // pblock <= 64
    __shared__ int32_t rel_s[kAsg];        // pattern of a vector relative to the block, -1 outside it
    const int tid = threadIdx.x, ck = blockIdx.x, s = blockIdx.y, d = a.d;
    const int n_slices = kGenThreads / d, slice = tid / d, c = tid - slice * d;
    const int p0 = blockIdx.z * pblock, np = min(pblock, a.P - p0);
    const int t0 = ck * chunk, t1 = min(a.T, t0 + chunk);
    for (int i = tid; i < n_slices * (np + 1) * d; i += kGenThreads) acc[i] = 0.f;
    cnt[tid] = 0;
    __syncthreads();
    const int32_t *asg = a.assign_ws + (int64_t)s * a.T;
    const __half *x = a.x + (int64_t)s * a.set_stride;
    float *mine = acc + (slice < n_slices ? slice : 0) * (np + 1) * d;   // np rows and the spare one
    for (int b0 = t0; b0 < t1; b0 += kAsg) {   // the chunk in pieces of kAsg vectors
        const int b1 = min(t1, b0 + kAsg);
        __syncthreads();   // the previous piece's assignments have been used
        for (int t = b0 + tid; t < b1; t += kGenThreads) {
            int rel = asg[t] - p0;
            if (rel < 0 || rel >= np) rel = -1;
            rel_s[t - b0] = rel;
            if (rel >= 0) atomicAdd(&cnt[rel], 1);
        }
        __syncthreads();
        if (slice < n_slices) {
            const int len = (b1 - b0 + n_slices - 1) / n_slices;
            const int s0 = b0 + slice * len, s1 = min(b1, s0 + len);
            for (int t = s0; t < s1; t += 16) {
                // the vectors of sixteen steps are requested together, then added in order
                // (no branches: a vector outside the block, or past the slice, goes to a spare row nobody reads)
                int rowi[16];
                float v[16];
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const int tk = min(t + k, s1 - 1);
                    const int rel = t + k < s1 ? rel_s[tk - b0] : -1;
                    rowi[k] = (rel < 0 ? np : rel) * d + c;
                    v[k] = h2f(x[(int64_t)tk * d + c]);
                }
#pragma unroll
                for (int k = 0; k < 16; ++k) mine[rowi[k]] += v[k];
            }
        }
    }
    __syncthreads();
    float *ps = a.psum + (((int64_t)s * a.tsplit + ck) * a.P + p0) * d;
    int32_t *pc = a.pcnt + ((int64_t)s * a.tsplit + ck) * a.P + p0;
    for (int i = tid; i < np * d; i += kGenThreads) {
        float v = acc[i];
        for (int k = 1; k < n_slices; ++k) v += acc[k * (np + 1) * d + i];
        ps[i] = v;
    }
    if (tid < np) pc[tid] = cnt[tid];
}

// update: chunks in increasing order, mean in binary32, fp16 nearest even; an empty cluster keeps its centroid
__global__ __launch_bounds__(kGenThreads) void gen_mine_update_kernel(MineArgs a)
{
    const int p = blockIdx.x, s = blockIdx.y, c = threadIdx.x, d = a.d;
    if (c >= d) return;
    float sum = 0.f;
    int cnt = 0;
    for (int ts = 0; ts < a.tsplit; ++ts) {
        sum += a.psum[(((int64_t)s * a.tsplit + ts) * a.P + p) * d + c];
        cnt += a.pcnt[((int64_t)s * a.tsplit + ts) * a.P + p];
    }
    if (cnt > 0) a.patterns[((int64_t)s * a.P + p) * d + c] = __float2half_rn(sum / (float)cnt);
}

__global__ __launch_bounds__(256) void gen_mine_inertia_kernel(MineArgs a, int it)
{
    __shared__ float red[256];
    const int s = blockIdx.x, tid = threadIdx.x;
    const float *b = a.best + (int64_t)s * a.T;
    float acc = 0.f;
    for (int t = tid; t < a.T; t += 256) acc += b[t];
    red[tid] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (tid < w) red[tid] += red[tid + w];
        __syncthreads();
    }
    if (tid == 0) a.inertia[(int64_t)s * a.iters + it] = red[0];
}

__global__ __launch_bounds__(kGenThreads) void gen_window_pattern_kernel(const __half *x, int64_t set_stride, int n, int d,
                                                                        __half *out, int64_t out_stride)
{
    const int c = threadIdx.x;
    if (c >= d) return;
    const __half *xs = x + (int64_t)blockIdx.x * set_stride + c;
    float mn = INFINITY, mx = -INFINITY;
    for (int t = 0; t < n; ++t) {
        const float v = h2f(xs[(int64_t)t * d]);
        mn = fminf(mn, v);
        mx = fmaxf(mx, v);
    }
    out[(int64_t)blockIdx.x * out_stride + c] = __float2half_rn((mn + mx) * 0.5f);
}

// ---------------------------------------------------------------------------------------------- reconstruction
// code of channel c of the packed token at position pos
__device__ __forceinline__ int k_code_at(const CacheView &cv, int64_t pos, int c, int d, int bits)
{
    int code = 0;
    for (int j = 0; j < bits; ++j) code |= (int)((cv.k_codes[(pos * (d / 32) + (c >> 5)) * bits + j] >> (c & 31)) & 1u) << j;
    return code;
}
__device__ __forceinline__ int v_code_at(const CacheView &cv, int64_t pos, int c, int d, int bits)
{
    const uint32_t *vb = reinterpret_cast<const uint32_t *>(cv.v_codes);
    const int64_t word = (((pos >> 4) * 16 + (c & 15)) * (d / 16) + (c >> 4)) * (bits / 2);
    int code = 0;
    for (int j = 0; j < bits; ++j) code |= (int)((vb[word + j / 2] >> (16 * (j % 2) + (int)(pos & 15))) & 1u) << j;
    return code;
}
// K^[c], V^[c] of a packed token: M[k*] + (s * code + z), multiply, add, add in binary32
__device__ __forceinline__ float k_hat(const CacheView &cv, const __half *MK, int64_t pos, int c, int d, int bits, int G)
{
    const int64_t prow = (pos / G) * d + c;
    const float res = h2f(cv.k_scale[prow]) * (float)k_code_at(cv, pos, c, d, bits) + h2f(cv.k_zero[prow]);
    return h2f(MK[(int64_t)cv.k_idx[pos] * d + c]) + res;
}
__device__ __forceinline__ float v_hat(const CacheView &cv, const __half *MV, int64_t pos, int c, int d, int bits, int Gc,
                                       int thresholded)
{
    const int ng = d / Gc;
    const int64_t prow = ((pos >> 4) * ng + c / Gc) * 16 + (pos & 15);
    const float res = h2f(cv.v_scale[prow]) * (float)v_code_at(cv, pos, c, d, bits) + h2f(cv.v_zero[prow]);
    const int vi = cv.v_idx[pos];
    if (thresholded && vi == PK_NO_PATTERN) return res;
    return h2f(MV[(int64_t)vi * d + c]) + res;
}

__global__ __launch_bounds__(kGenThreads) void gen_dequant_kernel(DequantArgs a)
{
    const int t = a.t0 + blockIdx.x, n = blockIdx.y, c = threadIdx.x, d = a.d;
    if (c >= d) return;
    const int set = a.sets.set_of(n);
    const int Gc = a.G < d ? a.G : d;
    const int64_t pos = a.c.map.pos(n, t);
    const int64_t orow = ((int64_t)n * (a.t1 - a.t0) + (t - a.t0)) * d + c;
    if (a.k_out) a.k_out[orow] = k_hat(a.c, a.patterns_k + (int64_t)set * a.P * d, pos, c, d, a.bits, a.G);
    if (a.v_out) a.v_out[orow] = v_hat(a.c, a.patterns_v + (int64_t)set * a.P * d, pos, c, d, a.bits, Gc, a.v_thresholded);
}

// ---------------------------------------------------------------------------------------------- decode
// Decode attention (Sec. 3.4) in plain vector arithmetic.  The context of a stream is cut into the same slots as in
// the tuned path (equal splits of the shared prefix's packed part, of the own packed part, then the own tail and
// the prefix's tail); a workgroup takes one slot of one stream for up to R = 8 query heads of the KV head at once (more heads: further workgroups), so
// the codes are taken apart once for all of them, and leaves an unnormalised partial (o, per-pattern softmax mass
// W, running maximum m in the log2 domain, sum l); a second kernel merges the partials and adds W . M_V once per
// head.  Scores: thread <-> token, score = q.M_K[k*] (a table formed once per workgroup) + sum_c q_c (s_c code_c +
// z_c).  Values: thread <-> channel over the tokens of the pass, o += p_t (s_t code_tc + z_t).  The reference of
// the online softmax is the running maximum; when a pass raises it, o, l and W are rescaled.  W is summed in LDS
// as 64-bit fixed point (unit 2^-31, weights are <= 1) with integer atomics, so the result does not depend on the
// order in which the tokens arrive.
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kMassUnit = 2147483648.f;   // 2^31
constexpr int kPass = kGenThreads;           // tokens per pass

__device__ __forceinline__ float half_of(const uint4 &v, int e)   // element e (0..7) of eight packed fp16
{
    const uint32_t w = e < 2 ? v.x : e < 4 ? v.y : e < 6 ? v.z : v.w;
    return h2f(__ushort_as_half((unsigned short)((e & 1) ? w >> 16 : w & 0xffffu)));
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// LDS of a split workgroup, in this order (the 8-byte arrays first)
struct GenDecodeLds {
    unsigned long long *W;   // [P][R]   softmax mass per V pattern and head, fixed point
    long long *pos;          // [kPass]  packed position (or tail ring row) of the pass's tokens
    float *qf;               // [d][R]   the queries, channel-major; heads beyond the workgroup's are zero
    float *QM;               // [P][R]   q . M_K[p]
    float *sc;               // [kPass][R] softmax numerators of the pass
    float *red;              // [4][R]
    __device__ GenDecodeLds(unsigned char *base, int d, int P, int R)
    {
        W = reinterpret_cast<unsigned long long *>(base);
        pos = reinterpret_cast<long long *>(W + (size_t)P * R);
        qf = reinterpret_cast<float *>(pos + kPass);
        QM = qf + (size_t)d * R;
        sc = QM + (size_t)P * R;
        red = sc + (size_t)kPass * R;
    }
};
inline size_t gen_decode_lds_bytes(int d, int P, int R)
{
    return (size_t)P * R * 8 + (size_t)kPass * 8 + ((size_t)d * R + (size_t)P * R + (size_t)kPass * R + 4 * R) * 4;
}

template <int R, int BITS>
__global__ __launch_bounds__(kGenThreads) void gen_decode_split_kernel(DecodeArgs a)
{
    extern __shared__ __align__(16) unsigned char gen_decode_smem[];
    const int tid = threadIdx.x, d = a.d, P = a.P;
    const GenDecodeLds lds(gen_decode_smem, d, P, R);
    const int n = blockIdx.x, slot = blockIdx.y, h0 = blockIdx.z * R;   // the workgroup's first head of the KV head's r
    const int seq = n / a.n_kv_heads, head = n - seq * a.n_kv_heads;
    const int r = a.n_q_heads / a.n_kv_heads, nh = min(R, r - h0);
    const int n_packed = a.splits_prefix + a.splits_own, n_slots = n_packed + 2;
    const bool packed = slot < n_packed;
    const bool pre = slot < a.splits_prefix || slot == n_packed + 1;
    const CacheView &cv = pre ? a.prefix : a.own;
    int tq = cv.t_quant, tt = cv.t_tail, ts = cv.tail_start;
    if (!pre) own_state(a, seq, tq, tt, ts);
    const int stream = pre ? head : n;
    const int set = pre ? head : a.sets.set_of(n);
    int t_begin = 0, t_end = tt;
    if (packed) {
        t_begin = (pre ? slot : slot - a.splits_prefix) * a.chunk;
        t_end = min(tq, t_begin + a.chunk);
    }
    const int64_t pb = ((int64_t)n * n_slots + slot) * r + h0;   // partial of the workgroup's first query head
    if (t_end <= t_begin) {   // nothing in this slot: the merge skips partials whose sum is zero
        if (tid < nh) {
            a.part_ml[(pb + tid) * 2] = -INFINITY;
            a.part_ml[(pb + tid) * 2 + 1] = 0.f;
        }
        return;
    }
    const int Gc = a.G < d ? a.G : d, ng = d / Gc;
    const float scale2 = a.softmax_scale * kLog2e;

    for (int i = tid; i < d * R; i += kGenThreads) {
        const int c = i / R, h = i - c * R;
        lds.qf[i] = h < nh ? h2f(a.q[((int64_t)seq * a.n_q_heads + head * r + h0 + h) * d + c]) : 0.f;
    }
    for (int i = tid; i < P * R; i += kGenThreads) lds.W[i] = 0ull;
    __syncthreads();
    if (packed) {
        const __half *MK = a.patterns_k + (int64_t)set * P * d;
        for (int p = tid; p < P; p += kGenThreads) {
            float s[R];
#pragma unroll
            for (int h = 0; h < R; ++h) s[h] = 0.f;
            for (int c8 = 0; c8 < d / 8; ++c8) {
                const uint4 mv = *reinterpret_cast<const uint4 *>(MK + (int64_t)p * d + 8 * c8);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float x = half_of(mv, e);
#pragma unroll
                    for (int h = 0; h < R; ++h) s[h] = fmaf(lds.qf[(8 * c8 + e) * R + h], x, s[h]);
                }
            }
#pragma unroll
            for (int h = 0; h < R; ++h) lds.QM[p * R + h] = s[h];
        }
        __syncthreads();
    }

    float m_run[R], l_thr[R], acc[R];
#pragma unroll
    for (int h = 0; h < R; ++h) {
        m_run[h] = -INFINITY;
        l_thr[h] = 0.f;
        acc[h] = 0.f;
    }
    // value phase: thread <-> (channel, sub); the subs take the 16-token blocks (tail tokens) of a pass in turn
    const int n_sub = kGenThreads / d;
    const int vsub = tid / d, vc = tid - vsub * d;
    const bool v_active = vsub < n_sub;
    const uint32_t *vwords = reinterpret_cast<const uint32_t *>(cv.v_codes);

    for (int t0 = t_begin; t0 < t_end; t0 += kPass) {
        const int t = t0 + tid;
        const bool live = t < t_end;
        float s[R];
        int64_t where = 0;
#pragma unroll
        for (int h = 0; h < R; ++h) s[h] = -INFINITY;
        if (live && packed) {
            where = cv.map.pos(stream, t);
            const int idx = min((int)cv.k_idx[where], P - 1);
#pragma unroll
            for (int h = 0; h < R; ++h) s[h] = lds.QM[idx * R + h];
            const int64_t prow = (where / a.G) * d;
            for (int w = 0; w < d / 32; ++w) {
                uint32_t pl[BITS];
#pragma unroll
                for (int j = 0; j < BITS; ++j) pl[j] = cv.k_codes[(where * (d / 32) + w) * BITS + j];
#pragma unroll
                for (int o = 0; o < 4; ++o) {
                    const uint4 sv = *reinterpret_cast<const uint4 *>(cv.k_scale + prow + 32 * w + 8 * o);
                    const uint4 zv = *reinterpret_cast<const uint4 *>(cv.k_zero + prow + 32 * w + 8 * o);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int cc = 8 * o + e;
                        uint32_t code = 0;
#pragma unroll
                        for (int j = 0; j < BITS; ++j) code |= ((pl[j] >> cc) & 1u) << j;
                        const float val = half_of(sv, e) * (float)code + half_of(zv, e);
#pragma unroll
                        for (int h = 0; h < R; ++h) s[h] = fmaf(lds.qf[(32 * w + cc) * R + h], val, s[h]);
                    }
                }
            }
        } else if (live) {
            int sl = ts + t;
            if (sl >= cv.ring_len) sl -= cv.ring_len;
            where = (int64_t)stream * cv.ring_len + sl;
#pragma unroll
            for (int h = 0; h < R; ++h) s[h] = 0.f;
            for (int c8 = 0; c8 < d / 8; ++c8) {
                const uint4 kv = *reinterpret_cast<const uint4 *>(cv.tail_k + where * d + 8 * c8);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float x = half_of(kv, e);
#pragma unroll
                    for (int h = 0; h < R; ++h) s[h] = fmaf(lds.qf[(8 * c8 + e) * R + h], x, s[h]);
                }
            }
        }
        // maximum of the pass per head
#pragma unroll
        for (int h = 0; h < R; ++h) {
            s[h] *= scale2;   // -inf stays -inf
            const float wm = wave_max(s[h]);
            if ((tid & 63) == 0) lds.red[(tid >> 6) * R + h] = wm;
        }
        lds.pos[tid] = where;
        __syncthreads();
        bool raised = false;   // the same in every thread
        float alpha[R];
#pragma unroll
        for (int h = 0; h < R; ++h) {
            const float pm = fmaxf(fmaxf(lds.red[h], lds.red[R + h]), fmaxf(lds.red[2 * R + h], lds.red[3 * R + h]));
            alpha[h] = 1.f;
            if (pm > m_run[h]) {
                alpha[h] = exp2f(m_run[h] - pm);   // 0 the first time
                m_run[h] = pm;
                raised = true;
            }
        }
        if (raised) {
#pragma unroll
            for (int h = 0; h < R; ++h) {
                acc[h] *= alpha[h];
                l_thr[h] *= alpha[h];
            }
            if (packed) {
                for (int p = tid; p < P; p += kGenThreads) {
#pragma unroll
                    for (int h = 0; h < R; ++h)
                        lds.W[p * R + h] = (unsigned long long)((double)lds.W[p * R + h] * (double)alpha[h]);
                }
                __syncthreads();   // before this pass's atomics
            }
        }
        float pw[R];
#pragma unroll
        for (int h = 0; h < R; ++h) {
            pw[h] = live ? exp2f(s[h] - m_run[h]) : 0.f;
            l_thr[h] += pw[h];
            lds.sc[tid * R + h] = pw[h];
        }
        if (live && packed) {
            const int vi = cv.v_idx[where];
            if (!(a.v_thresholded && vi == PK_NO_PATTERN)) {   // a token quantized without a pattern carries no mass
                const int vp = min(vi, P - 1);
#pragma unroll
                for (int h = 0; h < R; ++h) atomicAdd(&lds.W[vp * R + h], (unsigned long long)(pw[h] * kMassUnit));
            }
        }
        __syncthreads();

        const int n_here = min(kPass, t_end - t0);
        if (v_active && packed) {
            for (int b = vsub; 16 * b < n_here; b += n_sub) {
                const int64_t w0 = lds.pos[16 * b];   // the 16 tokens of a block are stored together
                const int64_t word = (((w0 >> 4) * 16 + (vc & 15)) * (d / 16) + (vc >> 4)) * (BITS / 2);
                uint32_t cw[BITS / 2];
#pragma unroll
                for (int j = 0; j < BITS / 2; ++j) cw[j] = vwords[word + j];
                const int64_t prow = ((w0 >> 4) * ng + vc / Gc) * 16;
                const uint4 sv[2] = {*reinterpret_cast<const uint4 *>(cv.v_scale + prow),
                                     *reinterpret_cast<const uint4 *>(cv.v_scale + prow + 8)};
                const uint4 zv[2] = {*reinterpret_cast<const uint4 *>(cv.v_zero + prow),
                                     *reinterpret_cast<const uint4 *>(cv.v_zero + prow + 8)};
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    uint32_t code = 0;
#pragma unroll
                    for (int j = 0; j < BITS; ++j) code |= ((cw[j / 2] >> (16 * (j % 2) + k)) & 1u) << j;
                    const float val = half_of(sv[k >> 3], k & 7) * (float)code + half_of(zv[k >> 3], k & 7);
#pragma unroll
                    for (int h = 0; h < R; ++h) acc[h] = fmaf(lds.sc[(16 * b + k) * R + h], val, acc[h]);
                }
            }
        } else if (v_active) {
            for (int k = vsub; k < n_here; k += n_sub) {
                const float val = h2f(cv.tail_v[lds.pos[k] * d + vc]);
#pragma unroll
                for (int h = 0; h < R; ++h) acc[h] = fmaf(lds.sc[k * R + h], val, acc[h]);
            }
        }
        __syncthreads();   // sc and pos are rewritten by the next pass
    }

    // the partial: sums over the threads in a fixed order
#pragma unroll
    for (int h = 0; h < R; ++h) {
        const float ws = wave_sum(l_thr[h]);
        if ((tid & 63) == 0) lds.red[(tid >> 6) * R + h] = ws;
    }
    if (v_active && vsub > 0) {
#pragma unroll
        for (int h = 0; h < R; ++h) lds.sc[(vsub * d + vc) * R + h] = acc[h];
    }
    __syncthreads();
    if (tid < d) {
        for (int k = 1; k < n_sub; ++k) {
#pragma unroll
            for (int h = 0; h < R; ++h) acc[h] += lds.sc[(k * d + tid) * R + h];
        }
#pragma unroll
        for (int h = 0; h < R; ++h)
            if (h < nh) a.part_o[(pb + h) * d + tid] = acc[h];
    }
    if (packed) {
        for (int p = tid; p < P; p += kGenThreads) {
#pragma unroll
            for (int h = 0; h < R; ++h)
                if (h < nh) a.part_w[(pb + h) * P + p] = (float)lds.W[p * R + h] * (1.f / kMassUnit);
        }
    }
#pragma unroll
    for (int h = 0; h < R; ++h) {
        if (tid == h && h < nh) {
            a.part_ml[(pb + h) * 2] = m_run[h];
            a.part_ml[(pb + h) * 2 + 1] = (lds.red[h] + lds.red[R + h]) + (lds.red[2 * R + h] + lds.red[3 * R + h]);
        }
    }
}

// log-sum-exp merge of the partials of one (sequence, query head) and the pattern part of the values, W . M_V
__global__ __launch_bounds__(kGenThreads) void gen_decode_merge_kernel(DecodeArgs a)
{
    __shared__ float wslot[kMaxSlots];
    __shared__ float Wsum[2][kGenThreads];   // shared prefix, own cache
    __shared__ float red[8];
    const int u = blockIdx.x, tid = threadIdx.x, d = a.d, P = a.P;
    const int seq = u / a.n_q_heads, qh = u - seq * a.n_q_heads;
    const int r = a.n_q_heads / a.n_kv_heads, head = qh / r, hr = qh - head * r;
    const int n = seq * a.n_kv_heads + head;
    const int n_packed = a.splits_prefix + a.splits_own, n_slots = n_packed + 2;
    const int64_t base = (int64_t)n * n_slots;
    float M = -INFINITY;
    for (int s = tid; s < n_slots; s += kGenThreads) {
        const int64_t q = ((base + s) * r + hr) * 2;
        if (a.part_ml[q + 1] > 0.f) M = fmaxf(M, a.part_ml[q]);
    }
    M = wave_max(M);
    if ((tid & 63) == 0) red[tid >> 6] = M;
    __syncthreads();
    M = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float L = 0.f;
    for (int s = tid; s < n_slots; s += kGenThreads) {
        const int64_t q = ((base + s) * r + hr) * 2;
        const float l = a.part_ml[q + 1];
        const float w = l > 0.f ? exp2f(a.part_ml[q] - M) : 0.f;
        wslot[s] = w;
        L = fmaf(l, w, L);
    }
    L = wave_sum(L);
    if ((tid & 63) == 0) red[4 + (tid >> 6)] = L;
    __syncthreads();
    L = (red[4] + red[5]) + (red[6] + red[7]);
    for (int p = tid; p < P; p += kGenThreads) {
        float wp = 0.f, wo = 0.f;
        for (int s = 0; s < a.splits_prefix; ++s)
            if (wslot[s] > 0.f) wp = fmaf(a.part_w[((base + s) * r + hr) * P + p], wslot[s], wp);
        for (int s = a.splits_prefix; s < n_packed; ++s)
            if (wslot[s] > 0.f) wo = fmaf(a.part_w[((base + s) * r + hr) * P + p], wslot[s], wo);
        Wsum[0][p] = wp;
        Wsum[1][p] = wo;
    }
    __syncthreads();
    if (tid >= d) return;
    float acc = 0.f;
    for (int s = 0; s < n_slots; ++s)
        if (wslot[s] > 0.f) acc = fmaf(a.part_o[((base + s) * r + hr) * d + tid], wslot[s], acc);
    if (a.splits_prefix > 0) {
        const __half *MV = a.patterns_v + (int64_t)head * P * d;
        for (int p = 0; p < P; ++p) acc = fmaf(Wsum[0][p], h2f(MV[(int64_t)p * d + tid]), acc);
    }
    if (a.splits_own > 0) {
        const __half *MV = a.patterns_v + (int64_t)a.sets.set_of(n) * P * d;
        for (int p = 0; p < P; ++p) acc = fmaf(Wsum[1][p], h2f(MV[(int64_t)p * d + tid]), acc);
    }
    a.out[(int64_t)u * d + tid] = L > 0.f ? acc / L : 0.f;
    if (a.lse && tid == 0) a.lse[u] = L > 0.f ? (M + log2f(L)) * kLn2 : -INFINITY;
}

template <int R>
hipError_t launch_gen_decode_split(const DecodeArgs &a, dim3 grid, size_t lds, hipStream_t s)
{
    if (a.bits == 2)
        hipLaunchKernelGGL((gen_decode_split_kernel<R, 2>), grid, dim3(kGenThreads), lds, s, a);
    else
        hipLaunchKernelGGL((gen_decode_split_kernel<R, 4>), grid, dim3(kGenThreads), lds, s, a);
    return hipGetLastError();
}

}  // namespace

// ---------------------------------------------------------------------------------------------- launchers
template <int D>
static hipError_t launch_gen_assign(const QuantArgs &a, hipStream_t s)
{
    const dim3 grid((a.nq + kGenThreads - 1) / kGenThreads, a.n_streams);
    if (a.metric == PK_METRIC_MINMAX)
        hipLaunchKernelGGL((gen_assign_kernel<D, PK_METRIC_MINMAX>), grid, dim3(kGenThreads), 0, s, a);
    else
        hipLaunchKernelGGL((gen_assign_kernel<D, PK_METRIC_L2>), grid, dim3(kGenThreads), 0, s, a);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_gen_assign_mfma(const QuantArgs &a, hipStream_t s)
{
    static LdsOptIn opt_in;   // per instantiation: the most it needs is a table of 256 patterns
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&gen_assign_mfma_kernel<D>), opt_in, GenSearchLds<D>::bytes(256));
    if (e != hipSuccess) return e;
    // aim at ~2048 workgroups, each staging the table once for at least 16 and at most 256 tiles of 16 vectors
    const int n_tiles = a.nq / 16;
    const int64_t total = (int64_t)n_tiles * a.n_streams;
    int tpw = (int)((total + 2047) / 2048);
    tpw = tpw < 16 ? 16 : tpw > 256 ? 256 : tpw;
    hipLaunchKernelGGL(gen_assign_mfma_kernel<D>, dim3((n_tiles + tpw - 1) / tpw, a.n_streams), dim3(256), GenSearchLds<D>::bytes(a.P), s, a,
                       tpw);
    return hipGetLastError();
}

hipError_t launch_generic_quantize(const QuantArgs &a, bool v_side, hipStream_t s)
{
    if (a.nq <= 0) return hipSuccess;
    if (a.d != 96 && a.d != 256) return hipErrorInvalidValue;
    hipError_t e;
    if (a.metric == PK_METRIC_MINMAX)
        e = a.d == 96 ? launch_gen_assign<96>(a, s) : launch_gen_assign<256>(a, s);
    else
        e = a.d == 96 ? launch_gen_assign_mfma<96>(a, s) : launch_gen_assign_mfma<256>(a, s);
    if (e != hipSuccess) return e;
    const dim3 block(a.d <= 128 ? 128 : kGenThreads);   // thread <-> channel: two waves hold 96 channels (and the 128 indices of a group)
    if (v_side)
        hipLaunchKernelGGL(gen_quantize_v_kernel, dim3(a.nq / 16, a.n_streams), block, 0, s, a);
    else
        hipLaunchKernelGGL(gen_quantize_k_kernel, dim3(a.nq / a.G, a.n_streams), block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_generic_tail_copy(const TailCopyArgs &a, hipStream_t s)
{
    const int64_t work = (int64_t)(a.i1 - a.i0) * (a.d / 8);
    if (work <= 0) return hipSuccess;
    hipLaunchKernelGGL(gen_tail_copy_kernel, dim3((unsigned)((work + 255) / 256), a.n_streams, 2), dim3(256), 0, s, a);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_gen_mine_assign(const MineArgs &a, int last, hipStream_t s)
{
    static LdsOptIn opt_in;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&gen_mine_assign_mfma_kernel<D>), opt_in, GenSearchLds<D>::bytes(256));
    if (e != hipSuccess) return e;
    const int n_tiles = (a.T + 15) / 16;
    const int64_t total = (int64_t)n_tiles * a.n_sets;
    int tpw = (int)((total + 2047) / 2048);
    tpw = tpw < 16 ? 16 : tpw > 256 ? 256 : tpw;
    hipLaunchKernelGGL(gen_mine_assign_mfma_kernel<D>, dim3((n_tiles + tpw - 1) / tpw, a.n_sets), dim3(256), GenSearchLds<D>::bytes(a.P), s,
                       a, last, tpw);
    return hipGetLastError();
}

hipError_t launch_generic_mine(const MineArgs &a, hipStream_t s)
{
    hipError_t e;
    const int chunk = (a.T + a.tsplit - 1) / a.tsplit;
    if (!a.init_given) {
        hipLaunchKernelGGL(gen_mine_init_kernel, dim3((a.P * a.d + 255) / 256, a.n_sets), dim3(256), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    for (int it = 0; it < a.iters; ++it) {
        if ((e = a.d == 96 ? launch_gen_mine_assign<96>(a, it == a.iters - 1 ? 1 : 0, s)
                           : launch_gen_mine_assign<256>(a, it == a.iters - 1 ? 1 : 0, s)) != hipSuccess)
            return e;
        if (a.inertia) {
            hipLaunchKernelGGL(gen_mine_inertia_kernel, dim3(a.n_sets), dim3(256), 0, s, a, it);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        const int per = kSumsLdsFloats / ((kGenThreads / a.d) * a.d) - 1;   // 47 patterns at d = 256, 63 at d = 96 (two slices); a spare row
        const int pblock = a.P < per ? a.P : per;
        hipLaunchKernelGGL(gen_mine_sums_kernel, dim3(a.tsplit, a.n_sets, (a.P + pblock - 1) / pblock), dim3(kGenThreads), 0,
                           s, a, chunk, pblock);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(gen_mine_update_kernel, dim3(a.P, a.n_sets), dim3(kGenThreads), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_generic_window_pattern(const __half *x, int64_t set_stride, int n_sets, int n, int d, __half *out,
                                         int64_t out_stride, hipStream_t s)
{
    hipLaunchKernelGGL(gen_window_pattern_kernel, dim3(n_sets), dim3(kGenThreads), 0, s, x, set_stride, n, d, out, out_stride);
    return hipGetLastError();
}

hipError_t launch_generic_decode(const DecodeArgs &a, hipStream_t s)
{
    // heads of a KV head per workgroup: the power of two that holds them, eight at most; more heads per KV head
    // (up to 64 by the configuration check) go to further workgroups along z
    const int r = a.n_q_heads / a.n_kv_heads;
    const int R = r > 4 ? 8 : r > 2 ? 4 : r > 1 ? 2 : 1;
    const dim3 grid(a.n_seq * a.n_kv_heads, a.splits_prefix + a.splits_own + 2, (r + R - 1) / R);
    const size_t lds = gen_decode_lds_bytes(a.d, a.P, R);
    hipError_t e = R == 8   ? launch_gen_decode_split<8>(a, grid, lds, s)
                   : R == 4 ? launch_gen_decode_split<4>(a, grid, lds, s)
                   : R == 2 ? launch_gen_decode_split<2>(a, grid, lds, s)
                            : launch_gen_decode_split<1>(a, grid, lds, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(gen_decode_merge_kernel, dim3(a.n_seq * a.n_q_heads), dim3(kGenThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_generic_dequant(const DequantArgs &a, hipStream_t s)
{
    if (a.t1 <= a.t0) return hipSuccess;
    hipLaunchKernelGGL(gen_dequant_kernel, dim3(a.t1 - a.t0, a.n_streams), dim3(kGenThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace pk
