// Nearest-pattern search under the Euclidean metric on the matrix cores (Sec. 3.1 Eq. 4 assignment
// step; Sec. 3.2 Eq. 6 argmin in L2 mode).
//
// Ranking uses e = x.m - ||m||^2/2 - ||x||^2/2 = -||x - m||^2 / 2 from v_mfma_f32_16x16x32_f16: the
// accumulator starts at -(||m||^2 + ||x||^2)/2 and the four K-steps add x.m (fp16 products are exact in
// fp32; only the accumulation rounds).  The best and second best value are tracked; a token whose gap
// between the two is not safely above the rounding error of that form is re-evaluated exactly,
// sum_c (x_c - m_c)^2 in binary32 over all patterns, lowest index on ties.  A token that is not
// re-evaluated has a gap larger than any possible ranking error, so the result always equals the
// exact argmin.
//
// Operand layout (lane = 16*kb + n):  A = patterns, row n of the 16-pattern tile, K-step s covers
// channels 32*s + 8*kb + j;  B = vectors, column n = token n of the 16-token tile, same channels;
// D: column n = token, rows 4*kb + i = patterns 16*tile + 4*kb + i.
#pragma once

#include "pk_internal.h"

namespace pk {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

constexpr int kTabStride = kD + 16;   // halves per pattern row in LDS: 288 B = 72 words, the row skew at which 16-byte reads of 16 rows x 4 column groups run at full rate

__host__ __device__ constexpr int pad16(int p) { return (p + 15) & ~15; }

struct PatternTable {
    const __half *lds_rows;   // LDS copy, pad16(P) rows of stride kTabStride, rows past P are zero
    const float *nh;          // LDS [pad16(P)]: -||m_p||^2 / 2, -inf past P
    float norm2_max;          // max_p ||m_p||^2
    int P;
};

__device__ __forceinline__ floatx4_t mfma_f16(const uint4 &a, const uint4 &b, floatx4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
}

// Stage a pattern table into LDS (nthr threads, a multiple of 64 dividing pad16(P)*16... or not: the loop is
// guarded) and compute the row norms; red_s gets one maximum per wave.  Ends with a barrier.
// Work item i = (row i/16, 16-byte piece i%16): the 16 lanes of a row sum their squares.
__device__ __forceinline__ void stage_patterns(const __half *Mg, int P, __half *tab_s, float *nh_s, float *red_s,
                                               int nthr = 256)
{
    const int tid = threadIdx.x;
    float mx = 0.f;
    // pad16(P) * 16 is a multiple of 256, and every 16 consecutive work items sit in one wave: the row sums
    // below see whole rows (a trailing half round of a 512-thread group has whole waves idle)
    for (int i = tid; i < pad16(P) * kRowChunks; i += nthr) {
        const int r = i >> 4, ch = i & 15;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (r < P) v = *reinterpret_cast<const uint4 *>(Mg + (int64_t)r * kD + ch * 8);
        *reinterpret_cast<uint4 *>(tab_s + r * kTabStride + ch * 8) = v;   // rows past P are zero
        const half2_t *h = reinterpret_cast<const half2_t *>(&v);
        float acc = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) acc = __builtin_amdgcn_fdot2(h[k], h[k], acc, false);
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) acc += __shfl_xor(acc, off);
        if (ch == 0) nh_s[r] = r < P ? -0.5f * acc : -INFINITY;   // rows past the table never win
        mx = fmaxf(mx, acc);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if ((tid & 63) == 0) red_s[tid >> 6] = mx;
    __syncthreads();
}

// A operand and accumulator start of one 16-pattern tile.
struct PatternTile {
    uint4 a[4];
    float4 nh;
};

__device__ __forceinline__ void load_pattern_tile(const PatternTable &tb, int p0, int n, int kb, PatternTile &t)
{
    const __half *arow = tb.lds_rows + (p0 + n) * kTabStride + 8 * kb;
#pragma unroll
    for (int s = 0; s < 4; ++s) t.a[s] = *reinterpret_cast<const uint4 *>(arow + 32 * s);
    t.nh = *reinterpret_cast<const float4 *>(tb.nh + p0 + 4 * kb);
}

// Candidates are ranked as unsigned integer keys: the binary32 pattern of e with the low 8 mantissa bits
// replaced by the pattern index.  e <= 0 up to rounding; among negative floats the unsigned order of the
// patterns is the order of decreasing value, so the smallest key is the nearest pattern.  An e that
// rounding made slightly positive ranks below every negative one, which is right, and can only be
// mis-ordered against another such e: both are then inside the re-evaluation band.
__device__ __forceinline__ void rank_pattern_tile(const uint4 (&xb)[4], const PatternTile &t, float hx, int p0, uint32_t &k1,
                                                  uint32_t &k2)
{
    floatx4_t d = {t.nh.x - hx, t.nh.y - hx, t.nh.z - hx, t.nh.w - hx};
#pragma unroll
    for (int s = 0; s < 4; ++s) d = mfma_f16(t.a[s], xb[s], d);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // bytes 3..1 of e, byte 0 = index (one byte permute)
        const uint32_t key = __builtin_amdgcn_perm(__float_as_uint(d[i]), (uint32_t)(p0 + i), 0x07060500u);
        k2 = max(min(k1, k2), min(max(k1, k2), key));   // median of three = second smallest so far
        k1 = min(k1, key);
    }
}

// NT 16-token tiles held as B operands xb[j][4] (K-step s in xb[j][s]); every pattern tile read from the table
// serves all NT of them.  Returns, in every lane of column n, per tile: best index, best squared distance (from
// the expanded form, low 8 mantissa bits dropped), ||x||^2 and whether the token needs the exact re-evaluation.
template <int NT>
__device__ __forceinline__ void assign_tiles_mfma(const uint4 (&xb)[NT][4], const PatternTable &tb, int lane, int (&best_i)[NT],
                                                  float (&best_v)[NT], float (&x2)[NT], bool (&flag)[NT])
{
    const int n = lane & 15, kb = lane >> 4;
    float xx[NT], hx[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        float acc = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const half2_t *h = reinterpret_cast<const half2_t *>(&xb[j][s]);
#pragma unroll
            for (int k = 0; k < 4; ++k) acc = __builtin_amdgcn_fdot2(h[k], h[k], acc, false);
        }
        acc += __shfl_xor(acc, 16);
        acc += __shfl_xor(acc, 32);
        xx[j] = acc;
        hx[j] = 0.5f * acc;
    }

    // the key's index bits are p0 + i here; the lane's 4*kb is added after the loop (no carries: p0 % 16 == 0)
    uint32_t k1[NT], k2[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) k1[j] = k2[j] = 0xffffffffu;   // above every key
    const int Pp = pad16(tb.P);
    PatternTile ta, tc;
    load_pattern_tile(tb, 0, n, kb, ta);
    for (int p0 = 0;;) {   // two tiles per round, the next one in flight while the current is ranked
        if (p0 + 16 < Pp) load_pattern_tile(tb, p0 + 16, n, kb, tc);
#pragma unroll
        for (int j = 0; j < NT; ++j) rank_pattern_tile(xb[j], ta, hx[j], p0, k1[j], k2[j]);
        if ((p0 += 16) >= Pp) break;
        if (p0 + 16 < Pp) load_pattern_tile(tb, p0 + 16, n, kb, ta);
#pragma unroll
        for (int j = 0; j < NT; ++j) rank_pattern_tile(xb[j], tc, hx[j], p0, k1[j], k2[j]);
        if ((p0 += 16) >= Pp) break;
    }
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        uint32_t a1 = k1[j] | (uint32_t)kb << 2, a2 = k2[j] | (uint32_t)kb << 2;
        // merge the four lane groups of the column
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            const uint32_t o1 = (uint32_t)__shfl_xor((int)a1, off), o2 = (uint32_t)__shfl_xor((int)a2, off);
            a2 = min(min(a2, o2), max(a1, o1));
            a1 = min(a1, o1);
        }
        best_i[j] = (int)(a1 & 0xffu);
        best_v[j] = -2.f * __uint_as_float(a1 & 0xffffff00u);
        const float second = -2.f * __uint_as_float(a2 & 0xffffff00u);
        x2[j] = xx[j];
        // accumulation error of e is far below 2^-21 (|x|^2 + |m|^2), the keys drop 8 mantissa bits:
        // flag with a wide margin.  A single pattern has nothing to be confused with.
        flag[j] = tb.P > 1 && !(second - best_v[j] > 7.62939453125e-06f * (xx[j] + tb.norm2_max) + 6.103515625e-05f * second);
    }
}

// One 16-token tile.
__device__ __forceinline__ void assign_tile_mfma(const uint4 (&xb)[4], const PatternTable &tb, int lane, int &best_i,
                                                 float &best_v, float &x2, bool &flag)
{
    int bi[1];
    float bv[1], xx[1];
    bool fl[1];
    assign_tiles_mfma<1>(reinterpret_cast<const uint4 (&)[1][4]>(xb), tb, lane, bi, bv, xx, fl);
    best_i = bi[0];
    best_v = bv[0];
    x2 = xx[0];
    flag = fl[0];
}

// Exact re-evaluation of one token by a whole wave: xrow_s = its 128 channels (fp16) in LDS.
// Every lane returns the exact argmin (lowest index on ties) and its distance.
__device__ __forceinline__ void exact_argmin_wave(const __half *xrow_s, const PatternTable &tb, int lane, int &best_i,
                                                  float &best_d)
{
    float bd = INFINITY;
    int bi = 0x7fffffff;
    for (int p = lane; p < tb.P; p += 64) {
        // the pattern rows come from the LDS copy of the table (the same fp16 values): read from global memory they
        // missed L2 often enough to add a fifth to the HBM traffic of a mining step on a large job
        const __half *m = tb.lds_rows + p * kTabStride;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll 4
        for (int ch = 0; ch < kRowChunks; ++ch) {   // several row pieces in flight
            const uint4 mv = *reinterpret_cast<const uint4 *>(m + ch * 8);
            const uint4 xv = *reinterpret_cast<const uint4 *>(xrow_s + ch * 8);
            // (one v_fma_mix_f32 per difference instead of two conversions and a subtraction: the same value)
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
    best_i = bi;
    best_d = bd;
}

// Re-evaluate the flagged tokens of a tile.  xrow_s: per-wave LDS scratch of kD halves.
__device__ __forceinline__ void resolve_flagged(const uint4 (&xb)[4], bool flag, __half *xrow_s, const PatternTable &tb,
                                                int lane, int &best_i, float &best_d)
{
    const int n = lane & 15, kb = lane >> 4;
    unsigned long long todo = __ballot(flag) & 0xffffull;   // one bit per column
    while (todo) {
        const int col = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        if (n == col) {
#pragma unroll
            for (int s = 0; s < 4; ++s) *reinterpret_cast<uint4 *>(xrow_s + 32 * s + 8 * kb) = xb[s];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        int bi;
        float bd;
        exact_argmin_wave(xrow_s, tb, lane, bi, bd);
        if (n == col) {
            best_i = bi;
            best_d = bd;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

}  // namespace pk
