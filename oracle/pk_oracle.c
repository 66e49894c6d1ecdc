/*
 * pk_oracle.c -- plain CPU reference for the PatternKV hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is
 * compared against; nothing on the product path may call it.  It shares no
 * code, header, table or helper with the HIP sources.
 *
 * Every function is the paper's definition written out, one scalar operation
 * at a time, in the order the paper states it:
 *   - asymmetric n-bit min / zero-point quantization ........ Sec. 2.1, Eq. 1
 *   - K per channel (over a group of tokens), V per token .... Sec. 4.1,
 *                                                 "Quantization Settings"
 *   - pattern mining = Lloyd iterations on the K-means
 *     objective, Euclidean metric, centroid = pattern ........ Sec. 3.1, Eq. 4
 *   - pattern selection by the min-max distance d_mm and
 *     residual R = X - M* .................................... Sec. 3.2, Eq. 6
 *   - reconstruction X^ = M* + (s*Q + z) ...................... Sec. 3.2
 *   - decode attention = softmax(q.K^ / sqrt(d)) V^ over the
 *     reconstructed cache (what the two fused kernels of
 *     "System Optimization" compute together) ................ Sec. 3.4
 *
 * Points the paper leaves open, and the reading taken here (each one is also
 * listed in the design notes of the repository):
 *   - scale and zero are stored in fp16; the zero point is rounded towards
 *     -inf and the scale towards +inf, so that (r - z)/s always lies in
 *     [0, 2^n - 1] and the half-step error bound of App. C holds for the
 *     stored parameters;
 *   - a flat group (max == min after rounding) gets scale 0, all codes 0;
 *   - rounding to the nearest integer is half-to-even;
 *   - ties between patterns go to the lowest index;
 *   - Lloyd starts from the first P vectors, an empty cluster keeps its
 *     centroid, centroids are rounded to fp16 after every update.
 *
 * Compile: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define PKO_METRIC_L2 0
#define PKO_METRIC_MINMAX 1

/* ------------------------------------------------------------------------- */
/* IEEE binary16 <-> binary32, written from the format definition.            */
/* ------------------------------------------------------------------------- */

float pko_half_to_float(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24); /* subnormal: m * 2^-24 */
    else if (e == 31)
        v = m ? (double)NAN : (double)INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25); /* (1 + m/1024) * 2^(e-15) */
    return (float)(sign ? -v : v);
}

/* bits of a non-negative value that is exactly representable in binary16 */
static uint16_t encode_exact_nonneg(double v)
{
    if (v == 0.0)
        return 0;
    if (v < ldexp(1.0, -14))
        return (uint16_t)(v * ldexp(1.0, 24)); /* subnormal */
    int ex;
    double fr = frexp(v, &ex); /* v = fr * 2^ex, fr in [0.5,1) */
    int e = ex - 1 + 15;       /* biased exponent of 1.xxx * 2^(ex-1) */
    int m = (int)(fr * 2048.0) - 1024;
    return (uint16_t)((e << 10) | m);
}

/* mode: 0 = to nearest, ties to even; -1 = towards -inf; +1 = towards +inf */
static uint16_t float_to_half_mode(float f, int mode)
{
    if (isnan(f))
        return 0x7e00;
    double a = fabs((double)f);
    int neg = signbit(f) ? 1 : 0;
    /* rounding direction on the magnitude */
    int mag_mode = mode;
    if (neg)
        mag_mode = -mode;
    const double hmax = 65504.0;
    uint16_t bits;
    if (isinf(f)) {
        bits = 0x7c00;
    } else if (a == 0.0) {
        bits = 0;
    } else {
        int ex;
        (void)frexp(a, &ex);   /* a in [2^(ex-1), 2^ex) */
        int e = ex - 1;        /* floor(log2 a) */
        if (e < -14)
            e = -14;           /* subnormal quantum */
        double q = ldexp(1.0, e - 10); /* spacing of binary16 around a */
        double n = a / q;      /* exact: power-of-two scaling */
        double lo = floor(n), hi = ceil(n);
        double pick;
        if (lo == hi)
            pick = lo;
        else if (mag_mode < 0)
            pick = lo;
        else if (mag_mode > 0)
            pick = hi;
        else {
            double dl = n - lo, dh = hi - n;
            if (dl < dh)
                pick = lo;
            else if (dh < dl)
                pick = hi;
            else
                pick = (fmod(lo, 2.0) == 0.0) ? lo : hi;
        }
        double r = pick * q;
        if (r > hmax) {
            /* beyond the largest finite value */
            if (mag_mode < 0)
                bits = 0x7bff;
            else
                bits = 0x7c00;
        } else {
            bits = encode_exact_nonneg(r);
        }
    }
    /* round-down of a tiny negative magnitude to zero keeps the sign bit off
       only when the result is +0; -0 is returned for negative inputs that
       round to zero, which compares equal to 0 everywhere it is used.       */
    return (uint16_t)(bits | (neg ? 0x8000 : 0));
}

uint16_t pko_float_to_half_rne(float f) { return float_to_half_mode(f, 0); }
uint16_t pko_float_to_half_down(float f) { return float_to_half_mode(f, -1); }
uint16_t pko_float_to_half_up(float f) { return float_to_half_mode(f, +1); }

/* ------------------------------------------------------------------------- */
/* Pattern selection.                                                         */
/* ------------------------------------------------------------------------- */

/*
 * Distance of one vector x[d] to one pattern m[d].
 *   L2     : squared Euclidean distance, accumulated in double (the metric
 *            K-means minimises, Sec. 3.1 Eq. 4).
 *   MINMAX : d_mm(x,m) = max_i(x_i - m_i) - min_j(x_j - m_j), Sec. 3.2; each
 *            difference is one binary32 subtraction, max/min are exact.
 */
static double distance_one(const uint16_t *x, const uint16_t *m, int d, int metric)
{
    if (metric == PKO_METRIC_L2) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c) {
            double diff = (double)pko_half_to_float(x[c]) - (double)pko_half_to_float(m[c]);
            acc += diff * diff;
        }
        return acc;
    } else {
        float mx = -INFINITY, mn = INFINITY;
        for (int c = 0; c < d; ++c) {
            float diff = pko_half_to_float(x[c]) - pko_half_to_float(m[c]);
            if (diff > mx)
                mx = diff;
            if (diff < mn)
                mn = diff;
        }
        float w = mx - mn;
        return (double)w;
    }
}

/*
 * Nearest pattern for T vectors of one stream (Sec. 3.2 Eq. 6 argmin; the
 * assignment step of Lloyd for L2).  idx[t] is the lowest index attaining the
 * minimum.  best[t] / second[t] (optional) are the smallest and second
 * smallest distances, used by the tests to find near-ties.
 */
void pko_assign(const uint16_t *x, int64_t T, int d, const uint16_t *M, int P, int metric,
                int32_t *idx, double *best, double *second)
{
    for (int64_t t = 0; t < T; ++t) {
        double b1 = INFINITY, b2 = INFINITY;
        int arg = 0;
        for (int p = 0; p < P; ++p) {
            double D = distance_one(x + t * d, M + (int64_t)p * d, d, metric);
            if (D < b1) {
                b2 = b1;
                b1 = D;
                arg = p;
            } else if (D < b2) {
                b2 = D;
            }
        }
        idx[t] = arg;
        if (best)
            best[t] = b1;
        if (second)
            second[t] = b2;
    }
}

/* ------------------------------------------------------------------------- */
/* Pattern mining: Lloyd iterations for the objective of Sec. 3.1 Eq. 4.      */
/* ------------------------------------------------------------------------- */

/*
 * x[T][d] fp16, one pattern set.  M[P][d]: if init_given == 0 it is first set
 * to the first P vectors, else used as passed.  Each iteration: assign every
 * vector to its nearest centroid (Euclidean), then replace every non-empty
 * cluster's centroid by the mean of its members, rounded to fp16.
 * assign[T]  : assignment of the LAST assignment step (i.e. with respect to
 *              the centroids before the last update).
 * inertia[i] : within-cluster sum of squares seen by assignment step i.
 * counts[P]  : cluster sizes of the last assignment step.
 */
void pko_mine(const uint16_t *x, int64_t T, int d, int P, int iters, int init_given,
              uint16_t *M, int32_t *assign, double *inertia, int32_t *counts)
{
    if (!init_given)
        for (int p = 0; p < P; ++p)
            memcpy(M + (int64_t)p * d, x + (int64_t)p * d, sizeof(uint16_t) * d);
    double *sum = (double *)malloc(sizeof(double) * P * d);
    int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * P);
    double *best = (double *)malloc(sizeof(double) * T);
    for (int it = 0; it < iters; ++it) {
        pko_assign(x, T, d, M, P, PKO_METRIC_L2, assign, best, NULL);
        double J = 0.0;
        memset(sum, 0, sizeof(double) * P * d);
        memset(cnt, 0, sizeof(int64_t) * P);
        for (int64_t t = 0; t < T; ++t) {
            int a = assign[t];
            J += best[t];
            cnt[a] += 1;
            for (int c = 0; c < d; ++c)
                sum[(int64_t)a * d + c] += (double)pko_half_to_float(x[t * d + c]);
        }
        if (inertia)
            inertia[it] = J;
        for (int p = 0; p < P; ++p) {
            if (counts)
                counts[p] = (int32_t)cnt[p];
            if (cnt[p] == 0)
                continue;
            for (int c = 0; c < d; ++c) {
                float mean = (float)(sum[(int64_t)p * d + c] / (double)cnt[p]);
                M[(int64_t)p * d + c] = pko_float_to_half_rne(mean);
            }
        }
    }
    free(sum);
    free(cnt);
    free(best);
}

/* ------------------------------------------------------------------------- */
/* Residual + asymmetric quantization (Sec. 2.1 Eq. 1 on R = X - M*).         */
/* ------------------------------------------------------------------------- */

/* scale / zero of one group from its residual min and max */
static void group_params(float mn, float mx, int bits, uint16_t *s16, uint16_t *z16)
{
    uint16_t z = pko_float_to_half_down(mn);            /* z = min(R), stored fp16 */
    float zf = pko_half_to_float(z);
    float s32 = (mx - zf) / (float)((1 << bits) - 1);   /* s = (max - z)/(2^n - 1) */
    uint16_t s = pko_float_to_half_up(s32);
    *s16 = s;
    *z16 = z;
}

static uint8_t quantize_one(float r, uint16_t s16, uint16_t z16, int bits)
{
    float s = pko_half_to_float(s16);
    if (s == 0.0f)
        return 0;
    float z = pko_half_to_float(z16);
    float inv = 1.0f / s;
    float q = rintf((r - z) * inv); /* round to nearest, ties to even */
    float qmax = (float)((1 << bits) - 1);
    if (q < 0.0f)
        q = 0.0f;
    if (q > qmax)
        q = qmax;
    return (uint8_t)q;
}

/*
 * K side: n tokens (n a multiple of G) of one stream; one (s,z) per channel
 * and group of G consecutive tokens.
 *   codes[n][d] (one byte each), scale/zero[n/G][d] fp16 bits.
 */
void pko_quantize_k(const uint16_t *x, int n, int d, const uint16_t *M, const int32_t *idx,
                    int bits, int G, uint8_t *codes, uint16_t *scale, uint16_t *zero)
{
    float *r = (float *)malloc(sizeof(float) * (size_t)G * d);
    for (int g = 0; g < n / G; ++g) {
        for (int i = 0; i < G; ++i) {
            int t = g * G + i;
            const uint16_t *m = M + (int64_t)idx[t] * d;
            for (int c = 0; c < d; ++c)
                r[i * d + c] = pko_half_to_float(x[(int64_t)t * d + c]) - pko_half_to_float(m[c]);
        }
        for (int c = 0; c < d; ++c) {
            float mn = r[c], mx = r[c];
            for (int i = 1; i < G; ++i) {
                float v = r[i * d + c];
                if (v < mn)
                    mn = v;
                if (v > mx)
                    mx = v;
            }
            uint16_t s16, z16;
            group_params(mn, mx, bits, &s16, &z16);
            scale[(int64_t)g * d + c] = s16;
            zero[(int64_t)g * d + c] = z16;
            for (int i = 0; i < G; ++i)
                codes[(int64_t)(g * G + i) * d + c] = quantize_one(r[i * d + c], s16, z16, bits);
        }
    }
    free(r);
}

/*
 * V side: per token, one (s,z) per group of Gc consecutive channels
 * (Gc = min(G, d)).  codes[n][d]; scale/zero are stored in slices of 16 tokens,
 * [n/16][d/Gc][16]: the parameter of token t and channel group j is at
 * ((t/16)*(d/Gc) + j)*16 + t%16.
 */
static int64_t v_param(int64_t t, int j, int ng) { return ((t / 16) * ng + j) * 16 + t % 16; }

/*
 * V side with the adaptive threshold of Sec. 3.3 ("Adaptive Threshold for V"): a token keeps its
 * pattern only if the range of the residual is at most rho times the range of the raw vector,
 *     R_flat = max_c r_c - min_c r_c ,  R_raw = max_c x_c - min_c x_c ,  R_flat <= rho * R_raw
 * (one binary32 multiply, ranges over all d channels of the token); otherwise the raw vector is
 * quantized and the index becomes PKO_NO_PATTERN.  rho = rho_*(d, alpha) of Sec. 3.3 is the caller's;
 * rho <= 0 switches the test off.
 */
#define PKO_NO_PATTERN 255

void pko_quantize_v(const uint16_t *x, int n, int d, const uint16_t *M, int32_t *idx,
                    int bits, int Gc, float rho, uint8_t *codes, uint16_t *scale, uint16_t *zero)
{
    int ng = d / Gc;
    float *r = (float *)malloc(sizeof(float) * d);
    for (int t = 0; t < n; ++t) {
        const uint16_t *m = M + (int64_t)idx[t] * d;
        for (int c = 0; c < d; ++c)
            r[c] = pko_half_to_float(x[(int64_t)t * d + c]) - pko_half_to_float(m[c]);
        if (rho > 0.0f) {
            float rmn = r[0], rmx = r[0];
            float xmn = pko_half_to_float(x[(int64_t)t * d]), xmx = xmn;
            for (int c = 1; c < d; ++c) {
                float xv = pko_half_to_float(x[(int64_t)t * d + c]);
                if (r[c] < rmn) rmn = r[c];
                if (r[c] > rmx) rmx = r[c];
                if (xv < xmn) xmn = xv;
                if (xv > xmx) xmx = xv;
            }
            float r_flat = rmx - rmn, r_raw = xmx - xmn;
            if (!(r_flat <= rho * r_raw)) {
                for (int c = 0; c < d; ++c)
                    r[c] = pko_half_to_float(x[(int64_t)t * d + c]);
                idx[t] = PKO_NO_PATTERN;
            }
        }
        for (int j = 0; j < ng; ++j) {
            float mn = r[j * Gc], mx = r[j * Gc];
            for (int c = j * Gc + 1; c < (j + 1) * Gc; ++c) {
                if (r[c] < mn)
                    mn = r[c];
                if (r[c] > mx)
                    mx = r[c];
            }
            uint16_t s16, z16;
            group_params(mn, mx, bits, &s16, &z16);
            scale[v_param(t, j, ng)] = s16;
            zero[v_param(t, j, ng)] = z16;
            for (int c = j * Gc; c < (j + 1) * Gc; ++c)
                codes[(int64_t)t * d + c] = quantize_one(r[c], s16, z16, bits);
        }
    }
    free(r);
}

/*
 * Decode-stage pattern of a window of vectors (Sec. 3.1 "Decoding Stage", Eq. 5): per channel the
 * Chebyshev centre of the window's values, (min_i x_ic + max_i x_ic) / 2, computed in binary32 (the sum
 * of two fp16 values and the halving are exact) and rounded to fp16, ties to even.
 */
void pko_window_pattern(const uint16_t *x, int n, int d, uint16_t *out)
{
    for (int c = 0; c < d; ++c) {
        float mn = pko_half_to_float(x[c]), mx = mn;
        for (int t = 1; t < n; ++t) {
            float v = pko_half_to_float(x[(int64_t)t * d + c]);
            if (v < mn) mn = v;
            if (v > mx) mx = v;
        }
        out[c] = pko_float_to_half_rne((mn + mx) * 0.5f);
    }
}

/* ------------------------------------------------------------------------- */
/* Bit-plane packing.  The paper does not fix a storage format; this is the   */
/* format of this repository, defined by the two index formulas below.        */
/* ------------------------------------------------------------------------- */

/*
 * K codes: one row of (d/32)*bits little-endian 32-bit words per token.
 * Word (w, j) of token t sits at  out[(t*(d/32) + w)*bits + j];  its bit i is
 * bit j of the code of channel 32*w + i.
 */
void pko_pack_k(const uint8_t *codes, int n, int d, int bits, uint32_t *out)
{
    int W = d / 32;
    memset(out, 0, sizeof(uint32_t) * (size_t)n * W * bits);
    for (int t = 0; t < n; ++t)
        for (int c = 0; c < d; ++c)
            for (int j = 0; j < bits; ++j)
                if ((codes[(int64_t)t * d + c] >> j) & 1)
                    out[((int64_t)t * W + c / 32) * bits + j] |= (uint32_t)1 << (c % 32);
}

void pko_unpack_k(const uint32_t *in, int n, int d, int bits, uint8_t *codes)
{
    int W = d / 32;
    for (int t = 0; t < n; ++t)
        for (int c = 0; c < d; ++c) {
            int v = 0;
            for (int j = 0; j < bits; ++j)
                v |= (int)((in[((int64_t)t * W + c / 32) * bits + j] >> (c % 32)) & 1) << j;
            codes[(int64_t)t * d + c] = (uint8_t)v;
        }
}

/*
 * V codes: the bit planes run along the tokens.  Tokens are packed in blocks of
 * 64 = 4 units of 16; one little-endian 32-bit word holds two planes of one
 * channel for the 16 tokens of a unit: bit (16*(j%2) + t%16) of word
 *     (((t/64)*4 + (t%64)/16)*16 + c%16) * (d/16)*(bits/2) + (c/16)*(bits/2) + j/2
 * is bit j of the code of channel c of token t.  A block occupies
 * 64*d*bits/8 bytes, the same as 64 K rows.
 */
static int64_t v_word(int64_t t, int c, int j, int d, int bits)
{
    int64_t unit = (t / 64) * 4 + (t % 64) / 16;
    return ((unit * 16 + c % 16) * (d / 16) + c / 16) * (bits / 2) + j / 2;
}

void pko_pack_v(const uint8_t *codes, int n, int d, int bits, uint32_t *out)
{
    memset(out, 0, (size_t)n * d * bits / 8);
    for (int t = 0; t < n; ++t)
        for (int c = 0; c < d; ++c)
            for (int j = 0; j < bits; ++j)
                if ((codes[(int64_t)t * d + c] >> j) & 1)
                    out[v_word(t, c, j, d, bits)] |= (uint32_t)1 << (16 * (j % 2) + t % 16);
}

void pko_unpack_v(const uint32_t *in, int n, int d, int bits, uint8_t *codes)
{
    for (int t = 0; t < n; ++t)
        for (int c = 0; c < d; ++c) {
            int v = 0;
            for (int j = 0; j < bits; ++j)
                v |= (int)((in[v_word(t, c, j, d, bits)] >> (16 * (j % 2) + t % 16)) & 1) << j;
            codes[(int64_t)t * d + c] = (uint8_t)v;
        }
}

/* ------------------------------------------------------------------------- */
/* Reconstruction  X^ = M* + (s*Q + z)   (Sec. 3.2), binary32, in that order. */
/* ------------------------------------------------------------------------- */

void pko_dequant_k(const uint8_t *codes, const uint16_t *scale, const uint16_t *zero,
                   const int32_t *idx, const uint16_t *M, int n, int d, int G, float *out)
{
    for (int t = 0; t < n; ++t)
        for (int c = 0; c < d; ++c) {
            float s = pko_half_to_float(scale[(int64_t)(t / G) * d + c]);
            float z = pko_half_to_float(zero[(int64_t)(t / G) * d + c]);
            float res = s * (float)codes[(int64_t)t * d + c] + z;
            out[(int64_t)t * d + c] = pko_half_to_float(M[(int64_t)idx[t] * d + c]) + res;
        }
}

/* thresholded != 0: tokens whose index is PKO_NO_PATTERN were quantized raw (Sec. 3.3), no pattern is added */
void pko_dequant_v(const uint8_t *codes, const uint16_t *scale, const uint16_t *zero,
                   const int32_t *idx, const uint16_t *M, int n, int d, int Gc, int thresholded, float *out)
{
    int ng = d / Gc;
    for (int t = 0; t < n; ++t)
        for (int c = 0; c < d; ++c) {
            float s = pko_half_to_float(scale[v_param(t, c / Gc, ng)]);
            float z = pko_half_to_float(zero[v_param(t, c / Gc, ng)]);
            float res = s * (float)codes[(int64_t)t * d + c] + z;
            if (thresholded && idx[t] == PKO_NO_PATTERN)
                out[(int64_t)t * d + c] = res;
            else
                out[(int64_t)t * d + c] = pko_half_to_float(M[(int64_t)idx[t] * d + c]) + res;
        }
}

/* ------------------------------------------------------------------------- */
/* Decode attention over reconstructed K^, V^ (binary32 values), in double.   */
/* ------------------------------------------------------------------------- */

/*
 * One query head: q[d] fp16, Khat/Vhat[T][d] float, softmax_scale (1/sqrt d).
 * out[d] = sum_t softmax_t(scale * q.Khat_t) * Vhat_t ;  lse = log sum exp.
 */
void pko_attend_head(const uint16_t *q, const float *Khat, const float *Vhat, int64_t T, int d,
                     double softmax_scale, float *out, float *lse)
{
    double *s = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
    double mx = -INFINITY;
    for (int64_t t = 0; t < T; ++t) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c)
            acc += (double)pko_half_to_float(q[c]) * (double)Khat[t * d + c];
        s[t] = acc * softmax_scale;
        if (s[t] > mx)
            mx = s[t];
    }
    double den = 0.0;
    for (int64_t t = 0; t < T; ++t) {
        s[t] = exp(s[t] - mx);
        den += s[t];
    }
    for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int64_t t = 0; t < T; ++t)
            acc += s[t] * (double)Vhat[t * d + c];
        out[c] = (float)(T > 0 ? acc / den : 0.0);
    }
    if (lse)
        *lse = (float)(T > 0 ? mx + log(den) : -INFINITY);
    free(s);
}

/* ------------------------------------------------------------------------- */
/* Batched drivers: the same per-stream functions, looped over independent    */
/* streams (sequence x KV head).  OpenMP is used across streams only.         */
/* ------------------------------------------------------------------------- */

int pko_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}

/* x[S][T][d]; M[S][P][d]; assign[S][T]; inertia[S][iters]; counts[S][P] */
void pko_mine_sets(const uint16_t *x, int S, int64_t T, int d, int P, int iters, int init_given,
                   uint16_t *M, int32_t *assign, double *inertia, int32_t *counts)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < S; ++s)
        pko_mine(x + (int64_t)s * T * d, T, d, P, iters, init_given, M + (int64_t)s * P * d,
                 assign + (int64_t)s * T, inertia ? inertia + (int64_t)s * iters : NULL,
                 counts ? counts + (int64_t)s * P : NULL);
}

/*
 * Assign + quantize + pack n tokens of each of N streams.
 *   x[N][n][d]; set_of[N] = pattern set of each stream; M[sets][P][d].
 *   side: 0 = K (groups of G tokens per channel), 1 = V (groups of Gc channels).
 * Outputs (per stream, contiguous): idx[N][n] int32, best/second[N][n]
 * (optional), codes_unpacked[N][n][d] (optional), packed[N][n*d*bits/8 bytes],
 * scale/zero[N][(n/G)*d] (K) or [N][(n/16)*(d/Gc)*16] (V).
 */
void pko_quantize_streams(const uint16_t *x, int N, int n, int d, const int32_t *set_of,
                          const uint16_t *M, int P, int metric, int bits, int G, int side, float v_rho,
                          int32_t *idx, double *best, double *second, uint8_t *codes_unpacked,
                          uint8_t *packed, uint16_t *scale, uint16_t *zero)
{
    int Gc = G < d ? G : d;
    int64_t nparam = side == 0 ? (int64_t)(n / G) * d : (int64_t)n * (d / Gc);
    int64_t npacked = (int64_t)n * d * bits / 8;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < N; ++s) {
        const uint16_t *xs = x + (int64_t)s * n * d;
        const uint16_t *Ms = M + (int64_t)set_of[s] * P * d;
        int32_t *ix = idx + (int64_t)s * n;
        uint8_t *codes = (uint8_t *)malloc((size_t)n * d);
        pko_assign(xs, n, d, Ms, P, metric, ix, best ? best + (int64_t)s * n : NULL,
                   second ? second + (int64_t)s * n : NULL);
        if (side == 0) {
            pko_quantize_k(xs, n, d, Ms, ix, bits, G, codes, scale + s * nparam, zero + s * nparam);
            pko_pack_k(codes, n, d, bits, (uint32_t *)(packed + s * npacked));
        } else {
            pko_quantize_v(xs, n, d, Ms, ix, bits, Gc, v_rho, codes, scale + s * nparam, zero + s * nparam);
            pko_pack_v(codes, n, d, bits, (uint32_t *)(packed + s * npacked));
        }
        if (codes_unpacked)
            memcpy(codes_unpacked + (int64_t)s * n * d, codes, (size_t)n * d);
        free(codes);
    }
}

/*
 * Attention for n_seq sequences: q[n_seq][Hq][d]; Khat/Vhat[n_seq][Hkv][T][d];
 * query head h reads KV head h / (Hq/Hkv).  out[n_seq][Hq][d], lse[n_seq][Hq].
 */
void pko_attend_streams(const uint16_t *q, const float *Khat, const float *Vhat, int n_seq,
                        int Hq, int Hkv, int64_t T, int d, double softmax_scale, float *out,
                        float *lse)
{
    int r = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < n_seq * Hq; ++u) {
        int s = u / Hq, h = u % Hq;
        int64_t kv = (int64_t)s * Hkv + h / r;
        pko_attend_head(q + (int64_t)u * d, Khat + kv * T * d, Vhat + kv * T * d, T, d,
                        softmax_scale, out + (int64_t)u * d, lse ? lse + u : NULL);
    }
}
