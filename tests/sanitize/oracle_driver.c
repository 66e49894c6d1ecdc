/* Drives every entry point of oracle/pk_oracle.c once on small seeded inputs, with exactly sized heap buffers, so
 * that AddressSanitizer / UndefinedBehaviorSanitizer see any access past a buffer, misaligned access, signed overflow
 * or invalid shift.  Built and run by tests/test_sanitizers_cpu.py; prints "ok" and exits 0. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

float pko_half_to_float(uint16_t h);
uint16_t pko_float_to_half_rne(float f);
uint16_t pko_float_to_half_down(float f);
uint16_t pko_float_to_half_up(float f);
void pko_mine_sets(const uint16_t *x, int S, int64_t T, int d, int P, int iters, int init_given, uint16_t *M,
                   int32_t *assign, double *inertia, int32_t *counts);
void pko_quantize_streams(const uint16_t *x, int N, int n, int d, const int32_t *set_of, const uint16_t *M, int P,
                          int metric, int bits, int G, int side, float v_rho, int32_t *idx, double *best, double *second,
                          uint8_t *codes_unpacked, uint8_t *packed, uint16_t *scale, uint16_t *zero);
void pko_unpack_k(const uint32_t *in, int n, int d, int bits, uint8_t *codes);
void pko_unpack_v(const uint32_t *in, int n, int d, int bits, uint8_t *codes);
void pko_dequant_k(const uint8_t *codes, const uint16_t *scale, const uint16_t *zero, const int32_t *idx, const uint16_t *M,
                   int n, int d, int G, float *out);
void pko_dequant_v(const uint8_t *codes, const uint16_t *scale, const uint16_t *zero, const int32_t *idx, const uint16_t *M,
                   int n, int d, int Gc, int thresholded, float *out);
void pko_window_pattern(const uint16_t *x, int n, int d, uint16_t *out);
void pko_attend_streams(const uint16_t *q, const float *Khat, const float *Vhat, int n_seq, int Hq, int Hkv, int64_t T, int d,
                        double softmax_scale, float *out, float *lse);

static uint32_t rng_state = 12345u;
static float rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return ((rng_state >> 8) & 0xffff) / 32768.0f - 1.0f;
}

int main(void)
{
    const int d = 128, P = 7, n = 192, N = 3, iters = 3;
    uint16_t *x = malloc(sizeof(uint16_t) * N * n * d);
    for (int i = 0; i < N * n * d; ++i) x[i] = pko_float_to_half_rne(3.0f * rnd() + ((i % d) == 5 ? 20.0f : 0.0f));
    if (pko_half_to_float(pko_float_to_half_down(0.1f)) > 0.1f || pko_half_to_float(pko_float_to_half_up(0.1f)) < 0.1f) return 2;
    uint16_t *M = malloc(sizeof(uint16_t) * N * P * d);
    int32_t *assign = malloc(sizeof(int32_t) * N * n), *counts = malloc(sizeof(int32_t) * N * P);
    double *inertia = malloc(sizeof(double) * N * iters);
    pko_mine_sets(x, N, n, d, P, iters, 0, M, assign, inertia, counts);
    int32_t set_of[3] = {0, 1, 2};
    for (int metric = 0; metric < 2; ++metric)
        for (int bits = 2; bits <= 4; bits += 2)
            for (int side = 0; side < 2; ++side)
                for (int G = 32; G <= 128; G *= 2) {
                    if (n % G) continue;
                    const int Gc = G < d ? G : d;
                    const size_t nparam = side == 0 ? (size_t)(n / G) * d : (size_t)n * (d / Gc);
                    int32_t *idx = malloc(sizeof(int32_t) * N * n);
                    double *best = malloc(sizeof(double) * N * n), *second = malloc(sizeof(double) * N * n);
                    uint8_t *codes = malloc((size_t)N * n * d), *packed = malloc((size_t)N * n * d * bits / 8);
                    uint16_t *scale = malloc(sizeof(uint16_t) * N * nparam), *zero = malloc(sizeof(uint16_t) * N * nparam);
                    pko_quantize_streams(x, N, n, d, set_of, M, P, metric, bits, G, side, side ? 0.9f : 0.0f, idx, best, second,
                                         codes, packed, scale, zero);
                    uint8_t *back = malloc((size_t)n * d);
                    float *deq = malloc(sizeof(float) * n * d);
                    for (int s = 0; s < N; ++s) {
                        const uint32_t *pk = (const uint32_t *)(packed + (size_t)s * n * d * bits / 8);
                        if (side == 0) {
                            pko_unpack_k(pk, n, d, bits, back);
                            pko_dequant_k(back, scale + s * nparam, zero + s * nparam, idx + s * n, M + (size_t)s * P * d, n, d, G, deq);
                        } else {
                            pko_unpack_v(pk, n, d, bits, back);
                            pko_dequant_v(back, scale + s * nparam, zero + s * nparam, idx + s * n, M + (size_t)s * P * d, n, d, Gc, 1, deq);
                        }
                        for (int i = 0; i < n * d; ++i)
                            if (back[i] != codes[(size_t)s * n * d + i]) return 3;
                    }
                    free(idx); free(best); free(second); free(codes); free(packed); free(scale); free(zero); free(back); free(deq);
                }
    uint16_t *wp = malloc(sizeof(uint16_t) * d);
    pko_window_pattern(x, n, d, wp);
    /* attention: 1 sequence, 3 KV heads, 6 query heads over the raw vectors widened to float */
    float *Kh = malloc(sizeof(float) * N * n * d), *out = malloc(sizeof(float) * 6 * d), *lse = malloc(sizeof(float) * 6);
    for (int i = 0; i < N * n * d; ++i) Kh[i] = pko_half_to_float(x[i]);
    uint16_t *q = malloc(sizeof(uint16_t) * 6 * d);
    for (int i = 0; i < 6 * d; ++i) q[i] = pko_float_to_half_rne(rnd());
    pko_attend_streams(q, Kh, Kh, 1, 6, 3, n, d, 0.0883883, out, lse);
    pko_attend_streams(q, Kh, Kh, 1, 6, 3, 0, d, 0.0883883, out, lse);   /* empty context */
    free(x); free(M); free(assign); free(counts); free(inertia); free(wp); free(Kh); free(out); free(lse); free(q);
    puts("ok");
    return 0;
}
