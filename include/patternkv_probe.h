/*
 * patternkv_probe.h -- machine-peak probes exported by libpatternkv.so next to the hot path.
 *
 * Not part of the method: four tiny kernels that measure what this GPU sustains, so that the rates of
 * the hot-path kernels can be quoted against measured peaks as well as against the published ones
 * (HBM 8 TB/s, dense fp16 MFMA 2.5 PFLOP/s, fp32 vector 157.3 TFLOP/s with packed operations).
 * All pointers are DEVICE pointers, 16-byte aligned; calls enqueue on `stream` and return without
 * synchronising; nothing is allocated.  The caller times them (events on the same stream).
 * Return value: 0 = enqueued, 1 = bad argument, 8 = launch refused (the pk_status values).
 */
#ifndef PATTERNKV_PROBE_H
#define PATTERNKV_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Streaming read of `bytes` (multiple of 16) with 16-byte loads; a 16-byte checksum per workgroup goes to
 * sink (at least 16 * 2048 bytes).  HBM bytes moved: bytes. */
int pk_probe_read(const void *src, size_t bytes, void *sink, void *stream);

/* Streaming copy of `bytes` (multiple of 16), 16-byte loads and stores.  HBM bytes moved: 2 * bytes. */
int pk_probe_copy(void *dst, const void *src, size_t bytes, void *stream);

/* 2048 workgroups x 256 threads, every thread runs `iters` rounds of 16 independent binary32 fused
 * multiply-adds (v_fma_f32; this library is built without packed-fp32 instructions).  Flops:
 * 2 * 16 * iters * 2048 * 256.  sink: at least 2048 * 256 floats. */
int pk_probe_fma_f32(float *sink, int32_t iters, void *stream);

/* 2048 workgroups x 256 threads, every wave runs `iters` rounds of 8 independent
 * v_mfma_f32_16x16x32_f16.  Flops: 2 * 16 * 16 * 32 * 8 * iters * 2048 * 4.  sink: at least 2048 * 256 floats. */
int pk_probe_mfma_f16(float *sink, int32_t iters, void *stream);

/* The quantizer's two division sequences (Sec. 2.1 Eq. 1: s = (max - z)/(2^b - 1), and 1/s), which replace the
 * IEEE divisions by a reciprocal estimate with one correction step, evaluated on n plain values so that a test
 * can compare them with IEEE division: recip[i] = 1/x[i] (meant for positive fp16-representable x),
 * by3[i] = x[i]/3, by15[i] = x[i]/15 (finite x >= 0).  All arrays hold n floats. */
int pk_probe_divisions(const float *x, size_t n, float *recip, float *by3, float *by15, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PATTERNKV_PROBE_H */
