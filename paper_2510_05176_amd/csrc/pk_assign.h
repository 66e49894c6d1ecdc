// Nearest-pattern search for a tile of vectors held in LDS (vector-ALU form).
//
// Sec. 3.2 Eq. 6 (argmin over patterns) with either the Euclidean metric of the
// mining objective (Sec. 3.1 Eq. 4) or the min-max distance d_mm of Sec. 3.2.
// Distances are formed directly, sum_c (x_c - m_c)^2 in binary32, so there is no
// cancellation between large norms; ties go to the lowest pattern index.
#pragma once

#include "pk_internal.h"

namespace pk {

constexpr int kXsStride = kD + 8;      // LDS row stride (halves) of a staged fp16 tile
constexpr int kPatTile = 16;           // patterns converted to fp32 and staged per round

struct AssignScratch {
    float pat[kPatTile][kD];           // current pattern tile, fp32
    float cand_d[128];
    int cand_i[128];
};

// Cooperative load of n_rows fp16 rows into LDS (128 threads), 16 bytes per access.
template <class RowFn>
__device__ __forceinline__ void stage_rows(__half *xs, int n_rows, RowFn rowptr)
{
    for (int i = threadIdx.x; i < n_rows * kRowChunks; i += 128) {
        const int r = i >> 4, ch = i & 15;
        const uint4 v = *reinterpret_cast<const uint4 *>(rowptr(r) + ch * 8);
        *reinterpret_cast<uint4 *>(xs + r * kXsStride + ch * 8) = v;
    }
}

// SLOTS = token slots of the tile (32, 64 or 128); 128 threads.  Starts with a barrier, so the
// caller may stage xs right before the call.  Thread t works on
// token slot t % SLOTS and on the patterns p with p % (128/SLOTS) == t / SLOTS.
// On return (after the trailing barrier) idx_s[slot] (and best_s[slot] if not null)
// are valid for slot < n_tok.
template <int SLOTS>
__device__ void assign_tile(const __half *xs, int n_tok, const __half *Mg, int P, int metric,
                            AssignScratch &sc, int *idx_s, float *best_s)
{
    constexpr int PARTS = 128 / SLOTS;
    const int tid = threadIdx.x;
    const int slot = tid % SLOTS, part = tid / SLOTS;
    const bool active = slot < n_tok;

    __syncthreads();   // the staged tile is complete
    float xr[kD];
    if (active) {
#pragma unroll
        for (int c = 0; c < kD; c += 2) {
            const __half2 h = *reinterpret_cast<const __half2 *>(xs + slot * kXsStride + c);
            xr[c] = __low2float(h);
            xr[c + 1] = __high2float(h);
        }
    } else {
#pragma unroll
        for (int c = 0; c < kD; ++c) xr[c] = 0.f;
    }

    float bd = INFINITY;
    int bi = 0x7fffffff;
    for (int p0 = 0; p0 < P; p0 += kPatTile) {
        __syncthreads();   // previous tile fully consumed
        const int np = min(kPatTile, P - p0);
        for (int i = tid; i < np * kRowChunks; i += 128) {
            const int r = i >> 4, ch = i & 15;
            const uint4 v = *reinterpret_cast<const uint4 *>(Mg + (int64_t)(p0 + r) * kD + ch * 8);
            const __half2 *h = reinterpret_cast<const __half2 *>(&v);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                sc.pat[r][ch * 8 + 2 * k] = __low2float(h[k]);
                sc.pat[r][ch * 8 + 2 * k + 1] = __high2float(h[k]);
            }
        }
        __syncthreads();
        if (active) {
            for (int r = part; r < np; r += PARTS) {
                const float4 *pm = reinterpret_cast<const float4 *>(sc.pat[r]);
                float dist;
                if (metric == PK_METRIC_L2) {
                    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
                    for (int c4 = 0; c4 < kD / 4; ++c4) {
                        const float4 m = pm[c4];
                        const float d0 = xr[4 * c4] - m.x, d1 = xr[4 * c4 + 1] - m.y;
                        const float d2 = xr[4 * c4 + 2] - m.z, d3 = xr[4 * c4 + 3] - m.w;
                        a0 = fmaf(d0, d0, a0);
                        a1 = fmaf(d1, d1, a1);
                        a2 = fmaf(d2, d2, a2);
                        a3 = fmaf(d3, d3, a3);
                    }
                    dist = (a0 + a1) + (a2 + a3);
                } else {
                    float mx = -INFINITY, mn = INFINITY;
#pragma unroll
                    for (int c4 = 0; c4 < kD / 4; ++c4) {
                        const float4 m = pm[c4];
                        const float d0 = xr[4 * c4] - m.x, d1 = xr[4 * c4 + 1] - m.y;
                        const float d2 = xr[4 * c4 + 2] - m.z, d3 = xr[4 * c4 + 3] - m.w;
                        mx = fmaxf(fmaxf(mx, d0), fmaxf(d1, fmaxf(d2, d3)));
                        mn = fminf(fminf(mn, d0), fminf(d1, fminf(d2, d3)));
                    }
                    dist = mx - mn;
                }
                if (dist < bd) {   // patterns are visited in increasing order: strict < keeps the lowest
                    bd = dist;
                    bi = p0 + r;
                }
            }
        }
    }
    // combine the PARTS candidates of each slot: smallest distance, then lowest index
    sc.cand_d[tid] = bd;
    sc.cand_i[tid] = bi;
    __syncthreads();
    if (part == 0 && active) {
#pragma unroll
        for (int k = 1; k < PARTS; ++k) {
            const float d2 = sc.cand_d[slot + k * SLOTS];
            const int i2 = sc.cand_i[slot + k * SLOTS];
            if (d2 < bd || (d2 == bd && i2 < bi)) {
                bd = d2;
                bi = i2;
            }
        }
        idx_s[slot] = bi;
        if (best_s) best_s[slot] = bd;
    }
    __syncthreads();
}

}  // namespace pk
