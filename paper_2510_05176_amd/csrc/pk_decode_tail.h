// fp16 tail of a stream in decode attention (vector ALUs): the body shared by the stand-alone tail kernel and by
// the tail workgroups that ride along in the launch of the packed kernel.
#pragma once
#include "pk_internal.h"

namespace pk {
namespace {

constexpr int kTile = 128;   // tokens per inner tile of the tail kernel
constexpr float kTailLog2e = 1.4426950408889634f;

template <int RP>
struct TailShared {
    float ps[kTile][RP];      // scores, then softmax numerators of the tile
    float mt[RP];
    float red[RP][2];
    float osum[4][RP][kD];    // output partials of the four waves
};

// Sum over the 16 lanes of a row with data-parallel-primitive shifts (row_shr 1, 2, 4, 8; lanes shifted in from
// outside the row read 0): an inclusive scan, so the row's last lane ends with the total.  No LDS traffic.
__device__ __forceinline__ float row_sum_to_last(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x111, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x112, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x114, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x118, 0xf, 0xf, true));
    return v;
}

// fp16 tail of one stream (own cache or shared prefix): plain q.k / softmax / p.v, 256 threads.
// Thread (cg, tg) = (tid % 16, tid / 16) owns channels 8cg .. 8cg+7 of the tokens tg, tg+16, ... of a tile, in
// the score phase and in the value phase alike: the 16 lanes of a token read its 256-byte row in 16-byte
// pieces, scores are summed over those lanes, outputs over the token groups at the end.
// grp: which of the stream's head_groups groups of query heads (r of them each) the workgroup takes.
template <int RP>
__device__ __forceinline__ void decode_tail_body(const DecodeArgs &a, int which, int n, int grp, TailShared<RP> &sh)
{
    const int tid = threadIdx.x;
    const int n_slots = a.splits_prefix + a.splits_own + 2;
    const int r_all = a.n_q_heads / a.n_kv_heads, r = r_all / a.head_groups, head0 = grp * r;
    const int seq = n / a.n_kv_heads, head = n - seq * a.n_kv_heads;
    const CacheView &cv = which == 0 ? a.own : a.prefix;
    const int cstream = which == 0 ? n : head;
    const int slot = n_slots - 2 + which;
    int t_end = cv.t_tail, tail_start = cv.tail_start;
    if (which == 0) {   // a ragged batch: this sequence's own fill state
        int tq;
        own_state(a, seq, tq, t_end, tail_start);
    }
    const int cg = tid & 15, tg = tid >> 4, lane = tid & 63, wave = tid >> 6;

    float qr[RP][8];
#pragma unroll
    for (int h = 0; h < RP; ++h) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (h < r) v = *reinterpret_cast<const uint4 *>(a.q + ((int64_t)seq * a.n_q_heads + head * r_all + head0 + h) * kD + 8 * cg);
        const __half2 *h2 = reinterpret_cast<const __half2 *>(&v);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            qr[h][2 * k] = __low2float(h2[k]);
            qr[h][2 * k + 1] = __high2float(h2[k]);
        }
    }
    float m_run[RP], l_thr[RP], acc[RP][8];
#pragma unroll
    for (int h = 0; h < RP; ++h) {
        m_run[h] = -INFINITY;
        l_thr[h] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
    }
    const __half *tail_k = cv.tail_k + (int64_t)cstream * cv.ring_len * kD + 8 * cg;
    const __half *tail_v = cv.tail_v + (int64_t)cstream * cv.ring_len * kD + 8 * cg;

    for (int t0 = 0; t0 < t_end; t0 += kTile) {
        const int n_valid = min(kTile, t_end - t0);
        __syncthreads();   // the previous tile's numerators have been used
        // ---- scores
#pragma unroll
        for (int i = 0; i < kTile / 16; ++i) {
            const int tk = tg + 16 * i;
            const bool valid = tk < n_valid;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            int rs = tail_start + t0 + tk;   // ring slot: one wrap at most, since t0 + tk < t_tail <= ring_len
            if (rs >= cv.ring_len) rs -= cv.ring_len;
            if (valid) v = *reinterpret_cast<const uint4 *>(tail_k + (int64_t)rs * kD);
            const __half2 *h2 = reinterpret_cast<const __half2 *>(&v);
            float kf[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                kf[2 * k] = __low2float(h2[k]);
                kf[2 * k + 1] = __high2float(h2[k]);
            }
#pragma unroll
            for (int h = 0; h < RP; ++h) {
                float sdot = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) sdot = fmaf(qr[h][e], kf[e], sdot);
                sdot = row_sum_to_last(sdot);   // the token's 16 lanes; lane 15 of the row holds the sum
                if (cg == 15 && valid) sh.ps[tk][h] = sdot * a.softmax_scale;
            }
        }
        __syncthreads();
        if (tid < 64) {   // wave 0: tile maximum per head
#pragma unroll
            for (int h = 0; h < RP; ++h) {
                float m = -INFINITY;
                if (tid < n_valid) m = sh.ps[tid][h];
                if (tid + 64 < n_valid) m = fmaxf(m, sh.ps[tid + 64][h]);
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
                if (tid == 0) sh.mt[h] = m;
            }
        }
        __syncthreads();
        // ---- online softmax update; thread t < 128 turns the scores of token t into numerators
#pragma unroll
        for (int h = 0; h < RP; ++h) {
            const float m_new = fmaxf(m_run[h], sh.mt[h]);
            const float alpha = m_run[h] == -INFINITY ? 0.f : __expf(m_run[h] - m_new);
            m_run[h] = m_new;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[h][e] *= alpha;
            float pr = 0.f;
            if (tid < n_valid) {   // n_valid <= 128
                pr = __expf(sh.ps[tid][h] - m_new);
                sh.ps[tid][h] = pr;
            }
            l_thr[h] = l_thr[h] * alpha + pr;
        }
        __syncthreads();
        // ---- values
#pragma unroll
        for (int i = 0; i < kTile / 16; ++i) {
            const int tk = tg + 16 * i;
            if (tk < n_valid) {
                int rs = tail_start + t0 + tk;
                if (rs >= cv.ring_len) rs -= cv.ring_len;
                const uint4 v = *reinterpret_cast<const uint4 *>(tail_v + (int64_t)rs * kD);
                const __half2 *h2 = reinterpret_cast<const __half2 *>(&v);
                float vf[8];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    vf[2 * k] = __low2float(h2[k]);
                    vf[2 * k + 1] = __high2float(h2[k]);
                }
#pragma unroll
                for (int h = 0; h < RP; ++h) {
                    const float pw = sh.ps[tk][h];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[h][e] = fmaf(pw, vf[e], acc[h][e]);
                }
            }
        }
    }

    // ---- outputs: the four token groups of a wave by shuffles, the four waves through LDS
#pragma unroll
    for (int h = 0; h < RP; ++h) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = acc[h][e];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            if (lane < 16) sh.osum[wave][h][8 * cg + e] = v;
        }
        float l = l_thr[h];   // nonzero in threads 0..127 only
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off);
        if (lane == 0 && wave < 2) sh.red[h][wave] = l;
    }
    __syncthreads();
    if (tid < kD) {
        const int c = tid;
        const int64_t pbase = ((int64_t)n * n_slots + slot) * r_all + head0;
#pragma unroll
        for (int h = 0; h < RP; ++h) {
            if (h < r) {
                a.part_o[(pbase + h) * kD + c] = (sh.osum[0][h][c] + sh.osum[1][h][c]) + (sh.osum[2][h][c] + sh.osum[3][h][c]);
                if (c == 0) {
                    a.part_ml[(pbase + h) * 2] = m_run[h] * kTailLog2e;   // partials carry the maximum in the log2 domain
                    a.part_ml[(pbase + h) * 2 + 1] = sh.red[h][0] + sh.red[h][1];
                }
            }
        }
    }
}

}  // namespace
}  // namespace pk
