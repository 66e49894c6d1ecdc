// Decode attention: the fp16 tails (vector ALUs), the log-sum-exp merge of all partial results,
// and the launch sequence.  The packed part runs on the matrix cores (pk_decode_packed.hip).
//
// Every split of a stream's context writes an unnormalised partial per query head:
//   o[c] = sum_t 2^(S2_t - m) * (value part of token t),  m = max_t S2_t,  l = sum_t 2^(S2_t - m)
// with S2 = log2(e) * softmax_scale * q.k.  Packed splits leave the pattern part of V out of o and
// write the softmax mass per pattern W[p] instead, so that W . M_V is formed once per head here.
#include "pk_internal.h"

namespace pk {

hipError_t launch_decode_packed(const DecodeArgs &a, hipStream_t s);

namespace {

constexpr int kTile = 128;   // tokens per inner tile of the tail kernel
constexpr int kMaxP = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

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
template <int RP>
__global__ __launch_bounds__(256) void decode_tail_kernel(DecodeArgs a)
{
    __shared__ TailShared<RP> sh;
    const int which = blockIdx.x, n = blockIdx.y, tid = threadIdx.x;
    const int n_slots = a.splits_prefix + a.splits_own + 2;
    const int r = a.n_q_heads / a.n_kv_heads;
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
        if (h < r) v = *reinterpret_cast<const uint4 *>(a.q + ((int64_t)seq * a.n_q_heads + head * r + h) * kD + 8 * cg);
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
        const int64_t pbase = ((int64_t)n * n_slots + slot) * r;
#pragma unroll
        for (int h = 0; h < RP; ++h) {
            if (h < r) {
                a.part_o[(pbase + h) * kD + c] = (sh.osum[0][h][c] + sh.osum[1][h][c]) + (sh.osum[2][h][c] + sh.osum[3][h][c]);
                if (c == 0) {
                    a.part_ml[(pbase + h) * 2] = m_run[h] * kLog2e;   // partials carry the maximum in the log2 domain
                    a.part_ml[(pbase + h) * 2 + 1] = sh.red[h][0] + sh.red[h][1];
                }
            }
        }
    }
}

// log-sum-exp merge of the partials of one (sequence, query head); 128*NQ threads, thread <-> (channel c,
// part q).  The weights exp2(m_s - M) of the slots are formed once, in parallel, and kept in LDS; every loop
// over the slots or the patterns is then a run of independent loads, of which each of the NQ parts takes every
// NQ-th term (NQ = 4 when there are many slots or patterns, so that no thread walks a long chain alone); the
// parts are added in a fixed order.
template <int NQ>
__global__ __launch_bounds__(128 * NQ) void decode_merge_kernel(DecodeArgs a)
{
    __shared__ float Wq[NQ][2][kMaxP];   // softmax mass per pattern (shared prefix, own cache), per part
    __shared__ float accq[NQ][kD];
    __shared__ float wslot[kMaxSlots];
    __shared__ float red[2 * NQ];
    const int u = blockIdx.x, tid = threadIdx.x, c = tid & (kD - 1), q = tid >> 7;
    const int seq = u / a.n_q_heads, qh = u - seq * a.n_q_heads;
    const int r = a.n_q_heads / a.n_kv_heads, P = a.P;
    const int head = qh / r, hr = qh - head * r;
    const int n = seq * a.n_kv_heads + head;
    const int n_packed = a.splits_prefix + a.splits_own;
    const int64_t base = (int64_t)n * (n_packed + 2);
    // the two tail slots are written (and read here) only when there is a tail at all
    // (own tail at n_packed, prefix tail behind it; without a prefix tail only the own one is launched)
    const int n_slots = a.prefix.t_tail > 0 ? n_packed + 2 : a.own.t_tail > 0 ? n_packed + 1 : n_packed;
    // maximum over the slots that hold anything
    float M = -INFINITY;
    for (int s = tid; s < n_slots; s += 128 * NQ) {
        const int64_t pb = (base + s) * r + hr;
        if (a.part_ml[pb * 2 + 1] > 0.f) M = fmaxf(M, a.part_ml[pb * 2]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    if ((tid & 63) == 0) red[tid >> 6] = M;
    __syncthreads();
    M = red[0];
#pragma unroll
    for (int w = 1; w < 2 * NQ; ++w) M = fmaxf(M, red[w]);
    float L = 0.f;
    for (int s = tid; s < n_slots; s += 128 * NQ) {
        const int64_t pb = (base + s) * r + hr;
        const float l = a.part_ml[pb * 2 + 1];
        const float w = l > 0.f ? exp2f(a.part_ml[pb * 2] - M) : 0.f;
        wslot[s] = w;
        L = fmaf(l, w, L);
    }
    __syncthreads();   // also orders the reads of red above against the writes below
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) L += __shfl_xor(L, off);
    if ((tid & 63) == 0) red[tid >> 6] = L;
    float acc = 0.f;
#pragma unroll 4
    for (int s = q; s < n_slots; s += NQ) acc = fmaf(a.part_o[((base + s) * r + hr) * kD + c], wslot[s], acc);
    for (int p = c; p < P; p += 128) {
        float wp = 0.f, wo = 0.f;
#pragma unroll 4
        for (int s = q; s < a.splits_prefix; s += NQ) wp = fmaf(a.part_w[((base + s) * r + hr) * P + p], wslot[s], wp);
#pragma unroll 4
        for (int s = a.splits_prefix + q; s < n_packed; s += NQ) wo = fmaf(a.part_w[((base + s) * r + hr) * P + p], wslot[s], wo);
        Wq[q][0][p] = wp;
        Wq[q][1][p] = wo;
    }
    __syncthreads();
    L = red[0];
#pragma unroll
    for (int w = 1; w < 2 * NQ; ++w) L += red[w];
    if (NQ > 1) {
        for (int i = tid; i < 2 * P; i += 128 * NQ) {
            const int k = i >= P ? 1 : 0, p = i - k * P;
            float w = Wq[0][k][p];
#pragma unroll
            for (int j = 1; j < NQ; ++j) w += Wq[j][k][p];
            Wq[0][k][p] = w;
        }
        __syncthreads();
    }
    if (a.splits_prefix > 0) {
        const __half *MV = a.patterns_v + (int64_t)head * P * kD;
#pragma unroll 8
        for (int p = q; p < P; p += NQ) acc = fmaf(Wq[0][0][p], h2f(MV[(int64_t)p * kD + c]), acc);
    }
    if (a.splits_own > 0) {
        const __half *MV = a.patterns_v + (int64_t)a.sets.set_of(n) * P * kD;
#pragma unroll 8
        for (int p = q; p < P; p += NQ) acc = fmaf(Wq[0][1][p], h2f(MV[(int64_t)p * kD + c]), acc);
    }
    if (NQ > 1) {
        accq[q][c] = acc;
        __syncthreads();
        if (q > 0) return;
        acc = accq[0][c];
#pragma unroll
        for (int j = 1; j < NQ; ++j) acc += accq[j][c];
    }
    a.out[(int64_t)u * kD + c] = L > 0.f ? acc / L : 0.f;
    if (a.lse && c == 0) a.lse[u] = L > 0.f ? (M + log2f(L)) * kLn2 : -INFINITY;
}

}  // namespace

int decode_chunk(int64_t n_streams, int64_t t_packed_total, int P, int r)
{
    // Equal splits, their number k chosen for the shortest modelled time: the chip holds 512 workgroups at once
    // (two per CU), workgroups that run side by side take the same time, so k splits per stream cost
    // ceil(n_streams * k / 512) rounds of (split length + fixed part).  The fixed part - prologue (q.M_K table,
    // LDS clears), epilogue (merge of the four waves), the r*P pattern masses and r*128 outputs every split
    // writes - is worth about 1024 + r*P/2 tokens of block work.  A split holds at least r*P/2 tokens and one
    // 64-token block per wave, at most 32768 tokens.  (Unequal splits - a long one and a remainder - leave the
    // long ones of the last streams waiting for a slot: 0.78 against 0.54 ms on 432 streams x 32768.)
    const int64_t t = t_packed_total > 0 ? t_packed_total : 1;
    int64_t floor_c = (int64_t)r * P / 2;
    if (floor_c < 256) floor_c = 256;
    const int64_t fixed = 1024 + (int64_t)r * P / 2;
    int64_t best_c = 0, best_cost = 0;
    for (int64_t k = (t + 32767) / 32768; k <= 512; ++k) {
        int64_t c = ((t + k - 1) / k + 255) / 256 * 256;
        if (c < floor_c) c = (floor_c + 255) / 256 * 256;
        if (c > 32768) c = 32768;
        const int64_t splits = (t + c - 1) / c;
        const int64_t rounds = (n_streams * splits + 511) / 512;
        const int64_t cost = rounds * (c + fixed);
        if (best_c == 0 || cost < best_cost) {
            best_c = c;
            best_cost = cost;
        }
        if (c <= floor_c || c <= 256) break;   // shorter splits are not allowed
    }
    return (int)best_c;
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t s)
{
    const int r = a.n_q_heads / a.n_kv_heads;
    const int N = a.n_seq * a.n_kv_heads;
    hipError_t e;
    if ((e = launch_decode_packed(a, s)) != hipSuccess) return e;
    if (a.own.t_tail > 0 || a.prefix.t_tail > 0) {
        // x = 0: own tails, x = 1: the shared prefix's tail (launched only if there is one: workgroups that find
        // nothing to do still cost their dispatch, tens of nanoseconds each)
        const dim3 grid(a.prefix.t_tail > 0 ? 2 : 1, N);
        if (r <= 4)
            hipLaunchKernelGGL((decode_tail_kernel<4>), grid, dim3(256), 0, s, a);
        else
            hipLaunchKernelGGL((decode_tail_kernel<8>), grid, dim3(256), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    // four parts per channel when a thread would otherwise walk many slots or patterns alone and the
    // (sequence, head) pairs are too few to fill the chip with 128-thread workgroups
    if (a.splits_prefix + a.splits_own + a.P >= 96 && a.n_seq * a.n_q_heads <= 2048)
        hipLaunchKernelGGL(decode_merge_kernel<4>, dim3(a.n_seq * a.n_q_heads), dim3(512), 0, s, a);
    else
        hipLaunchKernelGGL(decode_merge_kernel<1>, dim3(a.n_seq * a.n_q_heads), dim3(128), 0, s, a);
    return hipGetLastError();
}

}  // namespace pk
