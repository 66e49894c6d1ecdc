// Decode attention over the packed cache (Sec. 3.4 "Decode-stage KV reconstruction").
//
// For one KV stream and its r = n_q_heads / n_kv_heads query heads:
//   score[h][t] = scale * ( q_h . M_K[k*_t]  +  sum_c (q_h[c] s[g][c]) code[t][c]  +  q_h . z[g] )
//   out[h]      = sum_p W[h][p] M_V[p]  +  sum_t p[h][t] (s_V[t] code_V[t] + z_V[t])  +  tail terms
// with W[h][p] the softmax mass of the tokens whose V pattern is p.  The context is
// cut into splits (shared prefix | own packed | the two fp16 tails); every split
// keeps a running max / sum (online softmax) and writes an unnormalised partial,
// and a merge kernel combines the partials by log-sum-exp.
#include "pk_internal.h"

namespace pk {

namespace {

constexpr int kTile = 128;   // tokens per inner tile
constexpr int kMaxP = 256;

template <int RP>
struct DecodeShared {
    float q[RP][kD];
    float QM[RP][kMaxP];
    float W[RP][kMaxP];
    float qs[4][kD][RP];        // per K group of the tile: q[h][c] * s[g][c]
    float qz[4][RP];            // per K group: q[h] . z[g]
    float ps[kTile][RP];        // scores, then softmax numerators of the tile
    float half_acc[kTile][RP];  // second channel half's partial dot products; later output halves
    float vs[kTile][4], vz[kTile][4];
    float mt[RP];
    float red[RP][4];
};

// wave 0 reduces the tile's scores to one max per head
template <int RP>
__device__ __forceinline__ void tile_max(DecodeShared<RP> &sh, int n_valid)
{
    const int tid = threadIdx.x;
    if (tid < 64) {
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
}

// One split of one stream.  TAIL = false: packed tokens [t_begin, t_end) of cache view cv.
// TAIL = true: the fp16 tail of cv.  256 threads.
template <int RP, int BITS, bool TAIL>
__device__ void decode_split(const DecodeArgs &a, const CacheView &cv, int cstream, int set, int n,
                             int t_begin, int t_end, int slot, int n_slots, DecodeShared<RP> &sh)
{
    const int tid = threadIdx.x;
    const int r = a.n_q_heads / a.n_kv_heads;
    const int seq = n / a.n_kv_heads, head = n - seq * a.n_kv_heads;
    const int G = a.G, P = a.P;
    const int Gc = G < kD ? G : kD, ng = kD / Gc;
    const __half *MK = a.patterns_k + (int64_t)set * P * kD;
    const __half *MV = a.patterns_v + (int64_t)set * P * kD;

    // ---- preamble: queries, q.M_K, W = 0
    for (int i = tid; i < RP * kD; i += 256) {
        const int h = i / kD, c = i - h * kD;
        sh.q[h][c] = h < r ? h2f(a.q[((int64_t)seq * a.n_q_heads + head * r + h) * kD + c]) : 0.f;
    }
    __syncthreads();
    if (!TAIL) {
        for (int p = tid; p < P; p += 256) {
            float acc[RP];
#pragma unroll
            for (int h = 0; h < RP; ++h) acc[h] = 0.f;
            for (int c8 = 0; c8 < kD; c8 += 8) {
                const uint4 v = *reinterpret_cast<const uint4 *>(MK + (int64_t)p * kD + c8);
                const __half2 *h2 = reinterpret_cast<const __half2 *>(&v);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float m0 = __low2float(h2[k]), m1 = __high2float(h2[k]);
#pragma unroll
                    for (int h = 0; h < RP; ++h)
                        acc[h] = fmaf(sh.q[h][c8 + 2 * k], m0, fmaf(sh.q[h][c8 + 2 * k + 1], m1, acc[h]));
                }
            }
#pragma unroll
            for (int h = 0; h < RP; ++h) {
                sh.QM[h][p] = acc[h];
                sh.W[h][p] = 0.f;
            }
        }
    }

    float m_run[RP], l_thr[RP], o[RP];
#pragma unroll
    for (int h = 0; h < RP; ++h) {
        m_run[h] = -INFINITY;
        l_thr[h] = 0.f;
        o[h] = 0.f;
    }
    const int tt = tid & (kTile - 1), hf = tid >> 7;   // K phase: token slot, channel half; V phase: channel, token half

    for (int t0 = t_begin; t0 < t_end; t0 += kTile) {
        const int n_valid = min(kTile, t_end - t0);
        __syncthreads();   // previous tile's LDS fully consumed (and preamble published)
        if (!TAIL) {
            // fold the K scales into the queries, q.z per group; V parameters of the tile
            const int groups = (n_valid + G - 1) / G;
            for (int i = tid; i < 4 * RP; i += 256) sh.qz[i / RP][i % RP] = 0.f;
            __syncthreads();
            for (int i = tid; i < groups * kD; i += 256) {
                const int gl = i >> 7, c = i & (kD - 1);
                const int64_t prow = ((int64_t)cstream * (cv.t_capacity / G) + (t0 / G + gl)) * kD + c;
                const float s = h2f(cv.k_scale[prow]), z = h2f(cv.k_zero[prow]);
#pragma unroll
                for (int h = 0; h < RP; ++h) {
                    const float qh = sh.q[h][c];
                    sh.qs[gl][c][h] = qh * s;
                    float pz = qh * z;
#pragma unroll
                    for (int off = 32; off > 0; off >>= 1) pz += __shfl_xor(pz, off);
                    if ((tid & 63) == 0) atomicAdd(&sh.qz[gl][h], pz);
                }
            }
            for (int i = tid; i < n_valid * ng; i += 256) {
                const int tk = i / ng, gg = i - tk * ng;
                const int64_t prow = ((int64_t)cstream * cv.t_capacity + t0 + tk) * ng + gg;
                sh.vs[tk][gg] = h2f(cv.v_scale[prow]);
                sh.vz[tk][gg] = h2f(cv.v_zero[prow]);
            }
            __syncthreads();
        }

        // ---- K phase: thread (token slot tt, channel half hf)
        float acc[RP];
#pragma unroll
        for (int h = 0; h < RP; ++h) acc[h] = 0.f;
        const bool valid = tt < n_valid;
        if (valid) {
            if (TAIL) {
                int slotk = cv.tail_start + t0 + tt;
                if (slotk >= cv.ring_len) slotk -= cv.ring_len;
                const __half *krow = cv.tail_k + ((int64_t)cstream * cv.ring_len + slotk) * kD + hf * 64;
#pragma unroll
                for (int c8 = 0; c8 < 64; c8 += 8) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(krow + c8);
                    const __half2 *h2 = reinterpret_cast<const __half2 *>(&v);
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float k0 = __low2float(h2[k]), k1 = __high2float(h2[k]);
                        const int c = hf * 64 + c8 + 2 * k;
#pragma unroll
                        for (int h = 0; h < RP; ++h) acc[h] = fmaf(sh.q[h][c], k0, fmaf(sh.q[h][c + 1], k1, acc[h]));
                    }
                }
            } else {
                const int gl = tt / G;
                const uint32_t *krow = cv.k_codes + (((int64_t)cstream * cv.t_capacity + t0 + tt) * 4 + 2 * hf) * BITS;
                uint32_t wds[2 * BITS];
#pragma unroll
                for (int k = 0; k < 2 * BITS / 4; ++k) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(krow + 4 * k);
                    wds[4 * k] = v.x; wds[4 * k + 1] = v.y; wds[4 * k + 2] = v.z; wds[4 * k + 3] = v.w;
                }
#pragma unroll
                for (int wl = 0; wl < 2; ++wl) {
#pragma unroll 8
                    for (int i = 0; i < 32; ++i) {
                        int code = 0;
#pragma unroll
                        for (int j = 0; j < BITS; ++j) code |= (int)((wds[wl * BITS + j] >> i) & 1u) << j;
                        const float fc = (float)code;
                        const float *qv = sh.qs[gl][(2 * hf + wl) * 32 + i];
#pragma unroll
                        for (int h = 0; h < RP; ++h) acc[h] = fmaf(qv[h], fc, acc[h]);
                    }
                }
            }
        }
        if (hf == 1) {
#pragma unroll
            for (int h = 0; h < RP; ++h) sh.half_acc[tt][h] = acc[h];
        }
        __syncthreads();
        if (hf == 0) {
            if (valid) {
                int kidx = 0, gl = 0;
                if (!TAIL) {
                    kidx = cv.k_idx[(int64_t)cstream * cv.t_capacity + t0 + tt];
                    gl = tt / G;
                }
#pragma unroll
                for (int h = 0; h < RP; ++h) {
                    float sdot = acc[h] + sh.half_acc[tt][h];
                    if (!TAIL) sdot += sh.QM[h][kidx] + sh.qz[gl][h];
                    sh.ps[tt][h] = sdot * a.softmax_scale;
                }
            }
        }
        __syncthreads();
        tile_max<RP>(sh, n_valid);
        __syncthreads();

        // ---- online softmax update
        float alpha[RP];
#pragma unroll
        for (int h = 0; h < RP; ++h) {
            const float m_new = fmaxf(m_run[h], sh.mt[h]);
            alpha[h] = m_run[h] == -INFINITY ? 0.f : __expf(m_run[h] - m_new);
            m_run[h] = m_new;
            o[h] *= alpha[h];
        }
        if (!TAIL) {
            for (int i = tid; i < RP * P; i += 256) {
                const int h = i / P, p = i - h * P;
                sh.W[h][p] *= alpha[h];
            }
        }
        float pr[RP];
        if (hf == 0) {
#pragma unroll
            for (int h = 0; h < RP; ++h) {
                pr[h] = valid ? __expf(sh.ps[tt][h] - m_run[h]) : 0.f;
                l_thr[h] = l_thr[h] * alpha[h] + pr[h];
            }
        }
        __syncthreads();   // W rescaled, scores consumed
        if (hf == 0) {
#pragma unroll
            for (int h = 0; h < RP; ++h) sh.ps[tt][h] = pr[h];
            if (!TAIL && valid) {
                const int vidx = cv.v_idx[(int64_t)cstream * cv.t_capacity + t0 + tt];
#pragma unroll
                for (int h = 0; h < RP; ++h) atomicAdd(&sh.W[h][vidx], pr[h]);
            }
        }
        __syncthreads();

        // ---- V phase: thread (channel c, token half hf)
        const int c = tt;
        const int tk_end = min(n_valid, hf * 64 + 64);
        if (TAIL) {
            for (int tk = hf * 64; tk < tk_end; ++tk) {
                int slotv = cv.tail_start + t0 + tk;
                if (slotv >= cv.ring_len) slotv -= cv.ring_len;
                const float v = h2f(cv.tail_v[((int64_t)cstream * cv.ring_len + slotv) * kD + c]);
#pragma unroll
                for (int h = 0; h < RP; ++h) o[h] = fmaf(sh.ps[tk][h], v, o[h]);
            }
        } else {
            const int gg = c / Gc;
            const uint8_t *vbase = cv.v_codes + (int64_t)cstream * cv.t_capacity * (kD * BITS / 8);
            for (int tk8 = hf * 64; tk8 < tk_end; tk8 += 8) {
                const int64_t unit = ((int64_t)((t0 + tk8) >> 3) * 16 + (c & 15)) * (kD / 16) + (c >> 4);
                uint32_t planes;
                if (BITS == 2)
                    planes = *reinterpret_cast<const uint16_t *>(vbase + unit * 2);
                else
                    planes = *reinterpret_cast<const uint32_t *>(vbase + unit * 4);
                const int lim = min(8, tk_end - tk8);
                for (int k = 0; k < lim; ++k) {
                    int code = 0;
#pragma unroll
                    for (int j = 0; j < BITS; ++j) code |= (int)((planes >> (8 * j + k)) & 1u) << j;
                    const float val = fmaf(sh.vs[tk8 + k][gg], (float)code, sh.vz[tk8 + k][gg]);
#pragma unroll
                    for (int h = 0; h < RP; ++h) o[h] = fmaf(sh.ps[tk8 + k][h], val, o[h]);
                }
            }
        }
    }

    // ---- epilogue: combine the two token halves, add the pattern sums, write the partial
    __syncthreads();
    const int c = tt;
    if (hf == 1) {
#pragma unroll
        for (int h = 0; h < RP; ++h) sh.half_acc[c][h] = o[h];
    }
    // sum of the softmax numerators: 128 threads -> 2 waves -> LDS
    if (hf == 0) {
#pragma unroll
        for (int h = 0; h < RP; ++h) {
            float l = l_thr[h];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off);
            if ((tid & 63) == 0) sh.red[h][tid >> 6] = l;
        }
    }
    __syncthreads();
    if (hf == 0) {
        const int64_t pbase = ((int64_t)n * n_slots + slot) * r;
#pragma unroll
        for (int h = 0; h < RP; ++h) {
            float oo = o[h] + sh.half_acc[c][h];
            if (!TAIL) {
                float wm = 0.f;
                for (int p = 0; p < P; ++p) wm = fmaf(sh.W[h][p], h2f(MV[(int64_t)p * kD + c]), wm);
                oo += wm;
            }
            if (h < r) {
                a.part_o[(pbase + h) * kD + c] = oo;
                if (c == 0) {
                    a.part_ml[(pbase + h) * 2] = m_run[h];
                    a.part_ml[(pbase + h) * 2 + 1] = sh.red[h][0] + sh.red[h][1];
                }
            }
        }
    }
}

template <int RP, int BITS>
__global__ __launch_bounds__(256) void decode_packed_kernel(DecodeArgs a)
{
    __shared__ DecodeShared<RP> sh;
    const int split = blockIdx.x, n = blockIdx.y;
    const int n_slots = a.splits_prefix + a.splits_own + 2;
    if (split < a.splits_prefix) {
        const int head = n % a.n_kv_heads;
        const int tb = split * a.chunk;
        decode_split<RP, BITS, false>(a, a.prefix, head, head, n, tb, min(a.prefix.t_quant, tb + a.chunk), split, n_slots, sh);
    } else {
        const int tb = (split - a.splits_prefix) * a.chunk;
        decode_split<RP, BITS, false>(a, a.own, n, a.sets.set_of(n), n, tb, min(a.own.t_quant, tb + a.chunk), split, n_slots, sh);
    }
}

template <int RP>
__global__ __launch_bounds__(256) void decode_tail_kernel(DecodeArgs a)
{
    __shared__ DecodeShared<RP> sh;
    const int which = blockIdx.x, n = blockIdx.y;
    const int n_slots = a.splits_prefix + a.splits_own + 2;
    if (which == 0) {
        decode_split<RP, 2, true>(a, a.own, n, 0, n, 0, a.own.t_tail, n_slots - 2, n_slots, sh);
    } else {
        const int head = n % a.n_kv_heads;
        decode_split<RP, 2, true>(a, a.prefix, head, 0, n, 0, a.prefix.t_tail, n_slots - 1, n_slots, sh);
    }
}

// log-sum-exp merge of the partials of one (sequence, query head); thread <-> channel
__global__ __launch_bounds__(128) void decode_merge_kernel(DecodeArgs a)
{
    const int u = blockIdx.x, c = threadIdx.x;
    const int seq = u / a.n_q_heads, qh = u - seq * a.n_q_heads;
    const int r = a.n_q_heads / a.n_kv_heads;
    const int n = seq * a.n_kv_heads + qh / r, hr = qh % r;
    const int n_slots = a.splits_prefix + a.splits_own + 2;
    float M = -INFINITY;
    for (int s = 0; s < n_slots; ++s) {
        const int64_t pb = ((int64_t)n * n_slots + s) * r + hr;
        if (a.part_ml[pb * 2 + 1] > 0.f) M = fmaxf(M, a.part_ml[pb * 2]);
    }
    float L = 0.f, acc = 0.f;
    for (int s = 0; s < n_slots; ++s) {
        const int64_t pb = ((int64_t)n * n_slots + s) * r + hr;
        const float l = a.part_ml[pb * 2 + 1];
        if (l > 0.f) {
            const float w = __expf(a.part_ml[pb * 2] - M);
            L = fmaf(l, w, L);
            acc = fmaf(a.part_o[pb * kD + c], w, acc);
        }
    }
    a.out[(int64_t)u * kD + c] = L > 0.f ? acc / L : 0.f;
    if (a.lse && c == 0) a.lse[u] = L > 0.f ? M + __logf(L) : -INFINITY;
}

}  // namespace

int decode_chunk(int64_t n_streams, int64_t t_packed_total)
{
    // aim at ~2048 workgroups; at least one 128-token tile pair, at most 8192 tokens per split
    int64_t c = (n_streams * t_packed_total + 2047) / 2048;
    c = (c + 255) / 256 * 256;
    if (c < 256) c = 256;
    if (c > 8192) c = 8192;
    return (int)c;
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t s)
{
    const int r = a.n_q_heads / a.n_kv_heads;
    const int N = a.n_seq * a.n_kv_heads;
    const int splits = a.splits_prefix + a.splits_own;
    hipError_t e;
    if (splits > 0) {
        const dim3 grid(splits, N), block(256);
#define PK_LAUNCH_D(RP, BB)                                                          \
    if ((r <= 4) == (RP == 4) && a.bits == BB)                                       \
        hipLaunchKernelGGL((decode_packed_kernel<RP, BB>), grid, block, 0, s, a);
        PK_LAUNCH_D(4, 2) PK_LAUNCH_D(8, 2) PK_LAUNCH_D(4, 4) PK_LAUNCH_D(8, 4)
#undef PK_LAUNCH_D
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (r <= 4)
        hipLaunchKernelGGL((decode_tail_kernel<4>), dim3(2, N), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL((decode_tail_kernel<8>), dim3(2, N), dim3(256), 0, s, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(decode_merge_kernel, dim3(a.n_seq * a.n_q_heads), dim3(128), 0, s, a);
    return hipGetLastError();
}

}  // namespace pk
