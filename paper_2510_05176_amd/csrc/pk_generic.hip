// The hot path for head dimensions other than 128 (96 and 256, the other two that Sec. 3.3 names): plain kernels,
// thread <-> channel or thread <-> token, no matrix cores, no LDS tiling.  They compute the same definitions with
// the same arithmetic where it decides an integer (the quantizer's parameters and codes come from the shared
// pk_quant_arith.h; pattern selection evaluates the metric in binary32 over all patterns, lowest index on ties) and
// store the same cache format (head_dim enters the layout formulas), so they meet the same parity bars; they are
// not tuned, and the tuned kernels of the other files keep their fixed head dimension.
// Uniform appends, decode (with shared prefix and with per-sequence fill states), mining, the window pattern and
// dequantize are covered, on contiguous and on paged caches.
#pragma clang fp contract(off)

#include "pk_quant_arith.h"

namespace pk {

namespace {

constexpr int kGenThreads = 256;   // >= the largest head dimension

__device__ __forceinline__ float wave_min(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fminf(v, __shfl_xor(v, off));
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

// Distance of the fp16 vector x (d elements, LDS or global) to pattern row m under the metric: the sum of squared
// binary32 differences in channel order, or d_mm = max - min of the differences (Sec. 3.2).
__device__ __forceinline__ float metric_distance(const __half *x, const __half *m, int d, int metric)
{
    if (metric == PK_METRIC_MINMAX) {
        float mx = -INFINITY, mn = INFINITY;
        for (int c = 0; c < d; ++c) {
            const float r = h2f(x[c]) - h2f(m[c]);
            mx = fmaxf(mx, r);
            mn = fminf(mn, r);
        }
        return mx - mn;
    }
    float acc = 0.f;
    for (int c = 0; c < d; ++c) {
        const float r = h2f(x[c]) - h2f(m[c]);
        acc = fmaf(r, r, acc);
    }
    return acc;
}

// argmin over the patterns for the vector in xs (LDS): lane <-> pattern, then a wave reduction (lowest index on ties)
__device__ __forceinline__ void wave_nearest(const __half *xs, const __half *M, int P, int d, int metric, int lane, int &best_i,
                                             float &best_d)
{
    float bd = INFINITY;
    int bi = 0x7fffffff;
    for (int p = lane; p < P; p += 64) {
        const float dist = metric_distance(xs, M + (int64_t)p * d, d, metric);
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

// ---------------------------------------------------------------------------------------------- quantize-append
// Pattern index of every vector to quantize: one wave per vector, four vectors per workgroup.
__global__ __launch_bounds__(256) void gen_assign_kernel(QuantArgs a)
{
    __shared__ __half xs[4][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, ns = blockIdx.y;
    const int i = blockIdx.x * 4 + wave;
    if (i >= a.nq) return;
    const __half *row = a.src.row_d(ns, i, a.d);
    for (int c = lane; c < a.d; c += 64) xs[wave][c] = row[c];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    int bi;
    float bd;
    wave_nearest(xs[wave], a.patterns + (int64_t)a.sets.set_of(ns) * a.P * a.d, a.P, a.d, a.metric, lane, bi, bd);
    if (lane == 0) a.idx[a.map.pos(ns, a.t0 + i)] = (uint8_t)bi;
}

// K: one workgroup per (group of G tokens, stream), thread <-> channel.  Two passes over the group's residuals (the
// second recomputes them): minimum / maximum -> parameters, then codes; a plane word of 32 channels is a wave ballot.
__global__ __launch_bounds__(kGenThreads) void gen_quantize_k_kernel(QuantArgs a)
{
    const int c = threadIdx.x, lane = c & 63, ns = blockIdx.y, g = blockIdx.x, d = a.d, G = a.G;
    const bool on = c < d;
    const __half *M = a.patterns + (int64_t)a.sets.set_of(ns) * a.P * d;
    const int64_t p0 = a.map.pos(ns, a.t0 + g * G);   // a group never straddles a page
    float mn = INFINITY, mx = -INFINITY;
    for (int t = 0; t < G; ++t) {
        const int idx = a.idx[p0 + t];
        if (on) {
            const float r = h2f(a.src.row_d(ns, g * G + t, d)[c]) - h2f(M[(int64_t)idx * d + c]);
            mn = fminf(mn, r);
            mx = fmaxf(mx, r);
        }
    }
    GroupParams gp = group_params(on ? mn : 0.f, on ? mx : 0.f, a.bits);
    if (on) {
        a.scale[(p0 / G) * d + c] = __ushort_as_half(gp.s16);
        a.zero[(p0 / G) * d + c] = __ushort_as_half(gp.z16);
    }
    const int words = d / 32;
    for (int t = 0; t < G; ++t) {
        const int idx = a.idx[p0 + t];
        int code = 0;
        if (on) code = quantize_one(h2f(a.src.row_d(ns, g * G + t, d)[c]) - h2f(M[(int64_t)idx * d + c]), gp, a.bits);
        for (int j = 0; j < a.bits; ++j) {
            const unsigned long long m = __ballot((code >> j) & 1);   // bit l <-> channel 64 * wave + l
            const int w = (c >> 6) * 2 + (lane >> 5);
            if ((lane & 31) == 0 && w < words) a.codes_k[((p0 + t) * words + w) * a.bits + j] = (uint32_t)(m >> (lane & 32));
        }
    }
}

// V: one workgroup per (16-token unit, stream), thread <-> channel.  Per token: residual, the adaptive threshold of
// Sec. 3.3 if it is on, minimum / maximum per group of Gc channels (one thread per group walks its channels in LDS),
// parameters, code; every thread collects the bits of its channel's 16 tokens in the words it then stores.
__global__ __launch_bounds__(kGenThreads) void gen_quantize_v_kernel(QuantArgs a)
{
    __shared__ float rs[kGenThreads], xr[kGenThreads];
    __shared__ float pz[8], pinv[8], ps[8];
    __shared__ int keep_s;
    const int c = threadIdx.x, ns = blockIdx.y, u = blockIdx.x, d = a.d;
    const bool on = c < d;
    const int Gc = a.G < d ? a.G : d, NG = d / Gc;
    const __half *M = a.patterns + (int64_t)a.sets.set_of(ns) * a.P * d;
    const int64_t p0 = a.map.pos(ns, a.t0 + u * 16);
    uint32_t word[2] = {0u, 0u};
    for (int i = 0; i < 16; ++i) {
        int idx = a.idx[p0 + i];
        float x = 0.f, r = 0.f;
        if (on) {
            x = h2f(a.src.row_d(ns, u * 16 + i, d)[c]);
            r = x - h2f(M[(int64_t)idx * d + c]);
        }
        __syncthreads();   // the previous token's parameters have been read
        rs[c] = r;
        xr[c] = x;
        __syncthreads();
        if (a.v_rho > 0.f) {
            if (c == 0) {
                float rmn = INFINITY, rmx = -INFINITY, xmn = INFINITY, xmx = -INFINITY;
                for (int k = 0; k < d; ++k) {
                    rmn = fminf(rmn, rs[k]);
                    rmx = fmaxf(rmx, rs[k]);
                    xmn = fminf(xmn, xr[k]);
                    xmx = fmaxf(xmx, xr[k]);
                }
                keep_s = (rmx - rmn) <= a.v_rho * (xmx - xmn) ? 1 : 0;
            }
            __syncthreads();
            if (!keep_s) {   // the vector itself is quantized, stored under the index that says so
                idx = PK_NO_PATTERN;
                r = x;
                __syncthreads();
                rs[c] = r;
                __syncthreads();
            }
        }
        if (c < NG) {
            float mn = INFINITY, mx = -INFINITY;
            for (int k = c * Gc; k < (c + 1) * Gc; ++k) {
                mn = fminf(mn, rs[k]);
                mx = fmaxf(mx, rs[k]);
            }
            const GroupParams gp = group_params(mn, mx, a.bits);
            pz[c] = gp.z;
            ps[c] = gp.s;
            pinv[c] = gp.inv;
            a.scale[((p0 >> 4) * NG + c) * 16 + i] = __ushort_as_half(gp.s16);
            a.zero[((p0 >> 4) * NG + c) * 16 + i] = __ushort_as_half(gp.z16);
        }
        if (c == 0) a.idx[p0 + i] = (uint8_t)idx;
        __syncthreads();
        if (on) {
            GroupParams gp;
            gp.z = pz[c / Gc];
            gp.s = ps[c / Gc];
            gp.inv = pinv[c / Gc];
            const int code = quantize_one(r, gp, a.bits);
            for (int j = 0; j < a.bits; ++j) word[j >> 1] |= (uint32_t)((code >> j) & 1) << (16 * (j & 1) + i);
        }
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

// assignment step: one wave per vector
__global__ __launch_bounds__(256) void gen_mine_assign_kernel(MineArgs a, int last)
{
    __shared__ __half xs[4][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, s = blockIdx.y;
    const int t = blockIdx.x * 4 + wave;
    if (t >= a.T) return;
    const __half *row = a.x + (int64_t)s * a.set_stride + (int64_t)t * a.d;
    for (int c = lane; c < a.d; c += 64) xs[wave][c] = row[c];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    int bi;
    float bd;
    wave_nearest(xs[wave], a.patterns + (int64_t)s * a.P * a.d, a.P, a.d, PK_METRIC_L2, lane, bi, bd);
    if (lane == 0) {
        a.assign_ws[(int64_t)s * a.T + t] = bi;
        if (last && a.assign) a.assign[(int64_t)s * a.T + t] = bi;
        a.best[(int64_t)s * a.T + t] = bd;
    }
}

// cluster sums of one chunk of one set, vectors in order: thread <-> channel adds into the chunk's own [P][d] block
// of the workspace (only this thread ever touches its column), thread 0 counts
__global__ __launch_bounds__(kGenThreads) void gen_mine_sums_kernel(MineArgs a, int chunk)
{
    const int c = threadIdx.x, ck = blockIdx.x, s = blockIdx.y, d = a.d;
    const int t0 = ck * chunk, t1 = min(a.T, t0 + chunk);
    float *ps = a.psum + ((int64_t)s * a.tsplit + ck) * a.P * d;
    int32_t *pc = a.pcnt + ((int64_t)s * a.tsplit + ck) * a.P;
    if (c < d)
        for (int p = 0; p < a.P; ++p) ps[(int64_t)p * d + c] = 0.f;
    for (int p = c; p < a.P; p += kGenThreads) pc[p] = 0;
    __syncthreads();
    const int32_t *asg = a.assign_ws + (int64_t)s * a.T;
    const __half *x = a.x + (int64_t)s * a.set_stride;
    if (c < d)
        for (int t = t0; t < t1; ++t) ps[(int64_t)asg[t] * d + c] += h2f(x[(int64_t)t * d + c]);
    if (c == 0)
        for (int t = t0; t < t1; ++t) pc[asg[t]] += 1;
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
// One workgroup per (sequence, query head): the context [prefix packed | prefix tail | own packed | own tail] in
// chunks of 256 tokens.  Scores: thread <-> token (the reconstructed key against q, channel by channel); online
// softmax over the chunks; values: thread <-> channel over the chunk's tokens.  Everything in binary32.
__global__ __launch_bounds__(kGenThreads) void gen_decode_kernel(DecodeArgs a)
{
    __shared__ float qs[kGenThreads], pr[kGenThreads], red[kGenThreads];
    const int tid = threadIdx.x, d = a.d;
    const int seq = blockIdx.x / a.n_q_heads, qh = blockIdx.x - seq * a.n_q_heads;
    const int r = a.n_q_heads / a.n_kv_heads, head = qh / r;
    const int n_own = seq * a.n_kv_heads + head;
    const int Gc = a.G < d ? a.G : d;
    if (tid < d) qs[tid] = h2f(a.q[((int64_t)seq * a.n_q_heads + qh) * d + tid]);
    __syncthreads();
    float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
    for (int part = 0; part < 4; ++part) {
        const bool pre = part < 2, packed = (part & 1) == 0;
        const CacheView &cv = pre ? a.prefix : a.own;
        const int stream = pre ? head : n_own;
        const int set = pre ? head : a.sets.set_of(n_own);
        int tq = cv.t_quant, tt = cv.t_tail, ts = cv.tail_start;
        if (!pre) own_state(a, seq, tq, tt, ts);
        const int n_tok = packed ? tq : tt;
        const __half *MK = a.patterns_k + (int64_t)set * a.P * d, *MV = a.patterns_v + (int64_t)set * a.P * d;
        for (int t0 = 0; t0 < n_tok; t0 += kGenThreads) {
            const int t = t0 + tid;
            float sc = -INFINITY;
            int64_t where = 0;   // packed position, or row of the tail ring
            if (t < n_tok) {
                float dot = 0.f;
                if (packed) {
                    where = cv.map.pos(stream, t);
                    for (int c = 0; c < d; ++c) dot = fmaf(qs[c], k_hat(cv, MK, where, c, d, a.bits, a.G), dot);
                } else {
                    int slot = ts + t;
                    if (slot >= cv.ring_len) slot -= cv.ring_len;
                    where = (int64_t)stream * cv.ring_len + slot;
                    for (int c = 0; c < d; ++c) dot = fmaf(qs[c], h2f(cv.tail_k[where * d + c]), dot);
                }
                sc = dot * a.softmax_scale;
            }
            // chunk maximum
            red[tid] = sc;
            __syncthreads();
            for (int w = kGenThreads / 2; w > 0; w >>= 1) {
                if (tid < w) red[tid] = fmaxf(red[tid], red[tid + w]);
                __syncthreads();
            }
            const float m_new = fmaxf(m_run, red[0]);
            __syncthreads();
            const float p = t < n_tok ? __expf(sc - m_new) : 0.f;
            pr[tid] = p;
            red[tid] = p;
            // the positions of the chunk's tokens, for the value phase
            __syncthreads();
            for (int w = kGenThreads / 2; w > 0; w >>= 1) {
                if (tid < w) red[tid] += red[tid + w];
                __syncthreads();
            }
            const float alpha = m_run == -INFINITY ? 0.f : __expf(m_run - m_new);
            l_run = l_run * alpha + red[0];
            acc *= alpha;
            m_run = m_new;
            if (tid < d) {
                const int n_here = min(kGenThreads, n_tok - t0);
                for (int k = 0; k < n_here; ++k) {
                    const int tk = t0 + k;
                    float v;
                    if (packed) {
                        v = v_hat(cv, MV, cv.map.pos(stream, tk), tid, d, a.bits, Gc, a.v_thresholded);
                    } else {
                        int slot = ts + tk;
                        if (slot >= cv.ring_len) slot -= cv.ring_len;
                        v = h2f(cv.tail_v[((int64_t)stream * cv.ring_len + slot) * d + tid]);
                    }
                    acc = fmaf(pr[k], v, acc);
                }
            }
            __syncthreads();
        }
    }
    const int64_t u = (int64_t)seq * a.n_q_heads + qh;
    if (tid < d) a.out[u * d + tid] = l_run > 0.f ? acc / l_run : 0.f;
    if (a.lse && tid == 0) a.lse[u] = l_run > 0.f ? m_run + __logf(l_run) : -INFINITY;
}

}  // namespace

// ---------------------------------------------------------------------------------------------- launchers
hipError_t launch_generic_quantize(const QuantArgs &a, bool v_side, hipStream_t s)
{
    hipLaunchKernelGGL(gen_assign_kernel, dim3((a.nq + 3) / 4, a.n_streams), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (v_side)
        hipLaunchKernelGGL(gen_quantize_v_kernel, dim3(a.nq / 16, a.n_streams), dim3(kGenThreads), 0, s, a);
    else
        hipLaunchKernelGGL(gen_quantize_k_kernel, dim3(a.nq / a.G, a.n_streams), dim3(kGenThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_generic_tail_copy(const TailCopyArgs &a, hipStream_t s)
{
    const int64_t work = (int64_t)(a.i1 - a.i0) * (a.d / 8);
    if (work <= 0) return hipSuccess;
    hipLaunchKernelGGL(gen_tail_copy_kernel, dim3((unsigned)((work + 255) / 256), a.n_streams, 2), dim3(256), 0, s, a);
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
        hipLaunchKernelGGL(gen_mine_assign_kernel, dim3((a.T + 3) / 4, a.n_sets), dim3(256), 0, s, a, it == a.iters - 1 ? 1 : 0);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (a.inertia) {
            hipLaunchKernelGGL(gen_mine_inertia_kernel, dim3(a.n_sets), dim3(256), 0, s, a, it);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        hipLaunchKernelGGL(gen_mine_sums_kernel, dim3(a.tsplit, a.n_sets), dim3(kGenThreads), 0, s, a, chunk);
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
    hipLaunchKernelGGL(gen_decode_kernel, dim3(a.n_seq * a.n_q_heads), dim3(kGenThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_generic_dequant(const DequantArgs &a, hipStream_t s)
{
    if (a.t1 <= a.t0) return hipSuccess;
    hipLaunchKernelGGL(gen_dequant_kernel, dim3(a.t1 - a.t0, a.n_streams), dim3(kGenThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace pk
