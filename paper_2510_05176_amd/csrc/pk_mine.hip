// Pattern mining: Lloyd iterations for the K-means objective of Sec. 3.1 Eq. 4, one independent
// problem per pattern set (layer x KV head, K and V separately).
//
// One iteration = mine_step_kernel (assignment step and per-chunk cluster sums, both on the matrix
// cores) followed by mine_update_kernel (fixed-order reduction over the chunks, mean, fp16 rounding).
// Every sum is formed in a fixed order, so results are reproducible bit for bit.
#include "pk_assign_mfma.h"
#include "pk_internal.h"

namespace pk {

namespace {

// patterns[s][p] <- x[s][p], p < P  (initialisation from the first P vectors)
__global__ __launch_bounds__(256) void mine_init_kernel(MineArgs a)
{
    const int s = blockIdx.y;
    const int w = blockIdx.x * 256 + threadIdx.x;
    if (w >= a.P * kRowChunks) return;
    const int p = w >> 4, ch = w & 15;
    const uint4 v = *reinterpret_cast<const uint4 *>(a.x + (int64_t)s * a.set_stride + (int64_t)p * kD + ch * 8);
    *reinterpret_cast<uint4 *>(a.patterns + ((int64_t)s * a.P + p) * kD + ch * 8) = v;
}

// Assignment step + partial cluster sums of one chunk of one set.  64*NW threads.
// The chunk is walked in sub-tiles of 16*NT*NW vectors: every wave assigns 16*NT of them on the matrix cores
// (NT tiles per pass over the table) and leaves them, with their indices, in an LDS tile.  The cluster sums are a second contraction on the
// matrix cores, sums[p][c] += sum_t onehot[p][t] x[t][c].  The NW waves (4, or 8 when the table is large and
// only one workgroup fits a CU) split the pattern tiles (and, when there are fewer pattern tiles than waves,
// the 8 channel tiles as well), so each wave forms the one-hot operand of its own pattern rows only and keeps
// its accumulator tiles in registers for the whole chunk.  The vector operand is x transposed (the
// contraction runs over vectors, the tile is stored vector-major): it comes out of LDS with the transposing
// 64-bit read, in which lane i of a 16-lane group receives element i of four rows whose 32-byte pieces the
// group's lanes address four to a row.  The one-hot operand is formed in packed fp16 as
// clamp(1 - (idx_t - p)^2, 0, 1), which is exactly 1 or 0 for integers below 256; products are exact and the
// accumulation order is fixed by the instruction sequence, so the sums are reproducible.
// Dynamic LDS: [table pad16(P) rows] [-norm2/2 pad16(P)] [cnt pad16(P)] [xs 16 NT NW rows]
//              [idx 16 NT NW halves] [xrow NW*kD halves]
constexpr int kMineXs = kD + 16;   // halves per row of the vector tile: 72 words, so the eight rows that 32 lanes
                                   // of a transposing read touch (8 words each) fall on 64 distinct banks

typedef _Float16 half2m __attribute__((ext_vector_type(2)));
typedef short short4m __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4m *lds_short4_ptr;

template <int NPT, int NW, int NT>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(NT == 1 && NPT <= 4 ? 4 : 2))) void mine_step_kernel(MineArgs a, int chunk, int outputs)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int P = a.P;
    __half *tab_s = reinterpret_cast<__half *>(smem);
    float *norm_s = reinterpret_cast<float *>(smem + (size_t)pad16(P) * kTabStride * 2);
    int *cnt = reinterpret_cast<int *>(norm_s + pad16(P));
    __half *xs = reinterpret_cast<__half *>(cnt + pad16(P));
    constexpr int ST = 16 * NT * NW;     // vectors per sub-tile: NT 16-vector tiles per wave
    __half *idx_s = xs + ST * kMineXs;   // pattern index of every vector of the sub-tile, as an fp16 number
    __half *xrow_s = idx_s + ST;
    __shared__ float red_s[NW];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 15, kb = lane >> 4;
    const int ck = blockIdx.x, s = blockIdx.y;
    const int t_begin = ck * chunk, n_tok = min(chunk, a.T - t_begin);
    const __half *xg = a.x + (int64_t)s * a.set_stride + (int64_t)t_begin * kD;
    const __half *Mg = a.patterns + (int64_t)s * P * kD;

    auto load_tile = [&](int sub, uint4 (&xb)[NT][4]) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int tok = min(sub * ST + (wave * NT + j) * 16 + n, n_tok - 1);   // rows past the chunk repeat its last vector
#pragma unroll
            for (int k = 0; k < 4; ++k) xb[j][k] = *reinterpret_cast<const uint4 *>(xg + (int64_t)tok * kD + 32 * k + 8 * kb);
        }
    };
    uint4 xb[NT][4];
    load_tile(0, xb);

    for (int i = tid; i < pad16(P); i += 64 * NW) cnt[i] = 0;
    stage_patterns(Mg, P, tab_s, norm_s, red_s, 64 * NW);   // ends with a barrier
    PatternTable tb;
    tb.lds_rows = tab_s;
    tb.nh = norm_s;
    tb.norm2_max = red_s[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) tb.norm2_max = fmaxf(tb.norm2_max, red_s[w]);
    tb.P = P;

    // this wave's share of the sums: PW pattern tiles from pt0, CW channel tiles from ct0
    constexpr int PW = NPT >= NW ? NPT / NW : 1;
    constexpr int CW = NPT >= NW ? 8 : 8 * NPT / NW;
    const int pt0 = NPT >= NW ? wave * PW : wave % NPT;
    const int ct0 = NPT >= NW ? 0 : (wave / NPT) * CW;
    floatx4_t acc[PW][CW];
    half2m prow[PW];   // this lane's pattern row of every tile, as a packed pair
#pragma unroll
    for (int pi = 0; pi < PW; ++pi) {
#pragma unroll
        for (int ci = 0; ci < CW; ++ci) acc[pi][ci] = floatx4_t{0.f, 0.f, 0.f, 0.f};
        const _Float16 v = (_Float16)(float)(16 * (pt0 + pi) + n);
        prow[pi] = half2m{v, v};
    }
    const half2m one2 = {(_Float16)1.f, (_Float16)1.f};

    const int n_sub = (n_tok + ST - 1) / ST;
    for (int sub = 0; sub < n_sub; ++sub) {
        int bi[NT];
        float bv[NT], x2[NT];
        bool flag[NT];
        assign_tiles_mfma<NT>(xb, tb, lane, bi, bv, x2, flag);
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int tl = (wave * NT + j) * 16 + n, tok = sub * ST + tl;
            float bd = fmaxf(bv[j], 0.f);
            resolve_flagged(xb[j], flag[j], xrow_s + wave * kD, tb, lane, bi[j], bd);
#pragma unroll
            for (int k = 0; k < 4; ++k)   // a row past the chunk is stored as zeros, so it adds nothing to any sum
                *reinterpret_cast<uint4 *>(xs + tl * kMineXs + 32 * k + 8 * kb) = tok < n_tok ? xb[j][k] : make_uint4(0u, 0u, 0u, 0u);
            if (kb == 0) {
                idx_s[tl] = __float2half_rn((float)bi[j]);   // integers below 2048 are exact
                if (tok < n_tok) {
                    // per-vector outputs only where somebody reads them: indices from the last step (if asked
                    // for), distances when the objective is reported
                    if (outputs & 1) a.assign[(int64_t)s * a.T + t_begin + tok] = bi[j];
                    if (outputs & 2) a.best[(int64_t)s * a.T + t_begin + tok] = bd;
                    atomicAdd(&cnt[bi[j]], 1);
                }
            }
        }
        if (sub + 1 < n_sub) load_tile(sub + 1, xb);   // in flight during the accumulation
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < ST / 32; ++ks) {
            // 32 vectors per step; this lane's k-slots 0-3 are vectors ta .. ta+3, its slots 4-7 the ones 16 later
            const int ta = 32 * ks + 4 * kb;
            const uint2 ia = *reinterpret_cast<const uint2 *>(idx_s + ta);
            const uint2 ib = *reinterpret_cast<const uint2 *>(idx_s + ta + 16);
            const half2m idh[4] = {__builtin_bit_cast(half2m, ia.x), __builtin_bit_cast(half2m, ia.y),
                                   __builtin_bit_cast(half2m, ib.x), __builtin_bit_cast(half2m, ib.y)};
            uint4 av[PW];
#pragma unroll
            for (int pi = 0; pi < PW; ++pi) {
                uint32_t aop[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const half2m d = idh[j] - prow[pi];
                    half2m oh = one2 - d * d;                       // 1 where the index equals the row, <= 0 elsewhere
                    oh = __builtin_elementwise_min(__builtin_elementwise_max(oh, half2m{(_Float16)0.f, (_Float16)0.f}), one2);   // folds into the clamp bit
                    aop[j] = __builtin_bit_cast(uint32_t, oh);
                }
                av[pi] = make_uint4(aop[0], aop[1], aop[2], aop[3]);
            }
            // lane n of group kb addresses the 8-byte piece (n & 3) of row ta + n / 4 and receives column n of rows ta .. ta+3
            const __half *piece = xs + (ta + (n >> 2)) * kMineXs + 16 * ct0 + 4 * (n & 3);
#pragma unroll
            for (int ci = 0; ci < CW; ++ci) {
                const short4m lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(piece + 16 * ci));
                const short4m hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(piece + 16 * kMineXs + 16 * ci));
                const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
                const uint4 bop = make_uint4(l2.x, l2.y, h2.x, h2.y);
#pragma unroll
                for (int pi = 0; pi < PW; ++pi) acc[pi][ci] = mfma_f16(av[pi], bop, acc[pi][ci]);
            }
        }
        __syncthreads();
    }
    // partial sums of the chunk: D rows 4kb+i = pattern 16(pt0 + pi) + 4kb + i, column n = channel 16(ct0 + ci) + n
    const int64_t o = ((int64_t)s * a.tsplit + ck) * P;
#pragma unroll
    for (int pi = 0; pi < PW; ++pi) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int pr = 16 * (pt0 + pi) + 4 * kb + i;
            if (pr < P) {
#pragma unroll
                for (int ci = 0; ci < CW; ++ci) a.psum[(o + pr) * kD + 16 * (ct0 + ci) + n] = acc[pi][ci][i];
            }
        }
    }
    for (int i = tid; i < P; i += 64 * NW) a.pcnt[o + i] = cnt[i];
}

// update step: centroid = mean of members (binary32 division), rounded to fp16;
// an empty cluster keeps its centroid
__global__ __launch_bounds__(128) void mine_update_kernel(MineArgs a)
{
    const int p = blockIdx.x, s = blockIdx.y, c = threadIdx.x;
    const int64_t o0 = (int64_t)s * a.tsplit * a.P + p, step = a.P;
    // chunks in increasing order, eight loads in flight at a time; the order of the additions is fixed
    float sum = 0.f;
    int cnt = 0;
    int ts = 0;
    for (; ts + 8 <= a.tsplit; ts += 8) {
        float v[8];
        int k[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            v[u] = a.psum[(o0 + (ts + u) * step) * kD + c];
            k[u] = a.pcnt[o0 + (ts + u) * step];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            sum += v[u];
            cnt += k[u];
        }
    }
    for (; ts < a.tsplit; ++ts) {
        sum += a.psum[(o0 + ts * step) * kD + c];
        cnt += a.pcnt[o0 + ts * step];
    }
    if (cnt > 0) a.patterns[((int64_t)s * a.P + p) * kD + c] = __float2half_rn(sum / (float)cnt);
}

// inertia of one assignment step: fixed-order sum of the best distances
__global__ __launch_bounds__(256) void mine_inertia_kernel(MineArgs a, int it)
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

// Decode-stage pattern of a window (Sec. 3.1 "Decoding Stage", Eq. 5): per channel (min + max) / 2 over the
// window's vectors, in binary32 (exact for fp16 inputs), rounded to fp16.  One workgroup per window;
// thread <-> (channel, token parity).
__global__ __launch_bounds__(256) void window_pattern_kernel(const __half *x, int64_t set_stride, int n, __half *out,
                                                             int64_t out_stride)
{
    __shared__ float s_mn[kD], s_mx[kD];
    const int c = threadIdx.x & (kD - 1), par = threadIdx.x >> 7;
    const __half *xs = x + (int64_t)blockIdx.x * set_stride + c;
    float mn = INFINITY, mx = -INFINITY;
    for (int t = par; t < n; t += 2) {
        const float v = h2f(xs[(int64_t)t * kD]);
        mn = fminf(mn, v);
        mx = fmaxf(mx, v);
    }
    if (par == 1) {
        s_mn[c] = mn;
        s_mx[c] = mx;
    }
    __syncthreads();
    if (par == 0) {
        mn = fminf(mn, s_mn[c]);
        mx = fmaxf(mx, s_mx[c]);
        out[(int64_t)blockIdx.x * out_stride + c] = __float2half_rn((mn + mx) * 0.5f);
    }
}

size_t step_lds_bytes(int P, int nw, int nt)
{
    size_t b = (size_t)pad16(P) * kTabStride * 2;
    b += (size_t)pad16(P) * 4 + (size_t)pad16(P) * 4 + 16 * nw * nt * (size_t)kMineXs * 2 + 16 * nw * nt * 2 + (size_t)nw * kD * 2;
    return (b + 15) / 16 * 16;
}

}  // namespace

// Workgroups of the step kernel that one compute unit holds at a time: registers allow four 4-wave groups up
// to 64 patterns; the table and the vector tile in LDS allow two at 128 patterns and one 8-wave group above.
static int step_groups_per_cu(int P) { return P <= 64 ? 4 : P <= 128 ? 2 : 1; }

int mine_chunk(int T, int n_sets, int P)
{
    // One resident round of workgroups over the chip's 256 compute units: all chunks then run side by side and
    // take the same time, and every chunk writes its P*128 partial sums once, so fewer, longer chunks also
    // mean less traffic.  At most 64 chunks per set, none shorter than 256 vectors.
    const int64_t slots = 256 * step_groups_per_cu(P);
    const int64_t per_set = slots / n_sets > 1 ? slots / n_sets : 1;
    int64_t c = (T + per_set - 1) / per_set;
    if (c < (T + 63) / 64) c = (T + 63) / 64;
    c = (c + 127) / 128 * 128;
    if (c < 256) c = 256;
    return (int)c;
}

int mine_tsplit(int T, int n_sets, int P) { return (T + mine_chunk(T, n_sets, P) - 1) / mine_chunk(T, n_sets, P); }

template <int NPT, int NW, int NT>
static hipError_t launch_step(const MineArgs &a, int chunk, size_t lds, hipStream_t s, int outputs)
{
    hipLaunchKernelGGL((mine_step_kernel<NPT, NW, NT>), dim3(a.tsplit, a.n_sets), dim3(64 * NW), lds, s, a, chunk, outputs);
    return hipGetLastError();
}

template <int NPT, int NW, int NT>
static hipError_t prepare_step(const MineArgs &, int, size_t, hipStream_t, int)
{
    static LdsOptIn opt_in;   // the most this instantiation needs: a table of 16 * NPT patterns
    return allow_dynamic_lds(reinterpret_cast<const void *>(&mine_step_kernel<NPT, NW, NT>), opt_in, step_lds_bytes(16 * NPT, NW, NT));
}

hipError_t launch_mine(const MineArgs &a, hipStream_t s)
{
    if (a.d != kD) return launch_generic_mine(a, s);
    hipError_t e;
    const int chunk = mine_chunk(a.T, a.n_sets, a.P);
    const int npt = a.P <= 16 ? 1 : a.P <= 32 ? 2 : a.P <= 64 ? 4 : a.P <= 128 ? 8 : 16;
    // 8 waves share the table when only one workgroup fits a CU (P > 128; at 128 patterns two 4-wave workgroups
    // measured faster than one 8-wave group).  From 128 patterns on a wave assigns two 16-vector tiles per
    // table pass: reading the table out of LDS is what limits the assignment there, and every tile read then
    // serves 32 vectors (at 64 patterns and below the smaller tile and the higher occupancy win).
    const int nt = npt >= 8 ? 2 : 1;
    const int nw = a.P > 128 ? 8 : 4;
    const size_t lds = step_lds_bytes(a.P, nw, nt);
#define PK_STEP(CALL)                                                                                       \
    (npt == 1 ? CALL<1, 4, 1> : npt == 2 ? CALL<2, 4, 1> : npt == 4 ? CALL<4, 4, 1> : npt == 8 ? CALL<8, 4, 2> : CALL<16, 8, 2>)
    if ((e = PK_STEP(prepare_step)(a, chunk, lds, s, 0)) != hipSuccess) return e;
    if (!a.init_given) {
        hipLaunchKernelGGL(mine_init_kernel, dim3((a.P * kRowChunks + 255) / 256, a.n_sets), dim3(256), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    for (int it = 0; it < a.iters; ++it) {
        const int outputs = (a.assign && it == a.iters - 1 ? 1 : 0) | (a.inertia ? 2 : 0);
        if ((e = PK_STEP(launch_step)(a, chunk, lds, s, outputs)) != hipSuccess) return e;
        if (a.inertia) {
            hipLaunchKernelGGL(mine_inertia_kernel, dim3(a.n_sets), dim3(256), 0, s, a, it);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        hipLaunchKernelGGL(mine_update_kernel, dim3(a.P, a.n_sets), dim3(128), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
#undef PK_STEP
    return hipSuccess;
}

hipError_t launch_window_pattern(const __half *x, int64_t set_stride, int n_sets, int n, __half *out, int64_t out_stride,
                                 hipStream_t s)
{
    hipLaunchKernelGGL(window_pattern_kernel, dim3(n_sets), dim3(256), 0, s, x, set_stride, n, out, out_stride);
    return hipGetLastError();
}

}  // namespace pk
