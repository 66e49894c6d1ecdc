// Pattern mining: Lloyd iterations for the K-means objective of Sec. 3.1 Eq. 4, one independent
// problem per pattern set (layer x KV head, K and V separately).
//
// One iteration = mine_step_kernel (assignment step on the matrix cores + per-chunk cluster sums in
// LDS) followed by mine_update_kernel (fixed-order reduction over the chunks, mean, fp16 rounding).
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

// Assignment step + partial cluster sums of one chunk of one set.  256 threads.
// Dynamic LDS: [table pad16(P) rows (TAB_LDS only)] [-norm2/2 pad16(P)] [sums P*kD] [cnt P] [idx chunk bytes] [xrow 4*kD halves]
template <bool TAB_LDS>
__global__ __launch_bounds__(256) void mine_step_kernel(MineArgs a, int chunk)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int P = a.P;
    __half *tab_s = reinterpret_cast<__half *>(smem);
    float *norm_s = reinterpret_cast<float *>(smem + (TAB_LDS ? (size_t)pad16(P) * kTabStride * 2 : 0));
    float *sums = norm_s + pad16(P);
    int *cnt = reinterpret_cast<int *>(sums + (size_t)P * kD);
    uint8_t *idx_s = reinterpret_cast<uint8_t *>(cnt + P);
    __half *xrow_s = reinterpret_cast<__half *>(idx_s + chunk);
    __shared__ float red_s[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 15, kb = lane >> 4;
    const int ck = blockIdx.x, s = blockIdx.y;
    const int t_begin = ck * chunk, n_tok = min(chunk, a.T - t_begin);
    const __half *xg = a.x + (int64_t)s * a.set_stride + (int64_t)t_begin * kD;
    const __half *Mg = a.patterns + (int64_t)s * P * kD;

    for (int i = tid; i < P * kD; i += 256) sums[i] = 0.f;
    for (int i = tid; i < P; i += 256) cnt[i] = 0;
    stage_patterns(Mg, P, tab_s, norm_s, red_s, TAB_LDS);   // ends with a barrier
    PatternTable tb;
    tb.lds_rows = tab_s;
    tb.glb_rows = Mg;
    tb.nh = norm_s;
    tb.norm2_max = fmaxf(fmaxf(red_s[0], red_s[1]), fmaxf(red_s[2], red_s[3]));
    tb.P = P;

    // ---- assignment: wave w takes the 16-token tiles w, w+4, ...
    const int n_tiles = (n_tok + 15) >> 4;
    for (int tile = wave; tile < n_tiles; tile += 4) {
        const int tok = tile * 16 + n;
        const int tok_c = min(tok, n_tok - 1);
        uint4 xb[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) xb[k] = *reinterpret_cast<const uint4 *>(xg + (int64_t)tok_c * kD + 32 * k + 8 * kb);
        int bi;
        float bv, x2, bd;
        bool flag;
        assign_tile_mfma<TAB_LDS>(xb, tb, lane, bi, bv, x2, flag);
        bd = fmaxf(bv, 0.f);
        resolve_flagged(xb, flag, xrow_s + wave * kD, tb, Mg, lane, bi, bd);
        if (kb == 0 && tok < n_tok) {
            idx_s[tok] = (uint8_t)bi;
            a.assign[(int64_t)s * a.T + t_begin + tok] = bi;
            a.best[(int64_t)s * a.T + t_begin + tok] = bd;
        }
    }
    __syncthreads();

    // ---- cluster sums of the chunk: thread <-> channel, vectors in increasing order
    if (tid < kD) {
        const int c = tid;
        for (int t = 0; t < n_tok; t += 16) {
            __half xv[16];
            int id[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int tt = min(t + u, n_tok - 1);
                xv[u] = xg[(int64_t)tt * kD + c];
                id[u] = idx_s[tt];
            }
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (t + u < n_tok) atomicAdd(&sums[id[u] * kD + c], h2f(xv[u]));
        }
    } else if (tid == kD) {
        for (int t = 0; t < n_tok; ++t) cnt[idx_s[t]] += 1;
    }
    __syncthreads();
    const int64_t o = ((int64_t)s * a.tsplit + ck) * P;
    for (int i = tid; i < P * kD; i += 256) a.psum[o * kD + i] = sums[i];
    for (int i = tid; i < P; i += 256) a.pcnt[o + i] = cnt[i];
}

// update step: centroid = mean of members (binary32 division), rounded to fp16;
// an empty cluster keeps its centroid
__global__ __launch_bounds__(128) void mine_update_kernel(MineArgs a)
{
    const int p = blockIdx.x, s = blockIdx.y, c = threadIdx.x;
    float sum = 0.f;
    int cnt = 0;
    for (int ts = 0; ts < a.tsplit; ++ts) {
        const int64_t o = ((int64_t)s * a.tsplit + ts) * a.P + p;
        sum += a.psum[o * kD + c];
        cnt += a.pcnt[o];
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

size_t step_lds_bytes(int P, int chunk, bool tab_lds)
{
    size_t b = tab_lds ? (size_t)pad16(P) * kTabStride * 2 : 0;
    b += (size_t)pad16(P) * 4 + (size_t)P * kD * 4 + (size_t)P * 4 + (size_t)chunk + 4 * kD * 2;
    return (b + 15) / 16 * 16;
}

}  // namespace

int mine_chunk(int T)
{
    int c = (T / 64 + 255) / 256 * 256;   // at most 64 chunks per set
    if (c < 256) c = 256;
    return c;
}

int mine_tsplit(int T) { return (T + mine_chunk(T) - 1) / mine_chunk(T); }

hipError_t launch_mine(const MineArgs &a, hipStream_t s)
{
    hipError_t e;
    const int chunk = mine_chunk(a.T);
    const bool tab_lds = a.P <= 128;
    const size_t lds = step_lds_bytes(a.P, chunk, tab_lds);
    if (tab_lds)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&mine_step_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    else
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&mine_step_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    if (!a.init_given) {
        hipLaunchKernelGGL(mine_init_kernel, dim3((a.P * kRowChunks + 255) / 256, a.n_sets), dim3(256), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    for (int it = 0; it < a.iters; ++it) {
        if (tab_lds)
            hipLaunchKernelGGL((mine_step_kernel<true>), dim3(a.tsplit, a.n_sets), dim3(256), lds, s, a, chunk);
        else
            hipLaunchKernelGGL((mine_step_kernel<false>), dim3(a.tsplit, a.n_sets), dim3(256), lds, s, a, chunk);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (a.inertia) {
            hipLaunchKernelGGL(mine_inertia_kernel, dim3(a.n_sets), dim3(256), 0, s, a, it);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        hipLaunchKernelGGL(mine_update_kernel, dim3(a.P, a.n_sets), dim3(128), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace pk
