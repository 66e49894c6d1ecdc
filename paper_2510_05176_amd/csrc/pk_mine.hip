// Pattern mining: Lloyd iterations for the K-means objective of Sec. 3.1 Eq. 4,
// one independent problem per pattern set (layer x KV head, K and V separately).
// Every sum is formed in a fixed order, so results are reproducible bit for bit.
#include "pk_assign.h"
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

// assignment step: nearest centroid of each of 128 vectors per workgroup
__global__ __launch_bounds__(128) void mine_assign_kernel(MineArgs a)
{
    __shared__ __align__(16) __half xs[128 * kXsStride];
    __shared__ AssignScratch sc;
    __shared__ int idx_s[128];
    __shared__ float best_s[128];

    const int tile = blockIdx.x, s = blockIdx.y, tid = threadIdx.x;
    const int n_tok = min(128, a.T - tile * 128);
    const __half *xg = a.x + (int64_t)s * a.set_stride + (int64_t)tile * 128 * kD;
    stage_rows(xs, n_tok, [&](int r) { return xg + (int64_t)r * kD; });
    assign_tile<128>(xs, n_tok, a.patterns + (int64_t)s * a.P * kD, a.P, PK_METRIC_L2, sc, idx_s, best_s);
    if (tid < n_tok) {
        a.assign[(int64_t)s * a.T + tile * 128 + tid] = idx_s[tid];
        a.best[(int64_t)s * a.T + tile * 128 + tid] = best_s[tid];
    }
}

// partial sums of the members of cluster p inside one slice of the token range;
// thread <-> channel, tokens visited in increasing order
__global__ __launch_bounds__(128) void mine_sum_kernel(MineArgs a)
{
    __shared__ int as[128];
    const int p = blockIdx.x, ts = blockIdx.y, s = blockIdx.z, c = threadIdx.x;
    const int len = (a.T + a.tsplit - 1) / a.tsplit;
    const int t_begin = ts * len, t_end = min(a.T, t_begin + len);
    const int32_t *asg = a.assign + (int64_t)s * a.T;
    const __half *xg = a.x + (int64_t)s * a.set_stride;
    float sum = 0.f;
    int cnt = 0;
    for (int base = t_begin; base < t_end; base += 128) {
        __syncthreads();
        as[c] = base + c < t_end ? asg[base + c] : -1;
        __syncthreads();
        for (int k = 0; k < 128; ++k) {
            if (as[k] == p) {
                sum += h2f(xg[(int64_t)(base + k) * kD + c]);
                ++cnt;
            }
        }
    }
    const int64_t o = ((int64_t)s * a.tsplit + ts) * a.P + p;
    a.psum[o * kD + c] = sum;
    if (c == 0) a.pcnt[o] = cnt;
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

}  // namespace

int mine_tsplit(int T)
{
    int ts = T / 2048;
    if (ts < 1) ts = 1;
    if (ts > 16) ts = 16;
    return ts;
}

hipError_t launch_mine(const MineArgs &a, hipStream_t s)
{
    hipError_t e;
    if (!a.init_given) {
        hipLaunchKernelGGL(mine_init_kernel, dim3((a.P * kRowChunks + 255) / 256, a.n_sets), dim3(256), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    for (int it = 0; it < a.iters; ++it) {
        hipLaunchKernelGGL(mine_assign_kernel, dim3((a.T + 127) / 128, a.n_sets), dim3(128), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (a.inertia) {
            hipLaunchKernelGGL(mine_inertia_kernel, dim3(a.n_sets), dim3(256), 0, s, a, it);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        hipLaunchKernelGGL(mine_sum_kernel, dim3(a.P, a.tsplit, a.n_sets), dim3(128), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(mine_update_kernel, dim3(a.P, a.n_sets), dim3(128), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace pk
