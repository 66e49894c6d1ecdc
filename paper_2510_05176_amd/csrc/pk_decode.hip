// Decode attention: the fp16 tails (vector ALUs), the log-sum-exp merge of all partial results,
// and the launch sequence.  The packed part runs on the matrix cores (pk_decode_packed.hip).
//
// Every split of a stream's context writes an unnormalised partial per query head:
//   o[c] = sum_t 2^(S2_t - m) * (value part of token t),  m = max_t S2_t,  l = sum_t 2^(S2_t - m)
// with S2 = log2(e) * softmax_scale * q.k.  Packed splits leave the pattern part of V out of o and
// write the softmax mass per pattern W[p] instead, so that W . M_V is formed once per head here.
#include "pk_internal.h"
#include "pk_decode_tail.h"

namespace pk {

hipError_t launch_decode_packed(const DecodeArgs &a, hipStream_t s);

namespace {

constexpr int kMaxP = 256;
constexpr float kLn2 = 0.6931471805599453f;

// Stand-alone launch of the tails, for decodes without a packed part or with too many tails to ride along in the
// packed kernel's launch (decode_tails_ride_along).  x = 0: own tails, x = 1: the shared prefix's tail; y: stream;
// z: group of query heads.
template <int RP>
__global__ __launch_bounds__(256) void decode_tail_kernel(DecodeArgs a)
{
    __shared__ TailShared<RP> sh;
    decode_tail_body<RP>(a, blockIdx.x, blockIdx.y, blockIdx.z, sh);
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

// Ragged batch: rank of every sequence by the length of its packed part, longest first (ties by index), by
// counting; one workgroup, n_seq <= kMaxOrdered.  Workgroups are dispatched in grid order, so starting the long
// streams first keeps the last round from consisting of a few long ones running alone.
__global__ __launch_bounds__(kMaxOrdered) void decode_order_kernel(DecodeArgs a, int32_t *order)
{
    __shared__ int32_t key[kMaxOrdered];
    const int i = threadIdx.x, n = a.n_seq;
    int mine = 0;
    if (i < n) {
        int tq, tt, ts;
        own_state(a, i, tq, tt, ts);
        mine = tq;
        key[i] = tq;
    }
    __syncthreads();
    if (i >= n) return;
    int rank = 0;
    for (int j = 0; j < n; ++j) {
        const int k = key[j];
        rank += (k > mine || (k == mine && j < i)) ? 1 : 0;
    }
    order[rank] = i;
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
    const int64_t k_min = (t + 32767) / 32768;   // the fewest splits the length limit allows
    for (int64_t k = k_min; k < k_min + 512; ++k) {
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
    // the matrix-core kernel holds the (head, V channel group) pairs of a group of heads in the 16 columns of one tile
    // and takes up to 8 heads per group, the heads of a KV head in one group or two; what does not fit (5 or 7 heads
    // with 32-channel groups, an odd head count above 8, more than 16 heads) and the other head dimensions run the
    // plain kernels
    const int rg = r / a.head_groups;
    if (a.d != kD || rg > 8 || rg * (kD / (a.G < kD ? a.G : kD)) > 16) return launch_generic_decode(a, s);
    const int N = a.n_seq * a.n_kv_heads;
    hipError_t e;
    if (a.seq_order && a.splits_prefix + a.splits_own > 0) {
        hipLaunchKernelGGL(decode_order_kernel, dim3(1), dim3(kMaxOrdered), 0, s, a, const_cast<int32_t *>(a.seq_order));
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if ((e = launch_decode_packed(a, s)) != hipSuccess) return e;
    if ((a.own.t_tail > 0 || a.prefix.t_tail > 0) && !decode_tails_ride_along(a)) {
        // (launched for the prefix only if it has a tail: workgroups that find nothing to do still cost their
        // dispatch, tens of nanoseconds each)
        const dim3 grid(a.prefix.t_tail > 0 ? 2 : 1, N, a.head_groups);
        if (rg <= 4)
            hipLaunchKernelGGL((decode_tail_kernel<4>), grid, dim3(256), 0, s, a);
        else
            hipLaunchKernelGGL((decode_tail_kernel<8>), grid, dim3(256), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    // four parts per channel when a thread would otherwise walk many slots or patterns alone and the
    // (sequence, head) pairs are too few to fill the chip with 128-thread workgroups; eight when there are hundreds
    // of slots and patterns for a few heads only (config 5: 28 heads, 130 slots, 256 patterns: 17 -> 13 us)
    if (a.splits_prefix + a.splits_own + a.P >= 256 && a.n_seq * a.n_q_heads <= 256)
        hipLaunchKernelGGL(decode_merge_kernel<8>, dim3(a.n_seq * a.n_q_heads), dim3(1024), 0, s, a);
    else if (a.splits_prefix + a.splits_own + a.P >= 96 && a.n_seq * a.n_q_heads <= 2048)
        hipLaunchKernelGGL(decode_merge_kernel<4>, dim3(a.n_seq * a.n_q_heads), dim3(512), 0, s, a);
    else
        hipLaunchKernelGGL(decode_merge_kernel<1>, dim3(a.n_seq * a.n_q_heads), dim3(128), 0, s, a);
    return hipGetLastError();
}

}  // namespace pk
