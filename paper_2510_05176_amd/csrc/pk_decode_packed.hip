// Decode attention over the packed part of the cache on the matrix cores
// (Sec. 3.4 "Decode-stage KV reconstruction": index restoration + dequantization + QK, and
// dequantization + index restoration + weights.V, fused; here softmax is fused in as well).
//
// For one KV stream and its r query heads, with NG = channel groups per V token:
//   score[h][t] = scale * ( QM[h][k*_t] + sum_c (q_h[c] s_K[g][c]) code_K[t][c] + q_h . z_K[g] )
//   out[h][c]   = sum_p W[h][p] M_V[p][c] + sum_t p[h][t] s_V[t][g(c)] code_V[t][c] + sum_t p[h][t] z_V[t][g(c)]
// Both code contractions run as v_mfma_f32_16x16x32_f16.  The 2-bit codes are never converted to
// floating point: two bit planes are merged into 2-bit fields with two bit-field inserts, and a
// field masked in place inside the mantissa of an fp16 with exponent field 0 *is* the subnormal
// number code * 2^(pos-24).  The power of two is folded into the other operand (q*s on the K side,
// p*s on the V side), which is built in packed fp16.
//
// Work split: a workgroup = 4 waves handles one split of one stream; each wave walks its own run
// of 64-token blocks with its own online-softmax state, and the four states are merged at the end.
// Lane roles inside a wave (lane = 16*kb + n):
//   K side  A operand: row n  <-> token 16*(n/4) + 4*x + n%4 of the block (tile x = 0..3),
//                      lane group kb <-> channels 32*kb .. 32*kb+31 (one plane word per plane)
//           B operand: column n <-> (head h = n % r, V channel group g = n / r), duplicated over g so
//                      that the softmax numerators come out of the MFMA already in the lanes that
//                      need them for the V side;  D: column n, rows 4*kb+i <-> token 16*kb + 4*x + i
//   V side  A operand: row n = (h, g), lane group kb <-> the 16 tokens of unit kb of the block
//           B operand: column n <-> channel 16*tile + n, lane group kb <-> the same 16 tokens
//           D (output accumulators): column n <-> channel 16*tile + n, rows 4*kb+i <-> (h, g) rows
//
// HALF variant (r * NG <= 8, one K group per block): the (h, g) pairs fill only eight of the sixteen columns, so
// column n and column n + 8 carry the same pair and the two halves of a lane group's 16 tokens are split between
// them: lanes n < 8 keep the scores of tokens 16*kb + 0..7 (score tiles x = 0, 1), lanes n >= 8 those of tokens
// 16*kb + 8..15 (tiles x = 2, 3).  Every per-token step after the K-side MFMAs (pattern-score gather, exponentials,
// per-pattern mass, V-side A operand) then runs on 8 values per lane instead of 16.  On the V side the two K = 32
// steps of a channel tile cover tokens 0..7 and 8..15 of the units, so lanes n < 8 feed the first step and lanes
// n >= 8 the second (the other operand is zero): output rows rho and rho + 8 are two partial sums of one (h, g)
// pair and are added in the epilogue.
#include "pk_internal.h"
#include "pk_decode_tail.h"

namespace pk {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t bfi(uint32_t m, uint32_t a, uint32_t b) { return (a & m) | (b & ~m); }

__device__ __forceinline__ floatx4 mfma16(const uint32_t *a, const uint32_t *b, floatx4 c)
{
    union { uint32_t u[4]; half8 h; } A, B;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        A.u[i] = a[i];
        B.u[i] = b[i];
    }
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(A.h, B.h, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack2(_Float16 lo, _Float16 hi)
{
    half2v v = {lo, hi};
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint32_t pk_mul(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2v, a) * __builtin_bit_cast(half2v, b));
}
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, a), __builtin_bit_cast(half2v, b), c, false);
}
__device__ __forceinline__ uint32_t cvt2(float lo, float hi)
{
    float2v f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, half2v));
}

// Sixteen 2-bit fields at the even bit positions of X -> eight operand registers.  Register v
// holds, in its low half, the field of X-bit e_lo(v) and, in its high half, the field of X-bit
// e_lo(v) + 16, both at mantissa position pos(v):
//   v = 0..4: e_lo = 2v, pos = 2v ;  v = 5..7: e_lo = 10 + 2(v-5), pos = 2(v-5).
__device__ __forceinline__ void fields_to_operand(uint32_t X, uint32_t *out)
{
    out[0] = X & 0x00030003u;
    out[1] = X & 0x000C000Cu;
    out[2] = X & 0x00300030u;
    out[3] = X & 0x00C000C0u;
    out[4] = X & 0x03000300u;
    const uint32_t Y = X >> 10;
    out[5] = Y & 0x00030003u;
    out[6] = Y & 0x000C000Cu;
    out[7] = Y & 0x00300030u;
}
__host__ __device__ constexpr int e_lo(int v) { return v < 5 ? 2 * v : 10 + 2 * (v - 5); }
__host__ __device__ constexpr int fpos(int v) { return v < 5 ? 2 * v : 2 * (v - 5); }

struct GroupOperand {
    uint32_t Bq[16];   // q[h][c] * s[g][c] * 2^(8-pos) rounded to fp16, operand order
    uint32_t Bl[16];   // what that rounding dropped (the product of two fp16 numbers has 22 significant bits), as fp16;
                       // formed and used only for groups whose scales are large enough for it to matter (lo_on)
    float qz;          // scale * log2(e) * q_h . z[g]
    bool lo_on;        // wave-uniform
};

// sum over the 64 lanes (row shifts, then the two row broadcasts of the wave), returned wave-uniform
__device__ __forceinline__ float wave_sum(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x111, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x112, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x114, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x118, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xa, 0xf, false));   // row_bcast:15 into rows 1 and 3
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xc, 0xf, false));   // row_bcast:31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// lo/hi half of (a * b - c) with the fp16 halves widened and one rounding at the end: for c = fp16(a * b) this is
// exactly the rounding error of the fp16 product (it has at most 11 significant bits), again as fp16
__device__ __forceinline__ uint32_t product_error(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t r;
    asm("v_fma_mixlo_f16 %0, %1, %2, -%3 op_sel:[0,0,0] op_sel_hi:[1,1,1]\n\t"
        "v_fma_mixhi_f16 %0, %1, %2, -%3 op_sel:[1,1,1] op_sel_hi:[1,1,1]"
        : "=&v"(r)
        : "v"(a), "v"(b), "v"(c));
    return r;
}

template <int BITS, bool G32, bool HALF, bool PAGED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void decode_packed_kernel(DecodeArgs a)
{
    static_assert(!(HALF && G32), "the split of a unit's tokens over column halves assumes one K group per block");
    constexpr int WPU = BITS / 2;   // 32-bit words per (channel, 16-token unit) of V; K: 4*BITS words per token
    constexpr int NTK = HALF ? 8 : 16;   // tokens of a block whose scores a lane keeps
    // second contraction pass with the rounding errors of q * s (see build_group); not with two K groups per block,
    // whose two operand sets leave no registers for it (32-token groups also have the smallest scales)
    constexpr bool COMP = !G32;
    // dynamic LDS: QMs [P][16] floats (q.M_K per pattern and column); Ws [4 waves][R][w_stride] 64-bit fixed-point
    // sums (softmax mass per V pattern, unit 2^-31).  Integer LDS atomics run at full rate on this chip, float
    // ones retire about one lane per 2.6 cycles (measured), which made the mass sums the slowest part of a block.
    extern __shared__ __align__(16) unsigned char dyn_smem[];
    __shared__ float stat_m[4][16], stat_l[4][16], stat_pz[4][16];

    // Rows of the grid behind the streams hold the workgroups of the fp16 tails (own tails first, then the shared
    // prefix's if it has one): they ride along in this launch and fill the slots that the last round of packed
    // splits leaves idle, instead of running as a kernel of their own afterwards.
    if ((int)blockIdx.y >= a.n_seq * a.n_kv_heads * a.head_groups) {
        const int N = a.n_seq * a.n_kv_heads;
        const int NG2 = N * a.head_groups;   // (stream, head group) pairs
        const int id = ((int)blockIdx.y - NG2) * (int)gridDim.x + (int)blockIdx.x;
        if (id >= NG2 * (a.prefix.t_tail > 0 ? 2 : 1)) return;
        const int which = id / NG2, sg = id - which * NG2;
        if (a.n_q_heads / a.n_kv_heads / a.head_groups <= 4)
            decode_tail_body<4>(a, which, sg / a.head_groups, sg % a.head_groups, *reinterpret_cast<TailShared<4> *>(dyn_smem));
        else
            decode_tail_body<8>(a, which, sg / a.head_groups, sg % a.head_groups, *reinterpret_cast<TailShared<8> *>(dyn_smem));
        return;
    }
    const int tid = threadIdx.x, lane = tid & 63, n = lane & 15, kb = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: block ranges and base addresses stay scalar
    const int split = blockIdx.x;
    // row y of the grid: stream y / head_groups, group y % head_groups of its query heads
    int ns = blockIdx.y;
    int head0 = 0;                                   // first head of the row's group inside the KV head
    const int R_all = a.n_q_heads / a.n_kv_heads;    // query heads per KV head
    if (a.head_groups > 1) {
        const int grp = ns % a.head_groups;
        ns /= a.head_groups;
        head0 = grp * (R_all / a.head_groups);
    }
    if (a.seq_order) {   // a ragged batch: row y of the grid is a head of the (y / heads)-th longest sequence
        const int rank = ns / a.n_kv_heads;
        ns = a.seq_order[rank] * a.n_kv_heads + (ns - rank * a.n_kv_heads);
    }
    const int n_slots = a.splits_prefix + a.splits_own + 2;
    const int seq = ns / a.n_kv_heads, head = ns - seq * a.n_kv_heads;
    const bool in_prefix = split < a.splits_prefix;
    const CacheView &cv = in_prefix ? a.prefix : a.own;
    const int cstream = in_prefix ? head : ns;
    const int set = in_prefix ? head : a.sets.set_of(ns);
    const int t_begin = (in_prefix ? split : split - a.splits_prefix) * a.chunk;
    int tq = cv.t_quant;
    if (!in_prefix) {   // a ragged batch: this sequence's own fill state; a split past its end has no blocks
        int tt, ts;
        own_state(a, seq, tq, tt, ts);
    }
    const int t_end = max(t_begin, min(tq, t_begin + a.chunk));
    if (t_end == t_begin) {   // nothing of this sequence in the split: an empty partial (mass 0; the merge skips it)
        const int R0 = R_all / a.head_groups;
        const int64_t pbase = ((int64_t)ns * n_slots + split) * R_all + head0;
        for (int e = tid; e < R0 * kD; e += 256) a.part_o[pbase * kD + e] = 0.f;
        for (int e = tid; e < R0 * a.P; e += 256) a.part_w[pbase * a.P + e] = 0.f;
        if (tid < R0) {
            a.part_ml[(pbase + tid) * 2] = -INFINITY;
            a.part_ml[(pbase + tid) * 2 + 1] = 0.f;
        }
        return;
    }

    const int R = R_all / a.head_groups, G = a.G, P = a.P;   // heads of this row
    const int lgG = 31 - __clz(G);   // G is a power of two
    const int Gc = G < kD ? G : kD, NG = kD / Gc;
    const int hcol = HALF ? (n & 7) : n;            // the (h, g) pair of this lane's column
    const bool second = HALF && n >= 8;             // this lane keeps the second half of its unit's tokens
    const uint32_t m_first = second ? 0u : 0xffffffffu, m_second = ~m_first;
    const bool col_ok = hcol < R * NG;
    const int h = col_ok ? hcol % R : 0, g = col_ok ? hcol / R : 0;
    const __half *MK = a.patterns_k + (int64_t)set * P * kD;
    const int WS = a.w_stride;   // P, or 256 when index 255 can occur (tokens quantized without a pattern)
    float *QMs = reinterpret_cast<float *>(dyn_smem);
    unsigned long long *Ws = reinterpret_cast<unsigned long long *>(QMs + P * 16);
    constexpr float kWUnit = 2147483648.f;   // 2^31: weights are at most 1

    // ---- this lane's slice of its query head: channels 32*kb .. 32*kb+31
    _Float16 qh[32];
    {
        const uint4 *qsrc = reinterpret_cast<const uint4 *>(a.q + ((int64_t)seq * a.n_q_heads + head * R_all + head0 + h) * kD + 32 * kb);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint4 v = qsrc[i];
            if (!col_ok) v = make_uint4(0, 0, 0, 0);
            const half2v *hv = reinterpret_cast<const half2v *>(&v);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                qh[8 * i + 2 * k] = hv[k][0];
                qh[8 * i + 2 * k + 1] = hv[k][1];
            }
        }
    }
    // The operands below multiply q by up to 2^8 and by the K scales in fp16: the head's query is brought to
    // max |q| in [1, 2) by a power of two first (exact), which is folded back into the softmax scale of the
    // column, so that only the stored scales bound the operands (s_K < 128, i.e. a K residual range per
    // channel and group below 3 * 128 at 2 bits).
    float lam = 1.f;
    {
        float qmax = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) qmax = fmaxf(qmax, fabsf((float)qh[i]));
        qmax = fmaxf(qmax, __shfl_xor(qmax, 16));
        qmax = fmaxf(qmax, __shfl_xor(qmax, 32));
        if (qmax > 0.f) {
            int e;
            (void)frexpf(qmax, &e);          // qmax = m * 2^e, m in [0.5, 1)
            lam = ldexpf(1.f, 1 - e);
        }
#pragma unroll
        for (int i = 0; i < 32; ++i) qh[i] = (_Float16)((float)qh[i] * lam);
    }
    const float sc2 = a.softmax_scale * kLog2e / lam;
    const float c1 = sc2 * 65536.f, inv_c1 = 1.f / c1;
    // sum_c s_c^2 of a K group above which the dropped parts of q * s are contracted as well: the estimated score
    // error softmax_scale * 4.2e-4 * sqrt(|q|^2 / d * sum_c s_c^2) then exceeds 6e-4 for some head of the stream
    float lo_threshold = INFINITY;
    if (COMP) {
        float qq = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) qq = fmaf((float)qh[i], (float)qh[i], qq);
        qq += __shfl_xor(qq, 16);
        qq += __shfl_xor(qq, 32);                                     // |lam q|^2 of the column's head
        const float per_head = a.softmax_scale * a.softmax_scale / (lam * lam) * qq * (1.f / kD);
        float worst = per_head;
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) worst = fmaxf(worst, __shfl_xor(worst, off));
        worst = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, worst)));
        lo_threshold = worst > 0.f ? 2.04f / worst : INFINITY;       // (6e-4 / 4.2e-4)^2
    }
    uint32_t qn[16], qp[16];   // natural channel order; operand order with the field scale folded in
#pragma unroll
    for (int i = 0; i < 16; ++i) qn[i] = pack2(qh[2 * i], qh[2 * i + 1]);
#pragma unroll
    for (int V = 0; V < 16; ++V) {
        const int v = V & 7, odd = V >> 3;
        const _Float16 c = (_Float16)(float)(1 << (8 - fpos(v)));
        qp[V] = pack2(qh[e_lo(v) + odd] * c, qh[e_lo(v) + 16 + odd] * c);
    }

    // ---- QM[p][n] = scale*log2e * q_h . M_K[p], one 16-pattern tile per wave and round
    for (int tp = wave; tp * 16 < P; tp += 4) {
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        const int p = tp * 16 + n;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint4 av = make_uint4(0, 0, 0, 0);
            if (p < P) av = *reinterpret_cast<const uint4 *>(MK + (int64_t)p * kD + 32 * kb + 8 * s);
            acc = mfma16(reinterpret_cast<const uint32_t *>(&av), &qn[4 * s], acc);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int pr = tp * 16 + 4 * kb + i;
            if (pr < P) QMs[pr * 16 + n] = acc[i] * sc2;
        }
    }
    for (int i = lane; i < R * WS; i += 64) Ws[wave * R * WS + i] = 0ull;
    // With two K groups per block, or the extra operands of 4-bit codes, the registers that q in natural order
    // would hold for the rest of the kernel are needed elsewhere (the kernel is at its 256-register limit and
    // spilled): it waits in LDS instead (identical in the four waves; [piece][lane]).
    constexpr bool Q_LDS = G32 || BITS == 4;
    __shared__ uint4 qn_s[Q_LDS ? 4 : 1][64];
    if (Q_LDS && wave == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) qn_s[i][lane] = make_uint4(qn[4 * i], qn[4 * i + 1], qn[4 * i + 2], qn[4 * i + 3]);
    }
    __syncthreads();

    // ---- this wave's run of 64-token blocks
    const int n_blocks = (t_end - t_begin) >> 6;
    const int per = (n_blocks + 3) >> 2;
    const int b0 = wave * per, b1 = min(n_blocks, b0 + per);

    // Online softmax state per column.  Scores are formed relative to m_run (the reference enters the
    // matrix-core accumulator), so the exponentials need no subtraction; the reference is raised only
    // when a block exceeds it.
    float m_run = 0.f, l_run = 0.f, pzacc = 0.f;
    bool started = false;
    floatx4 O[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) O[t] = floatx4{0.f, 0.f, 0.f, 0.f};
    GroupOperand ga, gb;   // gb: second K group of a block, only when G == 32

    // Base pointers (wave-uniform) such that base + offset(logical token) is the token's place: for contiguous
    // streams the stream's start, fixed; for a paged cache the start of the page part that holds the block,
    // minus the block's logical position, set anew for every block (a 64-token block and a K group never
    // straddle a page).  The K-side set runs one block ahead of the V-side set (K inputs are prefetched).
    // Offsets from a base fit 32 bits (the host refuses capacities for which they would not).
    // (PAGED is a template parameter: the re-basing branches cost the contiguous case 1 % when decided at run time)
    constexpr bool paged = PAGED;
    const char *kcodes, *kscale, *kzero, *kidx, *vcodes, *vscale, *vzero, *vidx;
    // (the page of a block is looked up one block ahead of its first use, so that the scalar load of the table entry
    // is not on the path of the block's loads: with the lookup in place a scrambled cache of 128-token pages read
    // 33 % slower than contiguous streams)
    auto set_k_bases = [&](int tb, int page) {
        const int64_t delta = cv.map.pos_in(page, cstream, tb) - tb;   // a multiple of the page size (or stream * capacity)
        kcodes = reinterpret_cast<const char *>(cv.k_codes + delta * 4 * BITS);
        kscale = reinterpret_cast<const char *>(cv.k_scale + (delta >> lgG) * kD);
        kzero = reinterpret_cast<const char *>(cv.k_zero + (delta >> lgG) * kD);
        kidx = reinterpret_cast<const char *>(cv.k_idx + delta);
    };
    auto set_v_bases = [&](int tb, int page) {
        const int64_t delta = cv.map.pos_in(page, cstream, tb) - tb;
        vcodes = reinterpret_cast<const char *>(cv.v_codes) + delta * (kD * BITS / 8);
        vscale = reinterpret_cast<const char *>(cv.v_scale + delta * NG);
        vzero = reinterpret_cast<const char *>(cv.v_zero + delta * NG);
        vidx = reinterpret_cast<const char *>(cv.v_idx + delta);
    };
    int pg_cur = paged ? cv.map.page_of(cstream, t_begin + (b0 << 6)) : 0, pg_next = pg_cur;   // pages of this wave's current / next block
    set_k_bases(t_begin + (b0 << 6), pg_cur);
    set_v_bases(t_begin + (b0 << 6), pg_cur);
    int pg_v = pg_cur;   // page the V-side bases stand for

    // parameters of one K group: raw loads, then the B operand
    struct GroupRaw {
        uint4 s[4], z[4];
        uint32_t own;   // the lane's own two of the group's 128 scales (lane <-> dword), for the sum of their squares
    };
    auto load_group_raw = [&](int grp, GroupRaw &gr) {
        // offsets inside a stream fit 32 bits (checked on the host): base pointer + 32-bit lane offset
        const uint32_t prow = ((uint32_t)grp * kD + 32 * kb) * 2;
        const uint4 *sp = reinterpret_cast<const uint4 *>(kscale + prow);
        const uint4 *zp = reinterpret_cast<const uint4 *>(kzero + prow);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            gr.s[i] = sp[i];
            gr.z[i] = zp[i];
        }
        if (COMP) gr.own = *reinterpret_cast<const uint32_t *>(kscale + (uint32_t)grp * kD * 2 + lane * 4);
    };
    auto build_group = [&](const GroupRaw &gr, GroupOperand &go) {
        _Float16 sh[32];
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const half2v *hv = reinterpret_cast<const half2v *>(&gr.s[i]);
            const uint32_t *zu = reinterpret_cast<const uint32_t *>(&gr.z[i]);
            uint4 qv;
            if (G32 || BITS == 4)
                qv = qn_s[i][lane];
            else
                qv = make_uint4(qn[4 * i], qn[4 * i + 1], qn[4 * i + 2], qn[4 * i + 3]);
            const uint32_t qw[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                sh[8 * i + 2 * k] = hv[k][0];
                sh[8 * i + 2 * k + 1] = hv[k][1];
                acc = dot2(qw[k], zu[k], acc);
            }
        }
#pragma unroll
        for (int V = 0; V < 16; ++V) {
            const int v = V & 7, odd = V >> 3;
            go.Bq[V] = pk_mul(qp[V], pack2(sh[e_lo(v) + odd], sh[e_lo(v) + 16 + odd]));
        }
        // The fp16 rounding of q * s (2^-12 relative per channel) leaves a score error of about
        // softmax_scale * 4.2e-4 * sqrt(sum_c q_c^2 s_c^2); where the group's scales make that matter (large-magnitude
        // channels: outliers over long groups, a RoPE sub-space), the dropped part of every product is formed too
        // and contracted in a second pass over the same code operand.  The test uses |q|^2 / d for q_c^2.
        go.lo_on = false;
        if (COMP) {
            const float s2 = wave_sum(dot2(gr.own, gr.own, 0.f));
            go.lo_on = s2 > lo_threshold;
            if (go.lo_on) {
#pragma unroll
                for (int V = 0; V < 16; ++V) {
                    const int v = V & 7, odd = V >> 3;
                    go.Bl[V] = product_error(qp[V], pack2(sh[e_lo(v) + odd], sh[e_lo(v) + 16 + odd]), go.Bq[V]);
                }
            }
        }
        acc += __shfl_xor(acc, 16);
        acc += __shfl_xor(acc, 32);
        go.qz = acc * sc2;
    };


    // K-side inputs of a block: plane words of this lane's 4 token rows, pattern indices of the tokens whose scores
    // it keeps (16, or its half of the unit: 8)
    uint32_t kw[4][BITS];
    uint32_t kidw[NTK / 4];
    auto load_k = [&](int tb) {
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int tok = tb + 16 * (n >> 2) + 4 * x + (n & 3);
            const char *src = kcodes + ((uint32_t)tok * 4 + kb) * BITS * 4;
            if (BITS == 2) {
                const uint2 v = *reinterpret_cast<const uint2 *>(src);
                kw[x][0] = v.x;
                kw[x][1] = v.y;
            } else {
                const uint4 v = *reinterpret_cast<const uint4 *>(src);
                kw[x][0] = v.x;
                kw[x][1] = v.y;
                kw[x][BITS - 2] = v.z;
                kw[x][BITS - 1] = v.w;
            }
        }
        if (HALF) {
            const uint2 v = *reinterpret_cast<const uint2 *>(kidx + (uint32_t)(tb + 16 * kb + (second ? 8 : 0)));
            kidw[0] = v.x;
            kidw[1] = v.y;
        } else {
            const uint4 v = *reinterpret_cast<const uint4 *>(kidx + (uint32_t)(tb + 16 * kb));
            kidw[0] = v.x;
            kidw[1] = v.y;
            kidw[NTK / 4 - 2] = v.z;
            kidw[NTK / 4 - 1] = v.w;
        }
    };

    if (b0 < b1) {
        const int tb = t_begin + (b0 << 6);
        load_k(tb);
        GroupRaw gr;
        load_group_raw(tb >> lgG, gr);
        build_group(gr, ga);
        if (G32) {
            load_group_raw((tb >> lgG) + 1, gr);
            build_group(gr, gb);
        }
    }

    // field scale 2^(8 - pos) of the V-side operand registers this lane builds: registers 0..7 of a unit, or
    // (HALF) the four of its token half
    constexpr int NAV = NTK / 2;
    uint32_t cfield[NAV];
#pragma unroll
    for (int V = 0; V < NAV; ++V) {
        const _Float16 c_lo = (_Float16)(float)(1 << (8 - fpos(V)));
        const _Float16 c_hi = (_Float16)(float)(1 << (8 - fpos(HALF ? V + 4 : V)));
        cfield[V] = second ? pack2(c_hi, c_hi) : pack2(c_lo, c_lo);
    }

    for (int b = b0; b < b1; ++b) {
        const int tb = t_begin + (b << 6);

        // ---- V-side loads of the block (used after the scores)
        if (paged) {   // bases change only where the walk enters another page
            if (pg_cur != pg_v) {
                set_v_bases(tb, pg_cur);
                pg_v = pg_cur;
            }
            if (b + 1 < b1 && ((tb + 64) & ((1 << cv.map.page_shift) - 1)) == 0) pg_next = cv.map.page_of(cstream, tb + 64);
        }
        const int unit = (tb >> 4) + kb;   // 16-token unit of this lane group
        uint32_t vidw[NTK / 4];
        if (HALF) {
            const uint2 v = *reinterpret_cast<const uint2 *>(vidx + (uint32_t)(tb + 16 * kb + (second ? 8 : 0)));
            vidw[0] = v.x;
            vidw[1] = v.y;
        } else {
            const uint4 v = *reinterpret_cast<const uint4 *>(vidx + (uint32_t)(tb + 16 * kb));
            vidw[0] = v.x;
            vidw[1] = v.y;
            vidw[NTK / 4 - 2] = v.z;
            vidw[NTK / 4 - 1] = v.w;
        }
        uint32_t vw[8 * WPU];
        {
            const uint4 *src = reinterpret_cast<const uint4 *>(vcodes + ((uint32_t)unit * 16 + n) * 8 * WPU * 4);
#pragma unroll
            for (int i = 0; i < 2 * WPU; ++i) {
                const uint4 v = src[i];
                vw[4 * i] = v.x;
                vw[4 * i + 1] = v.y;
                vw[4 * i + 2] = v.z;
                vw[4 * i + 3] = v.w;
            }
        }
        uint32_t sv[NAV], zv[NAV];   // scales / zero points of the lane's tokens, two per register
        {
            const uint32_t poff = ((uint32_t)unit * NG + g) * 32 + (second ? 16 : 0);
            const uint4 *sp = reinterpret_cast<const uint4 *>(vscale + poff);
            const uint4 *zp = reinterpret_cast<const uint4 *>(vzero + poff);
#pragma unroll
            for (int i = 0; i < NAV / 4; ++i) {
                const uint4 s4 = sp[i], z4 = zp[i];
                sv[4 * i] = s4.x; sv[4 * i + 1] = s4.y; sv[4 * i + 2] = s4.z; sv[4 * i + 3] = s4.w;
                zv[4 * i] = z4.x; zv[4 * i + 1] = z4.y; zv[4 * i + 2] = z4.z; zv[4 * i + 3] = z4.w;
            }
        }

        // ---- K side: scores of the 64 tokens relative to m_run (this lane: column n, tokens 16*kb + 0..15, or
        //      its half of them), log2 domain.  The accumulator starts at (q.z - m_run) / c1.
        float S[NTK];
        const float d0 = (ga.qz - m_run) * inv_c1;
        const float d02 = G32 ? (gb.qz - m_run) * inv_c1 : 0.f;
        floatx4 dfirst[HALF ? 2 : 1];   // HALF: score tiles 0 and 1 wait for tiles 2 and 3
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            uint32_t A16[16];
            fields_to_operand(bfi(0x55555555u, kw[x][0], kw[x][1] << 1), A16);
            fields_to_operand(bfi(0x55555555u, kw[x][0] >> 1, kw[x][1]), A16 + 8);
            floatx4 d = {d0, d0, d0, d0}, d2 = {d02, d02, d02, d02};
#pragma unroll
            for (int s = 0; s < 4; ++s) d = mfma16(&A16[4 * s], &ga.Bq[4 * s], d);
            if (COMP && ga.lo_on) {
#pragma unroll
                for (int s = 0; s < 4; ++s) d = mfma16(&A16[4 * s], &ga.Bl[4 * s], d);
            }
            if (G32) {
#pragma unroll
                for (int s = 0; s < 4; ++s) d2 = mfma16(&A16[4 * s], &gb.Bq[4 * s], d2);
            }
            if (BITS == 4) {
                uint32_t H16[16];
                fields_to_operand(bfi(0x55555555u, kw[x][BITS - 2], kw[x][BITS - 1] << 1), H16);
                fields_to_operand(bfi(0x55555555u, kw[x][BITS - 2] >> 1, kw[x][BITS - 1]), H16 + 8);
                floatx4 e = {0.f, 0.f, 0.f, 0.f}, e2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) e = mfma16(&H16[4 * s], &ga.Bq[4 * s], e);
                if (COMP && ga.lo_on) {
#pragma unroll
                    for (int s = 0; s < 4; ++s) e = mfma16(&H16[4 * s], &ga.Bl[4 * s], e);
                }
                d += 4.f * e;
                if (G32) {
#pragma unroll
                    for (int s = 0; s < 4; ++s) e2 = mfma16(&H16[4 * s], &gb.Bq[4 * s], e2);
                    d2 += 4.f * e2;
                }
            }
            if (G32 && kb >= 2) d = d2;
            if (HALF) {
                if (x < 2) {
                    dfirst[x] = d;
                } else {
                    // lanes n < 8 take tile x - 2 (tokens 4(x-2) + i of the unit), lanes n >= 8 tile x (tokens 8 + 4(x-2) + i)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t sel = (__float_as_uint(dfirst[x - 2][i]) & m_first) | (__float_as_uint(d[i]) & m_second);
                        const int id = (kidw[x - 2] >> (8 * i)) & 255;
                        S[4 * (x - 2) + i] = fmaf(__uint_as_float(sel), c1, QMs[id * 16 + n]);
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int id = (kidw[x] >> (8 * i)) & 255;
                    S[4 * x + i] = fmaf(d[i], c1, QMs[id * 16 + n]);
                }
            }
        }

        // ---- next block's K-side inputs and group parameters: in flight during the rest of this block
        const bool more = b + 1 < b1;
        const int tbn = tb + 64;
        const bool new_group = more && (G32 || (tbn >> lgG) != (tb >> lgG));
        GroupRaw gr;
        if (paged && more && pg_next != pg_cur) {
            set_k_bases(tbn, pg_next);
            pg_cur = pg_next;
        }
        if (more) load_k(tbn);
        if (new_group) load_group_raw(tbn >> lgG, gr);

        // ---- online softmax (per column; the lane groups, and with HALF the two column halves, hold different tokens)
        float bmax = fmaxf(S[0], S[1]);
#pragma unroll
        for (int k = 2; k < NTK; k += 2) bmax = fmaxf(fmaxf(bmax, S[k]), S[k + 1]);
        if (!started || __ballot(bmax > 0.f) != 0ull) {
            if (HALF) bmax = fmaxf(bmax, __shfl_xor(bmax, 8));
            bmax = fmaxf(bmax, __shfl_xor(bmax, 16));
            bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
            const float delta = started ? fmaxf(bmax, 0.f) : bmax;
            const float alpha = started ? __builtin_amdgcn_exp2f(-delta) : 0.f;
            l_run *= alpha;
            pzacc *= alpha;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float ar = __shfl(alpha, 4 * kb + i);   // column 4*kb+i owns output row 4*kb+i
#pragma unroll
                for (int t = 0; t < 8; ++t) O[t][i] *= ar;
            }
            if (started) {
                for (int hh = 0; hh < R; ++hh) {
                    const float ar = __shfl(alpha, hh);
                    for (int p = lane; p < P; p += 64) {
                        unsigned long long *w = &Ws[(wave * R + hh) * WS + p];
                        *w = (unsigned long long)((float)*w * ar);
                    }
                }
            }
            m_run += delta;
#pragma unroll
            for (int k = 0; k < NTK; ++k) S[k] -= delta;
            started = true;
        }
        float pr[NTK];
#pragma unroll
        for (int k = 0; k < NTK; ++k) pr[k] = __builtin_amdgcn_exp2f(S[k]);

        // ---- softmax mass per V pattern (the columns of channel group 0 carry every head once per token)
        if (hcol < R) {
#pragma unroll
            for (int k = 0; k < NTK; ++k)
                atomicAdd(&Ws[(wave * R + hcol) * WS + ((vidw[k >> 2] >> (8 * (k & 3))) & 255)],
                          (unsigned long long)(uint32_t)(pr[k] * kWUnit));   // pr <= 1: no overflow; truncation loses < 2^-31
        }

        // ---- V side
        uint32_t Ap[8], Ap4[8];
        const uint32_t ones = pack2((_Float16)1.f, (_Float16)1.f);
#pragma unroll
        for (int V = 0; V < NAV; ++V) {
            const uint32_t ph = cvt2(pr[2 * V], pr[2 * V + 1]);
            pzacc = dot2(ph, zv[V], pzacc);
            l_run = dot2(ph, ones, l_run);   // the denominator sums the same rounded weights the numerator uses
            const uint32_t av = pk_mul(pk_mul(ph, sv[V]), cfield[V]);
            if (HALF) {   // registers 0..3 feed the K step of tokens 0..7, registers 4..7 that of tokens 8..15
                Ap[V] = av & m_first;
                Ap[V + 4] = av & m_second;
            } else {
                Ap[V] = av;
            }
        }
        if (BITS == 4) {
#pragma unroll
            for (int V = 0; V < 8; ++V) Ap4[V] = pk_mul(Ap[V], pack2((_Float16)4.f, (_Float16)4.f));
        }
        if (G32 && new_group) {   // first group done here, so that one set of registers serves both loads
            build_group(gr, ga);
            load_group_raw((tbn >> lgG) + 1, gr);
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            // one word = plane 0 (bits 0..15) and plane 1 (bits 16..31) of 16 tokens of channel 16*t + n;
            // merge into 2-bit fields: even tokens in the low half, odd tokens in the high half
            uint32_t Bv[8];
            {
                const uint32_t D = vw[t * WPU];
                const uint32_t u = bfi(0x0000AAAAu, D >> 15, D);
                fields_to_operand(bfi(0x55550000u, D << 15, u), Bv);
            }
            O[t] = mfma16(&Ap[0], &Bv[0], O[t]);
            O[t] = mfma16(&Ap[4], &Bv[4], O[t]);
            if (BITS == 4) {
                const uint32_t D = vw[t * WPU + WPU - 1];
                const uint32_t u = bfi(0x0000AAAAu, D >> 15, D);
                fields_to_operand(bfi(0x55550000u, D << 15, u), Bv);
                O[t] = mfma16(&Ap4[0], &Bv[0], O[t]);
                O[t] = mfma16(&Ap4[4], &Bv[4], O[t]);
            }
        }

        // ---- B operand of the next block's K group(s)
        if (new_group) build_group(gr, G32 ? gb : ga);
    }
    if (!started) m_run = -INFINITY;   // a wave without blocks contributes nothing to the merge

    // ---- merge the four waves of the workgroup
    if (HALF) {   // the two column halves hold partial sums over different tokens
        l_run += __shfl_xor(l_run, 8);
        pzacc += __shfl_xor(pzacc, 8);
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    pzacc += __shfl_xor(pzacc, 16);
    pzacc += __shfl_xor(pzacc, 32);
    if (kb == 0) {
        stat_m[wave][n] = m_run;
        stat_l[wave][n] = l_run;
        stat_pz[wave][n] = pzacc;
    }
    __syncthreads();
    // (column rho of the score tile = head rho % R, channel group rho / R; the quotients are formed by comparison
    // and the channel tile's group by a shift - integer divisions by run-time values here once cost more than
    // the rest of the epilogue, 10 us per workgroup)
    const int lgGc = 31 - __clz(Gc);
    const int64_t pbase = ((int64_t)ns * n_slots + split) * R_all + head0;
    // pattern masses first: afterwards the table and mass area of the dynamic LDS is free for the outputs
    for (int e = tid; e < R * P; e += 256) {
        int hh = 0;
#pragma unroll
        for (int k = 1; k < 8; ++k) hh += (e >= k * P) ? 1 : 0;   // e / P without a division (R <= 8)
        const int pp = e - hh * P;
        const float M = fmaxf(fmaxf(stat_m[0][hh], stat_m[1][hh]), fmaxf(stat_m[2][hh], stat_m[3][hh]));
        float acc = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) acc = fmaf(__builtin_amdgcn_exp2f(stat_m[w][hh] - M), (float)Ws[(w * R + hh) * WS + pp], acc);
        a.part_w[pbase * P + e] = acc * (1.f / kWUnit);
    }
    __syncthreads();
    // every wave leaves its outputs, scaled to the workgroup's reference, in slabs of its own: Os[4][NH][R][kD]
    // floats over the start of the dynamic LDS (the launch sizes it for that); NH = 2 with HALF, where output rows
    // rho and rho + 8 are the two token halves of one (h, g) pair
    constexpr int NH = HALF ? 2 : 1;
    float *Os = reinterpret_cast<float *>(dyn_smem);
    {
        const int w = wave;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rho = 4 * kb + i, rc = HALF ? (rho & 7) : rho, half = HALF ? (rho >> 3) : 0;
            if (rc < R * NG) {
                const int gg = (rc >= R) + (rc >= 2 * R) + (rc >= 3 * R), hh = rc - gg * R;   // NG <= 4
                const float M = fmaxf(fmaxf(stat_m[0][rc], stat_m[1][rc]), fmaxf(stat_m[2][rc], stat_m[3][rc]));
                const float f = __builtin_amdgcn_exp2f(stat_m[w][rc] - M);
                const float pzv = half == 0 ? stat_pz[w][rc] : 0.f;   // the zero-point part is added once
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    if (((16 * t) >> lgGc) == gg) Os[((w * NH + half) * R + hh) * kD + 16 * t + n] = f * fmaf(O[t][i], 65536.f, pzv);
                }
            }
        }
    }
    __syncthreads();
    for (int e = tid; e < R * kD; e += 256) {   // slabs added in a fixed order: waves 0, 1, 2, 3 (first half, second half)
        float acc = Os[e];
#pragma unroll
        for (int k = 1; k < 4 * NH; ++k) acc += Os[k * R * kD + e];
        a.part_o[pbase * kD + e] = acc;
    }
    if (tid < R) {
        const float M = fmaxf(fmaxf(stat_m[0][tid], stat_m[1][tid]), fmaxf(stat_m[2][tid], stat_m[3][tid]));
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) L = fmaf(__builtin_amdgcn_exp2f(stat_m[w][tid] - M), stat_l[w][tid], L);
        a.part_ml[(pbase + tid) * 2] = M;
        a.part_ml[(pbase + tid) * 2 + 1] = L;
    }
}

}  // namespace

template <int BITS, bool G32, bool HALF, bool PAGED>
static hipError_t launch_variant(const DecodeArgs &a, dim3 grid, size_t lds, hipStream_t s)
{
    // the most any launch of this instantiation needs: 256 patterns, 8 heads per KV head, 256 mass slots per head
    static LdsOptIn opt_in;
    constexpr size_t kMaxLds = (size_t)256 * 16 * 4 + (size_t)4 * 8 * 256 * 8;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&decode_packed_kernel<BITS, G32, HALF, PAGED>), opt_in, kMaxLds);
    if (e != hipSuccess) return e;
    if (lds > kMaxLds) return hipErrorInvalidValue;
    hipLaunchKernelGGL((decode_packed_kernel<BITS, G32, HALF, PAGED>), grid, dim3(256), lds, s, a);
    return hipGetLastError();
}

// a paged cache of its own or a paged shared prefix: the variant that re-bases its pointers block by block
template <int BITS, bool G32, bool HALF>
static hipError_t launch_one(const DecodeArgs &a, dim3 grid, size_t lds, hipStream_t s)
{
    return a.own.map.page_table || a.prefix.map.page_table ? launch_variant<BITS, G32, HALF, true>(a, grid, lds, s)
                                                           : launch_variant<BITS, G32, HALF, false>(a, grid, lds, s);
}

hipError_t launch_decode_packed(const DecodeArgs &a, hipStream_t s)
{
    const int splits = a.splits_prefix + a.splits_own;
    if (splits == 0) return hipSuccess;
    const int N = a.n_seq * a.n_kv_heads;
    const int r = a.n_q_heads / a.n_kv_heads, NG = kD / (a.G < kD ? a.G : kD);
    const int R = r / a.head_groups;   // heads per row of the grid
    // tail workgroups (one per stream, another one per stream for the shared prefix's tail) in rows behind the streams
    const bool tails = decode_tails_ride_along(a);
    const int n_tail = tails ? N * a.head_groups * (a.prefix.t_tail > 0 ? 2 : 1) : 0;
    const dim3 grid(splits, N * a.head_groups + (n_tail + splits - 1) / splits);
    // eight or fewer (head, channel group) pairs leave half of the score columns free: they take the second half
    // of every unit's tokens
    const bool half = a.G != 32 && R * NG <= 8;
    size_t lds = (size_t)a.P * 16 * 4 + (size_t)4 * R * a.w_stride * 8;   // QMs, Ws
    const size_t out_slabs = (size_t)4 * (half ? 2 : 1) * R * kD * 4;     // reused for the waves' outputs at the end
    if (lds < out_slabs) lds = out_slabs;
    const size_t tail_lds = R <= 4 ? sizeof(TailShared<4>) : sizeof(TailShared<8>);
    if (tails && lds < tail_lds) lds = tail_lds;
    if (a.bits == 2 && a.G == 32) return launch_one<2, true, false>(a, grid, lds, s);
    if (a.bits == 2) return half ? launch_one<2, false, true>(a, grid, lds, s) : launch_one<2, false, false>(a, grid, lds, s);
    if (a.bits == 4 && a.G == 32) return launch_one<4, true, false>(a, grid, lds, s);
    if (a.bits == 4) return half ? launch_one<4, false, true>(a, grid, lds, s) : launch_one<4, false, false>(a, grid, lds, s);
    return hipErrorInvalidValue;
}

}  // namespace pk
