// Quantize-append kernels: pattern selection (Sec. 3.2 Eq. 6), residual, group
// min/max -> stored (s, z), asymmetric n-bit quantization (Sec. 2.1 Eq. 1), bit-plane
// packing.  K is quantized per channel over groups of G tokens, V per token over
// groups of Gc channels (Sec. 4.1 "Quantization Settings").
//
// The arithmetic that decides a code is a fixed sequence of binary32 operations
// (subtract, one division per group for s, one for 1/s, subtract, multiply, round
// half to even, clamp); contraction into FMAs is switched off for this file so
// that the sequence is exactly what is written.
//
// Kernels, in file order: assign_minmax_kernel (the min-max selection rule of Sec. 3.2 as a search of its own: it
// writes the indices and the quantizers below then take them as given); quantize_k_kernel (groups of 128 tokens,
// a workgroup of eight waves per tile) and quantize_k_wave_kernel (groups of 32 / 64 tokens, a wave per group); quantize_v_kernel
// (a wave per 16-token unit); tail_copy_kernel (the fp16 ring); seq_table_kernel (per-sequence launch parameters
// of a ragged append).  Under the Euclidean rule the quantizers search on the matrix cores (pk_assign_mfma.h).
#pragma clang fp contract(off)

#include "pk_assign_mfma.h"
#include "pk_quant_arith.h"
#include "pk_internal.h"

namespace pk {

namespace {

// ---------------------------------------------------------------------------
// Min-max metric (Sec. 3.2): d_mm(x, m) = max_c (x_c - m_c) - min_c (x_c - m_c), argmin over the patterns, lowest
// index on ties.  Every operation is exact in binary32 apart from one correctly rounded subtraction per
// channel (fp16 values widened exactly), so the result is the definition's, bit for bit; it is not a
// contraction and runs on the vector ALUs.  A wave takes 64 vectors, lane <-> vector, the vector's 128 channels
// in registers as binary32; a pattern row is wave-uniform and comes through the scalar data path as packed fp16,
// which the mixed-precision subtract (x * 1.0 - m with the fp16 half widened) reads directly: per pattern and
// vector 128 subtractions and 128 three-operand maxima / minima.  The indices go to the cache's index array; the
// quantizers below then skip their own search.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float sub_s_lo(float x, uint32_t m)   // x - half(m.lo), m wave-uniform
{
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,0] op_sel_hi:[0,0,1]" : "=v"(r) : "v"(x), "s"(m));
    return r;
}
__device__ __forceinline__ float sub_s_hi(float x, uint32_t m)   // x - half(m.hi)
{
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,1] op_sel_hi:[0,0,1]" : "=v"(r) : "v"(x), "s"(m));
    return r;
}

// Sixteen consecutive dwords through the scalar data path (read only; address wave-uniform, 4-byte aligned), and the
// wait for every scalar load issued so far; the values are tied to the wait so that no use can move ahead of it.
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
// Which run of tiles of its stream (blockIdx.y) a workgroup takes.  Workgroups go to the chip's eight XCDs in turn
// by their linear index, y * gridDim.x + x; with the run taken as x itself an XCD would get the runs x = k, k + 8, ...
// of EVERY stream, and when streams have different numbers of runs (a ragged append: the grid is sized for the
// longest sequence and the runs past a sequence's end return at once) the XCDs of low k get up to 55 % more
// work than the last one (measured: 16 prompts of 2 k to 32 k tokens ran 1.55x slower than the same bytes in
// equal lengths).  Rotating the run by the stream index gives every XCD every residue class in turn.
__device__ __forceinline__ int chunk_of_workgroup()
{
    return (int)((blockIdx.x + blockIdx.y) % gridDim.x);
}

__device__ __forceinline__ u32x16 sload16(const uint32_t *p)
{
    u32x16 r;
    asm volatile("s_load_dwordx16 %0, %1, 0x0" : "=s"(r) : "s"(p) : "memory");
    return r;
}
__device__ __forceinline__ void swait2(u32x16 &r0, u32x16 &r1)
{
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(r0), "+s"(r1));
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void assign_minmax_kernel(QuantArgs a, int tiles_per_wg)
{
    const int tid = threadIdx.x, lane = tid & 63, ns = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t *Mg = reinterpret_cast<const uint32_t *>(a.patterns + (int64_t)a.sets.set_of(ns) * a.P * kD);
    take_sequence_entry(a, ns);
    const int n_tiles = a.nq / 64;
    const int tile0 = chunk_of_workgroup() * tiles_per_wg, tile1 = min(n_tiles, tile0 + tiles_per_wg);
    for (int tile = tile0 + wave; tile < tile1; tile += 4) {
        // the lane's vector, widened
        float x[kD];
        {
            const __half *row = a.src.row(ns, tile * 64 + lane);
#pragma unroll
            for (int ch = 0; ch < kRowChunks; ++ch) {
                const uint4 v = *reinterpret_cast<const uint4 *>(row + 8 * ch);
                const __half2 *h2 = reinterpret_cast<const __half2 *>(&v);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    x[8 * ch + 2 * k] = __low2float(h2[k]);
                    x[8 * ch + 2 * k + 1] = __high2float(h2[k]);
                }
            }
        }
        float best = INFINITY;
        int best_p = 0;
        // A pattern row is taken in two halves of 64 channels (32 scalar registers each).  Scalar loads return
        // in any order, so a wait covers all that are outstanding: the next half is requested right after the
        // wait for the current one and arrives under the 192 vector operations of that half.
        u32x16 a0 = sload16(Mg), a1 = sload16(Mg + 16), b0, b1;
        // two running maxima and minima, so that consecutive operations do not wait for each other
        float mxa, mxb, mna, mnb;
        auto scan = [&](const u32x16 &m, int c0) {   // channels c0 .. c0+31
#pragma unroll
            for (int c4 = 0; c4 < 8; ++c4) {
                const int c = c0 + 4 * c4;
                const float d0 = sub_s_lo(x[c], m[2 * c4]), d1 = sub_s_hi(x[c + 1], m[2 * c4]);
                const float d2 = sub_s_lo(x[c + 2], m[2 * c4 + 1]), d3 = sub_s_hi(x[c + 3], m[2 * c4 + 1]);
                mxa = fmaxf(fmaxf(mxa, d0), d1);
                mna = fminf(fminf(mna, d0), d1);
                mxb = fmaxf(fmaxf(mxb, d2), d3);
                mnb = fminf(fminf(mnb, d2), d3);
            }
        };
        for (int p = 0; p < a.P; ++p) {
            const uint32_t *mrow = Mg + (size_t)p * (kD / 2);                                   // wave-uniform
            const uint32_t *mnext = Mg + (size_t)min(p + 1, a.P - 1) * (kD / 2);                // (the last round repeats the last row; unused)
            swait2(a0, a1);
            b0 = sload16(mrow + 32);
            b1 = sload16(mrow + 48);
            mxa = mxb = -INFINITY;
            mna = mnb = INFINITY;
            scan(a0, 0);
            scan(a1, 32);
            swait2(b0, b1);
            a0 = sload16(mnext);
            a1 = sload16(mnext + 16);
            scan(b0, 64);
            scan(b1, 96);
            const float dist = fmaxf(mxa, mxb) - fminf(mna, mnb);
            if (dist < best) {   // patterns in increasing order: strict < keeps the lowest index
                best = dist;
                best_p = p;
            }
        }
        swait2(a0, a1);   // nothing may be in flight into registers that the next tile reuses
        a.idx[a.map.pos(ns, a.t0 + tile * 64) + lane] = (uint8_t)best_p;
    }
}

// ===========================================================================
// Euclidean metric: nearest pattern on the matrix cores (pk_assign_mfma.h).  A wave owns 16-token
// tiles; lane 16*kb + n holds, of token n, the 32 channels 32*k + 8*kb + j (k < 4, j < 8) - the MFMA
// B-operand layout - and keeps the residuals of those channels in registers through quantization and
// bit-plane packing.
//
// K: residuals also go to an LDS tile so that the per-channel minimum / maximum over the group's tokens
//    is a column scan; the parameters come back through LDS; every lane then forms one byte of each
//    plane word (8 channels) and stores it.
// V: everything per token stays inside the wave: group minimum / maximum by two cross-lane steps,
//    16 codes per plane packed per lane, and a 16x16 bit transpose across the 16 token lanes turns
//    them into the words of 16 tokens per channel.
// ===========================================================================

constexpr int kRStride = kD + 4;           // floats per row of the residual tile (16-byte aligned rows, bank skew 4)

// (sub_lo / sub_hi, the fp16 differences with one rounding, live in pk_assign_mfma.h: the exact search uses them too)
__device__ __forceinline__ float subz_lo(float x, uint32_t z)   // x - half(z.lo)
{
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,0] op_sel_hi:[0,0,1]" : "=v"(r) : "v"(x), "v"(z));
    return r;
}
__device__ __forceinline__ float subz_hi(float x, uint32_t z)   // x - half(z.hi)
{
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,1] op_sel_hi:[0,0,1]" : "=v"(r) : "v"(x), "v"(z));
    return r;
}

// Codes.  d = r - z >= 0 and d * (1/s) lies in [0, 2^b - 1] up to rounding because z <= min and
// s >= (max - z)/(2^b - 1), so the clamp of the definition never acts.  v_cvt_pk_u8_f32 rounds half to
// even like rintf (and saturates at 0 and 255) and drops the code into one byte of a word: four codes per
// word.  packed <- packed with code(d * inv) in byte `slot`.
__device__ __forceinline__ uint32_t put_code(float d, float inv, int slot, uint32_t packed)
{
    return __builtin_amdgcn_cvt_pk_u8_f32(d * inv, (uint32_t)slot, packed);
}

// Bits p of the 8 codes held in the bytes of (lo, hi), gathered into bits p .. p+7 of the result:
// two masked byte dot products with weights 1, 2, 4, .. 128.
__device__ __forceinline__ uint32_t plane_byte_shifted(uint32_t lo, uint32_t hi, int p)
{
    const uint32_t m = 0x01010101u << p;
    uint32_t acc = __builtin_amdgcn_udot4(lo & m, 0x08040201u, 0u, false);
    return __builtin_amdgcn_udot4(hi & m, 0x80402010u, acc, false);
}

struct TileShared {
    __half *tab;      // [pad16(P)][kTabStride]
    float *nh;        // [pad16(P)]
    unsigned char *wsc;   // V: [4 waves][kWaveScratch] (re-evaluation row, output staging)
    float *red;       // [8]: one maximum per wave from stage_patterns
    float *rt;        // K: [TT][kRStride]
    uint16_t *pz;     // K: [TT/G][kD] zero points (fp16 bits), then [TT/G][kD] scales
    float *pinv;      // K: [TT/G][kD] 1/s
};

// Per-wave output staging: the pieces a wave produces for its 16 tokens are put together in LDS so that
// every global store is one contiguous run of 8- or 16-byte lane pieces.
constexpr int kWsRow = 0;          // 256 B: one vector for the exact re-evaluation
constexpr int kWsCodes = 256;      // up to 1024 B: the unit's code words in memory order
constexpr int kWsIdx = 1280;       // 16 B: pattern indices
constexpr int kWsScale = 1296;     // up to 128 B: scales [group][16]
constexpr int kWsZero = 1424;      // up to 128 B: zero points [group][16]
constexpr int kWaveScratch = 1552;

// TT = 0: no residual tile (V)
__host__ __device__ inline size_t carve_offsets(int P, int TT, int G, size_t (&o)[7])
{
    size_t at = 0;
    o[0] = at; at += (size_t)pad16(P) * kTabStride * 2;
    o[1] = at; at += (size_t)pad16(P) * 4;
    o[2] = at; at += TT ? 0 : 4 * kWaveScratch;   // K stages in its own residual rows instead
    o[3] = at; at += 32;
    o[4] = at; at += (size_t)TT * kRStride * 4;
    const int ngrp = TT ? TT / G : 0;
    o[5] = at; at += (size_t)ngrp * kD * 2 * 2;
    o[6] = at; at += (size_t)ngrp * kD * 4;
    return at;
}

__device__ __forceinline__ TileShared carve(unsigned char *smem, int P, int TT, int G)
{
    size_t o[7];
    carve_offsets(P, TT, G, o);
    TileShared t;
    t.tab = reinterpret_cast<__half *>(smem + o[0]);
    t.nh = reinterpret_cast<float *>(smem + o[1]);
    t.wsc = smem + o[2];
    t.red = reinterpret_cast<float *>(smem + o[3]);
    t.rt = reinterpret_cast<float *>(smem + o[4]);
    t.pz = reinterpret_cast<uint16_t *>(smem + o[5]);
    t.pinv = reinterpret_cast<float *>(smem + o[6]);
    return t;
}

static size_t tile_lds_bytes(int P, int TT, int G)
{
    size_t o[7];
    return carve_offsets(P, TT, G, o);
}

__device__ __forceinline__ PatternTable make_table(const TileShared &sh, const __half *Mg, int P)
{
    PatternTable tb;
    tb.lds_rows = sh.tab;
    tb.nh = sh.nh;
    tb.norm2_max = fmaxf(fmaxf(sh.red[0], sh.red[1]), fmaxf(sh.red[2], sh.red[3]));
    tb.P = P;
    return tb;
}

// B operand of one 16-token tile: vectors i0 .. i0+15 of stream ns.
__device__ __forceinline__ void load_tile(const QuantArgs &a, int ns, int i0, uint4 (&xb)[4])
{
    const int lane = threadIdx.x & 63, n = lane & 15, kb = lane >> 4;
    const __half *row = a.src.row(ns, i0 + n);
#pragma unroll
    for (int k = 0; k < 4; ++k) xb[k] = *reinterpret_cast<const uint4 *>(row + 32 * k + 8 * kb);
}

// Residuals r[8k + j] of channel 32k + 8kb + j of the lane's token against pattern bi.
__device__ __forceinline__ void residuals(const TileShared &sh, const __half *Mg, const uint4 (&xb)[4], int bi, float (&r)[32])
{
    const int kb = (threadIdx.x & 63) >> 4;
    const __half *mrow = sh.tab + bi * kTabStride + 8 * kb;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint4 mv = *reinterpret_cast<const uint4 *>(mrow + 32 * k);
        const uint4 xv = xb[k];
        r[8 * k + 0] = sub_lo(xv.x, mv.x);
        r[8 * k + 1] = sub_hi(xv.x, mv.x);
        r[8 * k + 2] = sub_lo(xv.y, mv.y);
        r[8 * k + 3] = sub_hi(xv.y, mv.y);
        r[8 * k + 4] = sub_lo(xv.z, mv.z);
        r[8 * k + 5] = sub_hi(xv.z, mv.z);
        r[8 * k + 6] = sub_lo(xv.w, mv.w);
        r[8 * k + 7] = sub_hi(xv.w, mv.w);
    }
}

// Nearest pattern of the tile's tokens (exact).
__device__ __forceinline__ int assign_index(const PatternTable &tb, const __half *Mg, const uint4 (&xb)[4], __half *xrow)
{
    const int lane = threadIdx.x & 63;
    int bi;
    float bv, x2, bd;
    bool flag;
    assign_tile_mfma(xb, tb, lane, bi, bv, x2, flag);
    resolve_flagged(xb, flag, xrow, tb, lane, bi, bd);
    return bi;
}

__device__ __forceinline__ int assign_residuals(const TileShared &sh, const PatternTable &tb, const __half *Mg,
                                                const uint4 (&xb)[4], __half *xrow, float (&r)[32])
{
    const int bi = assign_index(tb, Mg, xb, xrow);
    residuals(sh, Mg, xb, bi, r);
    return bi;
}

// All LDS writes of the wave so far are visible to its own later reads.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Codes of the lane's 32 channels of one token against the group's parameters in LDS (zero points as fp16
// bits, 1/s as binary32, indexed by channel); 8 channels = one byte of a plane word, written to the token's
// row of the staging area stg ([16 tokens][4 words][BITS planes] words, memory order).
template <int BITS>
__device__ __forceinline__ void k_codes_to_staging(const float (&r)[32], const uint16_t *pz, const float *pinv, uint8_t *stg)
{
    const int lane = threadIdx.x & 63, n = lane & 15, kb = lane >> 4;
    uint8_t *mine = stg + n * 16 * BITS + kb;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint4 zq = *reinterpret_cast<const uint4 *>(pz + 32 * k + 8 * kb);
        const float4 i0 = *reinterpret_cast<const float4 *>(pinv + 32 * k + 8 * kb);
        const float4 i1 = *reinterpret_cast<const float4 *>(pinv + 32 * k + 8 * kb + 4);
        uint32_t lo = 0u, hi = 0u;
        lo = put_code(subz_lo(r[8 * k + 0], zq.x), i0.x, 0, lo);
        lo = put_code(subz_hi(r[8 * k + 1], zq.x), i0.y, 1, lo);
        lo = put_code(subz_lo(r[8 * k + 2], zq.y), i0.z, 2, lo);
        lo = put_code(subz_hi(r[8 * k + 3], zq.y), i0.w, 3, lo);
        hi = put_code(subz_lo(r[8 * k + 4], zq.z), i1.x, 0, hi);
        hi = put_code(subz_hi(r[8 * k + 5], zq.z), i1.y, 1, hi);
        hi = put_code(subz_lo(r[8 * k + 6], zq.w), i1.z, 2, hi);
        hi = put_code(subz_hi(r[8 * k + 7], zq.w), i1.w, 3, hi);
#pragma unroll
        for (int p = 0; p < BITS; ++p) mine[(k * BITS + p) * 4] = (uint8_t)(plane_byte_shifted(lo, hi, p) >> p);
    }
}

// Staging area -> global: the 16 tokens' code words as one contiguous run, then their 16 indices.
template <int BITS>
__device__ __forceinline__ void k_store_staging(const QuantArgs &a, int64_t tok0, const uint8_t *stg)
{
    const int lane = threadIdx.x & 63;
    uint8_t *codes = reinterpret_cast<uint8_t *>(a.codes_k);
    if (BITS == 2)
        reinterpret_cast<uint2 *>(codes + tok0 * 32)[lane] = reinterpret_cast<const uint2 *>(stg)[lane];
    else
        reinterpret_cast<uint4 *>(codes + tok0 * 64)[lane] = reinterpret_cast<const uint4 *>(stg)[lane];
    if (lane == 0) *reinterpret_cast<uint4 *>(a.idx + tok0) = *reinterpret_cast<const uint4 *>(stg + 16 * 16 * BITS);
}

// K: workgroup = NW waves, tiles of TT = max(64, G) tokens of one stream; wave w owns the 16-token
// tiles w*NT .. w*NT + NT-1 of the tile.  Launched for groups of 128 tokens with NW = 8, one 16-token tile per
// wave: the 128-token residual tile (68 KB) beside the pattern table leaves room for one workgroup per CU from 128
// patterns on, and eight waves give every SIMD two (four waves measured 12 % slower, on a bulk job at 64 patterns
// as on the 4-stream job at 256).
template <int G, int BITS, int NW>
__global__ __launch_bounds__(64 * NW) void quantize_k_kernel(QuantArgs a, int tiles_per_wg)
{
    constexpr int TT = G == 128 ? 128 : 64, NT = TT / (16 * NW);
    static_assert(NT >= 1, "every wave takes at least one 16-token tile");
    constexpr int LPC = TT / 32;          // lanes that share one channel in the column scan, 32 tokens each
    constexpr int CPR = 64 * NW / LPC;    // channels per round of the scan
    constexpr int NGRP = TT / G;          // parameter groups per tile
    extern __shared__ __align__(16) unsigned char smem[];
    const TileShared sh = carve(smem, a.P, TT, G);
    const int tid = threadIdx.x, ns = blockIdx.y;
    const int lane = tid & 63, wave = tid >> 6, n = lane & 15, kb = lane >> 4;
    const __half *Mg = a.patterns + (int64_t)a.sets.set_of(ns) * a.P * kD;
    take_sequence_entry(a, ns);
    const int n_tiles = a.nq / TT;
    const int tile0 = chunk_of_workgroup() * tiles_per_wg, tile1 = min(n_tiles, tile0 + tiles_per_wg);
    if (tile0 >= n_tiles) return;   // a ragged append: this sequence has fewer tiles than the launch was sized for
    uint4 xb[NT][4];
#pragma unroll
    for (int j = 0; j < NT; ++j) load_tile(a, ns, tile0 * TT + (wave * NT + j) * 16, xb[j]);   // in flight while the table is staged

    stage_patterns(Mg, a.P, sh.tab, sh.nh, sh.red, 64 * NW);
    PatternTable tb = make_table(sh, Mg, a.P);
    if (NW == 8) tb.norm2_max = fmaxf(tb.norm2_max, fmaxf(fmaxf(sh.red[4], sh.red[5]), fmaxf(sh.red[6], sh.red[7])));

    const int q = tid % LPC, cc = tid / LPC;
    for (int tile = tile0; tile < tile1; ++tile) {
        const int64_t tq0 = (int64_t)a.t0 + (int64_t)tile * TT;
        const int64_t pq0 = a.map.pos(ns, (int)tq0);   // where the tile's first token is stored
        float r[NT][32];
        int bi[NT];
        if (a.idx_given) {   // searched beforehand (min-max metric)
#pragma unroll
            for (int j = 0; j < NT; ++j) bi[j] = a.idx[pq0 + (wave * NT + j) * 16 + n];
        } else {   // the wave's NT 16-token tiles in one pass over the pattern table
            float bv[NT], x2[NT];
            bool flag[NT];
            assign_tiles_mfma<NT>(xb, tb, lane, bi, bv, x2, flag);
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                float bd;
                // scratch for the exact re-evaluation: the tile's own residual rows, which are written only below
                resolve_flagged(xb[j], flag[j], reinterpret_cast<__half *>(sh.rt + (wave * NT + j) * 16 * kRStride), tb, lane,
                                bi[j], bd);
            }
        }
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int tl = (wave * NT + j) * 16 + n;   // token slot inside the tile
            residuals(sh, Mg, xb[j], bi[j], r[j]);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float4 *dst = reinterpret_cast<float4 *>(sh.rt + tl * kRStride + 32 * k + 8 * kb);
                dst[0] = make_float4(r[j][8 * k], r[j][8 * k + 1], r[j][8 * k + 2], r[j][8 * k + 3]);
                dst[1] = make_float4(r[j][8 * k + 4], r[j][8 * k + 5], r[j][8 * k + 6], r[j][8 * k + 7]);
            }
        }
        __syncthreads();
        if (tile + 1 < tile1) {   // next tile's vectors: hidden behind the rest of this tile
#pragma unroll
            for (int j = 0; j < NT; ++j) load_tile(a, ns, (tile + 1) * TT + (wave * NT + j) * 16, xb[j]);
        }

        // column scan: lane q of a channel takes tokens 32q .. 32q+31, in an order rotated by q*16/LPC so
        // that the lanes of a wave fall on distinct banks
#pragma unroll
        for (int rd = 0; rd < 128 / CPR; ++rd) {
            const int c = cc + rd * CPR;
            float mn = INFINITY, mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < 32; t += 2) {
                const float v0 = sh.rt[(32 * q + ((t + q * (16 / LPC)) & 31)) * kRStride + c];
                const float v1 = sh.rt[(32 * q + ((t + 1 + q * (16 / LPC)) & 31)) * kRStride + c];
                mn = fminf(fminf(mn, v0), v1);
                mx = fmaxf(fmaxf(mx, v0), v1);
            }
            if (G >= 64) {
                mn = fminf(mn, __shfl_xor(mn, 1));
                mx = fmaxf(mx, __shfl_xor(mx, 1));
            }
            if (G == 128) {
                mn = fminf(mn, __shfl_xor(mn, 2));
                mx = fmaxf(mx, __shfl_xor(mx, 2));
            }
            const GroupParams gp = group_params(mn, mx, BITS);
            const int grp = G == 32 ? q : 0;
            if (G == 32 || q == 0) {
                sh.pz[grp * kD + c] = gp.z16;
                sh.pz[(NGRP + grp) * kD + c] = gp.s16;
                sh.pinv[grp * kD + c] = gp.inv;
            }
        }
        __syncthreads();
        // stored parameters of the tile's groups: 16-byte pieces, zero points then scales
        if (wave == NW - 1 && lane < NGRP * 32) {
            const int grp = lane >> 5, arr = (lane >> 4) & 1, piece = lane & 15;
            const uint4 v = *reinterpret_cast<const uint4 *>(sh.pz + (arr * NGRP + grp) * kD + piece * 8);
            __half *dstp = (arr ? a.scale : a.zero) + (pq0 / G + grp) * kD + piece * 8;
            *reinterpret_cast<uint4 *>(dstp) = v;
        }

        // codes of the lane's 32 channels per token; 8 channels = one byte of a plane word.  The bytes of the
        // wave's 16 tokens are put together in its own residual rows (no longer read by anyone) and leave as
        // one contiguous store.
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int tl0 = (wave * NT + j) * 16;
            const int grp = G == 32 ? tl0 >> 5 : 0;
            uint8_t *stg = reinterpret_cast<uint8_t *>(sh.rt + tl0 * kRStride);
            k_codes_to_staging<BITS>(r[j], sh.pz + grp * kD, sh.pinv + grp * kD, stg);
            if (kb == 0) stg[16 * 16 * BITS + n] = (uint8_t)bi[j];
            wave_lds_sync();
            k_store_staging<BITS>(a, pq0 + tl0, stg);
        }
        // the residual tile is rewritten only after the next barrier-separated scan has been passed by
        // every wave: the scan of this tile ended before the barrier above
    }
}

// K, groups of 32 or 64 tokens: a wave owns whole groups, so nothing but the pattern table is shared in
// the workgroup and no workgroup barrier is needed after it is staged.  The group's NTG = G/16 tiles stay
// in registers as loaded (fp16); pass A assigns every tile and feeds its residuals, 32 channels at a time,
// through a small LDS tile to a per-channel running minimum / maximum, pass B forms the residuals again,
// quantizes and stores.  A tile's registers are refilled with the wave's next group as soon as pass B
// has used them.
constexpr int kWkStride = 32 + 4;                     // floats per row of the quarter-width residual tile
constexpr int kWkTile = 16 * kWkStride * 4;           // bytes: 16 tokens x 32 channels (also the output staging area)
constexpr int kWkWave = kWkTile + kD * 2 * 2 + kD * 4;   // + zero points, scales (fp16 bits), 1/s

static size_t wave_k_lds_bytes(int P)
{
    return (size_t)pad16(P) * kTabStride * 2 + (size_t)pad16(P) * 4 + 16 + 4 * (size_t)kWkWave;
}

template <int G, int BITS, int NTA>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(NTA > 2 ? 2 : 3))) void quantize_k_wave_kernel(QuantArgs a, int tiles_per_wg)
{
    constexpr int NTG = G / 16;
    static_assert(G == 32 || G == 64, "a wave holds the group's tiles in registers");
    static_assert(16 * 16 * BITS + 16 <= kWkTile, "output staging fits the residual tile");
    extern __shared__ __align__(16) unsigned char smem[];
    TileShared sh;
    size_t at = 0;
    sh.tab = reinterpret_cast<__half *>(smem);
    at += (size_t)pad16(a.P) * kTabStride * 2;
    sh.nh = reinterpret_cast<float *>(smem + at);
    at += (size_t)pad16(a.P) * 4;
    sh.red = reinterpret_cast<float *>(smem + at);
    at += 16;
    const int tid = threadIdx.x, ns = blockIdx.y;
    const int lane = tid & 63, wave = tid >> 6, n = lane & 15, kb = lane >> 4;
    unsigned char *mine = smem + at + (size_t)wave * kWkWave;
    float *rt = reinterpret_cast<float *>(mine);
    uint16_t *pz = reinterpret_cast<uint16_t *>(mine + kWkTile);   // [kD] zero points, then [kD] scales
    float *pinv = reinterpret_cast<float *>(mine + kWkTile + kD * 2 * 2);

    const __half *Mg = a.patterns + (int64_t)a.sets.set_of(ns) * a.P * kD;
    take_sequence_entry(a, ns);
    const int n_tiles = a.nq / 64;
    const int tile0 = chunk_of_workgroup() * tiles_per_wg, tile1 = min(n_tiles, tile0 + tiles_per_wg);
    if (tile0 >= n_tiles) return;   // a ragged append: this sequence has fewer tiles than the launch was sized for
    const int g_end = tile1 * (64 / G);
    int g = tile0 * (64 / G) + wave;
    uint4 xb[NTG][4];
    if (g < g_end) {
#pragma unroll
        for (int j = 0; j < NTG; ++j) load_tile(a, ns, g * G + j * 16, xb[j]);   // in flight while the table is staged
    }
    stage_patterns(Mg, a.P, sh.tab, sh.nh, sh.red);
    const PatternTable tb = make_table(sh, Mg, a.P);

    for (; g < g_end; g += 4) {
        const int64_t tq0 = (int64_t)a.t0 + (int64_t)g * G;   // logical position of the group's first token
        const int64_t pq0 = a.map.pos(ns, (int)tq0);            // where it is stored
        // ---- pass A: indices; running minimum / maximum per channel.  The residuals pass through the LDS tile a
        //      quarter (32 channels = one operand step) at a time; lane <-> (channel lane%32, token half lane/32)
        float mn[4] = {INFINITY, INFINITY, INFINITY, INFINITY}, mx[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        int bi[NTG];
        const int sc = lane & 31, sth = lane >> 5;
        if (a.idx_given) {   // searched beforehand (min-max metric)
#pragma unroll
            for (int j = 0; j < NTG; ++j) bi[j] = a.idx[pq0 + j * 16 + n];
        } else if (NTA > 1) {   // NTA tiles of the group per pass over the pattern table
#pragma unroll
            for (int j0 = 0; j0 < NTG; j0 += NTA) {
                float bv[NTA], x2[NTA];
                bool flag[NTA];
                int bj[NTA];
                assign_tiles_mfma<NTA>(reinterpret_cast<const uint4 (&)[NTA][4]>(xb[j0]), tb, lane, bj, bv, x2, flag);
#pragma unroll
                for (int j = 0; j < NTA; ++j) {
                    float bd;
                    resolve_flagged(xb[j0 + j], flag[j], reinterpret_cast<__half *>(rt), tb, lane, bj[j], bd);
                    bi[j0 + j] = bj[j];
                }
            }
        }
#pragma unroll
        for (int j = 0; j < NTG; ++j) {
            float r[32];
            if (NTA > 1 || a.idx_given)
                residuals(sh, Mg, xb[j], bi[j], r);
            else
                bi[j] = assign_residuals(sh, tb, Mg, xb[j], reinterpret_cast<__half *>(rt), r);
#pragma unroll
            for (int k = 0; k < 4; ++k) {   // channels 32k .. 32k+31
                float4 *dst = reinterpret_cast<float4 *>(rt + n * kWkStride + 8 * kb);
                dst[0] = make_float4(r[8 * k], r[8 * k + 1], r[8 * k + 2], r[8 * k + 3]);
                dst[1] = make_float4(r[8 * k + 4], r[8 * k + 5], r[8 * k + 6], r[8 * k + 7]);
                wave_lds_sync();
#pragma unroll
                for (int t = 0; t < 8; t += 2) {
                    const float v0 = rt[(8 * sth + t) * kWkStride + sc], v1 = rt[(8 * sth + t + 1) * kWkStride + sc];
                    mn[k] = fminf(fminf(mn[k], v0), v1);
                    mx[k] = fmaxf(fmaxf(mx[k], v0), v1);
                }
                wave_lds_sync();
            }
        }
        // ---- parameters of the group: the two token halves are combined, then lane (c, half) takes the channels
        //      32(2 half) + c and 32(2 half + 1) + c
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            mn[k] = fminf(mn[k], __shfl_xor(mn[k], 32));
            mx[k] = fmaxf(mx[k], __shfl_xor(mx[k], 32));
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const GroupParams gp = group_params(sth ? mn[2 + h] : mn[h], sth ? mx[2 + h] : mx[h], BITS);
            const int c = 32 * (2 * sth + h) + sc;
            pz[c] = gp.z16;
            pz[kD + c] = gp.s16;
            pinv[c] = gp.inv;
        }
        wave_lds_sync();
        if (lane < 32) {   // stored parameters: 16-byte pieces, zero points then scales
            const int arr = lane >> 4, piece = lane & 15;
            const uint4 v = *reinterpret_cast<const uint4 *>(pz + arr * kD + piece * 8);
            __half *dstp = (arr ? a.scale : a.zero) + (pq0 / G) * kD + piece * 8;
            *reinterpret_cast<uint4 *>(dstp) = v;
        }
        // ---- pass B: residuals again, codes, planes; the tile's registers then take the next group
        uint8_t *stg = reinterpret_cast<uint8_t *>(rt);
#pragma unroll
        for (int j = 0; j < NTG; ++j) {
            float r[32];
            residuals(sh, Mg, xb[j], bi[j], r);
            if (g + 4 < g_end) load_tile(a, ns, (g + 4) * G + j * 16, xb[j]);
            k_codes_to_staging<BITS>(r, pz, pinv, stg);
            if (kb == 0) stg[16 * 16 * BITS + n] = (uint8_t)bi[j];
            wave_lds_sync();
            k_store_staging<BITS>(a, pq0 + j * 16, stg);
            wave_lds_sync();   // the staging area is rewritten by the next tile
        }
    }
}

// 16x16 bit transpose across the 16 lanes of a row, on both 16-bit halves of x at once:
// on return bit t of a half in lane i is what bit i of that half was in lane t.
struct TransposeConst {
    uint32_t sh[4], keep[4];   // stage d = 8, 4, 2, 1: rotation of the partner's word, bits kept from the own word
};
__device__ __forceinline__ TransposeConst transpose_const(int n)
{
    TransposeConst c;
    const uint32_t m0[4] = {0x00ff00ffu, 0x0f0f0f0fu, 0x33333333u, 0x55555555u};   // positions with bit d clear
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int d = 8 >> s;
        const bool lo = (n & d) == 0;
        c.sh[s] = lo ? 32 - d : d;        // lo lanes take the partner's bits d places up, hi lanes d places down
        c.keep[s] = lo ? m0[s] : ~m0[s];
    }
    return c;
}
__device__ __forceinline__ uint32_t transpose16(uint32_t x, const TransposeConst &c)
{
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const uint32_t partner = (uint32_t)__shfl_xor((int)x, 8 >> s);
        const uint32_t rot = __builtin_amdgcn_alignbit(partner, partner, c.sh[s]);   // bits that cross a half are masked out
        x = (x & c.keep[s]) | (rot & ~c.keep[s]);
    }
    return x;
}

// V: workgroup = 256 threads, blocks of 64 tokens of one stream; wave w owns the 16-token unit w of the
// block.  NG = channel groups per token (kD / Gc).  NT = blocks taken together: the wave assigns its units of
// NT consecutive blocks in one pass over the pattern table (every table tile read from LDS serves all of
// them), then quantizes them one after the other.
template <int BITS, int NG, int NT>
__global__ __launch_bounds__(256) void quantize_v_kernel(QuantArgs a, int tiles_per_wg)
{
    constexpr int TT = 64, WPU = BITS / 2, BPG = 4 / NG;   // BPG = 32-channel blocks per group
    extern __shared__ __align__(16) unsigned char smem[];
    const TileShared sh = carve(smem, a.P, 0, 1);
    const int tid = threadIdx.x, ns = blockIdx.y;
    const int lane = tid & 63, wave = tid >> 6, n = lane & 15, kb = lane >> 4;
    const __half *Mg = a.patterns + (int64_t)a.sets.set_of(ns) * a.P * kD;
    take_sequence_entry(a, ns);
    const int n_tiles = a.nq / TT;
    const int tile0 = chunk_of_workgroup() * tiles_per_wg, tile1 = min(n_tiles, tile0 + tiles_per_wg);
    if (tile0 >= n_tiles) return;   // a ragged append: this sequence has fewer tiles than the launch was sized for
    uint4 xbs[NT][4];
#pragma unroll
    for (int j = 0; j < NT; ++j)   // a block past the workgroup's range repeats the last one; its result is not used
        load_tile(a, ns, min(tile0 + j, tile1 - 1) * TT + wave * 16, xbs[j]);

    stage_patterns(Mg, a.P, sh.tab, sh.nh, sh.red);
    const PatternTable tb = make_table(sh, Mg, a.P);
    const TransposeConst tc = transpose_const(n);
    unsigned char *wsc = sh.wsc + wave * kWaveScratch;

    // Contiguous stores of a finished unit (code words, parameters, indices) out of the wave's staging area.
    // They are issued at the start of the NEXT unit, after that unit's vectors have arrived and before the
    // loads for the one after are issued: the wait for those loads at the top of a round would otherwise also
    // wait for stores issued just before it (loads and stores retire through one in-order counter).
    int64_t pend_tok0 = -1;
    auto store_pending = [&]() {
        if (pend_tok0 < 0) return;
        const int64_t tok0 = pend_tok0;
        const uint32_t *stg = reinterpret_cast<const uint32_t *>(wsc + kWsCodes);
        if (BITS == 2)
            reinterpret_cast<uint2 *>(a.codes_v + tok0 * (kD * BITS / 8))[lane] = reinterpret_cast<const uint2 *>(stg)[lane];
        else
            reinterpret_cast<uint4 *>(a.codes_v + tok0 * (kD * BITS / 8))[lane] = reinterpret_cast<const uint4 *>(stg)[lane];
        if (lane < 4 * NG) {   // NG*32 bytes per array = 2*NG pieces of 16 bytes; scales first, then zero points
            const int arr = lane / (2 * NG), piece = lane % (2 * NG);
            const uint4 v = *reinterpret_cast<const uint4 *>(wsc + (arr ? kWsZero : kWsScale) + piece * 16);
            *reinterpret_cast<uint4 *>((arr ? a.zero : a.scale) + tok0 * NG + piece * 8) = v;
        }
        if (lane == 63) *reinterpret_cast<uint4 *>(a.idx + tok0) = *reinterpret_cast<const uint4 *>(wsc + kWsIdx);
        wave_lds_sync();   // the staging area is rewritten by the unit that follows
        pend_tok0 = -1;
    };

    for (int tile_base = tile0; tile_base < tile1; tile_base += NT) {
        int bis[NT];
        if (a.idx_given) {   // searched beforehand (min-max metric); a block past the range repeats the last one
#pragma unroll
            for (int j = 0; j < NT; ++j)
                bis[j] = a.idx[a.map.pos(ns, a.t0 + min(tile_base + j, tile1 - 1) * TT) + wave * 16 + n];
        } else {
            float bv[NT], x2[NT];
            bool flag[NT];
            assign_tiles_mfma<NT>(xbs, tb, lane, bis, bv, x2, flag);
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                float bd;
                resolve_flagged(xbs[j], flag[j], reinterpret_cast<__half *>(wsc + kWsRow), tb, lane, bis[j], bd);
            }
        }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int tile = tile_base + j;
        if (tile >= tile1) break;
        uint4 (&xb)[4] = xbs[j];
        float r[32];
        int bi = bis[j];
        store_pending();
        residuals(sh, Mg, xb, bi, r);
        if (a.v_rho > 0.f) {
            // adaptive threshold (Sec. 3.3): keep the pattern iff R_flat <= rho * R_raw, ranges over all d
            // channels of the token: lane-local over its 32 channels, then over the token's 4 lanes
            float rmn = fminf(r[0], r[1]), rmx = fmaxf(r[0], r[1]);
            half2_t xmn = __builtin_bit_cast(half2_t, xb[0].x), xmx = xmn;
#pragma unroll
            for (int e = 2; e < 32; e += 2) {
                rmn = fminf(fminf(rmn, r[e]), r[e + 1]);
                rmx = fmaxf(fmaxf(rmx, r[e]), r[e + 1]);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t w[4] = {xb[k].x, xb[k].y, xb[k].z, xb[k].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    xmn = __builtin_elementwise_min(xmn, __builtin_bit_cast(half2_t, w[i]));
                    xmx = __builtin_elementwise_max(xmx, __builtin_bit_cast(half2_t, w[i]));
                }
            }
            float x_lo = fminf((float)xmn[0], (float)xmn[1]), x_hi = fmaxf((float)xmx[0], (float)xmx[1]);
#pragma unroll
            for (int off = 16; off <= 32; off <<= 1) {
                rmn = fminf(rmn, __shfl_xor(rmn, off));
                rmx = fmaxf(rmx, __shfl_xor(rmx, off));
                x_lo = fminf(x_lo, __shfl_xor(x_lo, off));
                x_hi = fmaxf(x_hi, __shfl_xor(x_hi, off));
            }
            const bool keep = (rmx - rmn) <= a.v_rho * (x_hi - x_lo);
            if (!keep) {   // quantize the vector itself
                bi = PK_NO_PATTERN;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t w[4] = {xb[k].x, xb[k].y, xb[k].z, xb[k].w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const half2_t h = __builtin_bit_cast(half2_t, w[i]);
                        r[8 * k + 2 * i] = (float)h[0];
                        r[8 * k + 2 * i + 1] = (float)h[1];
                    }
                }
            }
        }
        if (tile + NT < tile1) load_tile(a, ns, (tile + NT) * TT + wave * 16, xb);   // else the registers keep this block

        // minimum / maximum per channel group: lane-local over its channels, then over the 4 lanes of the token
        float mn[NG], mx[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            mn[g] = INFINITY;
            mx[g] = -INFINITY;
#pragma unroll
            for (int e = 8 * BPG * g; e < 8 * BPG * (g + 1); e += 2) {
                mn[g] = fminf(fminf(mn[g], r[e]), r[e + 1]);
                mx[g] = fmaxf(fmaxf(mx[g], r[e]), r[e + 1]);
            }
#pragma unroll
            for (int off = 16; off <= 32; off <<= 1) {
                mn[g] = fminf(mn[g], __shfl_xor(mn[g], off));
                mx[g] = fmaxf(mx[g], __shfl_xor(mx[g], off));
            }
        }
        // lane kb works out the parameters of group kb % NG and stores them; the others fetch them
        float my_mn = mn[0], my_mx = mx[0];
#pragma unroll
        for (int g = 1; g < NG; ++g) {
            if ((kb & (NG - 1)) == g) {
                my_mn = mn[g];
                my_mx = mx[g];
            }
        }
        const GroupParams gp = group_params(my_mn, my_mx, BITS);
        if (kb < NG) {
            reinterpret_cast<uint16_t *>(wsc + kWsScale)[kb * 16 + n] = gp.s16;
            reinterpret_cast<uint16_t *>(wsc + kWsZero)[kb * 16 + n] = gp.z16;
        }
        if (kb == 0) wsc[kWsIdx + n] = (uint8_t)bi;
        float z[NG], inv[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            z[g] = NG == 1 ? gp.z : __shfl(gp.z, n + 16 * g);
            inv[g] = NG == 1 ? gp.inv : __shfl(gp.inv, n + 16 * g);
        }

        // block b = channels 32*(2b + i/8) + 8*kb + i%8, i < 16: codes -> planes -> transpose -> words, put in
        // memory order in the wave's staging area
        uint32_t *stg = reinterpret_cast<uint32_t *>(wsc + kWsCodes);
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            uint32_t cw[4] = {0u, 0u, 0u, 0u};   // codes of elements 4q .. 4q+3 in the bytes of cw[q]
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int e = 16 * b + i, g = (e / 8) / BPG;
                cw[i >> 2] = put_code(r[e] - z[g], inv[g], i & 3, cw[i >> 2]);
            }
            // channel of this lane after the transpose: i = n
            const int c = 32 * (2 * b + (n >> 3)) + 8 * kb + (n & 7);
            uint32_t *dst = stg + ((c & 15) * (kD / 16) + (c >> 4)) * WPU;
#pragma unroll
            for (int w = 0; w < WPU; ++w) {
                // t_p = (bits p of the 16 codes) << p; low half of x = plane 2w, high half = plane 2w+1
                const uint32_t t0 = (plane_byte_shifted(cw[2], cw[3], 2 * w) << 8) | plane_byte_shifted(cw[0], cw[1], 2 * w);
                const uint32_t t1 = (plane_byte_shifted(cw[2], cw[3], 2 * w + 1) << 8) | plane_byte_shifted(cw[0], cw[1], 2 * w + 1);
                const uint32_t x = (t0 >> (2 * w)) | (t1 << (15 - 2 * w));
                dst[w] = transpose16(x, tc);
            }
        }
        wave_lds_sync();
        pend_tok0 = a.map.pos(ns, a.t0 + tile * TT) + wave * 16;   // stored at the start of the next unit
      }
    }
    store_pending();
}

// ---------------------------------------------------------------------------
// Tail ring: place logical vectors [i0, i1) of an append into their ring slots.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void tail_copy_kernel(TailCopyArgs a)
{
    const int n = blockIdx.y, side = blockIdx.z;
    if (a.seq_table) {   // a ragged append: the ring state and the range of the stream's own sequence
        const int32_t *e = a.seq_table + (int64_t)(n / a.n_kv_heads) * kSeqEntry;
        a.ring_start = e[kSeqRingStart];
        a.n_ring = e[kSeqNRing];
        a.i0 = e[kSeqI0];
        a.i1 = e[kSeqI1];
    }
    const int64_t work = (int64_t)(a.i1 - a.i0) * kRowChunks;
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (w >= work) return;
    const int i = a.i0 + (int)(w >> 4), ch = (int)(w & 15);
    const __half *fresh = side == 0 ? a.fresh_k : a.fresh_v;
    __half *ring = side == 0 ? a.ring_k : a.ring_v;
    const uint4 v = *reinterpret_cast<const uint4 *>(fresh + (int64_t)n * a.fresh_stride +
                                                     (int64_t)(i - a.n_ring) * kD + ch * 8);
    const int slot = (int)(((int64_t)a.ring_start + i) % a.ring_len);
    *reinterpret_cast<uint4 *>(ring + ((int64_t)n * a.ring_len + slot) * kD + ch * 8) = v;
}

__global__ __launch_bounds__(kSeqChunk * kSeqEntry) void seq_table_kernel(SeqTableArgs a)
{
    const int i = threadIdx.x / kSeqEntry, f = threadIdx.x % kSeqEntry;
    if (i >= a.count) return;
    a.table[(int64_t)(a.first + i) * kSeqEntry + f] = a.entry[i][f];
    if (a.states_out && f < 4) a.states_out[(int64_t)(a.first + i) * 4 + f] = f < 3 ? a.state[i][f] : 0;
}

}  // namespace

hipError_t launch_seq_table(const SeqTableArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL(seq_table_kernel, dim3(1), dim3(kSeqChunk * kSeqEntry), 0, s, a);
    return hipGetLastError();
}

static int tiles_per_wg(int n_tiles, int n_streams)
{
    // aim at ~1024 workgroups, each staging the pattern table once for at most 16 tiles; a job of very many
    // tiles (8 or more resident rounds even then) takes 32 or 64 per workgroup: fewer prologues, and the last,
    // partly filled round stays a small share (-4 % on the V kernel of config 3, worse on small jobs)
    const int64_t total = (int64_t)n_tiles * n_streams;
    const int cap = total >= 64 * 768 * 8 ? 64 : total >= 32 * 768 * 8 ? 32 : 16;
    const int t = (int)((total + 1023) / 1024);
    return t < 1 ? 1 : (t > cap ? cap : t);
}

template <auto KERNEL, int THREADS = 256>
static hipError_t launch_tiled(const QuantArgs &a, int TT, size_t lds, size_t max_lds, hipStream_t s, int min_tiles = 1)
{
    static LdsOptIn opt_in;   // per kernel instantiation; max_lds: what it needs with a table of 256 patterns
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(KERNEL), opt_in, max_lds);
    if (e != hipSuccess) return e;
    int tpw = tiles_per_wg(a.nq / TT, a.n_streams);
    if (tpw < min_tiles) tpw = min_tiles;
    const int n_tiles = a.nq / TT;
    hipLaunchKernelGGL(KERNEL, dim3((n_tiles + tpw - 1) / tpw, a.n_streams), dim3(THREADS), lds, s, a, tpw);
    return hipGetLastError();
}

// Min-max metric: the search kernel fills the index array, the quantizers then take the indices from there.
static hipError_t launch_assign_minmax(const QuantArgs &a, hipStream_t s)
{
    const int n_tiles = a.nq / 64;
    int tpw = tiles_per_wg(n_tiles, a.n_streams);
    if (tpw < 4) tpw = 4;   // four waves, a 64-vector tile each per round
    hipLaunchKernelGGL(assign_minmax_kernel, dim3((n_tiles + tpw - 1) / tpw, a.n_streams), dim3(256), 0, s, a, tpw);
    return hipGetLastError();
}

hipError_t launch_quantize_k(const QuantArgs &a_in, hipStream_t s)
{
    if (a_in.d != kD) return launch_generic_quantize(a_in, false, s);
    QuantArgs a = a_in;
    if (a.metric == PK_METRIC_MINMAX) {
        const hipError_t e = launch_assign_minmax(a, s);
        if (e != hipSuccess) return e;
        a.idx_given = 1;
    }
    {
        // (the pattern table, at most 256 rows = 74 KB, lives in LDS)
        // Tiles of a group assigned per pass over the pattern table (every table tile read from LDS serves all of
        // them): pairs keep three waves per SIMD; the whole 64-token group takes two, which pays above 128
        // patterns; 32-token groups gain from pairs only once the table is large.
        const int kmulti = a.G == 64 ? (a.P > 128 ? 4 : 2) : (a.P >= 128 ? 2 : 1);
        // group 128 with a large table: one workgroup fills a CU's LDS and stages 64 KB of patterns, so a small
        // job is cut into one resident round (256 workgroups) rather than many short ones
        const int64_t tiles64k = (int64_t)(a.nq / 64) * a.n_streams;   // the same for the group-64 wave kernel above 128 patterns (one workgroup per CU)
        const int bigw = a.P > 128 && tiles64k <= 256 * 64 ? (int)((tiles64k + 255) / 256) : 1;
        const int64_t tiles128 = (int64_t)(a.nq / 128) * a.n_streams;
        const int big1 = a.P > 128 && tiles128 <= 256 * 64 ? (int)((tiles128 + 255) / 256) : 1;
#define PK_LAUNCH_K2(GG, BB)                                                                                       \
    if (a.G == GG && a.bits == BB) {                                                                               \
        constexpr int TT = GG == 128 ? 128 : 64;                                                                   \
        return launch_tiled<quantize_k_kernel<GG, BB, 8>, 512>(a, TT, tile_lds_bytes(a.P, TT, GG), tile_lds_bytes(256, TT, GG), s, big1); \
    }
#define PK_LAUNCH_KW(GG, BB)                                                                                       \
    if (a.G == GG && a.bits == BB) {                                                                               \
        /* a wave owns whole groups: at least four groups per workgroup */                                        \
        const size_t lds = wave_k_lds_bytes(a.P), mx = wave_k_lds_bytes(256);                                      \
        return kmulti == 4 && GG == 64 ? launch_tiled<quantize_k_wave_kernel<GG, BB, GG / 16>>(a, 64, lds, mx, s, bigw > GG / 16 ? bigw : GG / 16) \
               : kmulti >= 2 ? launch_tiled<quantize_k_wave_kernel<GG, BB, 2>>(a, 64, lds, mx, s, GG / 16)         \
                             : launch_tiled<quantize_k_wave_kernel<GG, BB, 1>>(a, 64, lds, mx, s, GG / 16);        \
    }
        PK_LAUNCH_KW(32, 2) PK_LAUNCH_KW(64, 2) PK_LAUNCH_K2(128, 2)
        PK_LAUNCH_KW(32, 4) PK_LAUNCH_KW(64, 4) PK_LAUNCH_K2(128, 4)
#undef PK_LAUNCH_KW
#undef PK_LAUNCH_K2
        return hipErrorInvalidValue;
    }
}

hipError_t launch_quantize_v(const QuantArgs &a_in, hipStream_t s)
{
    if (a_in.d != kD) return launch_generic_quantize(a_in, true, s);
    QuantArgs a = a_in;
    if (a.metric == PK_METRIC_MINMAX) {
        const hipError_t e = launch_assign_minmax(a, s);
        if (e != hipSuccess) return e;
        a.idx_given = 1;
    }
    {
        const int ng = kD / (a.G < kD ? a.G : kD);
        const size_t lds = tile_lds_bytes(a.P, 0, 1), mx = tile_lds_bytes(256, 0, 1);
        const bool two = a.P >= 128;   // two blocks per table pass (three waves per SIMD instead of four) pay from 128 patterns on
        // a large table (two workgroups per CU, 64 KB of patterns staged by each): a small job as one resident round
        const int64_t tiles64 = (int64_t)(a.nq / 64) * a.n_streams;
        const int big1 = a.P > 128 && tiles64 <= 512 * 64 ? (int)((tiles64 + 511) / 512) : 1;
#define PK_LAUNCH_V2(BB, NN)                                                                   \
    if (a.bits == BB && ng == NN)                                                              \
        return two ? launch_tiled<quantize_v_kernel<BB, NN, 2>>(a, 64, lds, mx, s, big1)       \
                   : launch_tiled<quantize_v_kernel<BB, NN, 1>>(a, 64, lds, mx, s);
        PK_LAUNCH_V2(2, 1) PK_LAUNCH_V2(2, 2) PK_LAUNCH_V2(2, 4)
        PK_LAUNCH_V2(4, 1) PK_LAUNCH_V2(4, 2) PK_LAUNCH_V2(4, 4)
#undef PK_LAUNCH_V2
        return hipErrorInvalidValue;
    }
}

hipError_t launch_tail_copy(const TailCopyArgs &a, hipStream_t s)
{
    if (a.d != kD) return launch_generic_tail_copy(a, s);
    const int64_t work = (int64_t)(a.i1 - a.i0) * kRowChunks;
    if (work <= 0) return hipSuccess;
    const dim3 grid((unsigned)((work + 255) / 256), a.n_streams, 2), block(256);
    hipLaunchKernelGGL(tail_copy_kernel, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace pk
