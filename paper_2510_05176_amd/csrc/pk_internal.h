// Internal declarations shared by the HIP translation units of libpatternkv.
// Not part of the public ABI (that is include/patternkv.h).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "patternkv.h"

namespace pk {

constexpr int kD = 128;          // head_dim supported by the kernels
constexpr int kRowChunks = 16;   // 16-byte chunks per fp16 row of kD elements

// Where the logical vectors of an append come from: first the old fp16 tail
// (a ring), then the freshly passed vectors.
struct RowSource {
    const __half *ring;        // [N][ring_len][kD]
    const __half *fresh;       // stream n at fresh + n*fresh_stride
    int64_t fresh_stride;      // elements
    int32_t ring_len;
    int32_t ring_start;        // slot of logical vector 0
    int32_t n_ring;            // logical vectors [0, n_ring) live in the ring

    __device__ __forceinline__ const __half *row(int n, int i) const
    {
        if (i < n_ring) {
            int slot = ring_start + i;
            if (slot >= ring_len) slot -= ring_len;
            return ring + ((int64_t)n * ring_len + slot) * kD;
        }
        return fresh + (int64_t)n * fresh_stride + (int64_t)(i - n_ring) * kD;
    }
    // the same for rows of d elements (the generic kernels for head dimensions other than kD)
    __device__ __forceinline__ const __half *row_d(int n, int i, int d) const
    {
        if (i < n_ring) {
            int slot = ring_start + i;
            if (slot >= ring_len) slot -= ring_len;
            return ring + ((int64_t)n * ring_len + slot) * d;
        }
        return fresh + (int64_t)n * fresh_stride + (int64_t)(i - n_ring) * d;
    }
};

// Where token `tok` of stream `stream` lives in the packed arrays, in tokens: stream * capacity + tok for contiguous
// streams; through the sequence's page table for a paged cache (a page = [n_kv_heads][page_tokens] tokens).  A table
// entry is clamped to the pool, so whatever the table holds the position stays inside the arrays.  Quantization
// groups, 64-token blocks and tiles never straddle a page (page_tokens is a power of two >= 128), so a kernel asks
// for the position of a tile's first token and adds offsets inside the tile.
struct PackedMap {
    const int32_t *page_table;   // device [n_seq][pages_per_seq], or null
    int32_t page_shift;          // log2(page_tokens)
    int32_t pages_per_seq, n_pages, n_kv_heads, t_capacity;
    // physical page of the stream's token (clamped to the pool); 0 for contiguous streams
    __device__ __forceinline__ int page_of(int stream, int tok) const
    {
        if (!page_table) return 0;
        const int page = page_table[(int64_t)(stream / n_kv_heads) * pages_per_seq + min(tok >> page_shift, pages_per_seq - 1)];
        return min(max(page, 0), n_pages - 1);
    }
    // position of the token given its page (as page_of returns it)
    __device__ __forceinline__ int64_t pos_in(int page, int stream, int tok) const
    {
        if (!page_table) return (int64_t)stream * t_capacity + tok;
        const int head = stream % n_kv_heads;
        return (((int64_t)page * n_kv_heads + head) << page_shift) + (tok & ((1 << page_shift) - 1));
    }
    __device__ __forceinline__ int64_t pos(int stream, int tok) const { return pos_in(page_of(stream, tok), stream, tok); }
};

struct SetMap {
    int32_t n_kv_heads;
    int32_t seqs_per_set;
    __host__ __device__ __forceinline__ int set_of(int stream) const
    {
        const int seq = stream / n_kv_heads, head = stream - seq * n_kv_heads;
        return (seqs_per_set == 0 ? 0 : seq / seqs_per_set) * n_kv_heads + head;
    }
};

// ---- fp16 helpers -----------------------------------------------------------

__device__ __forceinline__ float h2f(__half h) { return __half2float(h); }
__device__ __forceinline__ float hbits2f(unsigned short u) { return __half2float(__ushort_as_half(u)); }

// Differences with one rounding, as the binary32 subtraction of the widened values: v_fma_mix_f32
// computes a*1.0 + (-b) with fp16 sources widened exactly.
__device__ __forceinline__ float sub_lo(uint32_t x, uint32_t m)   // half(x.lo) - half(m.lo)
{
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,0] op_sel_hi:[1,0,1]" : "=v"(r) : "v"(x), "v"(m));
    return r;
}
__device__ __forceinline__ float sub_hi(uint32_t x, uint32_t m)   // half(x.hi) - half(m.hi)
{
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[1,0,1] op_sel_hi:[1,0,1]" : "=v"(r) : "v"(x), "v"(m));
    return r;
}
// largest binary16 value <= f
__device__ __forceinline__ unsigned short f2h_down(float f)
{
    unsigned short u = __half_as_ushort(__float2half_rn(f));
    if (hbits2f(u) > f) {
        if ((u & 0x7fffu) == 0) u = 0x8001u;   // +-0 -> smallest negative subnormal
        else if (u & 0x8000u) u += 1;          // negative: one step away from zero
        else u -= 1;                           // positive: one step towards zero
    }
    return u;
}

// smallest binary16 value >= f
__device__ __forceinline__ unsigned short f2h_up(float f)
{
    unsigned short u = __half_as_ushort(__float2half_rn(f));
    if (hbits2f(u) < f) {
        if ((u & 0x7fffu) == 0) u = 0x0001u;
        else if (u & 0x8000u) u -= 1;
        else u += 1;
    }
    return u;
}

// ---- launchers (host) -------------------------------------------------------

// A kernel that uses more than 64 KB of dynamic LDS has to be allowed to, per function and device.  This is done
// once per kernel instantiation and device, with the most that instantiation can ever be launched with, so
// that concurrent calls with different sizes cannot lower each other's limit and a launch costs no extra
// runtime call.
struct LdsOptIn {
    std::mutex m;
    uint64_t devices_done = 0;
};
inline hipError_t allow_dynamic_lds(const void *kernel, LdsOptIn &st, size_t max_bytes)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(st.m);
    if (dev < 64 && ((st.devices_done >> dev) & 1u)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_bytes);
    if (e == hipSuccess && dev < 64) st.devices_done |= 1ull << dev;
    return e;
}

struct QuantArgs {
    RowSource src;
    SetMap sets;
    const __half *patterns;   // [n_sets][P][kD]
    int32_t P, metric, bits, G;
    int32_t d;                // head dimension: kD runs the tuned kernels, 96 and 256 the generic ones (pk_generic.hip)
    int32_t idx_given;        // the index array already holds every vector's pattern (min-max metric: searched by a kernel of its own)
    float v_rho;              // V side: adaptive threshold (0 = off)
    int32_t n_streams;
    int32_t nq;               // vectors to quantize per stream (multiple of G)
    int32_t t0;               // first packed position to write (= t_quant)
    PackedMap map;            // where the packed tokens of a stream live
    uint32_t *codes_k;        // K side
    uint8_t *codes_v;         // V side
    __half *scale, *zero;
    uint8_t *idx;
    // A ragged append: per-sequence fill parameters, [n_seq][kSeqEntry] int32 in device memory (written by
    // seq_table_kernel from the host's plan): vectors to quantize, first packed position, ring start, vectors in
    // the ring, first and end logical vector of the tail copy.  nq above is then the largest of the batch (launch
    // sizing only).  Null for a uniform append.
    const int32_t *seq_table;
};
constexpr int kSeqEntry = 8;                                   // int32 per sequence in the table
enum { kSeqNq = 0, kSeqT0 = 1, kSeqRingStart = 2, kSeqNRing = 3, kSeqI0 = 4, kSeqI1 = 5 };

// The fill parameters of the workgroup's own sequence replace the uniform ones (wave-uniform loads).
__device__ __forceinline__ void take_sequence_entry(QuantArgs &a, int stream)
{
    if (a.seq_table) {
        const int32_t *e = a.seq_table + (int64_t)(stream / a.sets.n_kv_heads) * kSeqEntry;
        a.nq = e[kSeqNq];
        a.t0 = e[kSeqT0];
        a.src.ring_start = e[kSeqRingStart];
        a.src.n_ring = e[kSeqNRing];
    }
}

hipError_t launch_quantize_k(const QuantArgs &a, hipStream_t s);
hipError_t launch_quantize_v(const QuantArgs &a, hipStream_t s);

struct TailCopyArgs {
    const __half *fresh_k, *fresh_v;
    int64_t fresh_stride;
    __half *ring_k, *ring_v;
    int32_t ring_len, ring_start, n_ring;   // as in RowSource (state before the append)
    int32_t i0, i1;                          // logical vectors [i0, i1) to place into the ring
    int32_t n_streams;
    int32_t n_kv_heads;
    int32_t d;                               // head dimension
    const int32_t *seq_table;                // ragged append: as in QuantArgs (i0, i1 above: the widest range)
};
// Writes up to kSeqChunk entries of the per-sequence table, and (optionally) the fill states after the append in
// the form the ragged decode reads, from values that travel in the kernel arguments: no host buffer has to outlive
// the call and nothing is copied from pageable memory.
constexpr int kSeqChunk = 64;
struct SeqTableArgs {
    int32_t *table;          // [n_seq][kSeqEntry]
    int32_t *states_out;     // [n_seq][4] or null: t_quant, t_tail, tail_start, 0 after the append
    int32_t first, count;
    int32_t entry[kSeqChunk][kSeqEntry];
    int32_t state[kSeqChunk][3];
};
hipError_t launch_seq_table(const SeqTableArgs &a, hipStream_t s);
hipError_t launch_tail_copy(const TailCopyArgs &a, hipStream_t s);

struct MineArgs {
    const __half *x;
    int64_t set_stride;
    int32_t n_sets, T, P, iters, init_given;
    int32_t d;             // head dimension
    __half *patterns;
    int32_t *assign_ws;    // [n_sets][T] workspace (the generic path keeps every step's assignment there)
    int32_t *assign;       // [n_sets][T] caller's, or null
    float *best;           // [n_sets][T] workspace (written when inertia is asked for)
    float *psum;           // [n_sets][tsplit][P][kD]
    int32_t *pcnt;         // [n_sets][tsplit][P]
    float *inertia;        // optional [n_sets][iters]
    int32_t tsplit;
};
hipError_t launch_mine(const MineArgs &a, hipStream_t s);
int mine_tsplit(int T, int n_sets, int P);
hipError_t launch_window_pattern(const __half *x, int64_t set_stride, int n_sets, int n, __half *out, int64_t out_stride,
                                 hipStream_t s);

// Head dimensions other than kD (pk_generic.hip): plain kernels, thread <-> channel, same results to the same bars.
hipError_t launch_generic_quantize(const QuantArgs &a, bool v_side, hipStream_t s);
hipError_t launch_generic_tail_copy(const TailCopyArgs &a, hipStream_t s);
hipError_t launch_generic_mine(const MineArgs &a, hipStream_t s);
hipError_t launch_generic_window_pattern(const __half *x, int64_t set_stride, int n_sets, int n, int d, __half *out,
                                         int64_t out_stride, hipStream_t s);

struct CacheView {
    const uint32_t *k_codes;
    const __half *k_scale, *k_zero;
    const uint8_t *k_idx;
    const uint8_t *v_codes;
    const __half *v_scale, *v_zero;
    const uint8_t *v_idx;
    const __half *tail_k, *tail_v;
    int32_t t_capacity, t_quant, t_tail, tail_start, ring_len;
    PackedMap map;
};

struct DecodeArgs {
    CacheView own, prefix;        // prefix.t_quant == prefix.t_tail == 0 when unused
    SetMap sets;
    const __half *q;              // [n_seq][Hq][kD]
    const __half *patterns_k, *patterns_v;
    int32_t n_seq, n_kv_heads, n_q_heads, P, bits, G;
    int32_t d;                    // head dimension
    int32_t v_thresholded;        // v_idx may hold PK_NO_PATTERN (read by the generic decode; the tuned one needs no flag)
    float softmax_scale;
    int32_t chunk;                // packed tokens per split
    int32_t w_stride;             // entries per (wave, head) row of the per-pattern softmax mass in LDS: P, or 256
                                  // when v_idx may hold PK_NO_PATTERN
    int32_t splits_prefix, splits_own;   // packed splits; two more slots hold the tails
    int32_t head_groups;          // the matrix-core kernel takes the r query heads of a KV head in this many groups of
                                  // r / head_groups heads, a workgroup row per (stream, group): 1, or 2 when the
                                  // (head, V channel group) pairs of all r heads exceed a tile's 16 columns or r > 8
    float *part_o;                // [N][S][r][kD]  unnormalised partial outputs
    float *part_w;                // [N][S][r][P]   softmax mass per V pattern (packed splits only)
    float *part_ml;               // [N][S][r][2]   running maximum (log2 domain) and sum
    float *out, *lse;
    const int32_t *seq_order;     // optional, device [n_seq]: sequences from the longest packed part to the shortest (a
                                  // ragged batch of at most kMaxOrdered sequences: the packed kernel takes its
                                  // streams in this order, so that the long ones start first)
    const int32_t *seq_state;     // optional, device [n_seq][4]: t_quant, t_tail, tail_start, 0 of every sequence's own
                                  // cache; own.t_quant / own.t_tail are then upper bounds
};
// Fill state of sequence seq's own cache: the uniform one, or the sequence's entry clamped to the bounds the
// launch was sized for (t_quant to whole 64-token blocks), so that a bad entry cannot lead outside the cache.
__device__ __forceinline__ void own_state(const DecodeArgs &a, int seq, int &t_quant, int &t_tail, int &tail_start)
{
    t_quant = a.own.t_quant;
    t_tail = a.own.t_tail;
    tail_start = a.own.tail_start;
    if (a.seq_state) {
        const int4 v = *reinterpret_cast<const int4 *>(a.seq_state + 4 * seq);
        t_quant = min(max(v.x, 0), a.own.t_quant) & ~63;
        t_tail = min(max(v.y, 0), a.own.t_tail);
        tail_start = min(max(v.z, 0), a.own.ring_len - 1);
    }
}
constexpr int kMaxOrdered = 1024;   // sequences a single workgroup ranks by counting
hipError_t launch_decode(const DecodeArgs &a, hipStream_t s);
// Whether the workgroups of the fp16 tails are part of the packed kernel's launch (rows of its grid behind the
// streams) instead of a kernel of their own.  They then run at that kernel's occupancy (two workgroups per CU),
// which suits a few hundred tails that fill slots the packed splits leave idle (config 4: -7 % per step) and does
// not suit thousands of them (config 3, 4096 tails: +8 % on the whole decode; the tail code hides its load
// latency by occupancy, eight workgroups per CU when launched alone).
inline bool decode_tails_ride_along(const DecodeArgs &a)
{
    const int n_tail = a.n_seq * a.n_kv_heads * a.head_groups * (a.prefix.t_tail > 0 ? 2 : 1);
    return a.splits_prefix + a.splits_own > 0 && (a.own.t_tail > 0 || a.prefix.t_tail > 0) && n_tail <= 1024;
}
int decode_chunk(int64_t n_streams, int64_t t_packed_total, int P, int r);
constexpr int kMaxSlots = 2304;   // partial slots per stream the merge kernel holds weights for (splits + 2)

struct DequantArgs {
    CacheView c;
    SetMap sets;
    const __half *patterns_k, *patterns_v;
    int32_t n_streams, P, bits, G, t0, t1;
    int32_t d;                // head dimension
    int32_t v_thresholded;    // v_idx == PK_NO_PATTERN marks a token quantized without a pattern
    float *k_out, *v_out;
};
hipError_t launch_dequant(const DequantArgs &a, hipStream_t s);
hipError_t launch_generic_decode(const DecodeArgs &a, hipStream_t s);
hipError_t launch_generic_dequant(const DequantArgs &a, hipStream_t s);

}  // namespace pk
