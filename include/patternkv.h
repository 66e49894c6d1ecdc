/*
 * patternkv.h -- C ABI of the PatternKV hot path for AMD MI355X (gfx950).
 *
 * PatternKV (arXiv 2510.05176) mines a few pattern vectors per attention head,
 * aligns every K/V vector to its nearest pattern and quantizes only the
 * residual (Sec. 3).  This library is the data-parallel part of that method:
 *
 *   pk_mine_patterns      Sec. 3.1 "Prefilling Stage", Eq. 4  (K-means / Lloyd)
 *   pk_quantize_append    Sec. 3.2 Eq. 6 (pattern selection, residual) followed
 *                         by Sec. 2.1 Eq. 1 (asymmetric n-bit quantization), with
 *                         K quantized per channel and V per token (Sec. 4.1)
 *   pk_decode_attention   Sec. 3.4 "Decode-stage KV reconstruction": attention
 *                         computed directly on the packed cache
 *   pk_decode_attention_ragged  the same over sequences filled to different lengths
 *   pk_decode_attention_noalloc the same with the partial results in a fixed array of the library
 *   pk_window_pattern     Sec. 3.1 "Decoding Stage", Eq. 5: the pattern of a window of
 *                         vectors (per-channel Chebyshev centre)
 *   pk_dequantize         the reconstruction rule below Eq. 6 (debug / parity)
 *
 * Conventions shared by every call
 *   - All tensor pointers are DEVICE pointers unless marked "host".  Structs
 *     (pk_config, pk_cache, pk_state, pk_layout) are HOST memory.
 *   - Tensors are dense, row-major, last index fastest; fp16 = IEEE binary16.
 *   - The caller owns every byte, including the workspace.  The library never
 *     allocates or frees device memory, keeps no global state and retains no
 *     pointer after a call returns.  (One exception, by design:
 *     pk_decode_attention_noalloc uses a fixed scratch array of the library.)
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and return without synchronising.  pk_state is updated on
 *     the host at enqueue time.
 *   - Every argument, shape, alignment (16 bytes for all device pointers),
 *     capacity and state error is detected on the host before anything is
 *     launched; the call then returns a status other than PK_OK and leaves
 *     pk_state and device memory untouched.  A launch the HIP runtime refuses
 *     gives PK_ERR_DEVICE: pk_state is unchanged then as well, but kernels
 *     launched earlier by the same call may already have written device memory
 *     (an append launches the K quantizer, the V quantizer and the tail copy in
 *     turn; what they wrote lies behind t_quant / outside the tail range that
 *     pk_state describes, so repeating the call overwrites it).  Nothing is
 *     printed, thrown or aborted.
 *   - Calls are re-entrant; calls that touch different caches on different
 *     streams may run concurrently.
 *
 * Streams and pattern sets
 *   A "stream" is the K (or V) history of one (sequence, KV head) pair; there
 *   are N = n_seq * n_kv_heads of them, stream index n = seq * n_kv_heads + head,
 *   all of the same length.  `n_seq` may flatten layers and batch.  A pattern
 *   table holds n_patterns vectors per pattern set; stream (seq, head) uses set
 *       (seqs_per_set == 0 ? 0 : seq / seqs_per_set) * n_kv_heads + head.
 *   seqs_per_set = 0 shares one table per KV head among all sequences (the
 *   paper's memory formula of App. H has no batch factor); seqs_per_set = batch
 *   gives one table per (layer, head) when n_seq = layers * batch.
 *
 * Packed cache format (the paper fixes none; d = head_dim, b = bits, G = group)
 *   k_codes [N][t_capacity][d/32][b] uint32   bit i of word (w,j) of token t is
 *                                             bit j of the code of channel 32w+i
 *   k_scale, k_zero [N][t_capacity/G][d] fp16 one (s,z) per channel and group of
 *                                             G consecutive tokens
 *   k_idx   [N][t_capacity] uint8             pattern index k* of every token
 *   v_codes [N][t_capacity*d*b/32] uint32     the bit planes of V run along the tokens:
 *                                             tokens in blocks of 64 = 4 units of 16; bit
 *                                             (16*(j%2) + t%16) of word
 *       (((t/64)*4 + (t%64)/16)*16 + c%16) * (d/16)*(b/2) + (c/16)*(b/2) + j/2
 *                                             is bit j of the code of channel c of token t
 *   v_scale, v_zero [N][t_capacity/16][d/Gc][16] fp16   Gc = min(G, d): one (s,z) per token
 *                                             and group of Gc channels, stored in slices of
 *                                             16 tokens
 *   v_idx   [N][t_capacity] uint8
 *   tail_k, tail_v [N][recent+flush][d] fp16  ring buffer of the most recent
 *                                             vectors, kept in full precision;
 *                                             logical tail token i is in slot
 *                                             (tail_start + i) % (recent+flush)
 * Paged cache (page_tokens > 0; the paper fixes no memory layout, serving engines allocate KV memory in pages)
 *   The packed arrays hold n_pages pages instead of N contiguous streams.  A page holds page_tokens consecutive
 *   tokens of ALL KV heads of one sequence, head after head; inside a (page, head) part every array is laid out
 *   exactly as a contiguous stream of page_tokens tokens above (so a page is [n_kv_heads][page_tokens] tokens and
 *   token t of stream (seq, head) lives at packed position
 *       (page_table[seq][t / page_tokens] * n_kv_heads + head) * page_tokens + t % page_tokens
 *   in units of tokens of the array concerned: k_codes [pos][d/32][b], k_scale [pos/G][d], k_idx [pos], v_codes in
 *   64-token blocks from pos, v_scale [pos/16][d/Gc][16], v_idx [pos]).  page_table is DEVICE int32
 *   [n_seq][t_capacity / page_tokens]; the kernels clamp every entry they read to [0, n_pages), so no table
 *   content can lead outside the arrays; entries of pages a sequence does not yet use are never read; giving two
 *   logical pages the same physical page is the caller's error (the later write wins).  The fp16 tails are not
 *   paged.  Quantization groups, 64-token blocks and flushes never straddle a page.
 *   Stored parameters: z = min of the residual group rounded to fp16 towards
 *   -inf; s = (max - z)/(2^b - 1) rounded to fp16 towards +inf; code =
 *   clamp(rint((r - z) * (1/s)), 0, 2^b - 1) in binary32, ties to even; a group
 *   with s == 0 has all codes 0.  Reconstruction: M[k*] + (s*code + z).
 */
#ifndef PATTERNKV_H
#define PATTERNKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PK_ABI_VERSION 5u

typedef enum {
    PK_OK = 0,
    PK_ERR_INVALID_ARG = 1, /* NULL where a pointer is required, negative size, bad enum        */
    PK_ERR_UNSUPPORTED = 2, /* head_dim / bits / group / GQA ratio outside the supported set    */
    PK_ERR_SHAPE = 3,       /* sizes inconsistent with each other (T < n_patterns, ...)         */
    PK_ERR_ALIGNMENT = 4,   /* a device pointer is not 16-byte aligned                          */
    PK_ERR_CAPACITY = 5,    /* the append would exceed t_capacity                               */
    PK_ERR_STATE = 6,       /* pk_state is not one this library could have produced             */
    PK_ERR_WORKSPACE = 7,   /* workspace missing or smaller than pk_workspace_bytes             */
    PK_ERR_DEVICE = 8       /* the HIP runtime refused a launch                                 */
} pk_status;

/* Pattern-selection metric.  L2 is the metric of the mining objective (Sec. 3.1
 * Eq. 4); MINMAX is d_mm(x,m) = max_i(x_i-m_i) - min_j(x_j-m_j) of Sec. 3.2.
 * Ties go to the lowest pattern index. */
typedef enum { PK_METRIC_L2 = 0, PK_METRIC_MINMAX = 1 } pk_metric;

typedef enum { PK_OP_MINE = 0, PK_OP_APPEND = 1, PK_OP_DECODE = 2 } pk_op;

typedef struct {
    int32_t n_seq;        /* sequences (layers x batch flattened), >= 1                       */
    int32_t n_kv_heads;   /* >= 1                                                             */
    int32_t n_q_heads;    /* multiple of n_kv_heads; r = n_q_heads/n_kv_heads in 1..64 (at d = 128 the matrix-core
                             decode kernel takes r <= 8 and even r up to 16, with G = 32 r = 1..4, 6 or 8; other head
                             counts decode through the plain kernels)                            */
    int32_t head_dim;     /* d: 128 (the tuned kernels), or 96 / 256 (the other head sizes of Sec. 3.3: plain
                             vector-ALU kernels; every call takes them).  min(G, d)
                             must divide d (d = 96: G = 32 or 128)                                  */
    int32_t n_patterns;   /* P: 1..256 (indices are stored in one byte)                       */
    int32_t seqs_per_set; /* see "Streams and pattern sets" above; >= 0                       */
    int32_t bits;         /* b: 2 or 4                                                        */
    int32_t group;        /* G: 32, 64 or 128                                                 */
    int32_t recent;       /* R >= 0: vectors always kept in fp16                              */
    int32_t flush;        /* F: multiple of G and of 64 (V codes and parameters are stored in
                             blocks of 64 tokens, so G = 32 with F = 32 is refused); vectors
                             quantized per flush                                              */
    int32_t t_capacity;   /* maximum packed tokens per stream, multiple of F, at most 2^25    */
    int32_t metric;       /* pk_metric                                                        */
    float v_rho;          /* adaptive threshold on V (Sec. 3.3, "Adaptive Threshold for V"): 0 = off.  With
                             0 < v_rho < 1 a V vector keeps its pattern only if
                             R_flat <= v_rho * R_raw, R = max - min over its d channels of the residual
                             (flat) and of the vector itself (raw), one binary32 multiply; otherwise the
                             vector itself is quantized and its index is PK_NO_PATTERN.  The caller passes
                             rho_*(d, alpha), the root in (0,1) of 1 - rho^2 = 2 z_{1-alpha}/sqrt(5d) *
                             sqrt(1 + rho^4).  Needs n_patterns <= 255.  K is never thresholded.        */
    int32_t page_tokens;  /* 0: every stream's packed part is contiguous (the layout above).  Otherwise the
                             packed arrays are a pool of pages, see "Paged cache" below: tokens per page, a
                             power of two >= 128 that divides t_capacity                              */
    int32_t n_pages;      /* pages in the pool (page_tokens > 0), >= 1                               */
} pk_config;

#define PK_NO_PATTERN 255 /* v_idx of a token quantized without a pattern (only when v_rho > 0)    */

/* Byte sizes of the cache arrays for a configuration (for the caller to allocate). */
typedef struct {
    uint64_t k_codes, k_scale, k_zero, k_idx;
    uint64_t v_codes, v_scale, v_zero, v_idx;
    uint64_t tail_k, tail_v;
    uint64_t total; /* sum of the above, each rounded up to `align`                           */
    uint32_t align; /* required alignment of every array (16)                                 */
} pk_layout;

/* Device pointers of one cache, each of at least the size pk_cache_layout reports. */
typedef struct {
    void *k_codes, *k_scale, *k_zero, *k_idx;
    void *v_codes, *v_scale, *v_zero, *v_idx;
    void *tail_k, *tail_v;
    const int32_t *page_table; /* device; required when page_tokens > 0, ignored otherwise          */
} pk_cache;

/* Host-side bookkeeping of a cache (all streams have the same lengths).  Start
 * from all zeros.  Invariants: t_quant is a multiple of flush, t_quant <=
 * t_capacity, 0 <= t_tail < recent + flush, 0 <= tail_start < recent + flush. */
typedef struct {
    int32_t t_quant;    /* tokens in the packed cache                                         */
    int32_t t_tail;     /* tokens in the fp16 tail                                            */
    int32_t tail_start; /* ring slot of the oldest tail token                                 */
} pk_state;

uint32_t pk_abi_version(void);
const char *pk_status_string(pk_status s);

/* Sizes of the cache arrays.  Host-only; never touches the device. */
pk_status pk_cache_layout(const pk_config *cfg, pk_layout *out /* host, out */);

/*
 * Bytes of device workspace the given operation needs.
 *   PK_OP_MINE  : a = tokens per set T, b = number of pattern sets
 *   PK_OP_APPEND: a, b unused: what pk_quantize_append_ragged needs (32 bytes per sequence); the uniform
 *                 pk_quantize_append needs none and ignores its workspace arguments
 *   PK_OP_DECODE: a = packed + tail tokens per stream of the cache itself,
 *                 b = the same for the shared prefix (0 if none)
 * Non-decreasing in a and b, so a workspace sized for the largest case serves
 * all smaller ones.  Returns 0 for an invalid configuration.
 */
size_t pk_workspace_bytes(const pk_config *cfg, pk_op op, int64_t a, int64_t b);

/*
 * How pk_decode_attention would cut a context (Sec. 3.4 leaves the work decomposition open): the length of the
 * equal splits that own_packed packed tokens per stream of the cache itself and prefix_packed of a shared prefix are
 * cut into, the number of partial-result slots per stream (splits of both plus two for the fp16 tails) and the
 * workspace bytes those slots take - never more than pk_workspace_bytes reports for the same or longer contexts,
 * and what has to fit PK_NOALLOC_SCRATCH_BYTES for pk_decode_attention_noalloc.  Host-only; never touches the
 * device.  Each out pointer may be NULL.  Errors: cfg NULL or a negative count -> PK_ERR_INVALID_ARG; an invalid
 * configuration -> its status.
 */
pk_status pk_decode_plan(const pk_config *cfg, int64_t own_packed, int64_t prefix_packed, int32_t *split_tokens /* host, out */,
                         int32_t *n_slots /* host, out */, size_t *bytes_needed /* host, out */);

/*
 * Pattern mining (Sec. 3.1, Eq. 4): `iters` Lloyd iterations of K-means under
 * the Euclidean metric on each of n_sets independent vector sets; the centroid
 * of each cluster is its pattern.  Uses cfg->head_dim and cfg->n_patterns only.
 *   x          [n_sets][T][d] fp16, set s starts at x + s*set_stride elements
 *   patterns   [n_sets][P][d] fp16.  init_given == 0: initialised from the first
 *              P vectors of each set (T >= P required); != 0: used as the
 *              starting centroids.  On return: the centroids after `iters`
 *              updates, each the mean of its members rounded to fp16 (nearest
 *              even); a cluster without members keeps its centroid.
 *   assign     optional [n_sets][T] int32: assignment of the last assignment
 *              step (taken against the centroids before the last update)
 *   inertia    optional [n_sets][iters] float: within-cluster sum of squares
 *              seen by each assignment step
 * Sums are formed in a fixed order: results are reproducible bit for bit.
 */
pk_status pk_mine_patterns(const pk_config *cfg, const void *x, int64_t set_stride, int32_t n_sets,
                           int32_t T, int32_t iters, int32_t init_given, void *patterns,
                           int32_t *assign, float *inertia, void *workspace, size_t workspace_bytes,
                           void *stream);

/*
 * Append n_new vectors per stream (Sec. 3.2): they join the fp16 tail; while
 * the tail holds at least recent + flush vectors its oldest `flush` vectors are
 * assigned to their nearest pattern (Eq. 6), residualised and quantized (Eq. 1;
 * K per channel over groups of G tokens, V per token over groups of Gc
 * channels), packed and written behind the t_quant tokens already there.
 *   k_new, v_new  [n_seq][n_kv_heads][n_new][d] fp16; stream n starts at
 *                 base + n*stream_stride elements (stream_stride 0 = n_new*d)
 *   patterns_k/_v [n_sets][P][d] fp16
 *   state         host, in/out
 * n_new == 0 is a no-op.  Prefill is one call with n_new = prompt length.
 */
pk_status pk_quantize_append(const pk_config *cfg, const pk_cache *cache, pk_state *state,
                             const void *k_new, const void *v_new, int32_t n_new,
                             int64_t stream_stride, const void *patterns_k, const void *patterns_v,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * pk_quantize_append for a batch whose sequences are filled to different lengths and receive different numbers
 * of new vectors in one call (prompts of different lengths prefilled together; continuous batching, where every
 * sequence is at a step of its own).  Sec. 3.2's computation is per stream and unchanged; every sequence keeps a
 * pk_state of its own and is treated exactly as pk_quantize_append would treat it alone.
 *   states          host, in/out, [n_seq]: the fill state of every sequence (each as for the uniform call)
 *   n_new           host, [n_seq]: new vectors of every sequence, >= 0 (0: the sequence is left as it is)
 *   k_new, v_new    [n_seq][n_kv_heads][n_max][d] fp16 with n_max >= max_i n_new[i]: sequence i uses the first
 *                   n_new[i] rows of each of its streams; stream n starts at base + n*stream_stride elements
 *                   (stream_stride 0 = max_i n_new[i] * d)
 *   seq_states_out  optional DEVICE int32 [n_seq][4], 16-byte aligned: receives t_quant, t_tail, tail_start (and
 *                   0) of every sequence after the append, in the form pk_decode_attention_ragged reads, so that
 *                   an append and a decode can follow each other without a host-to-device copy by the caller
 *   workspace       device, at least pk_workspace_bytes(cfg, PK_OP_APPEND, 0, 0) bytes (32 per sequence: the
 *                   per-sequence launch parameters, written by a small kernel from values that travel in its
 *                   arguments - no host buffer has to outlive the call)
 * All sequences are checked before anything is launched: a bad state -> PK_ERR_STATE, a negative count ->
 * PK_ERR_INVALID_ARG, a sequence whose flushes would exceed t_capacity -> PK_ERR_CAPACITY, a missing or small
 * workspace -> PK_ERR_WORKSPACE; states and device memory are then untouched.  Launch sizes follow the largest
 * sequence; workgroups beyond a shorter sequence's share return at once.
 */
pk_status pk_quantize_append_ragged(const pk_config *cfg, const pk_cache *cache, pk_state *states /* host [n_seq] */,
                                    const void *k_new, const void *v_new, const int32_t *n_new /* host [n_seq] */,
                                    int64_t stream_stride, const void *patterns_k, const void *patterns_v,
                                    int32_t *seq_states_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * One decode step of attention over [shared prefix | packed | tail] for every
 * query head (Sec. 3.4): out = softmax(softmax_scale * q.K^) V^ where K^, V^ are
 * the reconstructions M[k*] + (s*code + z) of the packed part and the fp16
 * vectors of the tail.  Nothing is reconstructed in memory: q.M is computed
 * once per pattern and gathered by index, q.(s*code + z) comes straight from
 * the packed codes, and the V side adds pattern sums weighted by the softmax
 * mass of each pattern to the weighted residuals.
 *   q        [n_seq][n_q_heads][d] fp16; query head h reads KV head h/(n_q/n_kv)
 *   prefix_* optional (all NULL if unused): a cache with n_seq == 1 whose
 *            streams precede every sequence's own cache (a shared prompt).  It
 *            must use the same head counts, head_dim, n_patterns, bits and group,
 *            and is read with pattern set = KV head of patterns_k / patterns_v.
 *   out      [n_seq][n_q_heads][d] float
 *   lse      optional [n_seq][n_q_heads] float: log-sum-exp of the scaled scores
 * A context of length 0 yields out = 0 and lse = -inf.
 * Arithmetic and supported range: scores and outputs are accumulated in binary32; the operands
 * of the two code contractions are fp16 products, q * s_K (q brought to max |q| in [1, 2) per
 * head by a power of two first, so any finite fp16 query is accepted) and p * s_V with p <= 1.
 * Both carry a factor of up to 2^8 for the position of a code inside its word, hence the stored
 * scales must satisfy s_K < 128 and s_V < 256 (a residual range below 384 resp. 768 per group at
 * 2 bits); larger scales overflow fp16 and give non-finite outputs.  The rounding of q * s_K is
 * compensated where it would exceed about 6e-4 in a score (groups of 64 or 128 tokens).
 */
pk_status pk_decode_attention(const pk_config *cfg, const pk_cache *cache, const pk_state *state,
                              const pk_config *prefix_cfg, const pk_cache *prefix,
                              const pk_state *prefix_state, const void *q, float softmax_scale,
                              const void *patterns_k, const void *patterns_v, float *out, float *lse,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same decode step for a batch whose sequences are filled to different lengths (the long-context and
 * test-time-scaling workloads of Sec. 4 batch requests whose prompts and generations differ in length;
 * Sec. 3.4's computation is per sequence and unchanged).  The caller fills each sequence through a cache
 * view of its own (the cache arrays are laid out stream by stream, so the part of sequence i is a cache with
 * n_seq == 1 whose pointers are offset by i times the per-sequence size) and keeps one pk_state per sequence.
 *   bound       host: t_quant and t_tail no smaller than any sequence's (t_quant a multiple of flush, both
 *               within what check of a uniform state allows), tail_start 0.  Launch sizes and the workspace
 *               (pk_workspace_bytes with these bounds) follow the bound.
 *   seq_states  DEVICE, int32 [n_seq][4], 16-byte aligned: t_quant, t_tail, tail_start of every sequence's
 *               own cache and one unused word.  Read by the kernels at run time, so the host cannot check the
 *               values: an entry is clamped to [0, bound] (t_quant to whole 64-token blocks, tail_start to
 *               the ring) before use, which keeps every access inside the cache whatever the array holds.
 * Everything else as pk_decode_attention (the shared prefix, if any, is uniform).  A sequence of length 0
 * yields out = 0 and lse = -inf.  Errors before any launch: as pk_decode_attention; seq_states or bound NULL
 * -> PK_ERR_INVALID_ARG; seq_states misaligned -> PK_ERR_ALIGNMENT; bound->tail_start != 0 -> PK_ERR_STATE.
 */
pk_status pk_decode_attention_ragged(const pk_config *cfg, const pk_cache *cache, const pk_state *bound,
                                     const int32_t *seq_states, const pk_config *prefix_cfg, const pk_cache *prefix,
                                     const pk_state *prefix_state, const void *q, float softmax_scale,
                                     const void *patterns_k, const void *patterns_v, float *out, float *lse,
                                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * pk_decode_attention for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * pk_decode_attention without the workspace: the per-split partial results (outputs, per-pattern softmax mass,
 * running maximum and sum) live in a fixed array of PK_NOALLOC_SCRATCH_BYTES inside the library's device image
 * (one copy per GPU, held until the process ends).  The call allocates and frees nothing; on the first call
 * on a device it looks up that device's copy of the array (hipGetSymbolAddress, with the calling thread's
 * current device, which must be the device of `stream` and of all pointers).
 *   - A decode whose partials (pk_workspace_bytes(cfg, PK_OP_DECODE, ...) for the cache's current fill) exceed
 *     PK_NOALLOC_SCRATCH_BYTES is refused with PK_ERR_WORKSPACE before anything is launched.
 *   - Every slot of the array that a call's merge reads was written by that call's own kernels first, so
 *     nothing needs clearing and what an earlier call left behind is never read.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or
 *     host threads) race on it.  Serialise them on one stream.
 * Errors: as pk_decode_attention; PK_ERR_DEVICE if the device's array cannot be located.
 */
#define PK_NOALLOC_SCRATCH_BYTES (32u << 20)
pk_status pk_decode_attention_noalloc(const pk_config *cfg, const pk_cache *cache, const pk_state *state,
                                      const pk_config *prefix_cfg, const pk_cache *prefix,
                                      const pk_state *prefix_state, const void *q, float softmax_scale,
                                      const void *patterns_k, const void *patterns_v, float *out, float *lse,
                                      void *stream);

/*
 * Decode-stage pattern update (Sec. 3.1 "Decoding Stage", Eq. 5): for each of n_sets windows of n
 * vectors, the per-channel Chebyshev centre  m_c = (min_i x_ic + max_i x_ic) / 2,  computed in binary32
 * (exact for fp16 inputs) and rounded to fp16, ties to even.  The caller merges the result into its
 * pattern table (one more row, n_patterns + 1 afterwards; tables are [sets][n_patterns][d] contiguous, so
 * growing one means re-laying it out) and uses the grown table for the following appends and decodes.
 *   x           device, fp16, window s at x + s*set_stride elements, n rows of head_dim contiguous
 *   pattern_out device, fp16, row s at pattern_out + s*out_stride elements (head_dim values)
 * Errors (before any launch): NULL pointers, n_sets < 1, n < 1 -> PK_ERR_INVALID_ARG; head_dim != 128 ->
 * PK_ERR_UNSUPPORTED; pointers or strides not 16-byte aligned -> PK_ERR_ALIGNMENT.  Asynchronous on `stream`.
 */
pk_status pk_window_pattern(const void *x, int64_t set_stride, int32_t n_sets, int32_t n, int32_t head_dim,
                            void *pattern_out, int64_t out_stride, void *stream);

/*
 * Reconstruct packed tokens [t0, t1) of every stream: X^ = M[k*] + (s*code + z)
 * in binary32, evaluated in that order (the rule below Eq. 6).  For parity
 * tests and debugging; not on the hot path.
 *   k_out, v_out [N][t1-t0][d] float (either may be NULL)
 */
pk_status pk_dequantize(const pk_config *cfg, const pk_cache *cache, const pk_state *state,
                        const void *patterns_k, const void *patterns_v, int32_t t0, int32_t t1,
                        float *k_out, float *v_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PATTERNKV_H */
