// Host side of the C ABI declared in include/patternkv.h: argument checking, cache
// layout, workspace carving and kernel launches.  Nothing here allocates device memory
// or synchronises with the device.
#include <cstring>
#include <vector>
#include <mutex>

#include "pk_internal.h"

using namespace pk;

// Partial results of pk_decode_attention_noalloc.  Part of the library's device image: every GPU the library
// runs on holds its own copy at its own address until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; the address kernels are given is the one that call returns.
static __device__ __align__(256) unsigned char scratch[PK_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];   // per device: address of that device's copy of `scratch`, once looked up

// Address of the current device's copy of the scratch array (looked up once per device), or nullptr.
void *scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

pk_status check_config(const pk_config *c)
{
    if (!c) return PK_ERR_INVALID_ARG;
    if (c->n_seq < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_patterns < 1 || c->seqs_per_set < 0 ||
        c->recent < 0 || c->flush < 1 || c->t_capacity < 0)
        return PK_ERR_INVALID_ARG;
    if (c->metric != PK_METRIC_L2 && c->metric != PK_METRIC_MINMAX) return PK_ERR_INVALID_ARG;
    if (c->head_dim != kD && c->head_dim != 96 && c->head_dim != 256) return PK_ERR_UNSUPPORTED;
    if (c->n_patterns > 256) return PK_ERR_UNSUPPORTED;
    if (!(c->v_rho >= 0.f) || !(c->v_rho < 1.f)) return PK_ERR_INVALID_ARG;   // also rejects NaN
    if (c->v_rho > 0.f && c->n_patterns > PK_NO_PATTERN) return PK_ERR_UNSUPPORTED;
    if (c->bits != 2 && c->bits != 4) return PK_ERR_UNSUPPORTED;
    if (c->group != 32 && c->group != 64 && c->group != 128) return PK_ERR_UNSUPPORTED;
    // V is quantized over contiguous groups of min(G, d) channels: they have to tile the head (d = 96: G = 32 or 128)
    if (c->head_dim % (c->group < c->head_dim ? c->group : c->head_dim) != 0) return PK_ERR_UNSUPPORTED;
    if (c->n_q_heads % c->n_kv_heads != 0) return PK_ERR_SHAPE;
    if (c->n_q_heads / c->n_kv_heads > 64) return PK_ERR_UNSUPPORTED;
    if ((int64_t)c->n_seq * c->n_kv_heads > 65535) return PK_ERR_UNSUPPORTED;
    if (c->flush % c->group != 0 || c->flush % 64 != 0) return PK_ERR_SHAPE;
    if (c->t_capacity % c->flush != 0) return PK_ERR_SHAPE;
    if (c->t_capacity > (1 << 25)) return PK_ERR_UNSUPPORTED;   // byte offsets inside a stream stay below 2^32
    if (c->page_tokens < 0 || c->n_pages < 0) return PK_ERR_INVALID_ARG;
    if (c->page_tokens > 0) {
        // a power of two of at least 128, so that no quantization group, 64-token block or tile straddles a page
        if (c->page_tokens < 128 || (c->page_tokens & (c->page_tokens - 1)) != 0) return PK_ERR_UNSUPPORTED;
        if (c->t_capacity % c->page_tokens != 0) return PK_ERR_SHAPE;
        if (c->n_pages < 1) return PK_ERR_INVALID_ARG;
        if ((int64_t)c->n_pages * c->n_kv_heads * c->page_tokens > ((int64_t)1 << 36)) return PK_ERR_UNSUPPORTED;
    }
    return PK_OK;
}

pk_status check_state(const pk_config *c, const pk_state *s)
{
    if (!s) return PK_ERR_INVALID_ARG;
    const int ring = c->recent + c->flush;
    if (s->t_quant < 0 || s->t_quant > c->t_capacity || s->t_quant % c->flush != 0) return PK_ERR_STATE;
    if (s->t_tail < 0 || s->t_tail >= ring) return PK_ERR_STATE;
    if (s->tail_start < 0 || s->tail_start >= ring) return PK_ERR_STATE;
    return PK_OK;
}

pk_status check_cache(const pk_cache *k)
{
    if (!k) return PK_ERR_INVALID_ARG;
    const void *p[10] = {k->k_codes, k->k_scale, k->k_zero, k->k_idx, k->v_codes,
                         k->v_scale, k->v_zero,  k->v_idx,  k->tail_k, k->tail_v};
    for (const void *q : p)
        if (!q) return PK_ERR_INVALID_ARG;
    for (const void *q : p)
        if (!aligned16(q)) return PK_ERR_ALIGNMENT;
    return PK_OK;
}

// a paged configuration needs its page table
pk_status check_paging(const pk_config *c, const pk_cache *k)
{
    if (c->page_tokens == 0) return PK_OK;
    if (!k->page_table) return PK_ERR_INVALID_ARG;
    return aligned16(k->page_table) ? PK_OK : PK_ERR_ALIGNMENT;
}

PackedMap make_map(const pk_config *c, const pk_cache *k)
{
    PackedMap m;
    m.page_table = c->page_tokens > 0 ? k->page_table : nullptr;
    m.page_shift = 0;
    while (c->page_tokens > 0 && (1 << m.page_shift) < c->page_tokens) ++m.page_shift;
    m.pages_per_seq = c->page_tokens > 0 ? c->t_capacity / c->page_tokens : 0;
    m.n_pages = c->n_pages;
    m.n_kv_heads = c->n_kv_heads;
    m.t_capacity = c->t_capacity;
    return m;
}

CacheView make_view(const pk_config *c, const pk_cache *k, const pk_state *s)
{
    CacheView v;
    v.map = make_map(c, k);
    v.k_codes = static_cast<const uint32_t *>(k->k_codes);
    v.k_scale = static_cast<const __half *>(k->k_scale);
    v.k_zero = static_cast<const __half *>(k->k_zero);
    v.k_idx = static_cast<const uint8_t *>(k->k_idx);
    v.v_codes = static_cast<const uint8_t *>(k->v_codes);
    v.v_scale = static_cast<const __half *>(k->v_scale);
    v.v_zero = static_cast<const __half *>(k->v_zero);
    v.v_idx = static_cast<const uint8_t *>(k->v_idx);
    v.tail_k = static_cast<const __half *>(k->tail_k);
    v.tail_v = static_cast<const __half *>(k->tail_v);
    v.t_capacity = c->t_capacity;
    v.t_quant = s->t_quant;
    v.t_tail = s->t_tail;
    v.tail_start = s->tail_start;
    v.ring_len = c->recent + c->flush;
    return v;
}

// the sequence order of a ragged batch lives behind the partials
uint64_t decode_order_bytes(int64_t n_seq) { return round_up((uint64_t)n_seq * 4, 256); }

// upper bound on the number of partial slots decode uses for up to a own / b prefix tokens
int64_t decode_slots_bound(int64_t N, int64_t a, int64_t b)
{
    const int64_t fine = (a + 255) / 256 + (b + 255) / 256;
    const int64_t target = 2048 / N + 4;
    const int64_t coarse = (a + 8191) / 8192 + (b + 8191) / 8192;
    int64_t s = fine < target ? fine : target;
    if (coarse > s) s = coarse;
    return s + 2;
}

struct MineCarve {
    size_t assign, best, psum, pcnt, total;
};
MineCarve mine_carve(int64_t S, int64_t T, int P, int d)
{
    MineCarve m;
    const int ts = mine_tsplit((int)T, (int)S, P);
    m.assign = 0;
    m.best = round_up(m.assign + (uint64_t)S * T * 4, 256);
    m.psum = round_up(m.best + (uint64_t)S * T * 4, 256);
    m.pcnt = round_up(m.psum + (uint64_t)S * ts * P * d * 4, 256);
    m.total = round_up(m.pcnt + (uint64_t)S * ts * P * 4, 256);
    return m;
}

}  // namespace

extern "C" {

uint32_t pk_abi_version(void) { return PK_ABI_VERSION; }

const char *pk_status_string(pk_status s)
{
    switch (s) {
    case PK_OK: return "ok";
    case PK_ERR_INVALID_ARG: return "invalid argument";
    case PK_ERR_UNSUPPORTED: return "unsupported configuration";
    case PK_ERR_SHAPE: return "inconsistent shapes";
    case PK_ERR_ALIGNMENT: return "device pointer not 16-byte aligned";
    case PK_ERR_CAPACITY: return "cache capacity exceeded";
    case PK_ERR_STATE: return "invalid cache state";
    case PK_ERR_WORKSPACE: return "workspace missing or too small";
    case PK_ERR_DEVICE: return "HIP launch failed";
    }
    return "unknown status";
}

pk_status pk_cache_layout(const pk_config *cfg, pk_layout *out)
{
    pk_status st = check_config(cfg);
    if (st != PK_OK) return st;
    if (!out) return PK_ERR_INVALID_ARG;
    const uint64_t N = (uint64_t)cfg->n_seq * cfg->n_kv_heads, d = cfg->head_dim, b = cfg->bits;
    const uint64_t G = cfg->group, Gc = G < d ? G : d;
    // packed token slots: N streams of t_capacity tokens, or a pool of pages of [n_kv_heads][page_tokens] tokens
    const uint64_t slots = cfg->page_tokens > 0 ? (uint64_t)cfg->n_pages * cfg->n_kv_heads * cfg->page_tokens
                                                : N * (uint64_t)cfg->t_capacity;
    out->align = 16;
    out->k_codes = slots * d * b / 8;
    out->k_scale = out->k_zero = (slots / G) * d * 2;
    out->k_idx = slots;
    out->v_codes = slots * d * b / 8;
    out->v_scale = out->v_zero = slots * (d / Gc) * 2;
    out->v_idx = slots;
    out->tail_k = out->tail_v = N * (uint64_t)(cfg->recent + cfg->flush) * d * 2;
    const uint64_t parts[10] = {out->k_codes, out->k_scale, out->k_zero, out->k_idx, out->v_codes,
                                out->v_scale, out->v_zero,  out->v_idx,  out->tail_k, out->tail_v};
    out->total = 0;
    for (uint64_t p : parts) out->total += round_up(p, out->align);
    return PK_OK;
}

size_t pk_workspace_bytes(const pk_config *cfg, pk_op op, int64_t a, int64_t b)
{
    if (!cfg || a < 0 || b < 0) return 0;
    if (op == PK_OP_MINE) {
        const int hd = cfg->head_dim;
        if ((hd != kD && hd != 96 && hd != 256) || cfg->n_patterns < 1 || cfg->n_patterns > 256 || b < 1) return 0;
        return mine_carve(b, a, cfg->n_patterns, hd).total;
    }
    if (check_config(cfg) != PK_OK) return 0;
    if (op == PK_OP_APPEND) return (size_t)cfg->n_seq * kSeqEntry * sizeof(int32_t);
    if (op == PK_OP_DECODE) {
        const int64_t N = (int64_t)cfg->n_seq * cfg->n_kv_heads, r = cfg->n_q_heads / cfg->n_kv_heads;
        const int64_t slots = decode_slots_bound(N, a, b);
        return round_up((uint64_t)N * slots * r * cfg->head_dim * 4, 256) + round_up((uint64_t)N * slots * r * cfg->n_patterns * 4, 256) +
               round_up((uint64_t)N * slots * r * 2 * 4, 256) + decode_order_bytes(cfg->n_seq);
    }
    return 0;
}

pk_status pk_decode_plan(const pk_config *cfg, int64_t own_packed, int64_t prefix_packed, int32_t *split_tokens,
                         int32_t *n_slots, size_t *bytes_needed)
{
    if (!cfg || own_packed < 0 || prefix_packed < 0) return PK_ERR_INVALID_ARG;
    const pk_status st = check_config(cfg);
    if (st != PK_OK) return st;
    const int64_t N = (int64_t)cfg->n_seq * cfg->n_kv_heads, r = cfg->n_q_heads / cfg->n_kv_heads;
    const int64_t c = decode_chunk(N, own_packed + prefix_packed, cfg->n_patterns, (int)r);
    const int64_t slots = (own_packed + c - 1) / c + (prefix_packed + c - 1) / c + 2;
    if (split_tokens) *split_tokens = (int32_t)c;
    if (n_slots) *n_slots = (int32_t)slots;
    if (bytes_needed)
        *bytes_needed = (size_t)(round_up((uint64_t)N * slots * r * cfg->head_dim * 4, 256) + round_up((uint64_t)N * slots * r * cfg->n_patterns * 4, 256) +
                                 round_up((uint64_t)N * slots * r * 2 * 4, 256) + decode_order_bytes(cfg->n_seq));
    return PK_OK;
}

pk_status pk_mine_patterns(const pk_config *cfg, const void *x, int64_t set_stride, int32_t n_sets, int32_t T,
                           int32_t iters, int32_t init_given, void *patterns, int32_t *assign, float *inertia,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    if (!cfg || !x || !patterns) return PK_ERR_INVALID_ARG;
    if (n_sets < 1 || T < 1 || iters < 0 || cfg->n_patterns < 1) return PK_ERR_INVALID_ARG;
    const int hd = cfg->head_dim;
    if ((hd != kD && hd != 96 && hd != 256) || cfg->n_patterns > 256 || n_sets > 65535) return PK_ERR_UNSUPPORTED;
    if (!init_given && T < cfg->n_patterns) return PK_ERR_SHAPE;
    if (set_stride < (int64_t)T * hd || set_stride % 8 != 0) return PK_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(patterns) || (assign && !aligned16(assign))) return PK_ERR_ALIGNMENT;
    const MineCarve mc = mine_carve(n_sets, T, cfg->n_patterns, hd);
    if (!workspace || workspace_bytes < mc.total) return PK_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PK_ERR_ALIGNMENT;

    char *ws = static_cast<char *>(workspace);
    MineArgs a;
    a.x = static_cast<const __half *>(x);
    a.set_stride = set_stride;
    a.n_sets = n_sets;
    a.T = T;
    a.P = cfg->n_patterns;
    a.iters = iters;
    a.init_given = init_given;
    a.d = hd;
    a.patterns = static_cast<__half *>(patterns);
    a.assign_ws = reinterpret_cast<int32_t *>(ws + mc.assign);
    a.assign = assign;   // optional: written by the last step only
    a.best = reinterpret_cast<float *>(ws + mc.best);
    a.psum = reinterpret_cast<float *>(ws + mc.psum);
    a.pcnt = reinterpret_cast<int32_t *>(ws + mc.pcnt);
    a.inertia = inertia;
    a.tsplit = mine_tsplit(T, n_sets, a.P);
    return launch_mine(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PK_OK : PK_ERR_DEVICE;
}

namespace {

// What an append launches: uniform values, or (seq_table set) the batch's largest counts for the launch sizes and
// a per-sequence table for everything else.
struct AppendPlan {
    int64_t nq;            // vectors to quantize per stream (largest of the batch)
    int32_t t0, ring_start, n_ring;
    int64_t i0, i1;        // tail copy: logical vectors [i0, i1) (ragged: 0 .. the widest range)
    const int32_t *seq_table;
};

pk_status launch_append(const pk_config *cfg, const pk_cache *cache, const AppendPlan &p, const void *k_new, const void *v_new,
                        int64_t stream_stride, const void *patterns_k, const void *patterns_v, hipStream_t hs)
{
    const int N = cfg->n_seq * cfg->n_kv_heads;
    const int64_t ring = (int64_t)cfg->recent + cfg->flush;
    if (p.nq > 0) {
        QuantArgs a;
        a.src.ring_len = (int32_t)ring;
        a.src.ring_start = p.ring_start;
        a.src.n_ring = p.n_ring;
        a.src.fresh_stride = stream_stride;
        a.sets.n_kv_heads = cfg->n_kv_heads;
        a.sets.seqs_per_set = cfg->seqs_per_set;
        a.P = cfg->n_patterns;
        a.metric = cfg->metric;
        a.idx_given = 0;
        a.v_rho = 0.f;
        a.bits = cfg->bits;
        a.G = cfg->group;
        a.d = cfg->head_dim;
        a.n_streams = N;
        a.nq = (int32_t)p.nq;
        a.t0 = p.t0;
        a.map = make_map(cfg, cache);
        a.seq_table = p.seq_table;
        // K
        a.src.ring = static_cast<const __half *>(cache->tail_k);
        a.src.fresh = static_cast<const __half *>(k_new);
        a.patterns = static_cast<const __half *>(patterns_k);
        a.codes_k = static_cast<uint32_t *>(cache->k_codes);
        a.codes_v = nullptr;
        a.scale = static_cast<__half *>(cache->k_scale);
        a.zero = static_cast<__half *>(cache->k_zero);
        a.idx = static_cast<uint8_t *>(cache->k_idx);
        if (launch_quantize_k(a, hs) != hipSuccess) return PK_ERR_DEVICE;
        // V
        a.src.ring = static_cast<const __half *>(cache->tail_v);
        a.src.fresh = static_cast<const __half *>(v_new);
        a.patterns = static_cast<const __half *>(patterns_v);
        a.codes_k = nullptr;
        a.codes_v = static_cast<uint8_t *>(cache->v_codes);
        a.scale = static_cast<__half *>(cache->v_scale);
        a.zero = static_cast<__half *>(cache->v_zero);
        a.idx = static_cast<uint8_t *>(cache->v_idx);
        a.v_rho = cfg->v_rho;
        if (launch_quantize_v(a, hs) != hipSuccess) return PK_ERR_DEVICE;
    }
    // what is left stays in (old tail vectors) or moves into (fresh vectors) the ring;
    // logical vector i always lives in slot (tail_start + i) % ring
    TailCopyArgs c;
    c.fresh_k = static_cast<const __half *>(k_new);
    c.fresh_v = static_cast<const __half *>(v_new);
    c.fresh_stride = stream_stride;
    c.ring_k = static_cast<__half *>(cache->tail_k);
    c.ring_v = static_cast<__half *>(cache->tail_v);
    c.ring_len = (int32_t)ring;
    c.ring_start = p.ring_start;
    c.n_ring = p.n_ring;
    c.i0 = (int32_t)p.i0;
    c.i1 = (int32_t)p.i1;
    c.n_streams = N;
    c.n_kv_heads = cfg->n_kv_heads;
    c.d = cfg->head_dim;
    c.seq_table = p.seq_table;
    if (launch_tail_copy(c, hs) != hipSuccess) return PK_ERR_DEVICE;
    return PK_OK;
}

}  // namespace

pk_status pk_quantize_append(const pk_config *cfg, const pk_cache *cache, pk_state *state, const void *k_new,
                             const void *v_new, int32_t n_new, int64_t stream_stride, const void *patterns_k,
                             const void *patterns_v, void *workspace, size_t workspace_bytes, void *stream)
{
    (void)workspace;
    (void)workspace_bytes;
    pk_status st = check_config(cfg);
    if (st != PK_OK) return st;
    if ((st = check_cache(cache)) != PK_OK) return st;
    if ((st = check_paging(cfg, cache)) != PK_OK) return st;
    if ((st = check_state(cfg, state)) != PK_OK) return st;
    if (n_new < 0) return PK_ERR_INVALID_ARG;
    if (n_new == 0) return PK_OK;
    if (!k_new || !v_new || !patterns_k || !patterns_v) return PK_ERR_INVALID_ARG;
    if (stream_stride == 0) stream_stride = (int64_t)n_new * cfg->head_dim;
    if (stream_stride < (int64_t)n_new * cfg->head_dim || stream_stride % 8 != 0) return PK_ERR_SHAPE;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(patterns_k) || !aligned16(patterns_v))
        return PK_ERR_ALIGNMENT;

    const int64_t R = cfg->recent, F = cfg->flush, ring = R + F;
    const int64_t L = (int64_t)state->t_tail + n_new;
    const int64_t nf = L >= R ? (L - R) / F : 0;
    const int64_t nq = nf * F;
    if ((int64_t)state->t_quant + nq > cfg->t_capacity) return PK_ERR_CAPACITY;

    AppendPlan p;
    p.nq = nq;
    p.t0 = state->t_quant;
    p.ring_start = state->tail_start;
    p.n_ring = state->t_tail;
    p.i0 = nq > state->t_tail ? nq : state->t_tail;
    p.i1 = L;
    p.seq_table = nullptr;
    if ((st = launch_append(cfg, cache, p, k_new, v_new, stream_stride, patterns_k, patterns_v, static_cast<hipStream_t>(stream))) != PK_OK)
        return st;

    state->t_quant += (int32_t)nq;
    state->tail_start = (int32_t)((state->tail_start + nq) % ring);
    state->t_tail = (int32_t)(L - nq);
    return PK_OK;
}

pk_status pk_quantize_append_ragged(const pk_config *cfg, const pk_cache *cache, pk_state *states, const void *k_new,
                                    const void *v_new, const int32_t *n_new, int64_t stream_stride, const void *patterns_k,
                                    const void *patterns_v, int32_t *seq_states_out, void *workspace, size_t workspace_bytes,
                                    void *stream)
{
    pk_status st = check_config(cfg);
    if (st != PK_OK) return st;
    if ((st = check_cache(cache)) != PK_OK) return st;
    if ((st = check_paging(cfg, cache)) != PK_OK) return st;
    if (!states || !n_new) return PK_ERR_INVALID_ARG;
    const int S = cfg->n_seq;
    int64_t max_new = 0;
    for (int i = 0; i < S; ++i) {
        if ((st = check_state(cfg, &states[i])) != PK_OK) return st;
        if (n_new[i] < 0) return PK_ERR_INVALID_ARG;
        if (n_new[i] > max_new) max_new = n_new[i];
    }
    if (seq_states_out && !aligned16(seq_states_out)) return PK_ERR_ALIGNMENT;
    const size_t table_bytes = (size_t)S * kSeqEntry * sizeof(int32_t);
    if (max_new > 0) {
        if (!k_new || !v_new || !patterns_k || !patterns_v) return PK_ERR_INVALID_ARG;
        if (stream_stride == 0) stream_stride = max_new * cfg->head_dim;
        if (stream_stride < max_new * cfg->head_dim || stream_stride % 8 != 0) return PK_ERR_SHAPE;
        if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(patterns_k) || !aligned16(patterns_v)) return PK_ERR_ALIGNMENT;
    }
    if (!workspace || workspace_bytes < table_bytes) return PK_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PK_ERR_ALIGNMENT;

    // the plan of every sequence, checked as a whole before anything is launched
    const int64_t R = cfg->recent, F = cfg->flush, ring = R + F;
    std::vector<int32_t> entry((size_t)S * kSeqEntry, 0), after((size_t)S * 3, 0);
    AppendPlan p;
    p.nq = 0;
    p.t0 = 0;
    p.ring_start = 0;
    p.n_ring = 0;
    p.i0 = 0;
    p.i1 = 0;
    for (int i = 0; i < S; ++i) {
        const pk_state &s = states[i];
        const int64_t L = (int64_t)s.t_tail + n_new[i];
        const int64_t nq = L >= R ? (L - R) / F * F : 0;
        if ((int64_t)s.t_quant + nq > cfg->t_capacity) return PK_ERR_CAPACITY;
        int32_t *e = &entry[(size_t)i * kSeqEntry];
        e[kSeqNq] = (int32_t)nq;
        e[kSeqT0] = s.t_quant;
        e[kSeqRingStart] = s.tail_start;
        e[kSeqNRing] = s.t_tail;
        e[kSeqI0] = (int32_t)(nq > s.t_tail ? nq : s.t_tail);
        e[kSeqI1] = (int32_t)L;
        after[(size_t)i * 3] = (int32_t)(s.t_quant + nq);
        after[(size_t)i * 3 + 1] = (int32_t)(L - nq);
        after[(size_t)i * 3 + 2] = (int32_t)((s.tail_start + nq) % ring);
        if (nq > p.nq) p.nq = nq;
        if (e[kSeqI1] - e[kSeqI0] > p.i1) p.i1 = e[kSeqI1] - e[kSeqI0];   // launch width of the tail copy
    }
    hipStream_t hs = static_cast<hipStream_t>(stream);
    p.seq_table = static_cast<const int32_t *>(workspace);
    for (int first = 0; first < S; first += kSeqChunk) {
        SeqTableArgs t;
        t.table = static_cast<int32_t *>(workspace);
        t.states_out = seq_states_out;
        t.first = first;
        t.count = S - first < kSeqChunk ? S - first : kSeqChunk;
        std::memset(t.entry, 0, sizeof(t.entry));
        std::memset(t.state, 0, sizeof(t.state));
        std::memcpy(t.entry, &entry[(size_t)first * kSeqEntry], (size_t)t.count * kSeqEntry * sizeof(int32_t));
        std::memcpy(t.state, &after[(size_t)first * 3], (size_t)t.count * 3 * sizeof(int32_t));
        if (launch_seq_table(t, hs) != hipSuccess) return PK_ERR_DEVICE;
    }
    if (max_new > 0 &&
        (st = launch_append(cfg, cache, p, k_new, v_new, stream_stride, patterns_k, patterns_v, hs)) != PK_OK)
        return st;
    for (int i = 0; i < S; ++i) {
        states[i].t_quant = after[(size_t)i * 3];
        states[i].t_tail = after[(size_t)i * 3 + 1];
        states[i].tail_start = after[(size_t)i * 3 + 2];
    }
    return PK_OK;
}

static pk_status decode_impl(const pk_config *cfg, const pk_cache *cache, const pk_state *state, const int32_t *seq_states,
                             const pk_config *prefix_cfg, const pk_cache *prefix, const pk_state *prefix_state,
                             const void *q, float softmax_scale, const void *patterns_k, const void *patterns_v,
                             float *out, float *lse, void *workspace, size_t workspace_bytes, void *stream)
{
    pk_status st = check_config(cfg);
    if (st != PK_OK) return st;
    if ((st = check_cache(cache)) != PK_OK) return st;
    if ((st = check_paging(cfg, cache)) != PK_OK) return st;
    if ((st = check_state(cfg, state)) != PK_OK) return st;
    if (!q || !patterns_k || !patterns_v || !out) return PK_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(patterns_k) || !aligned16(patterns_v) || !aligned16(out) ||
        (lse && !aligned16(lse)))
        return PK_ERR_ALIGNMENT;
    const bool has_prefix = prefix_cfg || prefix || prefix_state;
    if (has_prefix) {
        if (!prefix_cfg || !prefix || !prefix_state) return PK_ERR_INVALID_ARG;
        if ((st = check_config(prefix_cfg)) != PK_OK) return st;
        if ((st = check_cache(prefix)) != PK_OK) return st;
        if ((st = check_paging(prefix_cfg, prefix)) != PK_OK) return st;
        if ((st = check_state(prefix_cfg, prefix_state)) != PK_OK) return st;
        if (prefix_cfg->n_seq != 1 || prefix_cfg->n_kv_heads != cfg->n_kv_heads ||
            prefix_cfg->n_q_heads != cfg->n_q_heads || prefix_cfg->n_patterns != cfg->n_patterns ||
            prefix_cfg->bits != cfg->bits || prefix_cfg->group != cfg->group || prefix_cfg->head_dim != cfg->head_dim)
            return PK_ERR_SHAPE;
    }

    DecodeArgs a;
    a.own = make_view(cfg, cache, state);
    if (has_prefix) {
        a.prefix = make_view(prefix_cfg, prefix, prefix_state);
    } else {
        std::memset(&a.prefix, 0, sizeof(a.prefix));
        a.prefix.ring_len = 1;
    }
    const int64_t N = (int64_t)cfg->n_seq * cfg->n_kv_heads, r = cfg->n_q_heads / cfg->n_kv_heads;
    a.chunk = decode_chunk(N, (int64_t)a.own.t_quant + a.prefix.t_quant, cfg->n_patterns, (int)r);
    a.w_stride = (cfg->v_rho > 0.f || (has_prefix && prefix_cfg->v_rho > 0.f)) ? 256 : cfg->n_patterns;
    a.splits_own = (a.own.t_quant + a.chunk - 1) / a.chunk;
    a.splits_prefix = (a.prefix.t_quant + a.chunk - 1) / a.chunk;
    const int64_t slots = a.splits_own + a.splits_prefix + 2;
    if (slots > kMaxSlots) return PK_ERR_UNSUPPORTED;
    const uint64_t o_bytes = round_up((uint64_t)N * slots * r * cfg->head_dim * 4, 256);
    const uint64_t w_bytes = round_up((uint64_t)N * slots * r * cfg->n_patterns * 4, 256);
    const uint64_t ml_bytes = round_up((uint64_t)N * slots * r * 2 * 4, 256);
    const uint64_t order_bytes = decode_order_bytes(cfg->n_seq);
    if (!workspace || workspace_bytes < o_bytes + w_bytes + ml_bytes + order_bytes) return PK_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PK_ERR_ALIGNMENT;

    a.sets.n_kv_heads = cfg->n_kv_heads;
    a.sets.seqs_per_set = cfg->seqs_per_set;
    a.q = static_cast<const __half *>(q);
    a.patterns_k = static_cast<const __half *>(patterns_k);
    a.patterns_v = static_cast<const __half *>(patterns_v);
    a.n_seq = cfg->n_seq;
    a.n_kv_heads = cfg->n_kv_heads;
    a.n_q_heads = cfg->n_q_heads;
    a.P = cfg->n_patterns;
    a.bits = cfg->bits;
    a.G = cfg->group;
    a.d = cfg->head_dim;
    a.v_thresholded = (cfg->v_rho > 0.f || (has_prefix && prefix_cfg->v_rho > 0.f)) ? 1 : 0;
    {   // 6 or 8 heads per KV head over 32-channel groups, or 10 to 16 heads: two groups of heads, each with at
        // most 8 heads and 16 (head, V channel group) pairs
        const int64_t ng = kD / (cfg->group < kD ? cfg->group : kD);
        const bool one_fits = r <= 8 && r * ng <= 16;
        a.head_groups = (cfg->head_dim == kD && !one_fits && r % 2 == 0 && r / 2 <= 8 && (r / 2) * ng <= 16) ? 2 : 1;
    }
    a.softmax_scale = softmax_scale;
    a.part_o = reinterpret_cast<float *>(workspace);
    a.part_w = reinterpret_cast<float *>(static_cast<char *>(workspace) + o_bytes);
    a.part_ml = reinterpret_cast<float *>(static_cast<char *>(workspace) + o_bytes + w_bytes);
    a.out = out;
    a.lse = lse;
    a.seq_state = seq_states;
    a.seq_order = seq_states && cfg->n_seq > 1 && cfg->n_seq <= kMaxOrdered
                      ? reinterpret_cast<const int32_t *>(static_cast<char *>(workspace) + o_bytes + w_bytes + ml_bytes)
                      : nullptr;
    return launch_decode(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PK_OK : PK_ERR_DEVICE;
}

pk_status pk_decode_attention(const pk_config *cfg, const pk_cache *cache, const pk_state *state,
                              const pk_config *prefix_cfg, const pk_cache *prefix, const pk_state *prefix_state,
                              const void *q, float softmax_scale, const void *patterns_k, const void *patterns_v,
                              float *out, float *lse, void *workspace, size_t workspace_bytes, void *stream)
{
    return decode_impl(cfg, cache, state, nullptr, prefix_cfg, prefix, prefix_state, q, softmax_scale, patterns_k, patterns_v,
                       out, lse, workspace, workspace_bytes, stream);
}

pk_status pk_decode_attention_ragged(const pk_config *cfg, const pk_cache *cache, const pk_state *bound,
                                     const int32_t *seq_states, const pk_config *prefix_cfg, const pk_cache *prefix,
                                     const pk_state *prefix_state, const void *q, float softmax_scale,
                                     const void *patterns_k, const void *patterns_v, float *out, float *lse,
                                     void *workspace, size_t workspace_bytes, void *stream)
{
    if (!seq_states || !bound) return PK_ERR_INVALID_ARG;
    if (!aligned16(seq_states)) return PK_ERR_ALIGNMENT;
    if (bound->tail_start != 0) return PK_ERR_STATE;   // the bound carries sizes only; ring positions are per sequence
    return decode_impl(cfg, cache, bound, seq_states, prefix_cfg, prefix, prefix_state, q, softmax_scale, patterns_k,
                       patterns_v, out, lse, workspace, workspace_bytes, stream);
}

pk_status pk_decode_attention_noalloc(const pk_config *cfg, const pk_cache *cache, const pk_state *state,
                                      const pk_config *prefix_cfg, const pk_cache *prefix, const pk_state *prefix_state,
                                      const void *q, float softmax_scale, const void *patterns_k, const void *patterns_v,
                                      float *out, float *lse, void *stream)
{
    void *ptr = scratch_of_current_device();
    if (!ptr) return PK_ERR_DEVICE;
    // decode_impl refuses a decode whose partials do not fit (PK_ERR_WORKSPACE) before launching anything; every
    // partial slot the merge reads is written by this call's own kernels, so the array needs no clearing
    return decode_impl(cfg, cache, state, nullptr, prefix_cfg, prefix, prefix_state, q, softmax_scale, patterns_k, patterns_v,
                       out, lse, ptr, PK_NOALLOC_SCRATCH_BYTES, stream);
}

pk_status pk_window_pattern(const void *x, int64_t set_stride, int32_t n_sets, int32_t n, int32_t head_dim,
                            void *pattern_out, int64_t out_stride, void *stream)
{
    if (!x || !pattern_out || n_sets < 1 || n < 1 || set_stride < 0 || out_stride < 0) return PK_ERR_INVALID_ARG;
    if ((head_dim != kD && head_dim != 96 && head_dim != 256) || n_sets > 65535) return PK_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(pattern_out) || set_stride % 8 != 0 || out_stride % 8 != 0) return PK_ERR_ALIGNMENT;
    const __half *xs = static_cast<const __half *>(x);
    __half *po = static_cast<__half *>(pattern_out);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const hipError_t e = head_dim == kD ? launch_window_pattern(xs, set_stride, n_sets, n, po, out_stride, hs)
                                        : launch_generic_window_pattern(xs, set_stride, n_sets, n, head_dim, po, out_stride, hs);
    return e == hipSuccess ? PK_OK : PK_ERR_DEVICE;
}

pk_status pk_dequantize(const pk_config *cfg, const pk_cache *cache, const pk_state *state, const void *patterns_k,
                        const void *patterns_v, int32_t t0, int32_t t1, float *k_out, float *v_out, void *stream)
{
    pk_status st = check_config(cfg);
    if (st != PK_OK) return st;
    if ((st = check_cache(cache)) != PK_OK) return st;
    if ((st = check_paging(cfg, cache)) != PK_OK) return st;
    if ((st = check_state(cfg, state)) != PK_OK) return st;
    if (t0 < 0 || t1 < t0 || t1 > state->t_quant) return PK_ERR_SHAPE;
    if ((k_out && !patterns_k) || (v_out && !patterns_v)) return PK_ERR_INVALID_ARG;
    if ((k_out && !aligned16(k_out)) || (v_out && !aligned16(v_out))) return PK_ERR_ALIGNMENT;
    DequantArgs a;
    a.c = make_view(cfg, cache, state);
    a.sets.n_kv_heads = cfg->n_kv_heads;
    a.sets.seqs_per_set = cfg->seqs_per_set;
    a.patterns_k = static_cast<const __half *>(patterns_k);
    a.patterns_v = static_cast<const __half *>(patterns_v);
    a.n_streams = cfg->n_seq * cfg->n_kv_heads;
    a.P = cfg->n_patterns;
    a.bits = cfg->bits;
    a.G = cfg->group;
    a.d = cfg->head_dim;
    a.v_thresholded = cfg->v_rho > 0.f ? 1 : 0;
    a.t0 = t0;
    a.t1 = t1;
    a.k_out = k_out;
    a.v_out = v_out;
    return launch_dequant(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PK_OK : PK_ERR_DEVICE;
}

}  // extern "C"
