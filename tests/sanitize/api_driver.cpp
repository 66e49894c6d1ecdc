// Host side of the C ABI (pk_api.hip: argument checks, layout and workspace arithmetic, state updates) under
// AddressSanitizer / UndefinedBehaviorSanitizer, without a GPU: the kernel launchers are replaced by the stubs
// below, which record that they were reached, so every pointer handed over may be fake.  Built and run by
// tests/test_sanitizers_cpu.py; prints "ok" and exits 0.
#include <cstdio>
#include <cstring>

#include "pk_internal.h"

namespace pk {
static int g_launches = 0;
hipError_t launch_quantize_k(const QuantArgs &, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_quantize_v(const QuantArgs &, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_tail_copy(const TailCopyArgs &, hipStream_t) { ++g_launches; return hipSuccess; }
static int32_t g_table[64][kSeqEntry], g_after[64][3];
hipError_t launch_seq_table(const SeqTableArgs &a, hipStream_t)
{
    ++g_launches;
    for (int i = 0; i < a.count && a.first + i < 64; ++i) {
        std::memcpy(g_table[a.first + i], a.entry[i], sizeof(g_table[0]));
        std::memcpy(g_after[a.first + i], a.state[i], sizeof(g_after[0]));
    }
    return hipSuccess;
}
hipError_t launch_mine(const MineArgs &, hipStream_t) { ++g_launches; return hipSuccess; }
int mine_tsplit(int T, int, int) { return (T + 255) / 256; }
hipError_t launch_window_pattern(const __half *, int64_t, int, int, __half *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_generic_window_pattern(const __half *, int64_t, int, int, int, __half *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_decode(const DecodeArgs &, hipStream_t) { ++g_launches; return hipSuccess; }
int decode_chunk(int64_t, int64_t, int, int) { return 256; }
hipError_t launch_dequant(const DequantArgs &, hipStream_t) { ++g_launches; return hipSuccess; }
}  // namespace pk

#define CHECK(cond)                                                  \
    do {                                                             \
        if (!(cond)) {                                               \
            std::printf("failed at line %d: %s\n", __LINE__, #cond); \
            return 1;                                                \
        }                                                            \
    } while (0)

int main()
{
    pk_config c;
    std::memset(&c, 0, sizeof(c));
    c.n_seq = 2; c.n_kv_heads = 2; c.n_q_heads = 8; c.head_dim = 128; c.n_patterns = 16; c.bits = 2; c.group = 64;
    c.recent = 32; c.flush = 128; c.t_capacity = 1024; c.metric = PK_METRIC_L2;
    pk_layout lay;
    CHECK(pk_cache_layout(&c, &lay) == PK_OK && lay.total > 0 && lay.align == 16);
    CHECK(pk_cache_layout(nullptr, &lay) == PK_ERR_INVALID_ARG);
    pk_config bad = c;
    bad.head_dim = 64;
    CHECK(pk_cache_layout(&bad, &lay) == PK_ERR_UNSUPPORTED);
    bad = c; bad.t_capacity = 1000;
    CHECK(pk_cache_layout(&bad, &lay) == PK_ERR_SHAPE);
    CHECK(pk_workspace_bytes(&c, PK_OP_DECODE, 1024, 0) >= pk_workspace_bytes(&c, PK_OP_DECODE, 256, 0));
    CHECK(pk_workspace_bytes(&c, PK_OP_MINE, 4096, 4) > 0 && pk_workspace_bytes(&c, PK_OP_MINE, -1, 4) == 0);

    char *base = reinterpret_cast<char *>(0x100000);   // never dereferenced: the launchers are stubs
    pk_cache k = {base, base + 0x1000, base + 0x2000, base + 0x3000, base + 0x4000,
                  base + 0x5000, base + 0x6000, base + 0x7000, base + 0x8000, base + 0x9000};
    pk_state st = {0, 0, 0};
    // appends: bookkeeping of the fp16 window and the flushes
    CHECK(pk_quantize_append(&c, &k, &st, base, base, 100, 0, base, base, nullptr, 0, nullptr) == PK_OK);
    CHECK(st.t_quant == 0 && st.t_tail == 100);
    CHECK(pk_quantize_append(&c, &k, &st, base, base, 300, 0, base, base, nullptr, 0, nullptr) == PK_OK);
    CHECK(st.t_quant == 256 && st.t_tail == 144 && st.tail_start == 256 % 160);
    const pk_state before = st;
    CHECK(pk_quantize_append(&c, &k, &st, base, base, 4000, 0, base, base, nullptr, 0, nullptr) == PK_ERR_CAPACITY);
    CHECK(std::memcmp(&before, &st, sizeof(st)) == 0);
    CHECK(pk_quantize_append(&c, &k, &st, base + 2, base, 1, 0, base, base, nullptr, 0, nullptr) == PK_ERR_ALIGNMENT);
    pk_state wrong = {100, 0, 0};
    CHECK(pk_quantize_append(&c, &k, &wrong, base, base, 1, 0, base, base, nullptr, 0, nullptr) == PK_ERR_STATE);
    // one append for sequences at different fill: every sequence's plan is what the uniform call would do for it
    {
        pk_state ss[2] = {{0, 0, 0}, {256, 144, 96}};
        const int32_t nn[2] = {100, 300};
        const size_t wa = pk_workspace_bytes(&c, PK_OP_APPEND, 0, 0);
        CHECK(wa == 2 * 32);
        CHECK(pk_quantize_append_ragged(&c, &k, ss, base, base, nn, 0, base, base, nullptr, base, wa, nullptr) == PK_OK);
        CHECK(ss[0].t_quant == 0 && ss[0].t_tail == 100 && ss[0].tail_start == 0);
        CHECK(ss[1].t_quant == 256 + 384 && ss[1].t_tail == 444 - 384 && ss[1].tail_start == (96 + 384) % 160);
        CHECK(pk::g_table[1][pk::kSeqNq] == 384 && pk::g_table[1][pk::kSeqT0] == 256 && pk::g_table[1][pk::kSeqI0] == 384 &&
              pk::g_table[1][pk::kSeqI1] == 444 && pk::g_table[0][pk::kSeqNq] == 0 && pk::g_table[0][pk::kSeqI1] == 100);
        CHECK(pk::g_after[1][0] == 640 && pk::g_after[1][1] == 60);
        const pk_state keep0 = ss[0], keep1 = ss[1];
        const int32_t too_many[2] = {1, 4000};
        CHECK(pk_quantize_append_ragged(&c, &k, ss, base, base, too_many, 0, base, base, nullptr, base, wa, nullptr) == PK_ERR_CAPACITY);
        CHECK(std::memcmp(&keep0, &ss[0], sizeof(keep0)) == 0 && std::memcmp(&keep1, &ss[1], sizeof(keep1)) == 0);
        CHECK(pk_quantize_append_ragged(&c, &k, ss, base, base, nn, 0, base, base, nullptr, base, wa - 1, nullptr) == PK_ERR_WORKSPACE);
        const int32_t neg[2] = {1, -1};
        CHECK(pk_quantize_append_ragged(&c, &k, ss, base, base, neg, 0, base, base, nullptr, base, wa, nullptr) == PK_ERR_INVALID_ARG);
        const int32_t none[2] = {0, 0};
        CHECK(pk_quantize_append_ragged(&c, &k, ss, nullptr, nullptr, none, 0, nullptr, nullptr, nullptr, base, wa, nullptr) == PK_OK);
        CHECK(std::memcmp(&keep0, &ss[0], sizeof(keep0)) == 0);
    }
    // decode: workspace check, prefix consistency
    const size_t ws = pk_workspace_bytes(&c, PK_OP_DECODE, st.t_quant + st.t_tail, 0);
    float *out = reinterpret_cast<float *>(base);
    CHECK(pk_decode_attention(&c, &k, &st, nullptr, nullptr, nullptr, base, 0.1f, base, base, out, nullptr, base, ws, nullptr) == PK_OK);
    CHECK(pk_decode_attention(&c, &k, &st, nullptr, nullptr, nullptr, base, 0.1f, base, base, out, nullptr, base, 16, nullptr) == PK_ERR_WORKSPACE);
    pk_config pc = c;
    pc.n_seq = 1; pc.group = 32;
    pk_state pst = {0, 0, 0};
    CHECK(pk_decode_attention(&c, &k, &st, &pc, &k, &pst, base, 0.1f, base, base, out, nullptr, base, ws, nullptr) == PK_ERR_SHAPE);
    int32_t *seq_states = reinterpret_cast<int32_t *>(base);
    pk_state bound = {256, 159, 0};
    CHECK(pk_decode_attention_ragged(&c, &k, &bound, seq_states, nullptr, nullptr, nullptr, base, 0.1f, base, base, out, nullptr, base,
                                     pk_workspace_bytes(&c, PK_OP_DECODE, 415, 0), nullptr) == PK_OK);
    // mining, window pattern, dequantize
    const size_t wm = pk_workspace_bytes(&c, PK_OP_MINE, 4096, 4);
    CHECK(pk_mine_patterns(&c, base, 4096 * 128, 4, 4096, 5, 0, base, nullptr, nullptr, base, wm, nullptr) == PK_OK);
    CHECK(pk_mine_patterns(&c, base, 4096 * 128, 4, 8, 5, 0, base, nullptr, nullptr, base, wm, nullptr) == PK_ERR_SHAPE);
    CHECK(pk_window_pattern(base, 128 * 128, 4, 128, 128, base, 128, nullptr) == PK_OK);
    CHECK(pk_window_pattern(base, 128 * 128, 4, 128, 64, base, 128, nullptr) == PK_ERR_UNSUPPORTED);
    CHECK(pk_window_pattern(base, 128 * 96, 4, 128, 96, base, 96, nullptr) == PK_OK);
    CHECK(pk_dequantize(&c, &k, &st, base, base, 0, 256, out, out, nullptr) == PK_OK);
    CHECK(pk_dequantize(&c, &k, &st, base, base, 0, 512, out, out, nullptr) == PK_ERR_SHAPE);
    CHECK(pk::g_launches > 0);
    std::puts("ok");
    return 0;
}
