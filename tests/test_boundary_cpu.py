"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header
declares, computes layouts / workspace sizes, and turns bad arguments into status codes before any launch.
(Every error below is detected on the host; no kernel is ever launched from this file.)"""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "patternkv.h")
PROBE_HEADER = os.path.join(ROOT, "include", "patternkv_probe.h")
LIB = os.path.join(ROOT, "paper_2510_05176_amd", "libpatternkv.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libpatternkv.so not built")


@pytest.fixture(scope="module")
def pk():
    from paper_2510_05176_amd import patternkv
    return patternkv


def test_exports_every_declared_symbol(pk):
    src = open(HEADER).read() + open(PROBE_HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = set(re.findall(r"\b(pk_[a-z0-9_]+)\s*\(", src))
    assert {"pk_mine_patterns", "pk_quantize_append", "pk_quantize_append_ragged", "pk_decode_attention", "pk_dequantize", "pk_cache_layout",
            "pk_workspace_bytes", "pk_decode_plan", "pk_status_string", "pk_abi_version", "pk_window_pattern",
            "pk_decode_attention_ragged", "pk_decode_attention_noalloc", "pk_probe_read", "pk_probe_copy",
            "pk_probe_fma_f32", "pk_probe_mfma_f16", "pk_probe_divisions"} <= names
    lib = C.CDLL(LIB)
    for n in names:
        assert hasattr(lib, n), n
    assert pk.pk_abi_version() == 5


def test_status_strings(pk):
    seen = {pk.pk_status_string(s) for s in range(9)}
    assert len(seen) == 9 and "ok" in seen


def test_layout_byte_counts(pk):
    cfg = pk.Config(n_seq=2, n_kv_heads=8, n_q_heads=32, n_patterns=64, bits=2, group=64, recent=128, flush=128,
                    t_capacity=8192)
    lay = pk.pk_cache_layout(cfg)
    N = 16
    assert lay["k_codes"] == lay["v_codes"] == N * 8192 * 128 * 2 // 8
    assert lay["k_scale"] == lay["k_zero"] == N * (8192 // 64) * 128 * 2
    assert lay["v_scale"] == lay["v_zero"] == N * 8192 * 2 * 2
    assert lay["k_idx"] == lay["v_idx"] == N * 8192
    assert lay["tail_k"] == lay["tail_v"] == N * 256 * 128 * 2
    assert lay["align"] == 16
    # packed bytes per token and KV head (K+V, with parameters and index): 82 B at 2 bits, group 64
    per_tok = sum(lay[n] for n in ("k_codes", "k_scale", "k_zero", "k_idx", "v_codes", "v_scale", "v_zero", "v_idx")) / (N * 8192)
    assert per_tok == 82
    cfg4 = pk.Config(n_seq=1, n_kv_heads=1, n_q_heads=1, bits=4, group=64, flush=64, t_capacity=64)
    lay4 = pk.pk_cache_layout(cfg4)
    assert sum(lay4[n] for n in ("k_codes", "k_scale", "k_zero", "k_idx", "v_codes", "v_scale", "v_zero", "v_idx")) / 64 == 146


@pytest.mark.parametrize("field,value,status", [
    ("head_dim", 64, 2), ("bits", 3, 2), ("group", 48, 2), ("n_patterns", 257, 2), ("n_patterns", 0, 1),
    ("n_q_heads", 5, 3), ("n_q_heads", 260, 2), ("flush", 96, 3), ("t_capacity", 100, 3), ("metric", 7, 1),
    ("recent", -1, 1), ("n_seq", 0, 1), ("n_seq", 70000, 2),
    ("v_rho", -0.1, 1), ("v_rho", 1.0, 1), ("v_rho", float("nan"), 1),
])
def test_bad_config_is_refused(pk, field, value, status):
    kw = dict(n_seq=1, n_kv_heads=4, n_q_heads=4, n_patterns=16, bits=2, group=64, recent=0, flush=64, t_capacity=1024)
    kw[field] = value
    with pytest.raises(pk.PkError) as e:
        pk.pk_cache_layout(pk.Config(**kw))
    assert e.value.status == status
    assert pk.pk_workspace_bytes(pk.Config(**kw), pk.OP_DECODE, 1024) == 0


def test_paged_layout_and_its_config_checks(pk):
    """A paged configuration: the packed arrays are sized by the pool (n_pages x heads x page_tokens token slots), the
    tails by the streams; page sizes that a group or block could straddle, or that do not divide the capacity, are
    refused; a paged cache without a page table is refused before any launch."""
    kw = dict(n_seq=3, n_kv_heads=4, n_q_heads=8, n_patterns=16, bits=2, group=64, recent=32, flush=128, t_capacity=2048)
    lay = pk.pk_cache_layout(pk.Config(**kw, page_tokens=256, n_pages=10))
    slots = 10 * 4 * 256
    assert lay["k_codes"] == lay["v_codes"] == slots * 128 * 2 // 8
    assert lay["k_scale"] == slots // 64 * 128 * 2 and lay["v_scale"] == slots * 2 * 2 and lay["k_idx"] == slots
    assert lay["tail_k"] == 3 * 4 * 160 * 128 * 2
    for bad, status in [(dict(page_tokens=64, n_pages=10), 2), (dict(page_tokens=192, n_pages=10), 2),
                        (dict(page_tokens=4096, n_pages=10), 3), (dict(page_tokens=256, n_pages=0), 1),
                        (dict(page_tokens=-128, n_pages=4), 1)]:
        with pytest.raises(pk.PkError) as e:
            pk.pk_cache_layout(pk.Config(**kw, **bad))
        assert e.value.status == status, bad
    lib = C.CDLL(LIB)
    cfg = pk.Config(**kw, page_tokens=256, n_pages=10).c()
    cache, state = _fake_cache(pk), pk._State(0, 0, 0)          # page_table left NULL
    good = C.c_void_p(0x2000)
    st = lib.pk_quantize_append(C.byref(cfg), C.byref(cache), C.byref(state), good, good, C.c_int32(8), C.c_int64(0), good, good,
                                None, C.c_size_t(0), None)
    assert st == 1 and (state.t_quant, state.t_tail) == (0, 0)


def test_other_head_dimensions_in_the_layout_and_checks(pk):
    """Head dimensions 96 and 256: the layout formulas carry d, V's channel groups of min(G, d) must tile the head,
    the ragged append sizes its stride check by d."""
    kw = dict(n_seq=2, n_kv_heads=2, n_q_heads=4, n_patterns=16, bits=2, recent=0, flush=128, t_capacity=1024)
    lay = pk.pk_cache_layout(pk.Config(**kw, head_dim=256, group=64))
    N = 4
    assert lay["k_codes"] == lay["v_codes"] == N * 1024 * 256 * 2 // 8
    assert lay["k_scale"] == N * (1024 // 64) * 256 * 2 and lay["v_scale"] == N * 1024 * 4 * 2
    assert lay["tail_k"] == N * 128 * 256 * 2
    lay = pk.pk_cache_layout(pk.Config(**kw, head_dim=96, group=128))
    assert lay["k_codes"] == N * 1024 * 96 * 2 // 8 and lay["v_scale"] == N * 1024 * 1 * 2   # one V group of 96 channels
    with pytest.raises(pk.PkError) as e:
        pk.pk_cache_layout(pk.Config(**kw, head_dim=96, group=64))
    assert e.value.status == 2
    assert pk.pk_workspace_bytes(pk.Config(**kw, head_dim=256, group=64), pk.OP_MINE, 4096, 2) > \
        pk.pk_workspace_bytes(pk.Config(**kw, head_dim=128, group=64), pk.OP_MINE, 4096, 2)
    lib = C.CDLL(LIB)
    cfg = pk.Config(**kw, head_dim=256, group=64).c()
    cache = _fake_cache(pk)
    states = (pk._State * 2)(pk._State(0, 0, 0), pk._State(0, 0, 0))
    n_new = (C.c_int32 * 2)(8, 8)
    good = C.c_void_p(0x2000)
    # a stream stride that holds 8 vectors of 128 channels is too short for 8 vectors of 256: refused before any launch
    st = lib.pk_quantize_append_ragged(C.byref(cfg), C.byref(cache), states, good, good, n_new, C.c_int64(8 * 128), good, good,
                                       None, good, C.c_size_t(1024), None)
    assert st == 3


def test_v_threshold_needs_a_free_index(pk):
    # the adaptive threshold marks raw-quantized V tokens with index 255 (PK_NO_PATTERN)
    kw = dict(n_seq=1, n_kv_heads=4, n_q_heads=4, bits=2, group=64, recent=0, flush=64, t_capacity=1024, v_rho=0.9)
    pk.pk_cache_layout(pk.Config(n_patterns=255, **kw))
    with pytest.raises(pk.PkError) as e:
        pk.pk_cache_layout(pk.Config(n_patterns=256, **kw))
    assert e.value.status == 2
    assert pk.NO_PATTERN == 255


def test_workspace_sizes_are_monotone(pk):
    cfg = pk.Config(n_seq=4, n_kv_heads=8, n_q_heads=32, n_patterns=64, flush=64, t_capacity=1 << 20)
    prev = 0
    for t in [0, 1, 255, 256, 1000, 4096, 8192, 70000, 1 << 20]:
        w = pk.pk_workspace_bytes(cfg, pk.OP_DECODE, t, 0)
        assert w >= prev and w > 0
        assert pk.pk_workspace_bytes(cfg, pk.OP_DECODE, t, 4096) >= w
        prev = w
    prev = 0
    for t in [64, 1000, 8192, 131072]:
        w = pk.pk_workspace_bytes(cfg, pk.OP_MINE, t, 16)
        assert w > prev
        prev = w
    assert pk.pk_workspace_bytes(cfg, pk.OP_APPEND, 128) == 4 * 32   # the per-sequence table of the ragged form


def test_decode_plan_fits_the_workspace_bound(pk):
    """The split chooser of decode against the size the caller is told to allocate: for every stream count, context
    length (up to the largest capacity, with and without a shared prefix), table size and head ratio tried, the
    split is a positive multiple of 256 of at most 32768 tokens and the partial slots in use fit the workspace that
    pk_workspace_bytes reports for the same context."""
    n_cases = 0
    for n_seq, hkv in [(1, 1), (1, 4), (2, 1), (1, 8), (37, 1), (32, 8), (432, 1), (75, 8), (512, 8), (1500, 8)]:
        for P, r, G in [(1, 1, 64), (64, 4, 64), (128, 8, 64), (256, 7, 128), (64, 4, 32)]:
            cfg = pk.Config(n_seq=n_seq, n_kv_heads=hkv, n_q_heads=hkv * r, n_patterns=P, bits=2, group=G, recent=0,
                            flush=128, t_capacity=1 << 25)
            for t in [0, 128, 256, 1024, 4096, 8192, 12288, 32640, 32768, 65536, 131072, 1 << 20, (1 << 24) + 128, 1 << 25]:
                for pre in [0, 4096, 100096]:
                    split, slots, need = pk.pk_decode_plan(cfg, t, pre)
                    assert 0 < split <= 32768 and split % 256 == 0
                    assert slots == -(-t // split) + -(-pre // split) + 2
                    assert need <= pk.pk_workspace_bytes(cfg, pk.OP_DECODE, t, pre), (n_seq, hkv, P, r, t, pre, split, slots)
                    n_cases += 1
    assert n_cases == 10 * 5 * 14 * 3


def _fake_cache(pk, base=0x1000):
    return pk._Cache(*[base + 0x100 * i for i in range(10)])


def test_append_argument_errors_before_launch(pk):
    lib = pk._lib
    cfg = pk.Config(n_seq=1, n_kv_heads=2, n_q_heads=2, n_patterns=8, flush=64, group=64, t_capacity=128).c()
    cache, state = _fake_cache(pk), pk._State(0, 0, 0)
    good = C.c_void_p(0x2000)
    call = lambda **kw: lib.pk_quantize_append(
        C.byref(kw.get("cfg", cfg)), C.byref(kw.get("cache", cache)), C.byref(kw.get("state", state)),
        kw.get("k", good), kw.get("v", good), kw.get("n", 64), kw.get("stride", 0), kw.get("pk", good),
        kw.get("pv", good), None, 0, None)
    assert call(n=-1) == 1
    assert call(k=None) == 1
    assert call(k=C.c_void_p(0x2008)) == 4                      # misaligned
    assert call(cache=pk._Cache(*([0x1000] * 9 + [0]))) == 1     # a NULL cache array
    assert call(cache=pk._Cache(*([0x1000] * 9 + [0x1004]))) == 4
    assert call(state=pk._State(32, 0, 0)) == 6                  # t_quant not a multiple of flush
    assert call(state=pk._State(0, 64, 0)) == 6                  # tail longer than the ring allows
    assert call(state=pk._State(0, 0, 64)) == 6
    assert call(n=64, stride=100) == 3                           # stream stride shorter than the rows
    assert call(state=pk._State(128, 0, 0), n=64) == 5           # would exceed t_capacity
    st = pk._State(64, 0, 0)
    assert call(state=st, n=200) == 5 and (st.t_quant, st.t_tail, st.tail_start) == (64, 0, 0)   # state untouched
    assert call(n=0) == 0                                        # zero-length append is a no-op


def test_decode_and_mine_argument_errors_before_launch(pk):
    lib = pk._lib
    cfg = pk.Config(n_seq=1, n_kv_heads=2, n_q_heads=8, n_patterns=8, flush=64, group=64, t_capacity=128)
    c, cache, state = cfg.c(), _fake_cache(pk), pk._State(64, 3, 0)
    good = C.c_void_p(0x2000)

    def dec(**kw):
        return lib.pk_decode_attention(C.byref(c), C.byref(cache), C.byref(kw.get("state", state)),
                                       kw.get("pcfg"), kw.get("pcache"), kw.get("pstate"), kw.get("q", good),
                                       C.c_float(0.1), good, good, kw.get("out", good), None, kw.get("ws", good),
                                       kw.get("wsb", 0), None)
    assert dec(q=None) == 1
    assert dec(out=C.c_void_p(0x2004)) == 4
    assert dec(wsb=0) == 7                                       # workspace too small
    assert dec(ws=None, wsb=1 << 30) == 7
    pc = pk.Config(n_seq=1, n_kv_heads=2, n_q_heads=8, n_patterns=8, flush=64, group=32, t_capacity=128).c()
    assert dec(pcfg=C.byref(pc)) == 1                            # prefix arguments must come together
    pcache, pstate = _fake_cache(pk, 0x9000), pk._State(64, 0, 0)
    assert dec(pcfg=C.byref(pc), pcache=C.byref(pcache), pstate=C.byref(pstate), wsb=1 << 30) == 3   # group differs
    assert dec(state=pk._State(64, 64, 0)) == 6

    def rag(**kw):
        return lib.pk_decode_attention_ragged(C.byref(c), C.byref(cache), C.byref(kw.get("bound", state)),
                                              kw.get("states", good), None, None, None, kw.get("q", good), C.c_float(0.1),
                                              good, good, good, None, kw.get("ws", good), kw.get("wsb", 0), None)
    assert rag(states=None) == 1
    assert rag(states=C.c_void_p(0x2004)) == 4
    assert rag(bound=pk._State(64, 3, 5)) == 6                   # the bound carries no ring position
    assert rag(bound=pk._State(70, 3, 0)) == 6                   # not a multiple of flush
    assert rag(q=None) == 1
    assert rag(wsb=0) == 7

    def mine(**kw):
        return lib.pk_mine_patterns(C.byref(c), kw.get("x", good), kw.get("stride", 64 * 128), kw.get("S", 2),
                                    kw.get("T", 64), kw.get("iters", 3), 0, kw.get("pat", good), None, None,
                                    kw.get("ws", good), kw.get("wsb", 0), None)
    assert mine(x=None) == 1
    assert mine(T=4) == 3                                        # fewer vectors than patterns
    assert mine(stride=100) == 3
    assert mine(pat=C.c_void_p(0x2002)) == 4
    assert mine(wsb=16) == 7
    assert mine(iters=-1) == 1

    def deq(**kw):
        return lib.pk_dequantize(C.byref(c), C.byref(cache), C.byref(state), good, good, kw.get("t0", 0),
                                 kw.get("t1", 64), kw.get("k", good), good, None)
    assert deq(t1=65) == 3 and deq(t0=10, t1=5) == 3 and deq(k=C.c_void_p(0x2004)) == 4


def test_window_pattern_argument_errors_before_launch(pk):
    lib = pk._lib
    good, odd = C.c_void_p(0x2000), C.c_void_p(0x2002)

    def wp(x=good, ss=128 * 16, n_sets=2, n=16, d=128, out=good, os=128):
        return lib.pk_window_pattern(x, ss, n_sets, n, d, out, os, None)
    assert wp(x=None) == 1 and wp(out=None) == 1 and wp(n=0) == 1 and wp(n_sets=0) == 1
    assert wp(d=64) == 2
    assert wp(x=odd) == 4 and wp(out=odd) == 4 and wp(ss=100) == 4 and wp(os=130) == 4
