"""pk_decode_attention_noalloc (the entry point for callers that cannot allocate: partial results in a fixed
array of the library) against pk_decode_attention with a caller's workspace, through the C ABI.

Two calls in a row share the array, the second on a smaller input: the same kernels run on both sides with the
same split of the context, so the outputs must agree bit for bit; the attention bar of the parity tests
(2e-3 relative L2 per sequence and query head) is asserted as well.  A decode whose partials do not fit the
array is refused before any launch.
"""
import ctypes as C

import numpy as np
import pytest

from paper_2510_05176_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def pk():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2510_05176_amd import patternkv
    return patternkv


def dev(a_f16):
    return torch.from_numpy(np.ascontiguousarray(a_f16).view(np.int16)).cuda().view(torch.float16)


def build_case(pk, seed, n_seq, hkv, hq, T, P, bits, G, R, F, prefix_T=0, d=128):
    """Mine, append and return everything one decode call needs (all on the GPU, through the library)."""
    cap = -(-T // F) * F
    cfg = pk.Config(n_seq=n_seq, n_kv_heads=hkv, n_q_heads=hq, head_dim=d, n_patterns=P, seqs_per_set=0, bits=bits,
                    group=G, recent=R, flush=F, t_capacity=cap, metric=pk.METRIC_L2)
    K, V = synth.make_kv(seed, synth.KVSpec(1, n_seq, hkv, hq, T, d, 8))
    Kd, Vd = dev(K), dev(V)
    Mk = pk.pk_mine_patterns(cfg, Kd[0], 3)
    Mv = pk.pk_mine_patterns(cfg, Vd[0], 3)
    cache = pk.Cache(cfg)
    pk.pk_quantize_append(cfg, cache, Kd, Vd, Mk, Mv)
    prefix = None
    if prefix_T:
        pcfg = pk.Config(n_seq=1, n_kv_heads=hkv, n_q_heads=hq, head_dim=d, n_patterns=P, seqs_per_set=0, bits=bits,
                         group=G, recent=R, flush=F, t_capacity=-(-prefix_T // F) * F, metric=pk.METRIC_L2)
        Kp, Vp = synth.make_kv(seed + 100, synth.KVSpec(1, 1, hkv, hq, prefix_T, d, 8))
        prefix = pk.Cache(pcfg)
        pk.pk_quantize_append(pcfg, prefix, dev(Kp), dev(Vp), Mk, Mv)
    q = dev(synth.make_queries(seed, n_seq, hq, d))
    return cfg, cache, prefix, q, Mk, Mv


def both_ways(pk, case):
    cfg, cache, prefix, q, Mk, Mv = case
    scale = float(q.shape[-1]) ** -0.5
    lse_a = torch.empty(q.shape[:2], dtype=torch.float32, device="cuda")
    lse_b = torch.empty_like(lse_a)
    want = pk.pk_decode_attention(cfg, cache, q, scale, Mk, Mv, lse=lse_a, prefix=prefix)
    got = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    pk.pk_decode_attention_noalloc(cfg, cache, q, scale, Mk, Mv, got, lse=lse_b, prefix=prefix)
    torch.cuda.synchronize()
    want, got = want.cpu().numpy().astype(np.float64), got.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = np.linalg.norm(got - want, axis=-1) / np.maximum(np.linalg.norm(want, axis=-1), 1e-30)
    assert err.max() <= 2e-3, err.max()                       # the parity bar, per (sequence, query head)
    assert np.array_equal(got, want)                          # and in fact the same bits
    assert np.array_equal(lse_a.cpu().numpy(), lse_b.cpu().numpy())


def test_noalloc_matches_workspace_call_twice_in_a_row(pk):
    big = build_case(pk, 11, n_seq=3, hkv=2, hq=8, T=4096 + 200, P=32, bits=2, G=64, R=64, F=128, prefix_T=640)
    small = build_case(pk, 12, n_seq=1, hkv=2, hq=8, T=330, P=32, bits=2, G=64, R=0, F=64)
    both_ways(pk, big)
    both_ways(pk, small)     # smaller input over the array the first call left behind
    both_ways(pk, big)
    # the other kernels that write partials: two groups of query heads per KV head, and the plain kernels of
    # head dimension 256
    both_ways(pk, build_case(pk, 13, n_seq=2, hkv=1, hq=16, T=900, P=16, bits=2, G=64, R=16, F=64))
    both_ways(pk, build_case(pk, 14, n_seq=2, hkv=2, hq=4, T=1100, P=16, bits=4, G=128, R=0, F=128, prefix_T=300, d=256))
    both_ways(pk, small)


def test_noalloc_refuses_partials_beyond_the_array(pk):
    # 4096 streams x 32768 tokens: 6 slots x 4 heads x (128 + 128 + 2) floats per stream > 32 MiB.  The refusal comes
    # from the host-side size check, before any launch: the cache pointers below are never dereferenced.
    cfg = pk.Config(n_seq=512, n_kv_heads=8, n_q_heads=32, head_dim=128, n_patterns=128, seqs_per_set=16, bits=2,
                    group=64, recent=0, flush=128, t_capacity=32768, metric=pk.METRIC_L2)
    need = pk.pk_workspace_bytes(cfg, pk.OP_DECODE, 32768, 0)
    assert need > pk.NOALLOC_SCRATCH_BYTES
    fake = pk._Cache(*[0x10000 * (i + 1) for i in range(10)])
    state = pk._State(32768, 0, 0)
    cc = cfg.c()
    q = torch.zeros(16, dtype=torch.float16, device="cuda")
    st = pk._lib.pk_decode_attention_noalloc(C.byref(cc), C.byref(fake), C.byref(state), None, None, None,
                                             C.c_void_p(q.data_ptr()), C.c_float(0.1), C.c_void_p(q.data_ptr()),
                                             C.c_void_p(q.data_ptr()), C.c_void_p(q.data_ptr()), None, None)
    assert st == 7, pk.pk_status_string(st)   # PK_ERR_WORKSPACE
