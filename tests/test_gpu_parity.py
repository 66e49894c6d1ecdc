"""GPU-vs-oracle parity of the three hot-path calls, through the C ABI, on seeded synthetic KV.

Bars (the benchmark contract's): pattern indices bit-exact except where the oracle's top-2 distance gap
is < 1e-4 relative; given equal assignments, codes / packed bytes / fp16 scale and zero bit-exact;
reconstructed KV within 1e-3 absolute; attention outputs within 2e-3 relative L2.
"""
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


def host_u16(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


CACHE_ARRAYS = ("k_codes", "k_scale", "k_zero", "k_idx", "v_codes", "v_scale", "v_zero", "v_idx", "tail_k", "tail_v")


def gpu_arrays(gc, ocache):
    """GPU cache arrays as numpy arrays shaped like the oracle's."""
    out = {}
    for n in CACHE_ARRAYS:
        ref = getattr(ocache, n)
        raw = gc.array(n).cpu().numpy()
        out[n] = raw.view(ref.dtype).reshape(ref.shape)
    return out


def upload(gc, ocache):
    """Copy the oracle's cache into the GPU cache (to test decode on identical inputs)."""
    for n in CACHE_ARRAYS:
        raw = np.ascontiguousarray(getattr(ocache, n)).view(np.uint8).reshape(-1)
        gc.buf[n][: raw.size] = torch.from_numpy(raw.copy()).cuda()
    gc.state.t_quant, gc.state.t_tail, gc.state.tail_start = ocache.t_quant, ocache.t_tail, ocache.tail_start


def make_case(oracle, pk, seed, *, n_seq=1, hkv=2, hq=2, T=320, P=16, bits=2, G=64, R=0, F=None, metric=0,
              seqs_per_set=0, n_clusters=8, cap=None, mine_iters=3, v_rho=0.0):
    F = max(G, 64) if F is None else F
    cap = cap if cap is not None else -(-T // F) * F
    kw = dict(n_seq=n_seq, n_kv_heads=hkv, n_q_heads=hq, head_dim=128, n_patterns=P, seqs_per_set=seqs_per_set,
              bits=bits, group=G, recent=R, flush=F, t_capacity=cap, metric=metric, v_rho=v_rho)
    spec = synth.KVSpec(1, n_seq, hkv, hq, T, 128, n_clusters)
    K, V = synth.make_kv(seed, spec)
    ocfg, gcfg = oracle.Config(**kw), pk.Config(**kw)
    # patterns: oracle-mined on the first sequences of each set (inputs to both sides)
    set_of = ocfg.set_of()
    first_stream = [int(np.flatnonzero(set_of == s)[0]) for s in range(ocfg.n_sets)]
    Kf, Vf = K.reshape(-1, T, 128), V.reshape(-1, T, 128)
    Mk, _, _, _ = oracle.mine(Kf[first_stream].view(np.uint16), P, mine_iters)
    Mv, _, _, _ = oracle.mine(Vf[first_stream].view(np.uint16), P, mine_iters)
    return kw, ocfg, gcfg, K, V, Mk, Mv


def run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, pieces):
    oc, gc = oracle.Cache(ocfg), pk.Cache(gcfg)
    Kd, Vd = dev(K), dev(V)
    Mkd, Mvd = dev(Mk.view(np.float16)), dev(Mv.view(np.float16))
    pos = 0
    for n in pieces:
        oc.append(K[:, :, pos:pos + n].view(np.uint16), V[:, :, pos:pos + n].view(np.uint16), Mk, Mv)
        pk.pk_quantize_append(gcfg, gc, Kd[:, :, pos:pos + n], Vd[:, :, pos:pos + n], Mkd, Mvd)
        pos += n
        assert (gc.t_quant, gc.t_tail, gc.tail_start) == (oc.t_quant, oc.t_tail, oc.tail_start)
    torch.cuda.synchronize()
    return oc, gc, Mkd, Mvd


def compare_caches(oracle, oc, gc, metric):
    """Returns the number of tokens whose assignment differs (all inside the exemption band)."""
    cfg = oc.cfg
    N, d, b, G, tq = cfg.n_streams, cfg.head_dim, cfg.bits, cfg.group, oc.t_quant
    g = gpu_arrays(gc, oc)
    n_diff = 0
    for side in "kv" if tq else "":   # nothing packed yet: only the tails are compared
        oi, gi = getattr(oc, side + "_idx")[:, :tq], g[side + "_idx"][:, :tq]
        diff = oi != gi
        if diff.any():
            best, second = getattr(oc, side + "_best")[:, :tq], getattr(oc, side + "_second")[:, :tq]
            gap = (second - best) / np.maximum(second, 1e-30)
            assert metric == 0, "min-max selection uses exact binary32 operations on both sides"
            assert np.all(gap[diff] < 1e-4), f"{side}: assignment differs outside the near-tie band, gap {gap[diff].max()}"
            n_diff += int(diff.sum())
        same = ~diff
        if side == "k":
            grp_same = same.reshape(N, tq // G, G).all(axis=2)
            assert np.array_equal(g["k_scale"][:, :tq // G][grp_same], oc.k_scale[:, :tq // G][grp_same])
            assert np.array_equal(g["k_zero"][:, :tq // G][grp_same], oc.k_zero[:, :tq // G][grp_same])
            tok_same = np.repeat(grp_same, G, axis=1)
            assert np.array_equal(g["k_codes"][:, :tq][tok_same], oc.k_codes[:, :tq][tok_same])
        else:
            by_tok = lambda arr: arr[:, :tq // 16].transpose(0, 1, 3, 2).reshape(N, tq, -1)   # [N, t/16, groups, 16] -> [N, t, groups]
            assert np.array_equal(by_tok(g["v_scale"])[same], by_tok(oc.v_scale)[same])
            assert np.array_equal(by_tok(g["v_zero"])[same], by_tok(oc.v_zero)[same])
            bpt = d * b // 32
            if not diff.any():
                assert np.array_equal(g["v_codes"][:, :tq * bpt], oc.v_codes[:, :tq * bpt])   # packed bytes
            for s in range(N):
                cg = oracle.unpack_v(g["v_codes"][s, :tq * bpt], tq, d, b)
                co = oracle.unpack_v(oc.v_codes[s, :tq * bpt], tq, d, b)
                assert np.array_equal(cg[same[s]], co[same[s]])
    # tails (logical order)
    ring = cfg.recent + cfg.flush
    slots = (oc.tail_start + np.arange(oc.t_tail)) % ring
    assert np.array_equal(g["tail_k"][:, slots], oc.tail("k"))
    assert np.array_equal(g["tail_v"][:, slots], oc.tail("v"))
    return n_diff


def rel_l2(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b.astype(np.float64)) / max(np.linalg.norm(b.astype(np.float64)), 1e-30))


def assert_attention(got, want, elementwise=True, row_tol=2e-3):
    """The attention bar, applied to every (sequence, query head) row on its own: relative L2 error <= 2e-3, and
    (for runs on shared pattern tables) every element within 2e-3 of the row's largest magnitude."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape and np.isfinite(got).all()
    g2, w2 = got.reshape(-1, got.shape[-1]), want.reshape(-1, want.shape[-1])
    err = np.linalg.norm(g2 - w2, axis=1) / np.maximum(np.linalg.norm(w2, axis=1), 1e-30)
    assert err.max() <= row_tol, f"row {int(err.argmax())}: relative L2 error {err.max():.3e}"
    if elementwise:
        bound = row_tol * np.abs(w2).max(axis=1, keepdims=True)
        worst = (np.abs(g2 - w2) / np.maximum(bound, 1e-30)).max()
        assert worst <= 1.0, f"element error {worst:.3f} x the bound"


# ------------------------------------------------------------------------------ quantize-append

@pytest.mark.parametrize("bits,G,P,metric", [
    (2, 64, 16, 0), (4, 32, 16, 0), (2, 128, 64, 0), (4, 64, 33, 0), (2, 32, 1, 0), (2, 64, 256, 0),
    (2, 32, 200, 0), (4, 64, 128, 0), (2, 128, 130, 0),     # large tables: several tiles per pass over the table
    (2, 64, 16, 1), (4, 128, 40, 1), (2, 32, 7, 1),
])
def test_quantize_append_parity(oracle, pk, bits, G, P, metric):
    kw, ocfg, gcfg, K, V, Mk, Mv = make_case(oracle, pk, 100 + bits + G + P, T=384 + 17, P=P, bits=bits, G=G,
                                            metric=metric, n_seq=2, hkv=2, hq=2, n_clusters=max(4, min(P, 24)))
    oc, gc, Mkd, Mvd = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, [K.shape[2]])
    F = max(G, 64)
    assert oc.t_quant == (401 // F) * F and oc.t_tail == 401 - oc.t_quant
    n_diff = compare_caches(oracle, oc, gc, metric)
    assert n_diff <= 0.002 * oc.t_quant * ocfg.n_streams * 2 + 2
    # reconstruction (1e-3 absolute on tokens with equal assignment; the arithmetic is in fact identical)
    kg, vg = pk.pk_dequantize(gcfg, gc, Mkd, Mvd)
    ko, vo = oc.dequantize(Mk, Mv)
    g = gpu_arrays(gc, oc)
    tq = oc.t_quant
    same_k = np.repeat((g["k_idx"][:, :tq] == oc.k_idx[:, :tq]).reshape(ocfg.n_streams, tq // G, G).all(2), G, axis=1)
    same_v = g["v_idx"][:, :tq] == oc.v_idx[:, :tq]
    assert np.abs(kg.cpu().numpy() - ko)[same_k].max() <= 1e-3
    assert np.abs(vg.cpu().numpy() - vo)[same_v].max() <= 1e-3
    if n_diff == 0:
        assert np.array_equal(kg.cpu().numpy(), ko) and np.array_equal(vg.cpu().numpy(), vo)


@pytest.mark.parametrize("bits,G,P,metric,hq", [(2, 64, 4, 0, 8), (4, 32, 5, 0, 2), (2, 128, 3, 1, 4), (2, 32, 255, 0, 4)])
def test_v_adaptive_threshold_parity(oracle, pk, bits, G, P, metric, hq):
    """Sec. 3.3: V tokens whose flat range exceeds rho times their raw range are quantized without a pattern
    (index 255); fewer patterns than clusters make a large share of tokens take that branch."""
    rho = 0.8 if P < 255 else float(np.float32(oracle.rho_star(128, 0.05)))
    kw, ocfg, gcfg, K, V, Mk, Mv = make_case(oracle, pk, 500 + P + G, T=448, P=P, bits=bits, G=G, metric=metric,
                                            n_seq=2, hkv=2, hq=hq, n_clusters=12 if P < 255 else 40, v_rho=rho)
    oc, gc, Mkd, Mvd = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, [300, 148])
    raw_share = float((oc.v_idx[:, :oc.t_quant] == oracle.NO_PATTERN).mean())
    if P < 255:
        assert 0.05 < raw_share < 0.95
    n_diff = compare_caches(oracle, oc, gc, metric)
    assert n_diff <= 4
    assert not (oc.k_idx[:, :oc.t_quant] == oracle.NO_PATTERN).any() or P == 256   # K is never thresholded
    kg, vg = pk.pk_dequantize(gcfg, gc, Mkd, Mvd)
    ko, vo = oc.dequantize(Mk, Mv)
    if n_diff == 0:
        assert np.array_equal(kg.cpu().numpy(), ko) and np.array_equal(vg.cpu().numpy(), vo)
    q = synth.make_queries(9, 2, hq, 128)
    want, _ = oracle.decode_attention(oc, q.view(np.uint16), Mk, Mv, 128 ** -0.5)
    got = pk.pk_decode_attention(gcfg, gc, dev(q), 128 ** -0.5, Mkd, Mvd).cpu().numpy()
    assert_attention(got, want)


def test_streaming_appends_with_recent_window(oracle, pk):
    kw, ocfg, gcfg, K, V, Mk, Mv = make_case(oracle, pk, 7, T=700, P=16, bits=2, G=32, R=48, F=64, n_seq=3, hkv=2,
                                            hq=4, seqs_per_set=1, cap=704)
    pieces = [1, 1, 5, 40, 64, 100, 1, 300, 111, 77]
    assert sum(pieces) == 700
    oc, gc, Mkd, Mvd = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, pieces)
    assert oc.t_quant == 640 and oc.t_tail == 60
    compare_caches(oracle, oc, gc, 0)
    # the same tokens in one call give the same cache
    oc1, gc1, _, _ = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, [700])
    for n in ("k_codes", "k_scale", "k_zero", "k_idx", "v_codes", "v_scale", "v_zero", "v_idx"):
        assert torch.equal(gc.array(n), gc1.array(n)), n


def test_zero_residual_and_flat_groups(oracle, pk):
    # vectors that are exact copies of patterns: residual 0, scale 0, codes 0, exact reconstruction
    rng = np.random.default_rng(5)
    M = rng.standard_normal((2, 8, 128)).astype(np.float16)
    pick = rng.integers(0, 8, (1, 2, 128))
    K = np.stack([M[h][pick[0, h]] for h in range(2)])[None]
    V = K[:, ::-1].copy()
    kw = dict(n_seq=1, n_kv_heads=2, n_q_heads=2, head_dim=128, n_patterns=8, seqs_per_set=0, bits=2, group=64,
              recent=0, flush=64, t_capacity=128, metric=0)
    ocfg, gcfg = oracle.Config(**kw), pk.Config(**kw)
    Mv = M[::-1].copy()
    oc, gc, Mkd, Mvd = run_appends(oracle, pk, ocfg, gcfg, K, V, M.view(np.uint16), Mv.view(np.uint16), [128])
    assert compare_caches(oracle, oc, gc, 0) == 0
    g = gpu_arrays(gc, oc)
    assert not g["k_codes"].any() and not g["v_codes"].any() and not g["k_scale"].any() and not g["v_scale"].any()
    kg, vg = pk.pk_dequantize(gcfg, gc, Mkd, Mvd)
    assert np.array_equal(kg.cpu().numpy(), K.reshape(2, 128, 128).astype(np.float32))
    assert np.array_equal(vg.cpu().numpy(), V.reshape(2, 128, 128).astype(np.float32))


def test_append_is_reproducible_bit_for_bit(oracle, pk):
    kw, ocfg, gcfg, K, V, Mk, Mv = make_case(oracle, pk, 9, T=512, P=32, bits=2, G=64, n_seq=2, hkv=4, hq=4)
    _, g1, _, _ = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, [512])
    _, g2, _, _ = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, [512])
    for n in CACHE_ARRAYS:
        assert torch.equal(g1.array(n), g2.array(n)), n


def test_division_sequences_match_ieee_division(pk):
    """The quantizer forms s = (max - z)/(2^b - 1) and 1/s with a reciprocal estimate plus one correction step
    instead of the division instruction sequence; the codes are bit-exact only if both are correctly rounded.
    Checked here against IEEE binary32 division (numpy float32, the same operation the oracle's C code performs):
    1/s for every positive finite fp16 value, x/3 and x/15 for all 2^23 mantissas in each of seven binades that
    span fp16-sized ranges (2^-24 .. 2^17), and for every positive finite fp16 value."""
    import ctypes as C
    lib = pk._lib
    lib.pk_probe_divisions.restype = C.c_int
    lib.pk_probe_divisions.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    halves = np.arange(1, 0x7c00, dtype=np.uint16).view(np.float16).astype(np.float32)      # subnormals included
    mant = np.arange(1 << 23, dtype=np.uint32)
    sweeps = [((np.uint32(e + 127) << np.uint32(23)) | mant).view(np.float32) for e in (-24, -14, -7, -1, 0, 5, 17)]
    for x in [halves] + sweeps:
        xd = torch.from_numpy(x.copy()).cuda()
        outs = [torch.empty_like(xd) for _ in range(3)]
        rc = lib.pk_probe_divisions(xd.data_ptr(), xd.numel(), outs[0].data_ptr(), outs[1].data_ptr(), outs[2].data_ptr(),
                                    C.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0
        torch.cuda.synchronize()
        recip, by3, by15 = (o.cpu().numpy() for o in outs)
        assert np.array_equal(by3.view(np.uint32), (x / np.float32(3)).view(np.uint32))
        assert np.array_equal(by15.view(np.uint32), (x / np.float32(15)).view(np.uint32))
        if x is halves:
            assert np.array_equal(recip.view(np.uint32), (np.float32(1) / x).view(np.uint32))


# ------------------------------------------------------------------------------ decode attention

@pytest.mark.parametrize("hkv,hq,bits,G,P,R,T", [
    (2, 2, 2, 64, 16, 0, 401),        # r = 1, ragged tail
    (2, 8, 2, 64, 64, 128, 1500),     # r = 4, recent window, several tiles
    (1, 7, 2, 128, 40, 0, 1100),      # r = 7
    (1, 8, 4, 64, 16, 32, 700),       # r = 8, 4-bit
    (2, 8, 2, 32, 64, 0, 900),        # r = 4, group 32: four V channel groups, two K groups per 64-token block
    (1, 4, 4, 32, 16, 0, 333),        # 4-bit with group 32
    (2, 8, 4, 64, 64, 0, 640),        # 4-bit, r = 4, empty tail
    (1, 8, 2, 32, 16, 16, 700),       # r = 8 with group 32: 32 (head, channel group) pairs, two groups of four heads
    (2, 12, 4, 32, 24, 0, 500),       # r = 6 with group 32, 4-bit: two groups of three heads
    (1, 5, 4, 32, 8, 0, 1300),        # r = 5 with group 32, 4-bit, several splits
    (1, 16, 2, 64, 24, 32, 900),      # r = 16: two groups of eight heads
    (2, 24, 2, 128, 8, 0, 640),       # r = 12: two groups of six heads
    (1, 16, 2, 64, 8, 0, 50),         # r = 16, nothing packed yet: the tail kernel on its own, two head groups
    (1, 18, 2, 64, 8, 16, 700),       # r = 18: three groups of up to eight heads through the plain kernels
])
def test_decode_attention_parity(oracle, pk, hkv, hq, bits, G, P, R, T):
    kw, ocfg, gcfg, K, V, Mk, Mv = make_case(oracle, pk, 31 + hq + T, T=T, P=P, bits=bits, G=G, R=R, F=max(G, 64),
                                            n_seq=2, hkv=hkv, hq=hq, n_clusters=min(P, 16))
    oc, gc, Mkd, Mvd = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, [T])
    q = synth.make_queries(3, 2, hq, 128)
    scale = 128 ** -0.5
    want, want_lse = oracle.decode_attention(oc, q.view(np.uint16), Mk, Mv, scale)
    lse = torch.empty((2, hq), dtype=torch.float32, device="cuda")
    # (a) end to end: GPU-built cache
    got = pk.pk_decode_attention(gcfg, gc, dev(q), scale, Mkd, Mvd, lse=lse).cpu().numpy()
    assert_attention(got, want)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= 2e-3
    # (b) decode alone: the oracle's cache uploaded, so both sides read identical bytes
    gc2 = pk.Cache(gcfg)
    upload(gc2, oc)
    got2 = pk.pk_decode_attention(gcfg, gc2, dev(q), scale, Mkd, Mvd).cpu().numpy()
    assert_attention(got2, want)
    # reproducible
    got3 = pk.pk_decode_attention(gcfg, gc2, dev(q), scale, Mkd, Mvd).cpu().numpy()
    assert np.allclose(got2, got3, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("hkv,hq,bits,G", [(2, 8, 2, 64), (1, 8, 4, 64), (2, 8, 2, 32)])
def test_decode_large_query_and_key_range(oracle, pk, hkv, hq, bits, G):
    """Queries of magnitude ~150 against K scales of order 1..10: q * s_K exceeds 256 in many channels, which the
    fp16 operands of the score contraction (q * s * 2^8) survive only because the query is brought to [1, 2) by a
    power of two first.  The output must be finite and meet the usual bar."""
    T, P = 640, 16
    kw, ocfg, gcfg, K, V, Mk, Mv = make_case(oracle, pk, 77, T=T, P=P, bits=bits, G=G, F=max(G, 64), n_seq=2, hkv=hkv,
                                            hq=hq, n_clusters=8, mine_iters=1)
    K = (K.astype(np.float32) * 4).astype(np.float16)
    Mk = (Mk.view(np.float16).astype(np.float32) * 4).astype(np.float16).view(np.uint16)
    oc, gc, Mkd, Mvd = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, [T])
    s_k = oc.k_scale[:, :oc.t_quant // G].view(np.float16).astype(np.float32)
    q = (synth.make_queries(9, 2, hq, 128).astype(np.float32) * 40).astype(np.float16)
    assert np.abs(q.astype(np.float32)).max() * s_k.max() > 256     # the case the pre-scaling exists for
    scale = 128 ** -0.5 / 160
    want, want_lse = oracle.decode_attention(oc, q.view(np.uint16), Mk, Mv, scale)
    lse = torch.empty((2, hq), dtype=torch.float32, device="cuda")
    got = pk.pk_decode_attention(gcfg, gc, dev(q), scale, Mkd, Mvd, lse=lse).cpu().numpy()
    assert_attention(got, want)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= 2e-3 * max(1.0, np.abs(want_lse).max())


def test_decode_tail_only_and_empty_context(oracle, pk):
    kw, ocfg, gcfg, K, V, Mk, Mv = make_case(oracle, pk, 41, T=100, P=8, bits=2, G=64, R=64, F=64, n_seq=2, hkv=2,
                                            hq=8, cap=128)
    oc, gc, Mkd, Mvd = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, [100])
    assert oc.t_quant == 0 and oc.t_tail == 100
    q = synth.make_queries(4, 2, 8, 128)
    want, _ = oracle.decode_attention(oc, q.view(np.uint16), Mk, Mv, 128 ** -0.5)
    got = pk.pk_decode_attention(gcfg, gc, dev(q), 128 ** -0.5, Mkd, Mvd).cpu().numpy()
    assert_attention(got, want)
    # plain fp16 attention over the window
    Kd, Vd, Qd = K.astype(np.float64), V.astype(np.float64), q.astype(np.float64)
    for s in range(2):
        for h in range(8):
            sc = Kd[s, h // 4] @ Qd[s, h] * 128 ** -0.5
            p = np.exp(sc - sc.max()); p /= p.sum()
            assert np.allclose(got[s, h], p @ Vd[s, h // 4], rtol=2e-3, atol=2e-4)
    empty = pk.Cache(gcfg)
    lse = torch.zeros((2, 8), dtype=torch.float32, device="cuda")
    out = pk.pk_decode_attention(gcfg, empty, dev(q), 128 ** -0.5, Mkd, Mvd, lse=lse)
    assert not out.any() and torch.isinf(lse).all()


@pytest.mark.parametrize("G,hkv,hq", [
    (32, 2, 8),        # r = 4
    (32, 1, 8),        # r = 8 over 32-channel groups: two groups of query heads, in the prefix's splits and tails too
    (64, 1, 16),       # r = 16: two groups of eight heads
    (64, 1, 20),       # r = 20: the plain kernels
])
def test_decode_with_shared_prefix(oracle, pk, G, hkv, hq):
    # a shared prompt cache (n_seq = 1) in front of 3 sequences' own caches, same pattern tables
    P, bits = 32, 2
    own_kw = dict(n_seq=3, n_kv_heads=hkv, n_q_heads=hq, head_dim=128, n_patterns=P, seqs_per_set=0, bits=bits,
                  group=G, recent=0, flush=128, t_capacity=1024, metric=0)
    pre_kw = dict(own_kw, n_seq=1, flush=64, recent=16, t_capacity=512)
    spec = synth.KVSpec(1, 3, hkv, hq, 900, 128, 12, drift_sigma=0.05)
    K, V = synth.make_kv(77, spec)
    Kp, Vp = synth.make_kv(78, synth.KVSpec(1, 1, hkv, hq, 500, 128, 12))
    Mk, _, _, _ = oracle.mine(Kp[0].view(np.uint16), P, 4)
    Mv, _, _, _ = oracle.mine(Vp[0].view(np.uint16), P, 4)
    oo, go, Mkd, Mvd = run_appends(oracle, pk, oracle.Config(**own_kw), pk.Config(**own_kw), K, V, Mk, Mv, [700, 200])
    op, gp, _, _ = run_appends(oracle, pk, oracle.Config(**pre_kw), pk.Config(**pre_kw), Kp, Vp, Mk, Mv, [500])
    assert (op.t_quant, op.t_tail, oo.t_quant, oo.t_tail) == (448, 52, 896, 4)
    q = synth.make_queries(5, 3, hq, 128)
    want, want_lse = oracle.decode_attention(oo, q.view(np.uint16), Mk, Mv, 128 ** -0.5, prefix=op,
                                             prefix_patterns_k=Mk, prefix_patterns_v=Mv)
    lse = torch.empty((3, hq), dtype=torch.float32, device="cuda")
    got = pk.pk_decode_attention(pk.Config(**own_kw), go, dev(q), 128 ** -0.5, Mkd, Mvd, lse=lse, prefix=gp).cpu().numpy()
    assert_attention(got, want)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= 2e-3


def _ragged_batch(oracle, pk, kw, K, V, Mk, Mv, lens):
    """Fills sequence i of a GPU cache and an oracle cache of its own with the first lens[i] vectors."""
    gcfg = pk.Config(**dict(kw, n_seq=len(lens), seqs_per_set=len(lens)))
    gc = pk.Cache(gcfg)
    Kd, Vd = dev(K), dev(V)
    Mkd, Mvd = dev(Mk.view(np.float16)), dev(Mv.view(np.float16))
    ocs, states = [], []
    for i, n in enumerate(lens):
        oc = oracle.Cache(oracle.Config(**dict(kw, n_seq=1, seqs_per_set=0)))
        sub = gc.sequence(i)
        if n:
            oc.append(K[i:i + 1, :, :n].view(np.uint16), V[i:i + 1, :, :n].view(np.uint16), Mk, Mv)
            pk.pk_quantize_append(sub.cfg, sub, Kd[i:i + 1, :, :n], Vd[i:i + 1, :, :n], Mkd, Mvd)
        assert (sub.t_quant, sub.t_tail, sub.tail_start) == (oc.t_quant, oc.t_tail, oc.tail_start)
        ocs.append(oc)
        states.append([sub.t_quant, sub.t_tail, sub.tail_start, 0])
    torch.cuda.synchronize()
    return gcfg, gc, ocs, states, Mkd, Mvd


@pytest.mark.parametrize("hkv,hq,bits,G,P,R,lens", [
    (2, 8, 2, 64, 32, 32, [0, 70, 197, 1000, 517]),        # an empty sequence, a tail-only one, several splits
    (1, 4, 4, 32, 16, 0, [640, 64, 1, 333]),               # 4-bit, group 32, no recent window
    (2, 16, 2, 32, 16, 32, [300, 0, 900, 64]),             # r = 8 with group 32: the heads of a KV head in two groups
])
def test_decode_ragged_batch_parity(oracle, pk, hkv, hq, bits, G, P, R, lens):
    S, T = len(lens), max(lens)
    kw = dict(n_kv_heads=hkv, n_q_heads=hq, head_dim=128, n_patterns=P, bits=bits, group=G, recent=R, flush=64,
              t_capacity=-(-T // 64) * 64, metric=0)
    K, V = synth.make_kv(300 + P, synth.KVSpec(1, S, hkv, hq, T, 128, 12))
    Mk, _, _, _ = oracle.mine(K[0].view(np.uint16), P, 3)
    Mv, _, _, _ = oracle.mine(V[0].view(np.uint16), P, 3)
    gcfg, gc, ocs, states, Mkd, Mvd = _ragged_batch(oracle, pk, kw, K, V, Mk, Mv, lens)
    q = synth.make_queries(31, S, hq, 128)
    want, want_lse = oracle.decode_attention_ragged(ocs, q.view(np.uint16), Mk, Mv, 128 ** -0.5)
    st = torch.tensor(states, dtype=torch.int32, device="cuda")
    bq, bt = max(s[0] for s in states), max(s[1] for s in states)
    lse = torch.empty((S, hq), dtype=torch.float32, device="cuda")
    got = pk.pk_decode_attention_ragged(gcfg, gc, st, bq, bt, dev(q), 128 ** -0.5, Mkd, Mvd, lse=lse).cpu().numpy()
    glse = lse.cpu().numpy()
    for i, n in enumerate(lens):
        if n == 0:
            assert np.all(got[i] == 0) and np.all(np.isneginf(glse[i]))
        else:
            assert_attention(got[i], want[i])
            assert np.abs(glse[i] - want_lse[i]).max() <= 2e-3
    # entries beyond the bound are clamped to it: the longest sequence reads the same with an oversized entry
    big = int(np.argmax([s[0] for s in states]))
    st2 = st.clone()
    st2[big, 0] = bq + 640
    got2 = pk.pk_decode_attention_ragged(gcfg, gc, st2, bq, bt, dev(q), 128 ** -0.5, Mkd, Mvd).cpu().numpy()
    assert np.array_equal(got2, got)
    # a uniform state array reproduces the uniform entry point bit for bit
    full = gc.sequence(big)
    full.state = pk._State(*states[big][:3])
    one = pk.pk_decode_attention(full.cfg, full, dev(q[big:big + 1]), 128 ** -0.5, Mkd, Mvd).cpu().numpy()
    st1 = torch.tensor([states[big]], dtype=torch.int32, device="cuda")
    rag1 = pk.pk_decode_attention_ragged(full.cfg, full, st1, states[big][0], states[big][1], dev(q[big:big + 1]),
                                         128 ** -0.5, Mkd, Mvd).cpu().numpy()
    assert np.array_equal(one, rag1)


@pytest.mark.parametrize("d,hkv,hq,bits,G,P,R,F,metric,rounds", [
    (128, 2, 8, 2, 64, 32, 32, 64, 0, [[0, 70, 197, 1000, 517], [5, 0, 300, 64, 1], [1, 1, 1, 1, 1]]),
    (128, 1, 4, 4, 32, 16, 0, 128, 0, [[640, 64, 1, 333], [0, 0, 700, 127]]),
    (128, 2, 2, 2, 128, 200, 100, 128, 1, [[300, 1200, 40], [228, 1, 88]]),     # large table, group 128, min-max rule
    # more sequences than one launch of the table kernel carries (64)
    (128, 1, 2, 2, 64, 8, 16, 64, 0, [[(37 * i) % 211 for i in range(70)], [(91 * i) % 67 for i in range(70)]]),
    # the other head dimensions (plain kernels)
    (96, 2, 4, 2, 32, 16, 32, 64, 0, [[0, 70, 197, 700, 517], [5, 0, 300, 64, 1]]),
    (256, 1, 2, 4, 128, 24, 40, 128, 1, [[300, 900, 40], [228, 1, 88]]),
])
def test_quantize_append_ragged_parity(oracle, pk, d, hkv, hq, bits, G, P, R, F, metric, rounds):
    """One append call for sequences at different fill (prompts of different lengths, then steps of different size,
    a sequence that receives nothing): every sequence's part of the cache equals the oracle's cache of that sequence
    alone after the same appends; the fill states written for the ragged decode are the sequences' own; the decode
    that follows agrees with the oracle's."""
    S = len(rounds[0])
    total = [sum(r[i] for r in rounds) for i in range(S)]
    T = max(total)
    kw = dict(n_kv_heads=hkv, n_q_heads=hq, head_dim=d, n_patterns=P, bits=bits, group=G, recent=R, flush=F,
              t_capacity=-(-T // F) * F, metric=metric)
    K, V = synth.make_kv(500 + P, synth.KVSpec(1, S, hkv, hq, T, d, 12))
    Mk, _, _, _ = oracle.mine(K[0].view(np.uint16), P, 3)
    Mv, _, _, _ = oracle.mine(V[0].view(np.uint16), P, 3)
    gcfg = pk.Config(**dict(kw, n_seq=S, seqs_per_set=S))
    gc = pk.Cache(gcfg)
    Mkd, Mvd = dev(Mk.view(np.float16)), dev(Mv.view(np.float16))
    ocs = [oracle.Cache(oracle.Config(**dict(kw, n_seq=1, seqs_per_set=0))) for _ in range(S)]
    states = [[0, 0, 0] for _ in range(S)]
    done = [0] * S
    st_dev = torch.full((S, 4), -1, dtype=torch.int32, device="cuda")
    for n_new in rounds:
        n_max = max(n_new)
        Kn = np.zeros((S, hkv, n_max, d), np.float16)
        Vn = np.zeros_like(Kn)
        for i, n in enumerate(n_new):
            Kn[i, :, :n], Vn[i, :, :n] = K[i, :, done[i]:done[i] + n], V[i, :, done[i]:done[i] + n]
            if n:
                ocs[i].append(Kn[i:i + 1, :, :n].view(np.uint16), Vn[i:i + 1, :, :n].view(np.uint16), Mk, Mv)
            done[i] += n
        pk.pk_quantize_append_ragged(gcfg, gc, states, dev(Kn), dev(Vn), n_new, Mkd, Mvd, seq_states_out=st_dev)
        torch.cuda.synchronize()
        assert st_dev.cpu().tolist() == [s + [0] for s in states]
        for i, oc in enumerate(ocs):
            assert states[i] == [oc.t_quant, oc.t_tail, oc.tail_start]
            sub = gc.sequence(i)
            sub.state = pk._State(*states[i])
            compare_caches(oracle, oc, sub, metric)
    q = synth.make_queries(33, S, hq, d)
    want, _ = oracle.decode_attention_ragged(ocs, q.view(np.uint16), Mk, Mv, d ** -0.5)
    got = pk.pk_decode_attention_ragged(gcfg, gc, st_dev, max(s[0] for s in states), max(s[1] for s in states), dev(q),
                                        d ** -0.5, Mkd, Mvd).cpu().numpy()
    for i in range(S):
        assert_attention(got[i], want[i])


def test_decode_ragged_batch_with_shared_prefix(oracle, pk):
    """Samples of different generated length over one shared prompt cache (the breadth-sampling shape of Sec. 4.3)."""
    P, G, hkv, hq, lens = 32, 32, 2, 8, [130, 5, 300]
    kw = dict(n_kv_heads=hkv, n_q_heads=hq, head_dim=128, n_patterns=P, bits=2, group=G, recent=0, flush=128,
              t_capacity=384, metric=0)
    K, V = synth.make_kv(81, synth.KVSpec(1, 3, hkv, hq, 300, 128, 12, drift_sigma=0.05))
    Kp, Vp = synth.make_kv(82, synth.KVSpec(1, 1, hkv, hq, 500, 128, 12))
    Mk, _, _, _ = oracle.mine(Kp[0].view(np.uint16), P, 4)
    Mv, _, _, _ = oracle.mine(Vp[0].view(np.uint16), P, 4)
    pre_kw = dict(kw, n_seq=1, seqs_per_set=0, flush=64, recent=16, t_capacity=512)
    op, gp, _, _ = run_appends(oracle, pk, oracle.Config(**pre_kw), pk.Config(**pre_kw), Kp, Vp, Mk, Mv, [500])
    gcfg, gc, ocs, states, Mkd, Mvd = _ragged_batch(oracle, pk, kw, K, V, Mk, Mv, lens)
    q = synth.make_queries(32, 3, hq, 128)
    want, _ = oracle.decode_attention_ragged(ocs, q.view(np.uint16), Mk, Mv, 128 ** -0.5, prefix=op,
                                             prefix_patterns_k=Mk, prefix_patterns_v=Mv)
    st = torch.tensor(states, dtype=torch.int32, device="cuda")
    got = pk.pk_decode_attention_ragged(gcfg, gc, st, max(s[0] for s in states), max(s[1] for s in states), dev(q),
                                        128 ** -0.5, Mkd, Mvd, prefix=gp).cpu().numpy()
    for i in range(3):
        assert_attention(got[i], want[i])


# ------------------------------------------------------------------------------ decode-stage pattern update

def test_window_pattern_and_growing_tables(oracle, pk):
    """Sec. 3.1 "Decoding Stage": every flushed chunk of generated vectors contributes its Chebyshev centre as a
    new pattern of that stream's table; the grown tables serve the following appends and the decode."""
    P0, G, F, bits, hkv, hq, n_seq = 6, 32, 64, 2, 2, 4, 3
    spec = synth.KVSpec(1, n_seq, hkv, hq, 64 * 5, 128, 10, drift_sigma=0.2, drift_chunk=64)
    K, V = synth.make_kv(91, spec)
    N = n_seq * hkv
    Kf, Vf = K.reshape(N, -1, 128), V.reshape(N, -1, 128)
    # one table per stream (seqs_per_set = 1), started from the stream's first vectors
    Mk, Mv = Kf[:, :P0].copy().view(np.uint16), Vf[:, :P0].copy().view(np.uint16)
    Mkd, Mvd = dev(Mk.view(np.float16)), dev(Mv.view(np.float16))
    Kd, Vd = dev(K), dev(V)
    kw = dict(n_seq=n_seq, n_kv_heads=hkv, n_q_heads=hq, head_dim=128, n_patterns=P0, seqs_per_set=1, bits=bits,
              group=G, recent=0, flush=F, t_capacity=64 * 5, metric=0)
    oc, gc = oracle.Cache(oracle.Config(**kw)), pk.Cache(pk.Config(**kw))
    for step in range(5):
        sl = slice(64 * step, 64 * (step + 1))
        if step > 0:   # the window about to be flushed yields one more pattern per stream, K and V
            wk, wv = oracle.window_pattern(Kf[:, sl].view(np.uint16)), oracle.window_pattern(Vf[:, sl].view(np.uint16))
            gk = pk.pk_window_pattern(Kd.view(N, -1, 128)[:, sl])
            gv = pk.pk_window_pattern(Vd.view(N, -1, 128)[:, sl])
            assert np.array_equal(host_u16(gk), wk) and np.array_equal(host_u16(gv), wv)
            Mk, Mv = np.concatenate([Mk, wk[:, None]], 1), np.concatenate([Mv, wv[:, None]], 1)
            Mkd, Mvd = torch.cat([Mkd, gk[:, None]], 1).contiguous(), torch.cat([Mvd, gv[:, None]], 1).contiguous()
        kw["n_patterns"] = Mk.shape[1]
        oc.cfg, gc.cfg = oracle.Config(**kw), pk.Config(**kw)
        oc.append(K[:, :, sl].view(np.uint16), V[:, :, sl].view(np.uint16), Mk, Mv)
        pk.pk_quantize_append(gc.cfg, gc, Kd[:, :, sl], Vd[:, :, sl], Mkd, Mvd)
    assert Mk.shape[1] == P0 + 4 and oc.t_quant == 320
    compare_caches(oracle, oc, gc, 0)
    assert (oc.k_idx[:, 64:] >= P0).any() and oc.k_idx.max() < P0 + 4          # the added patterns are in use
    q = synth.make_queries(12, n_seq, hq, 128)
    want, _ = oracle.decode_attention(oc, q.view(np.uint16), Mk, Mv, 128 ** -0.5)
    got = pk.pk_decode_attention(gc.cfg, gc, dev(q), 128 ** -0.5, Mkd, Mvd).cpu().numpy()
    assert_attention(got, want)
    # strided output: straight into a row of a table
    tab = torch.zeros((N, 4, 128), dtype=torch.float16, device="cuda")
    pk.pk_window_pattern(Kd.view(N, -1, 128)[:, 64:128], out=tab[:, 2])
    assert np.array_equal(host_u16(tab[:, 2]), oracle.window_pattern(Kf[:, 64:128].view(np.uint16))) and not tab[:, 3].any()


# ------------------------------------------------------------------------------ second workload: MLA latent cache

@pytest.mark.parametrize("pre_rope,metric", [(False, 0), (True, 0), (False, 1)])
def test_mla_latent_cache_workload(oracle, pk, pre_rope, metric):
    """The cache that multi-head latent attention stores (appendix on ALiBi / MLA): one latent stream per sequence
    (n_kv_heads = 1) read by all 8 query heads, K = [latent | RoPE sub-space of larger magnitude], V = [latent | 0];
    with and without the rotation (pre-RoPE keys), Euclidean and min-max selection.  Whole path: patterns mined
    per layer by both sides from the same start, streaming appends with a recent window, decode."""
    spec = synth.MLASpec(n_layers=2, batch=2, n_q_heads=8, T=1400, pre_rope=pre_rope)
    K, V = synth.make_mla_kv(13, spec)
    P, bits, G, R, F = 32, 2, 64, 64, 128
    kw = dict(n_seq=4, n_kv_heads=1, n_q_heads=8, head_dim=128, n_patterns=P, seqs_per_set=2, bits=bits, group=G,
              recent=R, flush=F, t_capacity=1408, metric=metric)
    ocfg, gcfg = oracle.Config(**kw), pk.Config(**kw)
    # one table per layer, mined on the layer's first sequence: per-iteration agreement is covered by the mining
    # tests, here both sides quantize against the oracle's tables
    Mk, _, Jk, _ = oracle.mine(K[::2, 0].view(np.uint16), P, 4)
    Mv, _, _, _ = oracle.mine(V[::2, 0].view(np.uint16), P, 4)
    J = torch.empty((2, 4), dtype=torch.float32, device="cuda")
    pk.pk_mine_patterns(gcfg, dev(K[::2, 0]), 4, inertia=J)
    assert np.allclose(J.cpu().numpy(), Jk, rtol=1e-3)
    oc, gc, Mkd, Mvd = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, [700, 1, 450, 249])
    assert oc.t_quant == 1280 and oc.t_tail == 120
    assert compare_caches(oracle, oc, gc, metric) <= 8
    q = synth.make_queries(13, 4, 8, 128)
    want, want_lse = oracle.decode_attention(oc, q.view(np.uint16), Mk, Mv, 128 ** -0.5)
    lse = torch.empty((4, 8), dtype=torch.float32, device="cuda")
    got = pk.pk_decode_attention(gcfg, gc, dev(q), 128 ** -0.5, Mkd, Mvd, lse=lse).cpu().numpy()
    assert_attention(got, want)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= 2e-3


# ------------------------------------------------------------------------------ pattern mining

def _ulp_diff(a_u16, b_u16):
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7fff), u)
    return np.abs(key(a_u16) - key(b_u16))


@pytest.mark.parametrize("T,P,n_c", [(1000, 16, 16), (4096 + 37, 64, 32), (700, 128, 64), (640, 200, 64)])
def test_mining_parity_per_iteration(oracle, pk, T, P, n_c):
    spec = synth.KVSpec(1, 1, 3, 3, T, 128, n_c)
    K, V = synth.make_kv(50 + P, spec)
    x = np.concatenate([K[0], V[0, :1]])                      # 4 sets: 3 K heads and one V head
    xd = dev(x)
    gcfg = pk.Config(n_patterns=P)
    cur = x[:, :P].copy().view(np.uint16)
    for it in range(4):
        Mo, ao, Jo, cnt = oracle.mine(x.view(np.uint16), P, 1, init=cur)
        pat = dev(cur.view(np.float16)).clone()
        asg = torch.empty((4, T), dtype=torch.int32, device="cuda")
        J = torch.empty((4, 1), dtype=torch.float32, device="cuda")
        pk.pk_mine_patterns(gcfg, xd, 1, patterns=pat, init_given=True, assign=asg, inertia=J)
        ag, Mg = asg.cpu().numpy(), host_u16(pat)
        for s in range(4):
            diff = ag[s] != ao[s]
            if diff.any():
                _, best, second = oracle.assign(x[s].view(np.uint16), cur[s], 0)
                gap = (second - best) / np.maximum(second, 1e-30)
                assert np.all(gap[diff] < 1e-4)
            clean = np.ones(P, bool)
            clean[np.unique(np.concatenate([ag[s][diff], ao[s][diff]]))] = False   # clusters with equal member sets
            assert _ulp_diff(Mg[s][clean], Mo[s][clean]).max() <= 1
            assert np.abs(Mg[s].view(np.float16).astype(np.float32) - Mo[s].view(np.float16).astype(np.float32)).max() < 2e-2
            empty = cnt[s] == 0
            assert np.array_equal(Mg[s][empty & clean], cur[s][empty & clean])      # empty clusters keep their centroid
        assert np.allclose(J.cpu().numpy()[:, 0], Jo[:, 0], rtol=1e-4)
        cur = Mo                                                                    # both continue from the oracle's centroids


def _mining_step_parity(oracle, pk, x, P, cur, check_sets):
    """One Lloyd iteration on the GPU over all sets of x [S, T, d] from the centroids `cur` (uint16 [S, P, d]);
    the sets in check_sets are compared with the oracle's iteration from the same centroids.  Returns the
    oracle's new centroids of the checked sets ({set: uint16 [P, d]}): what a following iteration starts from."""
    S, T, _ = x.shape
    pat = dev(cur.view(np.float16)).clone()
    asg = torch.empty((S, T), dtype=torch.int32, device="cuda")
    J = torch.empty((S, 1), dtype=torch.float32, device="cuda")
    pk.pk_mine_patterns(pk.Config(n_patterns=P, head_dim=x.shape[2]), dev(x), 1, patterns=pat, init_given=True, assign=asg, inertia=J)
    ag, Mg, Jg = asg.cpu().numpy(), host_u16(pat), J.cpu().numpy()
    new = {}
    for s in check_sets:
        Mo, ao, Jo, cnt = oracle.mine(x[s:s + 1].view(np.uint16), P, 1, init=cur[s:s + 1])
        diff = ag[s] != ao[0]
        if diff.any():
            _, best, second = oracle.assign(x[s].view(np.uint16), cur[s], 0)
            gap = (second - best) / np.maximum(second, 1e-30)
            assert np.all(gap[diff] < 1e-4), (s, gap[diff].max())
        clean = np.ones(P, bool)
        clean[np.unique(np.concatenate([ag[s][diff], ao[0][diff]]))] = False   # clusters with equal member sets
        assert clean.sum() >= P - 2 * int(diff.sum())
        assert _ulp_diff(Mg[s][clean], Mo[0][clean]).max() <= 1, s
        empty = cnt[0] == 0
        assert np.array_equal(Mg[s][empty & clean], cur[s][empty & clean])      # empty clusters keep their centroid
        assert np.allclose(Jg[s, 0], Jo[0, 0], rtol=1e-4)
        new[s] = Mo[0]
    return new


def test_mining_parity_many_sets_several_subtiles(oracle, pk):
    """64 sets x 4133 vectors at P = 128: the launch cuts every set into 7 chunks of 640 vectors = five 128-vector
    sub-tiles each (prefetch of the next sub-tile, accumulators carried across barriers, a ragged last chunk)."""
    spec = synth.KVSpec(1, 8, 8, 8, 4096 + 37, 128, 48)
    K, _ = synth.make_kv(91, spec)
    x = K.reshape(64, 4096 + 37, 128)
    cur = x[:, :128].copy().view(np.uint16)
    checked = range(0, 64, 4)   # the GPU runs all 64 sets, the oracle every fourth (first, middle and last workgroups of the launch)
    for it in range(2):
        new = _mining_step_parity(oracle, pk, x, 128, cur, check_sets=checked)
        # both sides continue from the oracle's centroids; the sets the oracle skipped keep theirs (inputs never come from the GPU)
        cur = np.stack([new[s] if s in new else cur[s] for s in range(64)])


def test_mining_parity_256_patterns_long_chunks(oracle, pk):
    """One set of 65636 vectors at P = 256 (the 8-wave kernel): 57 chunks of 1152 vectors = 4.5 sub-tiles of 256."""
    spec = synth.KVSpec(1, 1, 1, 1, 65536 + 100, 128, 200)
    K, _ = synth.make_kv(92, spec)
    x = K.reshape(1, -1, 128)
    cur = x[:, :256].copy().view(np.uint16)
    for it in range(2):
        cur = _mining_step_parity(oracle, pk, x, 256, cur, check_sets=[0])[0][None]


def test_mining_end_to_end_and_reproducible(oracle, pk):
    spec = synth.KVSpec(1, 1, 2, 2, 3000, 128, 24)
    K, V = synth.make_kv(61, spec)
    x = np.concatenate([K[0], V[0]])
    P, iters = 32, 10
    Mo, ao, Jo, _ = oracle.mine(x.view(np.uint16), P, iters)
    gcfg = pk.Config(n_patterns=P)
    J = torch.empty((4, iters), dtype=torch.float32, device="cuda")
    asg = torch.empty((4, 3000), dtype=torch.int32, device="cuda")
    Mg = pk.pk_mine_patterns(gcfg, dev(x), iters, assign=asg, inertia=J)
    Jg = J.cpu().numpy()
    assert np.allclose(Jg[:, -1], Jo[:, -1], rtol=1e-3)
    assert np.all(Jg[:, 1:] <= Jg[:, :-1] * (1 + 1e-4))              # Lloyd never increases the objective (Sec. 3.1)
    # first assignment step starts from the first P vectors
    assert np.allclose(Jg[:, 0], Jo[:, 0], rtol=1e-4)
    J2 = torch.empty_like(J)
    Mg2 = pk.pk_mine_patterns(gcfg, dev(x), iters, inertia=J2)
    assert torch.equal(Mg, Mg2) and torch.equal(J, J2)                  # fixed summation order
    # the mined patterns serve quantization as well as the oracle's: compare objective on a fresh assignment
    for s in range(4):
        _, bo, _ = oracle.assign(x[s].view(np.uint16), Mo[s], 0)
        _, bg, _ = oracle.assign(x[s].view(np.uint16), host_u16(Mg)[s], 0)
        assert abs(bg.sum() - bo.sum()) <= 1e-3 * bo.sum()


# ------------------------------------------------------------------------------ contract configs 1 and 2

def test_config1_smoke_full_path(oracle, pk):
    """Config 1: 1 head, T=1024, P=16 from 10 Lloyd iterations, 4-bit, group 32; whole path on the GPU."""
    spec = synth.SPECS["cfg1"]
    K, V = synth.make_kv(0, spec)
    kw = dict(n_seq=1, n_kv_heads=1, n_q_heads=1, head_dim=128, n_patterns=16, seqs_per_set=0, bits=4, group=32,
              recent=0, flush=64, t_capacity=1024, metric=0)
    ocfg, gcfg = oracle.Config(**kw), pk.Config(**kw)
    Mk_o, _, _, _ = oracle.mine(K[0].view(np.uint16), 16, 10)
    Mv_o, _, _, _ = oracle.mine(V[0].view(np.uint16), 16, 10)
    Mk_g = pk.pk_mine_patterns(gcfg, dev(K[0]), 10)
    Mv_g = pk.pk_mine_patterns(gcfg, dev(V[0]), 10)
    q = synth.make_queries(0, 1, 1, 128)
    # GPU path end to end with its own patterns
    gc = pk.Cache(gcfg)
    pk.pk_quantize_append(gcfg, gc, dev(K), dev(V), Mk_g, Mv_g)
    got = pk.pk_decode_attention(gcfg, gc, dev(q), 128 ** -0.5, Mk_g, Mv_g).cpu().numpy()
    # oracle end to end with its own patterns
    oc = oracle.Cache(ocfg)
    oc.append(K.view(np.uint16), V.view(np.uint16), Mk_o, Mv_o)
    want, _ = oracle.decode_attention(oc, q.view(np.uint16), Mk_o, Mv_o, 128 ** -0.5)
    assert_attention(got, want, elementwise=False)   # each side on its own mined tables
    # and stage by stage on shared patterns
    oc2, gc2, Mkd, Mvd = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk_o, Mv_o, [1024])
    compare_caches(oracle, oc2, gc2, 0)


_CFG2 = {}


def _cfg2_inputs(oracle):
    if not _CFG2:
        K, V = synth.make_kv(2, synth.SPECS["cfg2"])
        Mk, _, Jk, _ = oracle.mine(K[0].view(np.uint16), 64, 10)
        Mv, _, _, _ = oracle.mine(V[0].view(np.uint16), 64, 10)
        _CFG2.update(K=K, V=V, Mk=Mk, Mv=Mv, Jk=Jk)
    return _CFG2


@pytest.mark.parametrize("bits", [2, 4])
def test_config2_llama_shaped_layer(oracle, pk, bits):
    """Config 2: T=8192, 8 KV heads, 32 query heads, P=64 from 10 Lloyd iterations, group 64, at full size."""
    c = _cfg2_inputs(oracle)
    K, V, Mk, Mv = c["K"], c["V"], c["Mk"], c["Mv"]
    kw = dict(n_seq=1, n_kv_heads=8, n_q_heads=32, head_dim=128, n_patterns=64, seqs_per_set=0, bits=bits, group=64,
              recent=0, flush=64, t_capacity=8192, metric=0)
    ocfg, gcfg = oracle.Config(**kw), pk.Config(**kw)
    oc, gc, Mkd, Mvd = run_appends(oracle, pk, ocfg, gcfg, K, V, Mk, Mv, [8192])
    n_diff = compare_caches(oracle, oc, gc, 0)
    assert n_diff <= 40
    q = synth.make_queries(2, 1, 32, 128)
    want, _ = oracle.decode_attention(oc, q.view(np.uint16), Mk, Mv, 128 ** -0.5)
    got = pk.pk_decode_attention(gcfg, gc, dev(q), 128 ** -0.5, Mkd, Mvd).cpu().numpy()
    assert_attention(got, want)
    if bits == 2:
        # mining at full size: objective after 10 iterations against the oracle's run from the same start
        J = torch.empty((8, 10), dtype=torch.float32, device="cuda")
        Mg = pk.pk_mine_patterns(gcfg, dev(K[0]), 10, inertia=J)
        assert np.allclose(J.cpu().numpy()[:, 0], c["Jk"][:, 0], rtol=1e-4)
        assert np.allclose(J.cpu().numpy()[:, -1], c["Jk"][:, -1], rtol=1e-3)
        # whole path on the GPU (its own patterns) against the whole path of the oracle
        Mvg = pk.pk_mine_patterns(gcfg, dev(V[0]), 10)
        gc2 = pk.Cache(gcfg)
        pk.pk_quantize_append(gcfg, gc2, dev(K), dev(V), Mg, Mvg)
        got2 = pk.pk_decode_attention(gcfg, gc2, dev(q), 128 ** -0.5, Mg, Mvg).cpu().numpy()
        assert_attention(got2, want, elementwise=False)   # each side on its own mined tables


# ------------------------------------------------------------------------------ paged cache

class PagedView:
    """The streams of a paged GPU cache gathered back into the contiguous layout (page after page through the page
    table), so that they compare with the oracle's cache, which knows nothing of pages."""

    def __init__(self, gc):
        self.gc = gc

    def array(self, name):
        raw = self.gc.array(name)
        if name.startswith("tail"):
            return raw
        cfg = self.gc.cfg
        hkv, PT = cfg.n_kv_heads, cfg.page_tokens
        parts = raw.view(cfg.n_pages * hkv, -1)                        # one row per (page, head)
        table = self.gc.page_table.long()                              # [n_seq, pages_per_seq]
        rows = table[:, None, :] * hkv + torch.arange(hkv, device=raw.device)[None, :, None]   # [n_seq, hkv, pages]
        return parts[rows.reshape(-1)].reshape(-1)                     # [n_seq][hkv][page][...] = stream-major


@pytest.mark.parametrize("d,bits,G,P,metric,R,PT,ragged", [
    (128, 2, 64, 32, 0, 32, 128, False),
    (128, 4, 32, 16, 0, 0, 256, False),
    (128, 2, 128, 130, 1, 100, 128, False),      # groups of 128 tokens = whole pages, large table, min-max rule
    (128, 2, 64, 32, 0, 32, 128, True),          # ragged appends and ragged decode over pages
    (256, 2, 64, 16, 0, 32, 128, False),         # the plain kernels of the other head dimensions over pages
    (96, 4, 32, 16, 0, 0, 256, True),            # ... with ragged appends and a ragged decode
])
def test_paged_cache_parity(oracle, pk, d, bits, G, P, metric, R, PT, ragged):
    """A cache whose packed arrays are a pool of pages, with a scrambled page table (more pages in the pool than
    the batch uses): appends in several pieces, then dequantize and decode.  Gathered back through the page table,
    every stream must equal the oracle's contiguous cache; attention and reconstruction must agree as usual."""
    S, hkv, hq, F, cap = 3, 2, 8, 128, 1024
    kw = dict(n_kv_heads=hkv, n_q_heads=hq, head_dim=d, n_patterns=P, bits=bits, group=G, recent=R, flush=F,
              t_capacity=cap, metric=metric)
    pages_per_seq = cap // PT
    n_pages = S * pages_per_seq + 5
    K, V = synth.make_kv(700 + P + PT, synth.KVSpec(1, S, hkv, hq, cap, d, 12))
    Mk, _, _, _ = oracle.mine(K[0].view(np.uint16), P, 3)
    Mv, _, _, _ = oracle.mine(V[0].view(np.uint16), P, 3)
    Mkd, Mvd = dev(Mk.view(np.float16)), dev(Mv.view(np.float16))
    gcfg = pk.Config(**dict(kw, n_seq=S, seqs_per_set=S, page_tokens=PT, n_pages=n_pages))
    gc = pk.Cache(gcfg)
    perm = np.random.default_rng(PT + P).permutation(n_pages)[:S * pages_per_seq].astype(np.int32)
    gc.page_table.copy_(torch.from_numpy(perm.reshape(S, pages_per_seq)))
    ocs = [oracle.Cache(oracle.Config(**dict(kw, n_seq=1, seqs_per_set=0))) for _ in range(S)]
    rounds = [[300, 900, 40], [500, 100, 1], [224, 24, 700]] if ragged else [[300] * S, [500] * S, [224] * S]
    states, done = [[0, 0, 0] for _ in range(S)], [0] * S
    for n_new in rounds:
        n_max = max(n_new)
        Kn, Vn = np.zeros((S, hkv, n_max, d), np.float16), np.zeros((S, hkv, n_max, d), np.float16)
        for i, n in enumerate(n_new):
            Kn[i, :, :n], Vn[i, :, :n] = K[i, :, done[i]:done[i] + n], V[i, :, done[i]:done[i] + n]
            ocs[i].append(Kn[i:i + 1, :, :n].view(np.uint16), Vn[i:i + 1, :, :n].view(np.uint16), Mk, Mv)
            done[i] += n
        if ragged:
            pk.pk_quantize_append_ragged(gcfg, gc, states, dev(Kn), dev(Vn), n_new, Mkd, Mvd)
        else:
            pk.pk_quantize_append(gcfg, gc, dev(Kn), dev(Vn), Mkd, Mvd)
            states = [[gc.t_quant, gc.t_tail, gc.tail_start] for _ in range(S)]
    torch.cuda.synchronize()
    gathered = PagedView(gc)
    for i, oc in enumerate(ocs):
        assert states[i] == [oc.t_quant, oc.t_tail, oc.tail_start]

        class One:   # sequence i of the gathered arrays, as a one-sequence cache
            def array(self, name, i=i):
                raw = gathered.array(name)
                per = raw.numel() // S
                return raw[i * per:(i + 1) * per]
        compare_caches(oracle, oc, One(), metric)
    q = synth.make_queries(34, S, hq, d)
    want, _ = oracle.decode_attention_ragged(ocs, q.view(np.uint16), Mk, Mv, d ** -0.5)
    if ragged:
        st = torch.tensor([s + [0] for s in states], dtype=torch.int32, device="cuda")
        got = pk.pk_decode_attention_ragged(gcfg, gc, st, max(s[0] for s in states), max(s[1] for s in states), dev(q),
                                            d ** -0.5, Mkd, Mvd).cpu().numpy()
    else:
        got = pk.pk_decode_attention(gcfg, gc, dev(q), d ** -0.5, Mkd, Mvd).cpu().numpy()
        # reconstruction through the page table
        kg, vg = pk.pk_dequantize(gcfg, gc, Mkd, Mvd)
        tq = gc.t_quant
        for i, oc in enumerate(ocs):
            ko, vo = oc.dequantize(Mk, Mv)
            dk = np.abs(kg[i * hkv:(i + 1) * hkv].cpu().numpy() - ko).max(axis=2)      # [hkv, tq]
            dv = np.abs(vg[i * hkv:(i + 1) * hkv].cpu().numpy() - vo).max(axis=2)
            # (a token whose assignment differs inside the near-tie band is reconstructed from another pattern)
            assert (dk > 1e-3).sum() <= 2 * G and (dv > 1e-3).sum() <= 2 and tq == oc.t_quant
    for i in range(S):
        assert_attention(got[i], want[i])


# ------------------------------------------------------------------------------ other head dimensions

@pytest.mark.parametrize("d,G,bits,P,metric,R,rho,with_prefix", [
    (96, 32, 2, 16, 0, 32, 0.0, False),
    (256, 64, 4, 40, 0, 0, 0.0, True),
    (256, 128, 2, 24, 1, 40, 0.0, False),       # min-max rule, groups of 128 tokens
    (96, 128, 4, 8, 0, 16, 0.8, False),         # one V group of all 96 channels, adaptive threshold on V
])
def test_other_head_dimensions_parity(oracle, pk, d, G, bits, P, metric, R, rho, with_prefix):
    """Head dimensions 96 and 256 (the generic kernels): two Lloyd iterations, appends in pieces, the window pattern,
    dequantize and decode (tail, optionally a shared prefix) against the oracle, to the bars of head dimension 128."""
    S, hkv, hq, T, F = 2, 2, 4, 400, 128
    K, V = synth.make_kv(900 + d + P, synth.KVSpec(1, S, hkv, hq, T, d, 12))
    # mining: per iteration from the oracle's centroids, K streams of the first sequence as sets
    x = np.ascontiguousarray(K[0])
    cur = x[:, :P].copy().view(np.uint16)
    for _ in range(2):
        new = _mining_step_parity(oracle, pk, x, P, cur, check_sets=range(hkv))
        cur = np.stack([new[s_] for s_ in range(hkv)])
    Mk = cur
    Mv, _, _, _ = oracle.mine(V[0].view(np.uint16), P, 2)
    # window pattern
    wp = pk.pk_window_pattern(dev(K[0][:, :100])).cpu().numpy().view(np.uint16)
    assert np.array_equal(wp, oracle.window_pattern(K[0][:, :100].view(np.uint16)))
    kw = dict(n_seq=S, n_kv_heads=hkv, n_q_heads=hq, head_dim=d, n_patterns=P, seqs_per_set=0, bits=bits, group=G,
              recent=R, flush=F, t_capacity=-(-T // F) * F, metric=metric, v_rho=rho)
    oc, gc, Mkd, Mvd = run_appends(oracle, pk, oracle.Config(**kw), pk.Config(**kw), K, V, Mk, Mv, [150, 1, 249])
    n_diff = compare_caches(oracle, oc, gc, metric)
    assert n_diff <= 4
    kg, vg = pk.pk_dequantize(pk.Config(**kw), gc, Mkd, Mvd)
    ko, vo = oc.dequantize(Mk, Mv)
    assert (np.abs(kg.cpu().numpy() - ko).max(axis=2) > 1e-3).sum() <= n_diff * G
    assert (np.abs(vg.cpu().numpy() - vo).max(axis=2) > 1e-3).sum() <= n_diff
    q = synth.make_queries(35, S, hq, d)
    op = gp = None
    if with_prefix:
        Kp, Vp = synth.make_kv(901, synth.KVSpec(1, 1, hkv, hq, 300, d, 12))
        pre_kw = dict(kw, n_seq=1, recent=16, t_capacity=384)
        op, gp, _, _ = run_appends(oracle, pk, oracle.Config(**pre_kw), pk.Config(**pre_kw), Kp, Vp, Mk, Mv, [300])
    want, want_lse = oracle.decode_attention(oc, q.view(np.uint16), Mk, Mv, d ** -0.5, prefix=op,
                                             prefix_patterns_k=Mk if with_prefix else None,
                                             prefix_patterns_v=Mv if with_prefix else None)
    lse = torch.empty((S, hq), dtype=torch.float32, device="cuda")
    got = pk.pk_decode_attention(pk.Config(**kw), gc, dev(q), d ** -0.5, Mkd, Mvd, lse=lse, prefix=gp).cpu().numpy()
    assert_attention(got, want)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= 2e-3


@pytest.mark.parametrize("d,hkv,hq,bits,G,P,R,lens", [
    (96, 2, 6, 2, 32, 16, 32, [0, 70, 1500, 517]),      # r = 3 (padded to four), empty and tail-only sequences, several splits
    (256, 1, 8, 4, 64, 8, 0, [1024, 333]),              # r = 8, 4-bit
    (256, 2, 2, 2, 128, 32, 40, [2048, 900, 129]),      # r = 1, groups of 128 tokens
    (96, 1, 7, 2, 128, 24, 0, [1100, 1100]),            # r = 7, one V group of all 96 channels
    (256, 1, 12, 2, 64, 8, 16, [1024, 333]),            # r = 12: two head groups per KV head, the second half filled
])
def test_other_head_dimensions_decode_splits(oracle, pk, d, hkv, hq, bits, G, P, R, lens):
    """Decode at head dimensions 96 and 256 over contexts of several splits and passes, with per-sequence fill states
    (splits past a sequence's end, sequences with only a tail or nothing), query-head counts that are no power of two, against the oracle; the uniform entry point on the longest sequence gives
    the ragged one's result bit for bit."""
    S, T = len(lens), max(lens)
    F = max(G, 64)
    kw = dict(n_kv_heads=hkv, n_q_heads=hq, head_dim=d, n_patterns=P, bits=bits, group=G, recent=R, flush=F,
              t_capacity=-(-T // F) * F, metric=0)
    K, V = synth.make_kv(700 + d + P, synth.KVSpec(1, S, hkv, hq, T, d, 12))
    Mk, _, _, _ = oracle.mine(K[0].view(np.uint16), P, 2)
    Mv, _, _, _ = oracle.mine(V[0].view(np.uint16), P, 2)
    gcfg, gc, ocs, states, Mkd, Mvd = _ragged_batch(oracle, pk, kw, K, V, Mk, Mv, lens)
    q = synth.make_queries(37, S, hq, d)
    want, want_lse = oracle.decode_attention_ragged(ocs, q.view(np.uint16), Mk, Mv, d ** -0.5)
    st = torch.tensor(states, dtype=torch.int32, device="cuda")
    bq, bt = max(s[0] for s in states), max(s[1] for s in states)
    split_tokens, n_slots, _ = pk.pk_decode_plan(gcfg, bq, 0)
    assert n_slots >= 4 or T < 1024             # the long cases run several packed splits
    lse = torch.empty((S, hq), dtype=torch.float32, device="cuda")
    got = pk.pk_decode_attention_ragged(gcfg, gc, st, bq, bt, dev(q), d ** -0.5, Mkd, Mvd, lse=lse).cpu().numpy()
    glse = lse.cpu().numpy()
    for i, n in enumerate(lens):
        if n == 0:
            assert np.all(got[i] == 0) and np.all(np.isneginf(glse[i]))
        else:
            assert_attention(got[i], want[i])
            assert np.abs(glse[i] - want_lse[i]).max() <= 2e-3
    again = pk.pk_decode_attention_ragged(gcfg, gc, st, bq, bt, dev(q), d ** -0.5, Mkd, Mvd).cpu().numpy()
    assert np.array_equal(again, got)           # fixed-point masses and fixed summation orders: reproducible
    big = int(np.argmax([s[0] for s in states]))
    full = gc.sequence(big)
    full.state = pk._State(*states[big][:3])
    one = pk.pk_decode_attention(full.cfg, full, dev(q[big:big + 1]), d ** -0.5, Mkd, Mvd).cpu().numpy()
    assert_attention(one[0], want[big])
