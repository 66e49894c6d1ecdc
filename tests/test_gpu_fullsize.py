"""Parity at the benchmark's full sizes, in the launch configurations bench.py times.

The oracle cannot run these workloads whole, so each test runs the GPU path on the complete input and
checks sampled KV streams one by one: the oracle quantizes the sampled stream on its own (its results do
not depend on the other streams) and must agree with the GPU's rows for that stream to the usual bars -
packed bytes, fp16 scale / zero and indices bit for bit outside the near-tie band, attention output of the
stream's query heads within 2e-3 relative L2.  Pattern tables are the first P vectors of each set's first
stream (a slice of the inputs, the same for both sides), so nothing the oracle reads comes from a kernel.
"""
import numpy as np
import pytest

from paper_2510_05176_amd import synth
from test_gpu_parity import _mining_step_parity, assert_attention, compare_caches, dev, host_u16   # noqa: F401  (shared helpers)

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def pk():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2510_05176_amd import patternkv
    return patternkv


class StreamView:
    """The rows of one KV stream inside a GPU cache, presented like a one-stream cache."""

    def __init__(self, gc, ns):
        self.gc, self.ns, self.N = gc, ns, gc.cfg.n_seq * gc.cfg.n_kv_heads

    def array(self, name):
        raw = self.gc.array(name)
        per = raw.numel() // self.N
        return raw[self.ns * per:(self.ns + 1) * per]


def check_stream(oracle, pk, gc, gcfg, kw, K, V, Mk, Mv, q, out, seq, head, appends, max_near_ties):
    """Oracle run of stream (seq, head) against the GPU's rows; q, out: the GPU's whole-batch query / output."""
    r = kw["n_q_heads"] // kw["n_kv_heads"]
    okw = dict(kw, n_seq=1, n_kv_heads=1, n_q_heads=r, seqs_per_set=0)
    ocfg = oracle.Config(**okw)
    ns = seq * kw["n_kv_heads"] + head
    set_id = (0 if kw["seqs_per_set"] == 0 else seq // kw["seqs_per_set"]) * kw["n_kv_heads"] + head
    Ks, Vs = host_u16(K[seq, head]), host_u16(V[seq, head])
    Mks, Mvs = host_u16(Mk[set_id])[None], host_u16(Mv[set_id])[None]
    oc = oracle.Cache(ocfg)
    t = 0
    for n_new in appends:
        oc.append(Ks[None, None, t:t + n_new], Vs[None, None, t:t + n_new], Mks, Mvs)
        t += n_new
    assert (oc.t_quant, oc.t_tail) == (gc.t_quant, gc.t_tail)
    n_diff = compare_caches(oracle, oc, StreamView(gc, ns), 0)
    assert n_diff <= max_near_ties
    qs = host_u16(q[seq, head * r:(head + 1) * r])[None]
    want, _ = oracle.decode_attention(oc, qs, Mks, Mvs, 128 ** -0.5)
    got = out[seq, head * r:(head + 1) * r].cpu().numpy()[None]
    assert_attention(got, want)
    return n_diff


def first_vectors(X, P, B):
    """[n_seq, H, T, d] -> [n_sets, P, d]: the first P vectors of the first batch element of every layer."""
    n_seq, H, T, d = X.shape
    return X[::B, :, :P].reshape(-1, P, d).contiguous()


def test_config3_long_context_batched_decode(oracle, pk):
    """Config 3 whole: 32 layers x batch 16 x T=32768, 8 KV / 32 query heads, P=128, 2 bits, group 64, 128 recent."""
    spec = synth.SPECS["cfg3"]
    L, B, Hkv, Hq, T, d, P = spec.n_layers, spec.batch, spec.n_kv_heads, spec.n_q_heads, spec.T, spec.d, 128
    kw = dict(n_seq=L * B, n_kv_heads=Hkv, n_q_heads=Hq, head_dim=d, n_patterns=P, seqs_per_set=B, bits=2, group=64,
              recent=128, flush=128, t_capacity=(T - 128) // 128 * 128, metric=0)
    gcfg = pk.Config(**kw)
    K = torch.empty((L * B, Hkv, T, d), dtype=torch.float16, device="cuda")
    V = torch.empty_like(K)
    one = synth.KVSpec(**{**spec.__dict__, "n_layers": 1})
    for layer in range(L):
        K[layer * B:(layer + 1) * B], V[layer * B:(layer + 1) * B] = synth.make_layer_device(3, layer, one, "cuda")
    Mk, Mv = first_vectors(K, P, B), first_vectors(V, P, B)
    q = dev(synth.make_queries(3, L * B, Hq, d))
    gc = pk.Cache(gcfg)
    pk.pk_quantize_append(gcfg, gc, K, V, Mk, Mv)
    out = pk.pk_decode_attention(gcfg, gc, q, d ** -0.5, Mk, Mv)
    torch.cuda.synchronize()
    assert gc.t_quant == T - 128 and gc.t_tail == 128
    for seq, head in [(0, 0), (301, 5), (L * B - 1, Hkv - 1)]:
        check_stream(oracle, pk, gc, gcfg, kw, K, V, Mk, Mv, q, out, seq, head, [T], max_near_ties=40)


def test_odd_tile_count_per_workgroup(oracle, pk):
    """64 streams x 2560 tokens at P=128: the quantize launches give every workgroup three 64-token blocks, so the
    kernels that take two blocks (V) or a pair of tiles (K) per pass over the pattern table end on a lone one."""
    Hkv, Hq, T, d, P, n_seq = 8, 32, 2560, 128, 128, 8
    kw = dict(n_seq=n_seq, n_kv_heads=Hkv, n_q_heads=Hq, head_dim=d, n_patterns=P, seqs_per_set=n_seq, bits=2, group=64,
              recent=0, flush=64, t_capacity=T, metric=0)
    gcfg = pk.Config(**kw)
    K, V = synth.make_layer_device(7, 0, synth.KVSpec(1, n_seq, Hkv, Hq, T, d, 48), "cuda")
    Mk, Mv = first_vectors(K, P, n_seq), first_vectors(V, P, n_seq)
    q = dev(synth.make_queries(7, n_seq, Hq, d))
    gc = pk.Cache(gcfg)
    pk.pk_quantize_append(gcfg, gc, K, V, Mk, Mv)
    out = pk.pk_decode_attention(gcfg, gc, q, d ** -0.5, Mk, Mv)
    torch.cuda.synchronize()
    for seq, head in [(0, 0), (3, 5), (n_seq - 1, Hkv - 1)]:
        check_stream(oracle, pk, gc, gcfg, kw, K, V, Mk, Mv, q, out, seq, head, [T], max_near_ties=10)


def test_config5_large_pattern_stress(oracle, pk):
    """Config 5 whole: T=131072, 4 KV / 28 query heads, P=256, 2 bits, group 128."""
    spec = synth.SPECS["cfg5"]
    Hkv, Hq, T, d, P = spec.n_kv_heads, spec.n_q_heads, spec.T, spec.d, 256
    kw = dict(n_seq=1, n_kv_heads=Hkv, n_q_heads=Hq, head_dim=d, n_patterns=P, seqs_per_set=0, bits=2, group=128,
              recent=0, flush=128, t_capacity=T, metric=0)
    gcfg = pk.Config(**kw)
    K, V = synth.make_layer_device(5, 0, spec, "cuda")
    Mk, Mv = first_vectors(K, P, 1), first_vectors(V, P, 1)
    q = dev(synth.make_queries(5, 1, Hq, d))
    gc = pk.Cache(gcfg)
    pk.pk_quantize_append(gcfg, gc, K, V, Mk, Mv)
    out = pk.pk_decode_attention(gcfg, gc, q, d ** -0.5, Mk, Mv)
    torch.cuda.synchronize()
    check_stream(oracle, pk, gc, gcfg, kw, K, V, Mk, Mv, q, out, 0, 2, [T], max_near_ties=80)


def test_config4_streaming_appends_over_shared_prompt(oracle, pk):
    """Config 4 at full breadth: 64 samples over one 4096-token prompt cache, P=64, 2 bits, group 32; generated
    tokens arrive one at a time and are flushed in 128-token chunks; decode runs over prompt + own cache."""
    spec = synth.SPECS["cfg4"]
    S, Hkv, Hq, d, P, Tp, Tg = spec.batch, spec.n_kv_heads, spec.n_q_heads, spec.d, 64, 4096, 300
    pkw = dict(n_seq=1, n_kv_heads=Hkv, n_q_heads=Hq, head_dim=d, n_patterns=P, seqs_per_set=0, bits=2, group=32,
               recent=0, flush=128, t_capacity=Tp, metric=0)
    kw = dict(pkw, n_seq=S, seqs_per_set=S, t_capacity=512)
    pcfg, gcfg = pk.Config(**pkw), pk.Config(**kw)
    prompt = synth.KVSpec(**{**spec.__dict__, "batch": 1, "T": Tp})
    Kp, Vp = synth.make_layer_device(4, 0, prompt, "cuda")
    Kg, Vg = synth.make_layer_device(4, 1, synth.KVSpec(**{**spec.__dict__, "T": Tg}), "cuda")
    Mk, Mv = first_vectors(Kp, P, 1), first_vectors(Vp, P, 1)
    pc, gc = pk.Cache(pcfg), pk.Cache(gcfg)
    pk.pk_quantize_append(pcfg, pc, Kp, Vp, Mk, Mv)
    appends = [1] * 130 + [126, 44]                       # crosses a flush with single tokens, then chunks
    t = 0
    for n_new in appends:
        pk.pk_quantize_append(gcfg, gc, Kg[:, :, t:t + n_new], Vg[:, :, t:t + n_new], Mk, Mv)
        t += n_new
    q = dev(synth.make_queries(4, S, Hq, d))
    out = pk.pk_decode_attention(gcfg, gc, q, d ** -0.5, Mk, Mv, prefix=pc)
    torch.cuda.synchronize()
    assert gc.t_quant == 256 and gc.t_tail == 44
    # oracle: the prompt cache of one head plus the sample's own cache
    r = Hq // Hkv
    for seq, head in [(0, 1), (37, 6), (S - 1, 0)]:
        okw = dict(pkw, n_kv_heads=1, n_q_heads=r)
        opc = oracle.Cache(oracle.Config(**okw))
        Mks, Mvs = host_u16(Mk[head])[None], host_u16(Mv[head])[None]
        opc.append(host_u16(Kp[0, head])[None, None], host_u16(Vp[0, head])[None, None], Mks, Mvs)
        compare_caches(oracle, opc, StreamView(pc, head), 0)
        ooc = oracle.Cache(oracle.Config(**dict(okw, t_capacity=512)))
        t = 0
        for n_new in appends:
            ooc.append(host_u16(Kg[seq, head, t:t + n_new])[None, None], host_u16(Vg[seq, head, t:t + n_new])[None, None], Mks, Mvs)
            t += n_new
        compare_caches(oracle, ooc, StreamView(gc, seq * Hkv + head), 0)
        qs = host_u16(q[seq, head * r:(head + 1) * r])[None]
        want, _ = oracle.decode_attention(ooc, qs, Mks, Mvs, d ** -0.5, prefix=opc, prefix_patterns_k=Mks,
                                          prefix_patterns_v=Mvs)
        got = out[seq, head * r:(head + 1) * r].cpu().numpy()[None]
        assert_attention(got, want)


def test_config5_mining_launch(oracle, pk):
    """Config 5's mining launch: 4 sets x 131072 vectors at P = 256 (64 chunks of 2048 vectors = 8 sub-tiles of the
    8-wave kernel per set).  The GPU runs two Lloyd iterations over all four sets; the oracle checks one set per
    iteration from the same centroids (assignments bit for bit outside the near-tie band, centroids within one
    fp16 step, objective)."""
    spec = synth.SPECS["cfg5"]
    K, _ = synth.make_kv(5, spec)
    x = K[0]                                                   # [4, 131072, 128]
    cur = x[:, :256].copy().view(np.uint16)
    for it, s in enumerate((2, 2)):
        new = _mining_step_parity(oracle, pk, x, 256, cur, check_sets=[s])
        cur = cur.copy()
        cur[s] = new[s]                                        # set 2 moves on with the oracle's centroids


def test_config3_mining_launch(oracle, pk):
    """Config 3's mining launch: 256 sets (32 layers x 8 KV heads) x 32768 vectors at P = 128, two chunks of 16384
    vectors = 128 sub-tiles per set; the oracle checks three sets of one iteration."""
    spec = synth.SPECS["cfg3"]
    one = synth.KVSpec(**{**spec.__dict__, "n_layers": 1, "batch": 1})
    x = torch.empty((256, spec.T, 128), dtype=torch.float16, device="cuda")
    for layer in range(32):
        x[layer * 8:(layer + 1) * 8] = synth.make_layer_device(3, layer, one, "cuda")[0][0]
    P = 128
    pat = x[:, :P].contiguous()
    cur = host_u16(pat)
    asg = torch.empty((256, spec.T), dtype=torch.int32, device="cuda")
    pk.pk_mine_patterns(pk.Config(n_patterns=P), x, 1, patterns=pat, init_given=True, assign=asg)
    Mg = host_u16(pat)
    for s in (0, 137, 255):
        xs = host_u16(x[s])
        Mo, ao, _, cnt = oracle.mine(xs[None], P, 1, init=cur[s:s + 1])
        ag = asg[s].cpu().numpy()
        diff = ag != ao[0]
        if diff.any():
            _, best, second = oracle.assign(xs, cur[s], 0)
            gap = (second - best) / np.maximum(second, 1e-30)
            assert np.all(gap[diff] < 1e-4), (s, gap[diff].max())
        clean = np.ones(P, bool)
        clean[np.unique(np.concatenate([ag[diff], ao[0][diff]]))] = False
        key = lambda u: np.where(u.astype(np.int32) & 0x8000, -(u.astype(np.int32) & 0x7fff), u.astype(np.int32))
        assert np.abs(key(Mg[s][clean]) - key(Mo[0][clean])).max() <= 1, s


def test_config4_decode_after_every_append(oracle, pk):
    """Config 4's schedule in small: 64 samples over the shared 4096-token prompt cache, one generated token
    appended per step and a decode after EVERY append, across two flushes of 128 tokens (260 steps).  The oracle
    replays three sampled streams step by step and checks every step's output of their query heads."""
    spec = synth.SPECS["cfg4"]
    S, Hkv, Hq, d, P, Tp, steps = spec.batch, spec.n_kv_heads, spec.n_q_heads, spec.d, 64, 4096, 260
    pkw = dict(n_seq=1, n_kv_heads=Hkv, n_q_heads=Hq, head_dim=d, n_patterns=P, seqs_per_set=0, bits=2, group=32,
               recent=0, flush=128, t_capacity=Tp, metric=0)
    kw = dict(pkw, n_seq=S, seqs_per_set=S, t_capacity=512)
    pcfg, gcfg = pk.Config(**pkw), pk.Config(**kw)
    Kp, Vp = synth.make_layer_device(4, 0, synth.KVSpec(**{**spec.__dict__, "batch": 1, "T": Tp}), "cuda")
    Kg, Vg = synth.make_layer_device(4, 1, synth.KVSpec(**{**spec.__dict__, "T": steps}), "cuda")
    Mk, Mv = first_vectors(Kp, P, 1), first_vectors(Vp, P, 1)
    pc, gc = pk.Cache(pcfg), pk.Cache(gcfg)
    pk.pk_quantize_append(pcfg, pc, Kp, Vp, Mk, Mv)
    q = dev(synth.make_queries(4, S, Hq, d))
    r = Hq // Hkv
    sampled = [(0, 1), (37, 6), (S - 1, 0)]
    outs = torch.empty((steps, len(sampled), r, d), dtype=torch.float32, device="cuda")
    out = torch.empty((S, Hq, d), dtype=torch.float32, device="cuda")
    ws = torch.empty(pk.pk_workspace_bytes(gcfg, pk.OP_DECODE, 512, Tp), dtype=torch.uint8, device="cuda")
    for t in range(steps):
        pk.pk_quantize_append(gcfg, gc, Kg[:, :, t:t + 1], Vg[:, :, t:t + 1], Mk, Mv)
        pk.pk_decode_attention(gcfg, gc, q, d ** -0.5, Mk, Mv, out=out, workspace=ws, prefix=pc)
        for i, (seq, head) in enumerate(sampled):
            outs[t, i] = out[seq, head * r:(head + 1) * r]
    torch.cuda.synchronize()
    assert gc.t_quant == 256 and gc.t_tail == 4
    got = outs.cpu().numpy()
    for i, (seq, head) in enumerate(sampled):
        okw = dict(pkw, n_kv_heads=1, n_q_heads=r)
        opc = oracle.Cache(oracle.Config(**okw))
        Mks, Mvs = host_u16(Mk[head])[None], host_u16(Mv[head])[None]
        opc.append(host_u16(Kp[0, head])[None, None], host_u16(Vp[0, head])[None, None], Mks, Mvs)
        ooc = oracle.Cache(oracle.Config(**dict(okw, t_capacity=512)))
        kg, vg = host_u16(Kg[seq, head]), host_u16(Vg[seq, head])
        qs = host_u16(q[seq, head * r:(head + 1) * r])[None]
        for t in range(steps):
            ooc.append(kg[None, None, t:t + 1], vg[None, None, t:t + 1], Mks, Mvs)
            want, _ = oracle.decode_attention(ooc, qs, Mks, Mvs, d ** -0.5, prefix=opc, prefix_patterns_k=Mks,
                                              prefix_patterns_v=Mvs)
            assert_attention(got[t, i][None], want)
        compare_caches(oracle, ooc, StreamView(gc, seq * Hkv + head), 0)


class PeriodView:
    """Tokens [j*Tp, (j+1)*Tp) of every stream of a GPU cache, presented like a cache of capacity Tp (every packed
    array is token-major inside a stream, so the part of a token range is a byte range of the same proportion)."""

    def __init__(self, gc, j, Tp):
        self.gc, self.j, self.Tp = gc, j, Tp
        self.N, self.cap = gc.cfg.n_seq * gc.cfg.n_kv_heads, gc.cfg.t_capacity

    def array(self, name):
        raw = self.gc.array(name)
        if name.startswith("tail"):
            return raw
        per = raw.numel() // self.N
        pp = per * self.Tp // self.cap
        return raw.view(self.N, per)[:, self.j * pp:(self.j + 1) * pp].contiguous().view(-1)


@pytest.mark.parametrize("bits,G,hq", [(2, 64, 8), (4, 32, 4)])
def test_maximum_capacity_periodic_stream(oracle, pk, bits, G, hq):
    """The largest capacity the interface accepts (2^25 packed tokens per stream; with 4-bit codes the last K and V
    code bytes of a stream sit just below 2^31, the second stream's behind it), filled by one append and read by
    one decode.  The streams repeat a 4096-token period 8192 times, which gives results the oracle can state
    from ONE period: every period of the packed cache equals the oracle's cache of that period (the quantizer
    works on groups of at most 128 tokens and 4096 is a multiple of every group and block size), and softmax
    attention over identical periods equals attention over one of them, with log-sum-exp larger by ln(8192)."""
    Tp, reps, hkv, P = 4096, 8192, 2, 64
    cap = Tp * reps
    assert cap == 1 << 25
    kw = dict(n_seq=1, n_kv_heads=hkv, n_q_heads=hq, head_dim=128, n_patterns=P, seqs_per_set=0, bits=bits, group=G,
              recent=0, flush=128, metric=0)
    spec = synth.KVSpec(1, 1, hkv, hq, Tp, 128, 16)
    Kp, Vp = synth.make_kv(11, spec)                       # [1, hkv, Tp, d] float16 (numpy)
    Mk, Mv = np.ascontiguousarray(Kp[0, :, :P]), np.ascontiguousarray(Vp[0, :, :P])
    ocfg = oracle.Config(**kw, t_capacity=Tp)
    oc = oracle.Cache(ocfg)
    oc.append(Kp.view(np.uint16), Vp.view(np.uint16), Mk.view(np.uint16), Mv.view(np.uint16))
    assert (oc.t_quant, oc.t_tail) == (Tp, 0)

    gcfg = pk.Config(**kw, t_capacity=cap)
    gc = pk.Cache(gcfg)
    Kd = torch.from_numpy(Kp).cuda().repeat(1, 1, reps, 1)  # [1, hkv, 2^25, d]: 8.6 GB per stream
    Vd = torch.from_numpy(Vp).cuda().repeat(1, 1, reps, 1)
    Mkd, Mvd = torch.from_numpy(Mk).cuda(), torch.from_numpy(Mv).cuda()
    pk.pk_quantize_append(gcfg, gc, Kd, Vd, Mkd, Mvd)
    torch.cuda.synchronize()
    del Kd, Vd
    assert (gc.t_quant, gc.t_tail) == (cap, 0)
    for j in (0, 1, reps // 2 - 1, reps // 2, reps - 1):   # first, around the middle (byte offset 2^30 / 2^31), last
        assert compare_caches(oracle, oc, PeriodView(gc, j, Tp), 0) <= 8, f"period {j}"

    rng = np.random.default_rng(5)
    q = rng.standard_normal((1, hq, 128)).astype(np.float16)
    want, want_lse = oracle.decode_attention(oc, q.view(np.uint16), Mk.view(np.uint16), Mv.view(np.uint16), 128 ** -0.5)
    lse = torch.empty((1, hq), dtype=torch.float32, device="cuda")
    out = pk.pk_decode_attention(gcfg, gc, torch.from_numpy(q).cuda(), 128 ** -0.5, Mkd, Mvd, lse=lse)
    assert_attention(out.cpu().numpy(), want)
    assert np.abs(lse.cpu().numpy() - (np.asarray(want_lse) + np.log(reps))).max() <= 2e-3
