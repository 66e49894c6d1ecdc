#!/usr/bin/env python3
"""Benchmark of the PatternKV hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic KV that is already resident in HBM:
mine the K and V pattern tables (Lloyd iterations), quantize-append the whole context against them, run one
decode-attention step over the packed cache for every query head.

Prints ONE JSON line.  The contract's metric has two quantities, KV quantize-append GB/s and decode-attention
tokens/s on the 2-bit cache, each as a fraction of the 8 TB/s HBM peak: `value` is the decode-attention
tokens/s (sequences of the batch that receive one token per decode step over all layers, divided by the time of
the decode call), `quantize_append_GBps` the other one; `ms_per_step` is the wall-clock time of a whole step
(mine + quantize-append + decode, back to back).  `roofline` describes the decode stage, `stage_rooflines` all
three.  Per-stage durations come from HIP events recorded on the launch stream around each library call, with a
cache flush (a 1 GiB fill, outside the events) before every timed call so that inputs come from HBM and not from
the 256 MB Infinity Cache.

Default workload: cfg3, the contract's long-context batched decode (32 layers x batch 16 x T = 32768, 8 KV / 32
query heads, P = 128, 2-bit, group 64, 128 recent fp16 tokens; 68.7 GB of fp16 source).  With the default
workload the line also carries `sweep` (the same stages on cfg2x32 - config 2's layer for all 32 layers of the
model in one launch, with 2- and with 4-bit codes -, cfg5, the MLA latent-cache workload, cfg4 at its full schedule of 8192 generated tokens
with a decode after every append, cfg3r - config 3 with sequences of different lengths: ragged prefill and ragged
decode -, and cfg2x32 with the min-max selection rule) and `measured_peaks` (streaming read / copy, fp32 FMA and
fp16 MFMA loops on this GPU).

Other modes (no GPU needed):
  bench.py --summarise-trace RESULTS.db --cmd "..."            per-kernel table of a rocprofv3 --kernel-trace --stats run
  bench.py --summarise-pmc FETCH.csv WRITE.csv --calls N --key K --cmd "..."
        HBM bytes per library call from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of
        `bench.py --traffic-probe`; writes profiles/<key>_hbm_traffic.txt and updates profiles/hbm_traffic.json,
        which `roofline.traffic` is read back from (a stored reading, not measured in the timed run).
  bench.py --summarise-counters COUNTERS.csv --cmd "..."       per-kernel averages per dispatch of any other --pmc run
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

METRIC = "KV quantize-append GB/s and decode-attention tokens/s on 2-bit cache, % HBM peak"
HBM_PEAK_GBPS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
# vector-ALU lane operations per second at one wave-wide instruction per SIMD every four cycles: 256 compute units
# x 4 SIMDs x 16 lanes x 2.4 GHz.  (The published 157.3 TFLOP/s counts 2 flops of an FMA at twice that issue rate,
# which plain add / multiply / fma / and / shift reach on this chip; min, max, the mixed-precision and three-operand
# forms issue every four cycles: 1.8 ns per wave instruction measured against 1.2 to 1.3; see measured_peaks.)
VALU_LANE_OPS_PEAK_T = 256 * 4 * 16 * 2.4e9 / 1e12

WORKLOADS = {
    "cfg2": dict(spec="cfg2", layers=1, batch=1, P=64, iters=10, group=64, recent=0, flush=64),
    "cfg2x32": dict(spec="cfg2", layers=32, batch=1, P=64, iters=10, group=64, recent=0, flush=64),
    # config 2's 32 layers at head dimensions 96 and 256: the plain kernels of pk_generic.hip
    "cfg2x32_d96": dict(spec="cfg2_d96", layers=32, batch=1, P=64, iters=10, group=32, recent=0, flush=64),
    "cfg2x32_d256": dict(spec="cfg2_d256", layers=32, batch=1, P=64, iters=10, group=64, recent=0, flush=64),
    "cfg3": dict(spec="cfg3", layers=32, batch=16, P=128, iters=10, group=64, recent=128, flush=128),
    "cfg5": dict(spec="cfg5", layers=1, batch=1, P=256, iters=20, group=128, recent=0, flush=128),
    # second workload: the latent cache of multi-head latent attention (one stream per sequence, 8 query heads)
    "mla": dict(spec="mla", layers=27, batch=16, P=128, iters=10, group=64, recent=128, flush=128),
    "mla_prerope": dict(spec="mla_prerope", layers=27, batch=16, P=128, iters=10, group=64, recent=128, flush=128),
    "cfg4": dict(spec="cfg4"),   # streaming: its own step, see run_streaming()
    "cfg3r": dict(spec="cfg3"),  # config 3's shape with a mix of sequence lengths: ragged prefill + ragged decode, see run_ragged()
}
DECODE_KERNELS = "decode_packed_kernel(+decode_tail_kernel+decode_merge_kernel)"


def stored_traffic(workload, bits):
    """HBM bytes per library call from rocprofv3 --pmc runs of this script (see --summarise-pmc): stored readings."""
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(tpath):
        return {}
    return json.load(open(tpath)).get("%s_%dbit" % (workload, bits), {})


def progress(msg):
    """One line on stderr per finished part of the run (the JSON line on stdout stays the only output there)."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def event_ms(torch, fn):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1)


# ------------------------------------------------------------------------------------------------------------
def run_static(name, args, torch, pk, synth, steps, warmup, metric=None, cpu_baseline=False, traffic_probe=False):
    """Mine, quantize-append the whole context, decode once; returns the result dictionary of the workload."""
    dev = "cuda"
    metric = pk.METRIC_L2 if metric is None else metric
    w = WORKLOADS[name]
    mla = w["spec"] in synth.MLA_SPECS
    if mla:
        spec = synth.MLASpec(**{**synth.MLA_SPECS[w["spec"]].__dict__, "n_layers": w["layers"], "batch": w["batch"]})
        L, B, Hkv, Hq, T, d = w["layers"], w["batch"], 1, spec.n_q_heads, spec.T, spec.d
    else:
        base = synth.SPECS[w["spec"]]
        spec = synth.KVSpec(**{**base.__dict__, "n_layers": w["layers"], "batch": w["batch"]})
        L, B, Hkv, Hq, T, d = w["layers"], w["batch"], spec.n_kv_heads, spec.n_q_heads, spec.T, spec.d
    P, iters, G, R, F, bits = w["P"], w["iters"], w["group"], w["recent"], w["flush"], args.bits
    n_seq = L * B
    N = n_seq * Hkv
    cap = (T - R) // F * F

    # ---------------------------------------------------------------- inputs, resident in HBM
    t_gen = time.time()
    if mla:
        K = torch.empty((n_seq, Hkv, T, d), dtype=torch.float16, device=dev)
        V = torch.empty_like(K)
        for layer in range(L):
            K[layer * B:(layer + 1) * B], V[layer * B:(layer + 1) * B] = synth.make_mla_layer_device(args.seed, layer, spec, dev)
    elif n_seq == 1:
        Kh, Vh = synth.make_kv(args.seed, spec)
        K = torch.from_numpy(Kh.view(np.int16)).to(dev).view(torch.float16)
        V = torch.from_numpy(Vh.view(np.int16)).to(dev).view(torch.float16)
    else:
        K = torch.empty((n_seq, Hkv, T, d), dtype=torch.float16, device=dev)
        V = torch.empty_like(K)
        one = synth.KVSpec(**{**spec.__dict__, "n_layers": 1})
        for layer in range(L):
            K[layer * B:(layer + 1) * B], V[layer * B:(layer + 1) * B] = synth.make_layer_device(args.seed, layer, one, dev)
    q = torch.from_numpy(synth.make_queries(args.seed, n_seq, Hq, d).view(np.int16)).to(dev).view(torch.float16)
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen
    progress(f"{name}: inputs resident ({t_gen:.1f} s)")

    PT = getattr(args, "page_tokens", 0)
    assert PT == 0 or cap % PT == 0, f"the packed capacity {cap} is not a multiple of --page-tokens {PT}"
    cfg = pk.Config(n_seq=n_seq, n_kv_heads=Hkv, n_q_heads=Hq, head_dim=d, n_patterns=P,
                    seqs_per_set=(B if L > 1 else 0), bits=bits, group=G, recent=R, flush=F, t_capacity=cap,
                    metric=metric, page_tokens=PT, n_pages=(n_seq * (cap // PT) if PT else 0))
    n_sets = cfg.n_sets
    cache = pk.Cache(cfg)
    if PT:   # a paged cache: the pool's pages in a seeded random order
        gen = torch.Generator(device=dev)
        gen.manual_seed(args.seed)
        cache.page_table.copy_(torch.randperm(cfg.n_pages, generator=gen, device=dev).to(torch.int32).view(n_seq, cap // PT))
    Mk = torch.empty((n_sets, P, d), dtype=torch.float16, device=dev)
    Mv = torch.empty_like(Mk)
    out = torch.empty((n_seq, Hq, d), dtype=torch.float32, device=dev)
    ws_mine = torch.empty(max(pk.pk_workspace_bytes(cfg, pk.OP_MINE, T, n_sets), 16), dtype=torch.uint8, device=dev)
    ws_dec = torch.empty(max(pk.pk_workspace_bytes(cfg, pk.OP_DECODE, T, 0), 16), dtype=torch.uint8, device=dev)
    flush_buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    scale = d ** -0.5

    # mining reads the first batch element of every layer: for a batch > 1 those streams are gathered once, at
    # set-up, into one uniformly strided tensor, so that all layers' tables are mined by one call per tensor
    Kmine = K.view(n_sets, T, d) if B == 1 else K[::B].reshape(n_sets, T, d).contiguous()
    Vmine = V.view(n_sets, T, d) if B == 1 else V[::B].reshape(n_sets, T, d).contiguous()

    def mine():
        pk.pk_mine_patterns(cfg, Kmine, iters, patterns=Mk, workspace=ws_mine)
        pk.pk_mine_patterns(cfg, Vmine, iters, patterns=Mv, workspace=ws_mine)

    def quantize():
        cache.state.t_quant = cache.state.t_tail = cache.state.tail_start = 0
        pk.pk_quantize_append(cfg, cache, K, V, Mk, Mv)

    def decode():
        pk.pk_decode_attention(cfg, cache, q, scale, Mk, Mv, out=out, workspace=ws_dec)

    stages = [("mine", mine), ("quantize_append", quantize), ("decode_attention", decode)]

    def timed_pass():
        ms = {}
        for sname, fn in stages:
            flush_buf.fill_(1)
            ms[sname] = event_ms(torch, fn)
        return ms

    for _ in range(warmup):
        for _, fn in stages:
            fn()
    torch.cuda.synchronize()
    # whole steps, back to back
    t0 = time.perf_counter()
    for _ in range(steps):
        for _, fn in stages:
            fn()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    progress(f"{name}: {steps} whole steps timed, {ms_per_step:.3f} ms each")
    # per-stage durations from HIP events, inputs evicted before every call
    cold = [timed_pass() for _ in range(steps)]
    progress(f"{name}: per-stage passes timed")
    stage_ms = {sname: float(np.mean([c[sname] for c in cold])) for sname, _ in stages}
    stage_ms_min = {sname: float(np.min([c[sname] for c in cold])) for sname, _ in stages}
    assert cache.t_quant == cap and cache.t_tail == T - cap

    # ---------------------------------------------------------------- algorithmic bytes / flops
    Gc = min(G, d)
    k_tok = bits * d / 8 + 2 * 2 * d / G + 1          # K: codes + (s,z) amortised over the group + index
    v_tok = bits * d / 8 + 2 * 2 * d / Gc + 1         # V: codes + (s,z) per channel group + index
    packed_per_tok = k_tok + v_tok                    # 82 B at 2 bits, group 64
    quant_bytes = N * (cap * (2 * d * 2 + packed_per_tok) + (T - cap) * 2 * d * 2 * 2)   # tail: read + write
    dec_bytes = N * (cap * packed_per_tok + (T - cap) * 2 * d * 2 + 2 * P * d * 2) + n_seq * Hq * d * (2 + 4)
    mine_flops = 2.0 * T * P * d * (2 * L * Hkv) * iters
    mine_bytes = 2.0 * L * Hkv * iters * T * d * 2            # per Lloyd iteration: one pass over x
    traffic = stored_traffic(name, bits) if metric == pk.METRIC_L2 else {}

    generic = d != 128   # head dimensions 96 and 256 run the plain kernels

    def roof(stage, bound, achieved, peak, unit, kernels):
        if generic:
            kernels = {"mine": "gen_mine_assign_kernel+gen_mine_sums_kernel+gen_mine_update_kernel",
                       "quantize_append": "gen_assign_kernel+gen_quantize_k_kernel+gen_quantize_v_kernel",
                       "decode_attention": "gen_decode_split_kernel+gen_decode_merge_kernel"}[stage]
        return {"bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": traffic.get(stage), "kernel": kernels}

    # mining: the distance contraction is a dense GEMM only at large P; below that the pass over x binds
    mine_s = stage_ms["mine"] * 1e-3
    if P >= 256:
        mine_roof = roof("mine", "mfma", mine_flops / mine_s / 1e12, MFMA_F16_PEAK_TFLOPS, "TFLOP/s", "mine_step_kernel")
    else:
        mine_roof = roof("mine", "hbm", mine_bytes / mine_s / 1e9, HBM_PEAK_GBPS, "GB/s", "mine_step_kernel")
    q_s = stage_ms["quantize_append"] * 1e-3
    if metric == pk.METRIC_L2:
        q_roof = roof("quantize_append", "hbm", quant_bytes / q_s / 1e9, HBM_PEAK_GBPS, "GB/s",
                      "quantize_k_wave_kernel+quantize_v_kernel")
    else:
        # d_mm of one vector against one pattern (Sec. 3.2) in its shortest instruction form: d binary32 subtractions,
        # d/2 three-operand maxima and d/2 three-operand minima = 2 lane operations per channel, for K and for V
        lane_ops = 2.0 * N * cap * P * 2 * d
        q_roof = roof("quantize_append", "alu", lane_ops / q_s / 1e12, round(VALU_LANE_OPS_PEAK_T, 2), "T lane-ops/s",
                      "assign_minmax_kernel(+quantize_k_wave_kernel+quantize_v_kernel)")
        q_roof["hbm_GB/s"] = round(quant_bytes / q_s / 1e9, 2)
    rl = {
        "mine": mine_roof,
        "quantize_append": q_roof,
        "decode_attention": roof("decode_attention", "hbm", dec_bytes / (stage_ms["decode_attention"] * 1e-3) / 1e9,
                                 HBM_PEAK_GBPS, "GB/s", DECODE_KERNELS),
    }
    stage_out = {
        "mine": {"ms": round(stage_ms["mine"], 4), "ms_min": round(stage_ms_min["mine"], 4),
                 "TFLOP/s": round(mine_flops / mine_s / 1e12, 3), "GB/s": round(mine_bytes / mine_s / 1e9, 2)},
        "quantize_append": {"ms": round(stage_ms["quantize_append"], 4), "ms_min": round(stage_ms_min["quantize_append"], 4),
                            "GB/s": round(quant_bytes / q_s / 1e9, 3), "frac_hbm_peak": round(quant_bytes / q_s / 1e9 / HBM_PEAK_GBPS, 4),
                            "algorithmic_bytes": int(quant_bytes)},
        "decode_attention": {"ms": round(stage_ms["decode_attention"], 4), "ms_min": round(stage_ms_min["decode_attention"], 4),
                             "GB/s": rl["decode_attention"]["achieved"], "frac_hbm_peak": rl["decode_attention"]["frac"],
                             "tokens/s": round(B / (stage_ms["decode_attention"] * 1e-3), 2),
                             "algorithmic_bytes": int(dec_bytes)},
    }
    result = {
        "ms_per_step": round(ms_per_step, 4),
        "config": {"workload": name, "layers": L, "batch": B, "n_kv_heads": Hkv, "n_q_heads": Hq, "T": T,
                   "head_dim": d, "n_patterns": P, "lloyd_iters": iters, "bits": bits, "group": G, "recent": R,
                   "flush": F, "metric": "L2" if metric == pk.METRIC_L2 else "MINMAX", "seed": args.seed,
                   **({"page_tokens": PT, "page_table": "scrambled"} if PT else {})},
        "stages": stage_out,
        "stage_rooflines": rl,
        "input_generation_s": round(t_gen, 2),
    }

    # ---------------------------------------------------------------- the oracle on the host, bounded sample
    if cpu_baseline:
        from oracle import pk_oracle as oracle
        heads = min(Hkv, 8)                                   # sample: the first `heads` KV heads of sequence 0
        r = Hq // Hkv
        Ts = min(T, 16384)
        it_s = 1 if P >= 128 else min(iters, 4)               # about 10-30 s of host work in all
        Ks = K[0, :heads, :Ts].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
        Vs = V[0, :heads, :Ts].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
        qs = q[0:1, :heads * r].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
        caps = (Ts - R) // F * F
        ocfg = oracle.Config(n_seq=1, n_kv_heads=heads, n_q_heads=heads * r, head_dim=d, n_patterns=P, seqs_per_set=0,
                             bits=bits, group=G, recent=R, flush=F, t_capacity=caps,
                             metric=0 if metric == pk.METRIC_L2 else 1)
        t0 = time.perf_counter()
        Mko, _, _, _ = oracle.mine(Ks, P, it_s)
        Mvo, _, _, _ = oracle.mine(Vs, P, it_s)
        t_mine_s = time.perf_counter() - t0
        t0 = time.perf_counter()
        oc = oracle.Cache(ocfg)
        oc.append(Ks[None], Vs[None], Mko, Mvo)
        t_q = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.decode_attention(oc, qs, Mko, Mvo, scale)
        t_d = time.perf_counter() - t0
        progress(f"{name}: oracle sample timed on the host ({t_mine_s + t_q + t_d:.1f} s)")
        # the sample scaled to the whole workload: streams, context length and Lloyd iterations are all linear
        factor = (N / heads) * (T / Ts)
        q_bytes_s = heads * (caps * (2 * d * 2 + packed_per_tok) + (Ts - caps) * 2 * d * 2 * 2)
        result["cpu_baseline"] = {
            "value": round(B / (t_d * factor), 4), "unit": "decode-attention tokens/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"sequence 0 of layer 0: {heads} of {N} KV streams, the first {Ts} of {T} tokens, {it_s} of {iters} "
                      f"Lloyd iterations; measured {t_mine_s + t_q + t_d:.2f} s; the decode time is scaled linearly to all "
                      f"streams and the full context (extrapolated)",
            "quantize_append_GB/s": round(q_bytes_s / t_q / 1e9, 4),
            "mine_s_full_extrapolated": round(t_mine_s * (iters / it_s) * (L * Hkv / heads) * (T / Ts), 1),
            "stage_seconds_sample": {"mine": round(t_mine_s, 3), "quantize_append": round(t_q, 3),
                                     "decode_attention": round(t_d, 3)},
        }
    if traffic_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
        dst = torch.empty_like(src)
        flush_buf.fill_(2)
        torch.cuda.synchronize()
        torch.bitwise_not(src, out=dst)      # one dispatch: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
    return result


# ------------------------------------------------------------------------------------------------------------
def run_streaming(args, torch, pk, synth, gen0, steps, warm):
    """Config 4: 64 samples share a 4096-token prompt cache (patterns mined once on the prompt, P=64); every step
    appends one generated token per sample (flushed to the packed cache in 128-token chunks, group 32, 2 bits)
    and runs decode attention over prompt + own cache.  A step here = one generation step of all samples; with
    gen0 = 0 and steps = 8192 the run is the contract's whole schedule."""
    dev = "cuda"
    spec = synth.SPECS["cfg4"]
    S, Hkv, Hq, d, P, Tp, G, F, bits = spec.batch, spec.n_kv_heads, spec.n_q_heads, spec.d, 64, 4096, 32, 128, args.bits
    t_all = gen0 + steps
    cap = -(-t_all // F) * F
    pcfg = pk.Config(n_seq=1, n_kv_heads=Hkv, n_q_heads=Hq, head_dim=d, n_patterns=P, seqs_per_set=0, bits=bits,
                     group=G, recent=0, flush=F, t_capacity=Tp, metric=pk.METRIC_L2)
    cfg = pk.Config(n_seq=S, n_kv_heads=Hkv, n_q_heads=Hq, head_dim=d, n_patterns=P, seqs_per_set=S, bits=bits,
                    group=G, recent=0, flush=F, t_capacity=cap, metric=pk.METRIC_L2)
    Kp, Vp = synth.make_layer_device(args.seed, 0, synth.KVSpec(**{**spec.__dict__, "batch": 1, "T": Tp}), dev)
    Kg, Vg = synth.make_layer_device(args.seed, 1, synth.KVSpec(**{**spec.__dict__, "T": t_all}), dev)
    Mk = pk.pk_mine_patterns(pcfg, Kp[0], 10)
    Mv = pk.pk_mine_patterns(pcfg, Vp[0], 10)
    pc, gc = pk.Cache(pcfg), pk.Cache(cfg)
    pk.pk_quantize_append(pcfg, pc, Kp, Vp, Mk, Mv)
    q = torch.from_numpy(synth.make_queries(args.seed, S, Hq, d).view(np.int16)).to(dev).view(torch.float16)
    out = torch.empty((S, Hq, d), dtype=torch.float32, device=dev)
    ws = torch.empty(max(pk.pk_workspace_bytes(cfg, pk.OP_DECODE, t_all, Tp), 16), dtype=torch.uint8, device=dev)
    scale = d ** -0.5

    def step(t):
        pk.pk_quantize_append(cfg, gc, Kg[:, :, t:t + 1], Vg[:, :, t:t + 1], Mk, Mv)
        pk.pk_decode_attention(cfg, gc, q, scale, Mk, Mv, out=out, workspace=ws, prefix=pc)

    def reset():
        gc.state.t_quant = gc.state.t_tail = gc.state.tail_start = 0
        if gen0:
            pk.pk_quantize_append(cfg, gc, Kg[:, :, :gen0], Vg[:, :, :gen0], Mk, Mv)

    reset()
    for i in range(warm):          # warm-up steps on the same cache, then the cache starts over
        step(gen0 + i)
    reset()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for t in range(gen0, gen0 + steps):
        step(t)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    progress(f"cfg4: {steps} generation steps timed, {ms_per_step:.4f} ms each")
    # the decode call on its own at the final length (HIP events on the launch stream, median of 20)
    dec_ms = float(np.median([event_ms(torch, lambda: pk.pk_decode_attention(cfg, gc, q, scale, Mk, Mv, out=out, workspace=ws, prefix=pc))
                              for _ in range(20)]))
    N = S * Hkv
    tq, tt = gc.t_quant, gc.t_tail
    per_tok = 2 * (bits * d / 8) + 2 * (2 * 2 * d / G) + 2
    dec_bytes = N * (tq * per_tok + tt * 2 * d * 2) + Hkv * (pc.t_quant * per_tok + 2 * P * d * 2) + S * Hq * d * 6
    flush_bytes = N * F * (2 * d * 2 + per_tok)
    roofl = {"bound": "hbm", "achieved": round(dec_bytes / dec_ms / 1e6, 3), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
             "frac": round(dec_bytes / dec_ms / 1e6 / HBM_PEAK_GBPS, 4), "traffic": None, "kernel": DECODE_KERNELS}
    return {
        "ms_per_step": round(ms_per_step, 4),
        "generated_tokens/s": round(S / (ms_per_step * 1e-3), 1),
        "config": {"workload": "cfg4", "samples": S, "n_kv_heads": Hkv, "n_q_heads": Hq, "prompt_tokens": Tp,
                   "generated_tokens_at_start": gen0, "generated_tokens_at_end": gen0 + steps, "head_dim": d,
                   "n_patterns": P, "bits": bits, "group": G, "flush": F, "metric": "L2", "seed": args.seed},
        "stages": {"step_ms_events": round(e0.elapsed_time(e1) / steps, 4),
                   "decode_attention_at_end": {"ms": round(dec_ms, 4), "GB/s": roofl["achieved"], "frac_hbm_peak": roofl["frac"],
                                               "tokens/s": round(S / (dec_ms * 1e-3), 1), "algorithmic_bytes": int(dec_bytes)},
                   "append_flush_bytes_every_128_steps": int(flush_bytes)},
        "stage_rooflines": {"decode_attention": roofl},
    }


# ------------------------------------------------------------------------------------------------------------
def run_ragged(args, torch, pk, synth):
    """Config 3's shape (32 layers x batch 16, 8 KV / 32 query heads, P=128, group 64, 128 recent fp16 tokens) with
    the batch's 16 sequences filled to different lengths, drawn once (seeded, uniform in [2048, 32768]; a sequence
    has the same length in every layer).  Each layer's 16 prompts are prefilled by ONE ragged append call (timed per
    layer with events, inputs resident; reported as quantize_append_ragged); the timed step is one ragged decode
    call over all 512 (layer, sequence) pairs."""
    dev = "cuda"
    base = synth.SPECS["cfg3"]
    L, B, Hkv, Hq, T, d = base.n_layers, base.batch, base.n_kv_heads, base.n_q_heads, base.T, base.d
    P, G, R, F, bits, iters = 128, 64, 128, 128, args.bits, 10
    lens = [int(v) for v in np.random.default_rng(args.seed).integers(2048, T + 1, size=B)]
    lens[0] = T                                               # the first sequence of a layer is the one mined on
    n_seq, cap = L * B, (T - R) // F * F
    cfg = pk.Config(n_seq=n_seq, n_kv_heads=Hkv, n_q_heads=Hq, head_dim=d, n_patterns=P, seqs_per_set=B, bits=bits,
                    group=G, recent=R, flush=F, t_capacity=cap, metric=pk.METRIC_L2)
    cache = pk.Cache(cfg)
    Mk = torch.empty((L * Hkv, P, d), dtype=torch.float16, device=dev)
    Mv = torch.empty_like(Mk)
    one = synth.KVSpec(**{**base.__dict__, "n_layers": 1})
    states, app_ms = [], 0.0
    st = torch.empty((n_seq, 4), dtype=torch.int32, device=dev)
    flush_buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    for layer in range(L):
        K, V = synth.make_layer_device(args.seed, layer, one, dev)
        mk, mv = Mk[layer * Hkv:(layer + 1) * Hkv], Mv[layer * Hkv:(layer + 1) * Hkv]
        sub0 = cache.sequence(layer * B)
        pk.pk_mine_patterns(sub0.cfg, K[0], iters, patterns=mk)
        pk.pk_mine_patterns(sub0.cfg, V[0], iters, patterns=mv)
        lay = cache.sequences(layer * B, B)
        lay_states = [[0, 0, 0] for _ in range(B)]
        flush_buf.fill_(layer)
        app_ms += event_ms(torch, lambda: pk.pk_quantize_append_ragged(lay.cfg, lay, lay_states, K, V, lens, mk, mv,
                                                                       seq_states_out=st[layer * B:(layer + 1) * B]))
        states += [s + [0] for s in lay_states]
        del K, V
    assert st.cpu().tolist() == states
    per_tok = 2 * (bits * d / 8) + 2 * (2 * 2 * d / G) + 2
    # per KV head: fp16 source read once, packed bytes written for the flushed part, the rest written to the tail
    app_bytes = Hkv * sum(s[0] * (2 * d * 2 + per_tok) + s[1] * 2 * d * 2 * 2 for s in states)
    bq, bt = max(s[0] for s in states), max(s[1] for s in states)
    q = torch.from_numpy(synth.make_queries(args.seed, n_seq, Hq, d).view(np.int16)).to(dev).view(torch.float16)
    out = torch.empty((n_seq, Hq, d), dtype=torch.float32, device=dev)
    ws = torch.empty(max(pk.pk_workspace_bytes(cfg, pk.OP_DECODE, bq + bt, 0), 16), dtype=torch.uint8, device=dev)
    scale = d ** -0.5

    def decode():
        pk.pk_decode_attention_ragged(cfg, cache, st, bq, bt, q, scale, Mk, Mv, out=out, workspace=ws)

    for _ in range(args.warmup):
        decode()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        decode()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    cold = []
    for _ in range(args.steps):
        flush_buf.fill_(1)
        cold.append(event_ms(torch, decode))
    dec_ms = float(np.mean(cold))
    dec_bytes = Hkv * sum(s[0] * per_tok + s[1] * 2 * d * 2 + 2 * P * d * 2 for s in states) + n_seq * Hq * d * 6
    roofl = {"bound": "hbm", "achieved": round(dec_bytes / dec_ms / 1e6, 3), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
             "frac": round(dec_bytes / dec_ms / 1e6 / HBM_PEAK_GBPS, 4), "traffic": None, "kernel": DECODE_KERNELS}
    return {
        "ms_per_step": round(ms_per_step, 4),
        "config": {"workload": "cfg3r", "layers": L, "batch": B, "n_kv_heads": Hkv, "n_q_heads": Hq, "lengths": lens,
                   "head_dim": d, "n_patterns": P, "bits": bits, "group": G, "recent": R, "flush": F, "metric": "L2",
                   "seed": args.seed},
        "stages": {"quantize_append_ragged": {"ms": round(app_ms, 4), "GB/s": round(app_bytes / app_ms / 1e6, 3),
                                              "frac_hbm_peak": round(app_bytes / app_ms / 1e6 / HBM_PEAK_GBPS, 4),
                                              "algorithmic_bytes": int(app_bytes),
                                              "note": "32 calls, one per layer: 16 prompts of different lengths each"},
                   "decode_attention": {"ms": round(dec_ms, 4), "ms_min": round(float(np.min(cold)), 4),
                                        "GB/s": roofl["achieved"], "frac_hbm_peak": roofl["frac"],
                                        "tokens/s": round(B / (dec_ms * 1e-3), 1), "algorithmic_bytes": int(dec_bytes)}},
        "stage_rooflines": {"decode_attention": roofl},
    }


# ------------------------------------------------------------------------------------------------------------
def measure_peaks(torch, pk):
    """What this GPU sustains on four plain kernels (include/patternkv_probe.h): best of 5 runs each."""
    import ctypes as C
    lib = pk._lib
    for fn in ("pk_probe_read", "pk_probe_copy", "pk_probe_fma_f32", "pk_probe_mfma_f16"):
        getattr(lib, fn).restype = C.c_int
    lib.pk_probe_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.pk_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.pk_probe_fma_f32.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    lib.pk_probe_mfma_f16.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    nbytes = 4 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty(nbytes // 2, dtype=torch.uint8, device="cuda")
    sink = torch.empty(2048 * 256, dtype=torch.float32, device="cuda")
    fma_iters, mfma_iters = 8192, 128

    def best(fn):
        fn()
        torch.cuda.synchronize()
        return min(event_ms(torch, fn) for _ in range(5))

    def checked(rc):
        assert rc == 0, rc

    t_read = best(lambda: checked(lib.pk_probe_read(src.data_ptr(), nbytes, sink.data_ptr(), stream)))
    t_copy = best(lambda: checked(lib.pk_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes // 2, stream)))
    t_fma = best(lambda: checked(lib.pk_probe_fma_f32(sink.data_ptr(), fma_iters, stream)))
    t_mfma = best(lambda: checked(lib.pk_probe_mfma_f16(sink.data_ptr(), mfma_iters, stream)))
    del src, dst
    return {
        "hbm_read_GB/s": round(nbytes / t_read / 1e6, 1), "hbm_copy_GB/s": round(nbytes / t_copy / 1e6, 1),
        "fma_f32_TFLOP/s": round(2.0 * 16 * fma_iters * 2048 * 256 / t_fma / 1e9, 2),
        "mfma_f16_TFLOP/s": round(2.0 * 16 * 16 * 32 * 8 * mfma_iters * 2048 * 4 / t_mfma / 1e9, 1),
        "note": "read: 4 GiB streamed once; copy: 2 GiB read + 2 GiB written; fma: plain v_fma_f32, 16 independent chains "
                "per lane (this build uses no packed fp32 instructions); mfma: v_mfma_f32_16x16x32_f16, 8 independent "
                "accumulators per wave",
    }


# ------------------------------------------------------------------------------------------------------------
def summarise_trace(db, cmd):
    import sqlite3
    cur = sqlite3.connect(db).cursor()
    print(f"command: {cmd}")
    print(f"{'kernel':100s} {'calls':>6s} {'total_us':>12s} {'avg_us':>10s} {'pct':>6s}")
    for kname, calls, tot, avg, pct in cur.execute("select * from top_kernels"):   # durations in microseconds
        if "at::native" in kname or "rocclr" in kname:
            continue
        print(f"{kname[:100]:100s} {calls:6d} {tot:12.1f} {avg:10.2f} {pct:6.2f}")


def summarise_pmc(fetch_csv, write_csv, n_calls, key, cmd):
    import collections
    import csv

    def load(path, counter):
        tot, cnt = collections.defaultdict(float), collections.Counter()
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] != counter:
                continue
            tot[r["Kernel_Name"]] += float(r["Counter_Value"])
            cnt[r["Kernel_Name"]] += 1
        return tot, cnt

    F, Fc = load(fetch_csv, "FETCH_SIZE")
    W, Wc = load(write_csv, "WRITE_SIZE")
    copyk = [k for k in F if "bitwise_not" in k]
    assert len(copyk) == 1 and Fc[copyk[0]] == 1, "the 1 GiB copy of --traffic-probe was not found"
    ck = copyk[0]
    f_scale, w_scale = float(1 << 20) / (F[ck] / Fc[ck]), float(1 << 20) / (W[ck] / Wc[ck])
    stages = {"mine": ["mine_"], "quantize_append": ["quantize_", "tail_copy"], "decode_attention": ["decode_"]}
    res = {}
    lines = [f"command (run twice, --pmc FETCH_SIZE and --pmc WRITE_SIZE): {cmd}",
             f"copy kernel: {ck[:80]}: FETCH_SIZE {F[ck] / Fc[ck]:.0f} KiB, WRITE_SIZE {W[ck] / Wc[ck]:.0f} KiB for 1048576 KiB "
             f"each way -> scale {f_scale:.4f} / {w_scale:.4f}",
             f"library calls per stage in the run: {n_calls}", "",
             f"{'kernel':70s} {'disp':>6s} {'fetch KiB/disp':>15s} {'write KiB/disp':>15s}"]
    for st, subs in stages.items():
        fb = wb = 0.0
        for k in sorted(F):
            if any(s in k for s in subs):
                fb += F[k] * f_scale
                wb += W.get(k, 0.0) * w_scale
                lines.append(f"{k[:70]:70s} {Fc[k]:6d} {F[k] / Fc[k] * f_scale:15.1f} {W.get(k, 0.0) / max(Wc.get(k, 1), 1) * w_scale:15.1f}")
        res[st] = int((fb + wb) * 1024 / n_calls)
        lines.append(f"  => {st}: {res[st] / 1e6:.2f} MB per library call (fetch {fb * 1024 / n_calls / 1e6:.2f} + write {wb * 1024 / n_calls / 1e6:.2f})")
    out_json = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    allj = json.load(open(out_json)) if os.path.exists(out_json) else {}
    allj[key] = res
    json.dump(allj, open(out_json, "w"), indent=1, sort_keys=True)
    open(os.path.join(ROOT, "profiles", key + "_hbm_traffic.txt"), "w").write("\n".join(lines) + "\n")
    print("\n".join(lines))


def summarise_counters(csv_path, cmd):
    """Per-kernel averages per dispatch of whatever counters one rocprofv3 --pmc run of this script collected."""
    import collections
    import csv
    tot, cnt = collections.defaultdict(float), collections.Counter()
    for r in csv.DictReader(open(csv_path)):
        tot[(r["Kernel_Name"], r["Counter_Name"])] += float(r["Counter_Value"])
        cnt[(r["Kernel_Name"], r["Counter_Name"])] += 1
    names = sorted({c for _, c in tot})
    print(f"command: {cmd}")
    print("average per dispatch; kernels of this library only")
    print(f"{'kernel':60s} {'disp':>5s} " + " ".join(f"{c[:18]:>18s}" for c in names))
    for k in sorted({k for k, _ in tot}):
        if "pk::" not in k:
            continue
        print(f"{k[:60]:60s} {cnt[(k, names[0])]:5d} " + " ".join(f"{tot[(k, c)] / max(cnt[(k, c)], 1):18.1f}" for c in names))


# ------------------------------------------------------------------------------------------------------------
def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg3", choices=sorted(WORKLOADS))
    ap.add_argument("--bits", type=int, default=2, choices=[2, 4])
    ap.add_argument("--metric", default="l2", choices=["l2", "minmax"],
                    help="pattern selection rule of quantize-append: l2 (matrix cores) or minmax (d_mm of Sec. 3.2, vector ALUs)")
    ap.add_argument("--page-tokens", type=int, default=0,
                    help="static workloads: run on a paged cache with pages of this many tokens (a power of two >= 128 "
                         "that divides the packed capacity) and a scrambled page table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="default workload only: leave out the other configs")
    ap.add_argument("--no-peaks", action="store_true")
    ap.add_argument("--seed", type=int, default=2)
    ap.add_argument("--gen-len", type=int, default=0, help="cfg4: generated tokens per sample before the timed steps")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run one 1 GiB elementwise copy kernel (bitwise_not) at the end: the known traffic that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings of this command are scaled by")
    ap.add_argument("--summarise-trace", metavar="DB")
    ap.add_argument("--summarise-pmc", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"))
    ap.add_argument("--summarise-counters", metavar="CSV")
    ap.add_argument("--calls", type=int, default=1)
    ap.add_argument("--key", default="")
    ap.add_argument("--cmd", default="")
    args = ap.parse_args()
    if args.summarise_trace:
        return summarise_trace(args.summarise_trace, args.cmd)
    if args.summarise_counters:
        return summarise_counters(args.summarise_counters, args.cmd)
    if args.summarise_pmc:
        return summarise_pmc(args.summarise_pmc[0], args.summarise_pmc[1], args.calls, args.key, args.cmd)
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no sharding or collectives are part of it)",
              file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2510_05176_amd import patternkv as pk
    from paper_2510_05176_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    # As timeit does: no pause of the host's cyclic collector inside a timed region.  (With it on, about one default
    # run in two had a pass of a short stage stretched by 1 to 57 ms: the host collected between the start event and
    # the library call, with the GPU idle meanwhile.  Reference counting still frees everything.)
    gc.collect()
    gc.disable()
    metric = pk.METRIC_L2 if args.metric == "l2" else pk.METRIC_MINMAX
    common = {"metric": METRIC, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True,
              "scaling": "weak", "vs_baseline": None, "dtype": "f16 in, f32 arithmetic, u%d codes" % args.bits,
              "data": "synthetic"}

    if args.workload == "cfg4":
        steps = args.steps if args.steps > 20 else 8192      # the contract's schedule unless a step count is asked for
        r = run_streaming(args, torch, pk, synth, args.gen_len, steps, args.warmup)
        line = {**common, "steps": steps, "value": r["generated_tokens/s"],
                "unit": "generated tokens/s (64 samples, one layer: one append + one decode attention per sample and step)",
                **r, "roofline": r["stage_rooflines"]["decode_attention"]}
        print(json.dumps(line))
        return
    if args.workload == "cfg3r":
        r = run_ragged(args, torch, pk, synth)
        line = {**common, "value": r["stages"]["decode_attention"]["tokens/s"],
                "unit": "decode-attention tokens/s (one ragged decode step of the 16-sequence batch over all 32 layers)",
                **r, "roofline": r["stage_rooflines"]["decode_attention"]}
        print(json.dumps(line))
        return

    r = run_static(args.workload, args, torch, pk, synth, args.steps, args.warmup, metric=metric,
                   cpu_baseline=not args.no_cpu_baseline, traffic_probe=args.traffic_probe)
    c = r["config"]
    line = {**common,
            "value": r["stages"]["decode_attention"]["tokens/s"],
            "unit": f"decode-attention tokens/s ({c['batch']} sequence(s) x one token per decode step over all {c['layers']} "
                    f"layer(s), {args.bits}-bit cache; = batch / time of the decode call)",
            "quantize_append_GBps": r["stages"]["quantize_append"]["GB/s"],
            "ms_per_step_covers": "mine + quantize-append + decode, back to back (wall clock)",
            **r, "roofline": r["stage_rooflines"]["decode_attention"]}
    torch.cuda.empty_cache()

    if args.workload == "cfg3" and not args.no_sweep and metric == pk.METRIC_L2:
        sweep = {}
        # (50 passes per stage on these short jobs: a single slow pass then moves an average by 2 %, not by 10)
        for wname in ("cfg2x32", "cfg5", "mla"):
            s = run_static(wname, args, torch, pk, synth, 50, 5)
            torch.cuda.empty_cache()
            sweep[wname] = {st: {"ms": s["stages"][st]["ms"], "bound": s["stage_rooflines"][st]["bound"],
                                 "achieved": s["stage_rooflines"][st]["achieved"], "unit": s["stage_rooflines"][st]["unit"],
                                 "frac": s["stage_rooflines"][st]["frac"]} for st in s["stages"]}
            sweep[wname]["decode_attention"]["tokens/s"] = s["stages"]["decode_attention"]["tokens/s"]
        import copy
        args4 = copy.copy(args)
        args4.bits = 4                                        # config 2 asks for both code widths
        s = run_static("cfg2x32", args4, torch, pk, synth, 50, 5)
        torch.cuda.empty_cache()
        sweep["cfg2x32_4bit"] = {st: {"ms": s["stages"][st]["ms"], "bound": s["stage_rooflines"][st]["bound"],
                                      "achieved": s["stage_rooflines"][st]["achieved"], "unit": s["stage_rooflines"][st]["unit"],
                                      "frac": s["stage_rooflines"][st]["frac"]} for st in ("quantize_append", "decode_attention")}
        sweep["cfg2x32_4bit"]["decode_attention"]["tokens/s"] = s["stages"]["decode_attention"]["tokens/s"]
        for wname in ("cfg2x32_d96", "cfg2x32_d256"):
            s = run_static(wname, args, torch, pk, synth, 5, 1)
            torch.cuda.empty_cache()
            sweep[wname] = {st: {"ms": s["stages"][st]["ms"], "bound": s["stage_rooflines"][st]["bound"],
                                 "achieved": s["stage_rooflines"][st]["achieved"], "unit": s["stage_rooflines"][st]["unit"],
                                 "frac": s["stage_rooflines"][st]["frac"], "kernel": s["stage_rooflines"][st]["kernel"]}
                            for st in s["stages"]}
        s = run_streaming(args, torch, pk, synth, 0, 8192, 8)
        torch.cuda.empty_cache()
        sweep["cfg4"] = {"schedule": "64 samples x 8192 generated tokens over a shared 4096-token prompt; one append and one "
                                     "decode per step, a 128-token flush every 128 steps",
                         "ms_per_step": s["ms_per_step"], "generated_tokens/s": s["generated_tokens/s"],
                         "decode_attention_at_end": {k: s["stages"]["decode_attention_at_end"][k] for k in ("ms", "GB/s", "frac_hbm_peak")}}
        s = run_ragged(args, torch, pk, synth)
        torch.cuda.empty_cache()
        progress("cfg3r: ragged prefill and decode timed")
        sweep["cfg3r"] = {"batch": "config 3's shape, the 16 sequences filled to different lengths (seeded, 2048 .. 32768)",
                          "quantize_append_ragged": {k: s["stages"]["quantize_append_ragged"][k] for k in ("ms", "GB/s", "frac_hbm_peak")},
                          "decode_attention_ragged": {k: s["stages"]["decode_attention"][k] for k in ("ms", "GB/s", "frac_hbm_peak", "tokens/s")}}
        s = run_static("cfg2x32", args, torch, pk, synth, 5, 1, metric=pk.METRIC_MINMAX)
        torch.cuda.empty_cache()
        rq = s["stage_rooflines"]["quantize_append"]
        sweep["cfg2x32_minmax"] = {"quantize_append": {"ms": s["stages"]["quantize_append"]["ms"], "bound": rq["bound"],
                                                       "achieved": rq["achieved"], "unit": rq["unit"], "peak": rq["peak"],
                                                       "frac": rq["frac"], "hbm_GB/s": rq["hbm_GB/s"]}}
        line["sweep"] = sweep
    if not args.no_peaks:
        line["measured_peaks"] = measure_peaks(torch, pk)
        progress("peak probes done")
    print(json.dumps(line))


if __name__ == "__main__":
    main()
