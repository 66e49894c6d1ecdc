#!/usr/bin/env python3
"""Benchmark of the PatternKV hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic KV that is already resident
in HBM: mine the K and V pattern tables (Lloyd iterations), quantize-append the whole context
against them, run one decode-attention step over the packed cache for every query head.

Prints ONE JSON line.  `value` is whole-path throughput (context tokens pushed through mining,
quantize-append and decode per second); the per-stage figures the contract's metric names
(quantize-append GB/s, decode-attention tokens/s, each as a fraction of the 8 TB/s HBM peak) are in
`stages`.  `roofline` describes the stage kernel that takes the most time in a step; `stage_rooflines`
has all three.  Per-stage durations come from HIP events recorded on the launch stream around each
library call, with a cache flush (a 1 GiB fill, outside the events) before every timed call so that
inputs come from HBM and not from the 256 MB Infinity Cache.

Workloads (--workload): cfg2x32 (default: the contract's config 2 - Llama-3-8B-shaped layer, batch 1, T=8192,
8 KV / 32 query heads, P=64, group 64 - for the model's 32 layers in one launch, 256 KV streams), cfg2 (one
layer of it: 8 streams, launch-bound), cfg3 (32 layers x batch 16 x T=32768, P=128), cfg5 (T=131072, P=256),
cfg4 (streaming: 64 samples over a shared 4096-token prompt cache, one token appended per step; use --steps 256).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBPS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0

WORKLOADS = {
    # name: (spec key, layers, batch, P, iters, group, recent, flush, default bits)
    "cfg2": dict(spec="cfg2", layers=1, batch=1, P=64, iters=10, group=64, recent=0, flush=64),
    "cfg2x32": dict(spec="cfg2", layers=32, batch=1, P=64, iters=10, group=64, recent=0, flush=64),
    "cfg3": dict(spec="cfg3", layers=32, batch=16, P=128, iters=10, group=64, recent=128, flush=128),
    "cfg5": dict(spec="cfg5", layers=1, batch=1, P=256, iters=20, group=128, recent=0, flush=128),
    "cfg4": dict(spec="cfg4"),   # streaming: its own step, see run_streaming()
    "cfg3r": dict(spec="cfg3"),  # config 3's shape with a mix of sequence lengths: decode only, see run_ragged()
}


def run_streaming(args, torch, pk, synth):
    """Config 4: 64 samples share a 4096-token prompt cache (patterns mined once on the prompt, P=64); every step
    appends one generated token per sample (flushed to the packed cache in 128-token chunks, group 32, 2 bits)
    and runs decode attention over prompt + own cache.  A step here = one generation step of all samples."""
    dev = "cuda"
    spec = synth.SPECS["cfg4"]
    S, Hkv, Hq, d, P, Tp, G, F, bits = spec.batch, spec.n_kv_heads, spec.n_q_heads, spec.d, 64, 4096, 32, 128, args.bits
    gen0, steps, warm = args.gen_len, args.steps, args.warmup
    t_all = gen0 + steps + warm
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
    pk.pk_quantize_append(cfg, gc, Kg[:, :, :gen0], Vg[:, :, :gen0], Mk, Mv)
    q = torch.from_numpy(synth.make_queries(args.seed, S, Hq, d).view(np.int16)).to(dev).view(torch.float16)
    out = torch.empty((S, Hq, d), dtype=torch.float32, device=dev)
    ws = torch.empty(max(pk.pk_workspace_bytes(cfg, pk.OP_DECODE, t_all, Tp), 16), dtype=torch.uint8, device=dev)
    scale = d ** -0.5

    def step(t):
        pk.pk_quantize_append(cfg, gc, Kg[:, :, t:t + 1], Vg[:, :, t:t + 1], Mk, Mv)
        pk.pk_decode_attention(cfg, gc, q, scale, Mk, Mv, out=out, workspace=ws, prefix=pc)

    t = gen0
    for _ in range(warm):
        step(t)
        t += 1
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        step(t)
        t += 1
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    # the two calls on their own at the final length (HIP events on the launch stream, median of 20)
    def med(fn):
        v = []
        for _ in range(20):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record(); b.synchronize()
            v.append(a.elapsed_time(b))
        return float(np.median(v))
    dec_ms = med(lambda: pk.pk_decode_attention(cfg, gc, q, scale, Mk, Mv, out=out, workspace=ws, prefix=pc))
    N = S * Hkv
    tq, tt = gc.t_quant, gc.t_tail
    per_tok = 2 * (bits * d / 8) + 2 * (2 * 2 * d / G) + 2
    dec_bytes = N * (tq * per_tok + tt * 2 * d * 2) + Hkv * (pc.t_quant * per_tok + 2 * P * d * 2) + S * Hq * d * 6
    flush_bytes = N * F * (2 * d * 2 + per_tok)
    result = {
        "metric": "KV quantize-append GB/s and decode-attention tokens/s on 2-bit cache, % HBM peak",
        "value": round(S * steps / (ms_per_step * steps * 1e-3), 1),
        "unit": "generated tokens/s (64 samples, one layer: append + decode attention per step)",
        "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16 in, f32 arithmetic, u%d codes" % bits,
        "data": "synthetic",
        "config": {"workload": "cfg4", "samples": S, "n_kv_heads": Hkv, "n_q_heads": Hq, "prompt_tokens": Tp,
                   "generated_tokens_at_end": t, "head_dim": d, "n_patterns": P, "bits": bits, "group": G, "flush": F,
                   "metric": "L2", "seed": args.seed},
        "stages": {"step_ms_events": round(e0.elapsed_time(e1) / steps, 4),
                   "decode_attention": {"ms": round(dec_ms, 4), "GB/s": round(dec_bytes / dec_ms / 1e6, 2),
                                        "frac_hbm_peak": round(dec_bytes / dec_ms / 1e6 / HBM_PEAK_GBPS, 4),
                                        "tokens/s": round(S / (dec_ms * 1e-3), 1), "algorithmic_bytes": int(dec_bytes)},
                   "append_flush_bytes_every_128_steps": int(flush_bytes)},
        "roofline": {"bound": "hbm", "achieved": round(dec_bytes / dec_ms / 1e6, 3), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(dec_bytes / dec_ms / 1e6 / HBM_PEAK_GBPS, 4), "traffic": None,
                     "kernel": "decode_packed_kernel(+decode_tail_kernel+decode_merge_kernel)"},
    }
    print(json.dumps(result))


def run_ragged(args, torch, pk, synth):
    """Config 3's shape (32 layers x batch 16, 8 KV / 32 query heads, P=128, group 64, 128 recent fp16 tokens) with
    the batch's 16 sequences filled to different lengths, drawn once (seeded, uniform in [2048, 32768]; a sequence
    has the same length in every layer).  Every sequence is appended through its own cache view; the timed step
    is one ragged decode call over all 512 (layer, sequence) pairs."""
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
    states = []
    for layer in range(L):
        K, V = synth.make_layer_device(args.seed, layer, one, dev)
        mk, mv = Mk[layer * Hkv:(layer + 1) * Hkv], Mv[layer * Hkv:(layer + 1) * Hkv]
        sub0 = cache.sequence(layer * B)
        pk.pk_mine_patterns(sub0.cfg, K[0], iters, patterns=mk)
        pk.pk_mine_patterns(sub0.cfg, V[0], iters, patterns=mv)
        for b in range(B):
            sub = cache.sequence(layer * B + b)
            pk.pk_quantize_append(sub.cfg, sub, K[b:b + 1, :, :lens[b]], V[b:b + 1, :, :lens[b]], mk, mv)
            states.append([sub.t_quant, sub.t_tail, sub.tail_start, 0])
        del K, V
    st = torch.tensor(states, dtype=torch.int32, device=dev)
    bq, bt = max(s[0] for s in states), max(s[1] for s in states)
    q = torch.from_numpy(synth.make_queries(args.seed, n_seq, Hq, d).view(np.int16)).to(dev).view(torch.float16)
    out = torch.empty((n_seq, Hq, d), dtype=torch.float32, device=dev)
    ws = torch.empty(max(pk.pk_workspace_bytes(cfg, pk.OP_DECODE, bq + bt, 0), 16), dtype=torch.uint8, device=dev)
    flush_buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
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
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); decode(); e1.record(); e1.synchronize()
        cold.append(e0.elapsed_time(e1))
    dec_ms = float(np.mean(cold))
    per_tok = 2 * (bits * d / 8) + 2 * (2 * 2 * d / G) + 2
    dec_bytes = Hkv * sum(s[0] * per_tok + s[1] * 2 * d * 2 + 2 * P * d * 2 for s in states) + n_seq * Hq * d * 6
    roof = {"bound": "hbm", "achieved": round(dec_bytes / dec_ms / 1e6, 3), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(dec_bytes / dec_ms / 1e6 / HBM_PEAK_GBPS, 4), "traffic": None,
            "kernel": "decode_packed_kernel(+decode_tail_kernel+decode_merge_kernel)"}
    print(json.dumps({
        "metric": "KV quantize-append GB/s and decode-attention tokens/s on 2-bit cache, % HBM peak",
        "value": round(B / (ms_per_step * 1e-3), 1),
        "unit": "generated tokens/s (one ragged decode step of the 16-sequence batch over all 32 layers)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 in, f32 arithmetic, u%d codes" % bits, "data": "synthetic",
        "config": {"workload": "cfg3r", "layers": L, "batch": B, "n_kv_heads": Hkv, "n_q_heads": Hq, "lengths": lens,
                   "head_dim": d, "n_patterns": P, "bits": bits, "group": G, "recent": R, "flush": F, "metric": "L2",
                   "seed": args.seed},
        "stages": {"decode_attention": {"ms": round(dec_ms, 4), "ms_min": round(float(np.min(cold)), 4),
                                        "GB/s": roof["achieved"], "frac_hbm_peak": roof["frac"],
                                        "tokens/s": round(B / (dec_ms * 1e-3), 1), "algorithmic_bytes": int(dec_bytes)}},
        "roofline": roof,
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg2x32", choices=sorted(WORKLOADS))
    ap.add_argument("--bits", type=int, default=2, choices=[2, 4])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=2)
    ap.add_argument("--gen-len", type=int, default=4096, help="cfg4: generated tokens per sample before the timed steps")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run one 1 GiB elementwise copy kernel (bitwise_not) at the end: the known traffic that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings of this command are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no sharding or collectives are part of it)",
              file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2510_05176_amd import patternkv as pk
    from paper_2510_05176_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.workload == "cfg4":
        return run_streaming(args, torch, pk, synth)
    if args.workload == "cfg3r":
        return run_ragged(args, torch, pk, synth)
    dev = "cuda"
    w = WORKLOADS[args.workload]
    base = synth.SPECS[w["spec"]]
    spec = synth.KVSpec(**{**base.__dict__, "n_layers": w["layers"], "batch": w["batch"]})
    L, B, Hkv, Hq, T, d = w["layers"], w["batch"], spec.n_kv_heads, spec.n_q_heads, spec.T, spec.d
    P, iters, G, R, F, bits = w["P"], w["iters"], w["group"], w["recent"], w["flush"], args.bits
    n_seq = L * B
    N = n_seq * Hkv
    cap = (T - R) // F * F

    # ---------------------------------------------------------------- inputs, resident in HBM
    t_gen = time.time()
    if n_seq == 1:
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

    cfg = pk.Config(n_seq=n_seq, n_kv_heads=Hkv, n_q_heads=Hq, head_dim=d, n_patterns=P,
                    seqs_per_set=(B if L > 1 else 0), bits=bits, group=G, recent=R, flush=F, t_capacity=cap,
                    metric=pk.METRIC_L2)
    n_sets = cfg.n_sets
    cache = pk.Cache(cfg)
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

    def timed_pass(cold):
        ms = {}
        for name, fn in stages:
            if cold:
                flush_buf.fill_(1)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            ms[name] = e0.elapsed_time(e1)
        return ms

    for _ in range(args.warmup):
        for _, fn in stages:
            fn()
    torch.cuda.synchronize()
    # whole steps, back to back
    t0 = time.perf_counter()
    for _ in range(args.steps):
        for _, fn in stages:
            fn()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    # per-stage durations from HIP events, inputs evicted before every call
    cold = [timed_pass(True) for _ in range(args.steps)]
    stage_ms = {name: float(np.mean([c[name] for c in cold])) for name, _ in stages}
    stage_ms_min = {name: float(np.min([c[name] for c in cold])) for name, _ in stages}
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

    # HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE, scaled by a copy of known
    # size): written by profiles/collect_traffic.py from runs of this script, read back here
    traffic = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("%s_%dbit" % (args.workload, bits), {})

    def roof(stage, bound, achieved, peak, unit, kernels):
        return {"bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": traffic.get(stage), "kernel": kernels}

    # mining: the distance contraction is a dense GEMM only at large P; below that the pass over x binds
    mine_s = stage_ms["mine"] * 1e-3
    if P >= 256:
        mine_roof = roof("mine", "mfma", mine_flops / mine_s / 1e12, MFMA_F16_PEAK_TFLOPS, "TFLOP/s", "mine_step_kernel")
    else:
        mine_roof = roof("mine", "hbm", mine_bytes / mine_s / 1e9, HBM_PEAK_GBPS, "GB/s", "mine_step_kernel")
    rl = {
        "mine": mine_roof,
        "quantize_append": roof("quantize_append", "hbm", quant_bytes / (stage_ms["quantize_append"] * 1e-3) / 1e9,
                                HBM_PEAK_GBPS, "GB/s", "quantize_k_wave_kernel+quantize_v_kernel"),
        "decode_attention": roof("decode_attention", "hbm", dec_bytes / (stage_ms["decode_attention"] * 1e-3) / 1e9,
                                 HBM_PEAK_GBPS, "GB/s", "decode_packed_kernel(+decode_tail_kernel+decode_merge_kernel)"),
    }
    dominant = max(stage_ms, key=stage_ms.get)
    stage_out = {
        "mine": {"ms": round(stage_ms["mine"], 4), "ms_min": round(stage_ms_min["mine"], 4),
                 "TFLOP/s": round(mine_flops / mine_s / 1e12, 3), "GB/s": round(mine_bytes / mine_s / 1e9, 2)},
        "quantize_append": {"ms": round(stage_ms["quantize_append"], 4), "ms_min": round(stage_ms_min["quantize_append"], 4),
                            "GB/s": rl["quantize_append"]["achieved"], "frac_hbm_peak": rl["quantize_append"]["frac"],
                            "algorithmic_bytes": int(quant_bytes)},
        "decode_attention": {"ms": round(stage_ms["decode_attention"], 4), "ms_min": round(stage_ms_min["decode_attention"], 4),
                             "GB/s": rl["decode_attention"]["achieved"], "frac_hbm_peak": rl["decode_attention"]["frac"],
                             "tokens/s": round(B / (stage_ms["decode_attention"] * 1e-3), 2),
                             "algorithmic_bytes": int(dec_bytes)},
    }

    result = {
        "metric": "KV quantize-append GB/s and decode-attention tokens/s on 2-bit cache, % HBM peak",
        "value": round(n_seq * T / (ms_per_step * 1e-3), 1),
        "unit": "context tokens/s through the whole path (mine + quantize-append + decode)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16 in, f32 arithmetic, u%d codes" % bits,
        "data": "synthetic",
        "config": {"workload": args.workload, "layers": L, "batch": B, "n_kv_heads": Hkv, "n_q_heads": Hq, "T": T,
                   "head_dim": d, "n_patterns": P, "lloyd_iters": iters, "bits": bits, "group": G, "recent": R,
                   "flush": F, "metric": "L2", "seed": args.seed},
        "stages": stage_out,
        "roofline": rl[dominant],
        "stage_rooflines": rl,
        "input_generation_s": round(t_gen, 2),
    }

    # ---------------------------------------------------------------- the oracle on the host, bounded sample
    if not args.no_cpu_baseline:
        from oracle import pk_oracle as oracle
        heads = min(Hkv, 8)                                   # sample: the first `heads` KV heads of sequence 0
        r = Hq // Hkv
        Ks = K[0, :heads].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
        Vs = V[0, :heads].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
        qs = q[0:1, :heads * r].cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
        Ts = min(T, 16384)
        it_s = min(iters, 4)
        Ks, Vs = np.ascontiguousarray(Ks[:, :Ts]), np.ascontiguousarray(Vs[:, :Ts])
        ocfg = oracle.Config(n_seq=1, n_kv_heads=heads, n_q_heads=heads * r, head_dim=d, n_patterns=P, seqs_per_set=0,
                             bits=bits, group=G, recent=R, flush=F, t_capacity=(Ts - R) // F * F, metric=0)
        t0 = time.perf_counter()
        Mko, _, _, _ = oracle.mine(Ks, P, it_s)
        Mvo, _, _, _ = oracle.mine(Vs, P, it_s)
        t_mine = (time.perf_counter() - t0) * iters / it_s
        t0 = time.perf_counter()
        oc = oracle.Cache(ocfg)
        oc.append(Ks[None], Vs[None], Mko, Mvo)
        t_q = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.decode_attention(oc, qs, Mko, Mvo, scale)
        t_d = time.perf_counter() - t0
        # scale the sample to the whole workload: streams and context length are both linear
        factor = (N / heads) * (T / Ts)
        t_full = (t_mine * (L * Hkv / heads) * (T / Ts)) + (t_q + t_d) * factor
        result["cpu_baseline"] = {
            "value": round(n_seq * T / t_full, 2), "unit": result["unit"], "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{heads} of {N} KV streams, {Ts} of {T} tokens, {it_s} of {iters} Lloyd iterations; "
                      f"measured {t_mine * it_s / iters + t_q + t_d:.2f} s, scaled linearly to the full workload",
            "stage_seconds_sample": {"mine": round(t_mine * it_s / iters, 3), "quantize_append": round(t_q, 3),
                                     "decode_attention": round(t_d, 3)},
        }
    if args.traffic_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
        dst = torch.empty_like(src)
        flush_buf.fill_(2)
        torch.cuda.synchronize()
        torch.bitwise_not(src, out=dst)      # one dispatch: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
