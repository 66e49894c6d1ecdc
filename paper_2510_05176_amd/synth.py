"""Seeded synthetic K/V/query generators shaped like the paper's workloads.

This module only draws random inputs; it contains none of the method's
arithmetic and is the one module both the tests of the GPU library and the
CPU oracle's tests read their inputs from.

Value structure (what the paper reports about real caches, Sec. 2.2):
  * K: a few stable high-magnitude "outlier" channels plus a per-channel
    offset that is a property of the head, not of the prompt (Insight 1), and
    vectors that gather around a modest number of centres which drift slowly
    along the sequence (Insight 2);
  * V: no outliers and no wide dynamic range, but clustered (Insight 3).

Recipe, per (layer, KV head), all draws from numpy PCG64 in this order:
  head stream  [seed, layer, head, 0]   : K centres N(0,1)[n_c,d]; K channel
        offsets N(0, offset_std^2)[d]; outlier channel ids (choice without
        replacement); V centres N(0,1)[n_c,d]
  token stream [seed, layer, head, 1+b] : (optional drift steps) ; cluster ids
        uniform[T]; K noise N(0,1)[T,d]; V cluster ids uniform[T]; V noise
  K = (centre[u] + sigma_k*noise + offset), outlier channels * outlier_scale
  V =  centre_v[u'] + sigma_v*noise
then rounded to fp16 (round to nearest even).  Centres, offsets and outlier
ids are shared by all batch elements of a head; tokens are not.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class KVSpec:
    n_layers: int = 1
    batch: int = 1
    n_kv_heads: int = 1
    n_q_heads: int = 1
    T: int = 1024
    d: int = 128
    n_clusters: int = 16
    sigma_k: float = 0.3
    sigma_v: float = 0.5
    n_outlier: int = 4
    outlier_scale: float = 8.0
    offset_std: float = 2.0
    drift_sigma: float = 0.0     # per-chunk random walk of the K/V centres
    drift_chunk: int = 128


def head_params(seed: int, layer: int, head: int, spec: KVSpec):
    rng = np.random.Generator(np.random.PCG64([seed, layer, head, 0]))
    ck = rng.standard_normal((spec.n_clusters, spec.d))
    off = rng.standard_normal(spec.d) * spec.offset_std
    out_idx = rng.choice(spec.d, size=spec.n_outlier, replace=False)
    cv = rng.standard_normal((spec.n_clusters, spec.d))
    return ck, off, out_idx, cv


def make_stream(seed: int, layer: int, head: int, b: int, spec: KVSpec, T: int | None = None):
    """One (layer, head, batch element) stream: K, V as float16 [T, d]."""
    T = spec.T if T is None else T
    ck, off, out_idx, cv = head_params(seed, layer, head, spec)
    rng = np.random.Generator(np.random.PCG64([seed, layer, head, 1 + b]))
    if spec.drift_sigma > 0:
        nchunk = -(-T // spec.drift_chunk)
        wk = np.cumsum(rng.standard_normal((nchunk, spec.n_clusters, spec.d)) * spec.drift_sigma, axis=0)
        wv = np.cumsum(rng.standard_normal((nchunk, spec.n_clusters, spec.d)) * spec.drift_sigma, axis=0)
    u = rng.integers(0, spec.n_clusters, size=T)
    nk = rng.standard_normal((T, spec.d))
    uv = rng.integers(0, spec.n_clusters, size=T)
    nv = rng.standard_normal((T, spec.d))
    k = ck[u] + spec.sigma_k * nk + off[None, :]
    v = cv[uv] + spec.sigma_v * nv
    if spec.drift_sigma > 0:
        chunk = np.arange(T) // spec.drift_chunk
        k = k + wk[chunk, u]
        v = v + wv[chunk, uv]
    k[:, out_idx] *= spec.outlier_scale
    return k.astype(np.float16), v.astype(np.float16)


def make_kv(seed: int, spec: KVSpec, T: int | None = None):
    """K, V as float16 [n_layers*batch, n_kv_heads, T, d]; sequence index = layer*batch + b."""
    T = spec.T if T is None else T
    n_seq = spec.n_layers * spec.batch
    K = np.empty((n_seq, spec.n_kv_heads, T, spec.d), np.float16)
    V = np.empty_like(K)
    for layer in range(spec.n_layers):
        for b in range(spec.batch):
            for h in range(spec.n_kv_heads):
                K[layer * spec.batch + b, h], V[layer * spec.batch + b, h] = make_stream(seed, layer, h, b, spec, T)
    return K, V


def make_queries(seed: int, n_seq: int, n_q_heads: int, d: int):
    rng = np.random.Generator(np.random.PCG64([seed, 977]))
    return rng.standard_normal((n_seq, n_q_heads, d)).astype(np.float16)


# The five workload shapes of the benchmark contract (config 1 = smoke).
SPECS = {
    "cfg1": KVSpec(1, 1, 1, 1, 1024, 128, 16, 0.3, 0.5, 4, 8.0),
    "cfg2": KVSpec(1, 1, 8, 32, 8192, 128, 32, 0.3, 0.5, 4, 8.0),
    # config 2's layer at the other two head sizes that Sec. 3.3 names
    "cfg2_d96": KVSpec(1, 1, 8, 32, 8192, 96, 32, 0.3, 0.5, 4, 8.0),
    "cfg2_d256": KVSpec(1, 1, 8, 32, 8192, 256, 32, 0.3, 0.5, 4, 8.0),
    "cfg3": KVSpec(32, 16, 8, 32, 32768, 128, 32, 0.3, 0.5, 4, 8.0),
    "cfg4": KVSpec(1, 64, 8, 32, 8192, 128, 32, 0.3, 0.5, 4, 8.0, drift_sigma=0.05, drift_chunk=128),
    "cfg5": KVSpec(1, 1, 4, 28, 131072, 128, 256, 0.3, 0.5, 8, 10.0),
}


# ---------------------------------------------------------------------------------------------------------------
# Second workload: the cache that multi-head latent attention actually stores (the paper's appendix on ALiBi / MLA
# states that the method applies to it directly).  Per token there is ONE vector shared by all query heads: a
# compressed latent (clustered, no outlier channels - it plays the role of V as well) followed by a small RoPE
# sub-space of larger magnitude whose pairs rotate with the position.  K = [latent | rope part], V = [latent | 0];
# n_kv_heads = 1 and every query head reads the same stream.  `pre_rope` leaves the rotation out (the pre-RoPE K
# variant of Sec. 4.1's setting discussion).
@dataclass(frozen=True)
class MLASpec:
    n_layers: int = 1
    batch: int = 1
    n_q_heads: int = 8
    T: int = 1024
    d: int = 128
    d_rope: int = 32
    n_clusters: int = 32
    sigma: float = 0.3
    rope_scale: float = 8.0
    rope_base: float = 10000.0
    pre_rope: bool = False


def mla_layer_params(seed: int, layer: int, spec: MLASpec):
    rng = np.random.Generator(np.random.PCG64([seed, layer, 4242, 0]))
    c_lat = rng.standard_normal((spec.n_clusters, spec.d - spec.d_rope))
    c_rope = rng.standard_normal((spec.n_clusters, spec.d_rope))
    return c_lat, c_rope


def _rope_angles(T: int, spec: MLASpec):
    i = np.arange(spec.d_rope // 2)
    return np.arange(T)[:, None] * spec.rope_base ** (-2.0 * i / spec.d_rope)[None, :]      # [T, d_rope/2]


def make_mla_stream(seed: int, layer: int, b: int, spec: MLASpec, T: int | None = None):
    """One (layer, sequence) latent stream: K, V as float16 [T, d]."""
    T = spec.T if T is None else T
    c_lat, c_rope = mla_layer_params(seed, layer, spec)
    rng = np.random.Generator(np.random.PCG64([seed, layer, 4242, 1 + b]))
    u = rng.integers(0, spec.n_clusters, size=T)
    lat = c_lat[u] + spec.sigma * rng.standard_normal((T, spec.d - spec.d_rope))
    ur = rng.integers(0, spec.n_clusters, size=T)
    kr = spec.rope_scale * (c_rope[ur] + spec.sigma * rng.standard_normal((T, spec.d_rope)))
    if not spec.pre_rope:
        ang = _rope_angles(T, spec)
        even, odd = kr[:, 0::2].copy(), kr[:, 1::2].copy()
        kr[:, 0::2] = even * np.cos(ang) - odd * np.sin(ang)
        kr[:, 1::2] = even * np.sin(ang) + odd * np.cos(ang)
    k = np.concatenate([lat, kr], axis=1)
    v = np.concatenate([lat, np.zeros((T, spec.d_rope))], axis=1)
    return k.astype(np.float16), v.astype(np.float16)


def make_mla_kv(seed: int, spec: MLASpec, T: int | None = None):
    """K, V as float16 [n_layers*batch, 1, T, d]; sequence index = layer*batch + b."""
    T = spec.T if T is None else T
    K = np.empty((spec.n_layers * spec.batch, 1, T, spec.d), np.float16)
    V = np.empty_like(K)
    for layer in range(spec.n_layers):
        for b in range(spec.batch):
            K[layer * spec.batch + b, 0], V[layer * spec.batch + b, 0] = make_mla_stream(seed, layer, b, spec, T)
    return K, V


def make_mla_layer_device(seed: int, layer: int, spec: MLASpec, device="cuda", T: int | None = None):
    """Device-side twin of make_mla_kv for one layer: K, V float16 [batch, 1, T, d] (layer parameters as in
    mla_layer_params; the per-token draws come from a torch generator and differ from the numpy stream)."""
    import torch

    T = spec.T if T is None else T
    dl = spec.d - spec.d_rope
    K = torch.zeros((spec.batch, 1, T, spec.d), dtype=torch.float16, device=device)
    V = torch.zeros_like(K)
    c_lat, c_rope = mla_layer_params(seed, layer, spec)
    c_lat_d = torch.from_numpy(c_lat).to(device=device, dtype=torch.float32)
    c_rope_d = torch.from_numpy(c_rope).to(device=device, dtype=torch.float32)
    ang = torch.from_numpy(_rope_angles(T, spec)).to(device=device, dtype=torch.float32)
    gen = torch.Generator(device=device)
    for b in range(spec.batch):
        gen.manual_seed((seed * 1009 + layer) * 100003 + 77 + b)
        u = torch.randint(0, spec.n_clusters, (T,), generator=gen, device=device)
        lat = c_lat_d[u] + spec.sigma * torch.randn((T, dl), generator=gen, device=device)
        ur = torch.randint(0, spec.n_clusters, (T,), generator=gen, device=device)
        kr = spec.rope_scale * (c_rope_d[ur] + spec.sigma * torch.randn((T, spec.d_rope), generator=gen, device=device))
        if not spec.pre_rope:
            even, odd = kr[:, 0::2].clone(), kr[:, 1::2].clone()
            kr[:, 0::2] = even * torch.cos(ang) - odd * torch.sin(ang)
            kr[:, 1::2] = even * torch.sin(ang) + odd * torch.cos(ang)
        K[b, 0, :, :dl] = lat.to(torch.float16)
        K[b, 0, :, dl:] = kr.to(torch.float16)
        V[b, 0, :, :dl] = lat.to(torch.float16)
    return K, V


# MLA-shaped long-context decode: 27 layers x batch 16 x T = 32768, one latent stream per sequence read by 8 query heads
MLA_SPECS = {
    "mla": MLASpec(27, 16, 8, 32768, 128, 32, 32, 0.3, 8.0),
    "mla_prerope": MLASpec(27, 16, 8, 32768, 128, 32, 32, 0.3, 8.0, pre_rope=True),
}


def make_layer_device(seed: int, layer: int, spec: KVSpec, device="cuda", T: int | None = None):
    """Device-side twin of make_kv for workloads too large for host memory: one layer's
    K, V as float16 [batch, n_kv_heads, T, d] on `device`.

    Head parameters (centres, offsets, outlier channels) are the numpy draws of head_params, so they
    match make_stream; the per-token draws (cluster ids, noise, drift) come from a torch generator
    seeded with (seed, layer, head, batch element) and therefore differ from the numpy stream.
    """
    import torch

    T = spec.T if T is None else T
    K = torch.empty((spec.batch, spec.n_kv_heads, T, spec.d), dtype=torch.float16, device=device)
    V = torch.empty_like(K)
    gen = torch.Generator(device=device)
    for h in range(spec.n_kv_heads):
        ck, off, out_idx, cv = head_params(seed, layer, h, spec)
        ck_d = torch.from_numpy(ck).to(device=device, dtype=torch.float32)
        cv_d = torch.from_numpy(cv).to(device=device, dtype=torch.float32)
        off_d = torch.from_numpy(off).to(device=device, dtype=torch.float32)
        mult = torch.ones(spec.d, device=device)
        mult[torch.from_numpy(out_idx).to(device)] = spec.outlier_scale
        for b in range(spec.batch):
            gen.manual_seed(((seed * 1009 + layer) * 1009 + h) * 100003 + b)
            u = torch.randint(0, spec.n_clusters, (T,), generator=gen, device=device)
            k = ck_d[u] + spec.sigma_k * torch.randn((T, spec.d), generator=gen, device=device) + off_d
            uv = torch.randint(0, spec.n_clusters, (T,), generator=gen, device=device)
            v = cv_d[uv] + spec.sigma_v * torch.randn((T, spec.d), generator=gen, device=device)
            if spec.drift_sigma > 0:
                nchunk = -(-T // spec.drift_chunk)
                chunk = torch.arange(T, device=device) // spec.drift_chunk
                wk = torch.cumsum(torch.randn((nchunk, spec.n_clusters, spec.d), generator=gen, device=device) * spec.drift_sigma, 0)
                wv = torch.cumsum(torch.randn((nchunk, spec.n_clusters, spec.d), generator=gen, device=device) * spec.drift_sigma, 0)
                k = k + wk[chunk, u]
                v = v + wv[chunk, uv]
            K[b, h] = (k * mult).to(torch.float16)
            V[b, h] = v.to(torch.float16)
    return K, V
