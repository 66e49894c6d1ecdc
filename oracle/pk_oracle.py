"""Python face of the CPU oracle (``pk_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``; never by the product package.
It imports nothing from the product package either.

The C file holds the arithmetic of the method (Sec. 2.1 Eq. 1, Sec. 3.1 Eq. 4,
Sec. 3.2 Eq. 6 and the reconstruction rule below it).  This module only
  * compiles / loads that file,
  * keeps the cache arrays and the append bookkeeping (which tokens are still
    in the full-precision window, which are flushed to the packed cache), and
  * lines up reconstructed K^ / V^ for the attention definition.

Append rule (the paper keeps the most recent vectors in full precision and
quantizes a window once it is complete, Sec. 3.1 "Decoding Stage"; the exact
window bookkeeping is this repository's): new vectors join the fp16 tail; as
long as the tail holds at least ``recent + flush`` vectors the oldest ``flush``
are assigned, residualised, quantized and packed.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pk_oracle.c")
_LIB = os.path.join(_HERE, "libpk_oracle.so")

METRIC_L2 = 0
METRIC_MINMAX = 1


def build(force: bool = False) -> str:
    """Compile pk_oracle.c with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared",
               "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.pko_half_to_float.restype = C.c_float
        _lib.pko_half_to_float.argtypes = [C.c_uint16]
        for name in ("pko_float_to_half_rne", "pko_float_to_half_down", "pko_float_to_half_up"):
            getattr(_lib, name).restype = C.c_uint16
            getattr(_lib, name).argtypes = [C.c_float]
        _lib.pko_num_threads.restype = C.c_int
    return _lib


def _p(a):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(lib().pko_num_threads())


# --------------------------------------------------------------------------
# thin array wrappers around the C functions
# --------------------------------------------------------------------------

def half_to_float(h: int) -> float:
    return float(lib().pko_half_to_float(int(h)))


def float_to_half(f: float, mode: str = "rne") -> int:
    return int(getattr(lib(), "pko_float_to_half_" + mode)(float(f)))


def assign(x_u16: np.ndarray, M_u16: np.ndarray, metric: int):
    """x[T,d], M[P,d] (fp16 bit patterns) -> idx[T] i32, best[T], second[T] f64."""
    x_u16 = np.ascontiguousarray(x_u16, dtype=np.uint16)
    M_u16 = np.ascontiguousarray(M_u16, dtype=np.uint16)
    T, d = x_u16.shape
    P = M_u16.shape[0]
    idx = np.empty(T, np.int32)
    best = np.empty(T, np.float64)
    second = np.empty(T, np.float64)
    lib().pko_assign(_p(x_u16), C.c_int64(T), d, _p(M_u16), P, metric, _p(idx), _p(best), _p(second))
    return idx, best, second


def mine(x_u16: np.ndarray, P: int, iters: int, init: np.ndarray | None = None):
    """x[S,T,d] -> M[S,P,d] u16, assign[S,T] i32, inertia[S,iters] f64, counts[S,P] i32."""
    x_u16 = np.ascontiguousarray(x_u16, dtype=np.uint16)
    S, T, d = x_u16.shape
    assert T >= P
    M = np.zeros((S, P, d), np.uint16) if init is None else np.ascontiguousarray(init, np.uint16).copy()
    a = np.empty((S, T), np.int32)
    J = np.zeros((S, max(iters, 1)), np.float64)
    cnt = np.zeros((S, P), np.int32)
    lib().pko_mine_sets(_p(x_u16), S, C.c_int64(T), d, P, iters, 0 if init is None else 1,
                        _p(M), _p(a), _p(J), _p(cnt))
    return M, a, J[:, :iters], cnt


def quantize_streams(x_u16, set_of, M_u16, metric, bits, G, side, want_codes=False, v_rho=0.0):
    """x[N,n,d]; M[sets,P,d].  side 0 = K, 1 = V.  Returns dict of arrays.

    v_rho > 0 (V side only): the adaptive threshold of Sec. 3.3; rejected tokens get index NO_PATTERN."""
    x_u16 = np.ascontiguousarray(x_u16, dtype=np.uint16)
    M_u16 = np.ascontiguousarray(M_u16, dtype=np.uint16)
    set_of = np.ascontiguousarray(set_of, dtype=np.int32)
    N, n, d = x_u16.shape
    P = M_u16.shape[1]
    Gc = min(G, d)
    assert n % 64 == 0 and (side == 1 or n % G == 0)
    idx = np.empty((N, n), np.int32)
    best = np.empty((N, n), np.float64)
    second = np.empty((N, n), np.float64)
    codes = np.empty((N, n, d), np.uint8) if want_codes else None
    packed = np.zeros((N, n * d * bits // 8), np.uint8)
    if side == 0:
        scale = np.empty((N, n // G, d), np.uint16)
    else:
        scale = np.empty((N, n // 16, d // Gc, 16), np.uint16)
    zero = np.empty_like(scale)
    assert v_rho <= 0 or P <= NO_PATTERN
    lib().pko_quantize_streams(_p(x_u16), N, n, d, _p(set_of), _p(M_u16), P, metric, bits, G, side,
                               C.c_float(v_rho if side == 1 else 0.0), _p(idx), _p(best), _p(second), _p(codes), _p(packed), _p(scale), _p(zero))
    return dict(idx=idx, best=best, second=second, codes=codes, packed=packed, scale=scale, zero=zero)


def v_params_by_token(a):
    """V scale / zero from the stored [n/16, groups, 16] slices to [n, groups]."""
    a = np.asarray(a)
    return a.transpose(0, 2, 1).reshape(-1, a.shape[1])


def pack_k(codes_u8, bits):
    n, d = codes_u8.shape
    out = np.zeros((n, d // 32, bits), np.uint32)
    lib().pko_pack_k(_p(np.ascontiguousarray(codes_u8)), n, d, bits, _p(out))
    return out


def unpack_k(words_u32, n, d, bits):
    out = np.empty((n, d), np.uint8)
    lib().pko_unpack_k(_p(np.ascontiguousarray(words_u32)), n, d, bits, _p(out))
    return out


def pack_v(codes_u8, bits):
    n, d = codes_u8.shape
    out = np.zeros(n * d * bits // 32, np.uint32)
    lib().pko_pack_v(_p(np.ascontiguousarray(codes_u8)), n, d, bits, _p(out))
    return out


def unpack_v(words_u32, n, d, bits):
    out = np.empty((n, d), np.uint8)
    lib().pko_unpack_v(_p(np.ascontiguousarray(words_u32)), n, d, bits, _p(out))
    return out


def dequant(side, codes_u8, scale, zero, idx_i32, M_u16, G, thresholded=False):
    """thresholded (V side): tokens with index NO_PATTERN were quantized raw and get no pattern added."""
    n, d = codes_u8.shape
    out = np.empty((n, d), np.float32)
    args = (_p(np.ascontiguousarray(codes_u8)), _p(np.ascontiguousarray(scale)), _p(np.ascontiguousarray(zero)),
            _p(np.ascontiguousarray(idx_i32, dtype=np.int32)), _p(np.ascontiguousarray(M_u16)), n, d)
    if side == 0:
        lib().pko_dequant_k(*args, G, _p(out))
    else:
        lib().pko_dequant_v(*args, min(G, d), 1 if thresholded else 0, _p(out))
    return out


def window_pattern(x_u16):
    """x[S, n, d] u16 -> [S, d] u16: the decode-stage pattern of each window (Sec. 3.1 Eq. 5, per-channel midrange)."""
    x_u16 = np.ascontiguousarray(x_u16, dtype=np.uint16)
    S, n, d = x_u16.shape
    out = np.empty((S, d), np.uint16)
    for s in range(S):
        lib().pko_window_pattern(_p(x_u16[s]), n, d, _p(out[s]))
    return out


NO_PATTERN = 255   # V index of a token the adaptive threshold sent to raw quantization


def rho_star(d: int, alpha: float) -> float:
    """Largest contraction ratio R_flat / R_raw at which flattening is kept (Sec. 3.3): the root in (0, 1) of
    1 - rho^2 = c sqrt(1 + rho^4), c = 2 z_{1-alpha} / sqrt(5 d).  With u = rho^2 the equality squares to
    (1 - c^2) u^2 - 2u + (1 - c^2) = 0, whose smaller root is the one with 1 - u >= 0."""
    from statistics import NormalDist
    c = 2.0 * NormalDist().inv_cdf(1.0 - alpha) / (5.0 * d) ** 0.5
    a = 1.0 - c * c
    assert a > 0, "the test rejects every ratio at this (d, alpha)"
    u = (1.0 - (1.0 - a * a) ** 0.5) / a
    return u ** 0.5


def attend(q_u16, Khat, Vhat, softmax_scale):
    """q[n_seq,Hq,d] u16; Khat,Vhat[n_seq,Hkv,T,d] f32 -> out[n_seq,Hq,d] f32, lse[n_seq,Hq] f32."""
    q_u16 = np.ascontiguousarray(q_u16, dtype=np.uint16)
    Khat = np.ascontiguousarray(Khat, dtype=np.float32)
    Vhat = np.ascontiguousarray(Vhat, dtype=np.float32)
    n_seq, Hq, d = q_u16.shape
    Hkv, T = Khat.shape[1], Khat.shape[2]
    out = np.empty((n_seq, Hq, d), np.float32)
    lse = np.empty((n_seq, Hq), np.float32)
    lib().pko_attend_streams(_p(q_u16), _p(Khat), _p(Vhat), n_seq, Hq, Hkv, C.c_int64(T), d,
                             C.c_double(softmax_scale), _p(out), _p(lse))
    return out, lse


# --------------------------------------------------------------------------
# cache + append bookkeeping
# --------------------------------------------------------------------------

@dataclass
class Config:
    n_seq: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    n_patterns: int
    seqs_per_set: int      # 0: every sequence shares one table per KV head; k>0: set = seq // k
    bits: int
    group: int
    recent: int
    flush: int
    t_capacity: int
    metric: int
    v_rho: float = 0.0     # > 0: adaptive threshold on V (Sec. 3.3), keep the pattern iff R_flat <= v_rho * R_raw

    @property
    def n_streams(self):
        return self.n_seq * self.n_kv_heads

    @property
    def n_sets(self):
        if self.seqs_per_set == 0:
            return self.n_kv_heads
        return -(-self.n_seq // self.seqs_per_set) * self.n_kv_heads

    def set_of(self):
        s = np.arange(self.n_seq)
        base = np.zeros_like(s) if self.seqs_per_set == 0 else s // self.seqs_per_set
        return (base[:, None] * self.n_kv_heads + np.arange(self.n_kv_heads)[None, :]).reshape(-1).astype(np.int32)


class Cache:
    """Packed cache + fp16 tail ring of N = n_seq*n_kv_heads streams, all the same length."""

    def __init__(self, cfg: Config):
        self.cfg = cfg
        N, d, b, G = cfg.n_streams, cfg.head_dim, cfg.bits, cfg.group
        cap, Gc = cfg.t_capacity, min(cfg.group, cfg.head_dim)
        assert cfg.flush % 64 == 0 and cfg.flush % cfg.group == 0 and cfg.t_capacity % cfg.flush == 0
        self.ring = cfg.recent + cfg.flush
        self.k_codes = np.zeros((N, cap, d // 32, b), np.uint32)
        self.k_scale = np.zeros((N, cap // G, d), np.uint16)
        self.k_zero = np.zeros((N, cap // G, d), np.uint16)
        self.k_idx = np.zeros((N, cap), np.uint8)
        self.v_codes = np.zeros((N, cap * d * b // 32), np.uint32)
        self.v_scale = np.zeros((N, cap // 16, d // Gc, 16), np.uint16)
        self.v_zero = np.zeros((N, cap // 16, d // Gc, 16), np.uint16)
        self.v_idx = np.zeros((N, cap), np.uint8)
        self.tail_k = np.zeros((N, self.ring, d), np.uint16)
        self.tail_v = np.zeros((N, self.ring, d), np.uint16)
        # distances of every quantized vector to its best / second-best pattern
        self.k_best = np.zeros((N, cap)); self.k_second = np.zeros((N, cap))
        self.v_best = np.zeros((N, cap)); self.v_second = np.zeros((N, cap))
        self.t_quant = 0
        self.t_tail = 0
        self.tail_start = 0

    # logical tail (oldest first)
    def tail(self, which):
        buf = self.tail_k if which == "k" else self.tail_v
        slots = (self.tail_start + np.arange(self.t_tail)) % self.ring
        return buf[:, slots, :]

    def append(self, k_new, v_new, patterns_k, patterns_v):
        """k_new, v_new: [n_seq, Hkv, n_new, d] u16; patterns: [sets, P, d] u16."""
        cfg = self.cfg
        N, d, b, G, R, F = cfg.n_streams, cfg.head_dim, cfg.bits, cfg.group, cfg.recent, cfg.flush
        k_new = np.asarray(k_new, np.uint16).reshape(N, -1, d)
        v_new = np.asarray(v_new, np.uint16).reshape(N, -1, d)
        n_new = k_new.shape[1]
        zk = np.concatenate([self.tail("k"), k_new], axis=1)
        zv = np.concatenate([self.tail("v"), v_new], axis=1)
        L = self.t_tail + n_new
        nf = max(0, (L - R) // F)
        nq = nf * F
        if self.t_quant + nq > cfg.t_capacity:
            raise ValueError("capacity exceeded")
        if nq:
            set_of = cfg.set_of()
            t0, t1 = self.t_quant, self.t_quant + nq
            rk = quantize_streams(zk[:, :nq], set_of, patterns_k, cfg.metric, b, G, 0)
            rv = quantize_streams(zv[:, :nq], set_of, patterns_v, cfg.metric, b, G, 1, v_rho=cfg.v_rho)
            self.k_codes[:, t0:t1] = rk["packed"].view(np.uint32).reshape(N, nq, d // 32, b)
            self.k_scale[:, t0 // G:t1 // G] = rk["scale"]
            self.k_zero[:, t0 // G:t1 // G] = rk["zero"]
            self.k_idx[:, t0:t1] = rk["idx"].astype(np.uint8)
            wpt = d * b // 32
            self.v_codes[:, t0 * wpt:t1 * wpt] = rv["packed"].view(np.uint32)
            self.v_scale[:, t0 // 16:t1 // 16] = rv["scale"]
            self.v_zero[:, t0 // 16:t1 // 16] = rv["zero"]
            self.v_idx[:, t0:t1] = rv["idx"].astype(np.uint8)
            self.k_best[:, t0:t1], self.k_second[:, t0:t1] = rk["best"], rk["second"]
            self.v_best[:, t0:t1], self.v_second[:, t0:t1] = rv["best"], rv["second"]
            self.t_quant = t1
        # new tail = what is left, written into the ring after advancing its start
        self.tail_start = (self.tail_start + nq) % self.ring
        self.t_tail = L - nq
        slots = (self.tail_start + np.arange(self.t_tail)) % self.ring
        self.tail_k[:, slots, :] = zk[:, nq:]
        self.tail_v[:, slots, :] = zv[:, nq:]
        return nq

    def dequantize(self, patterns_k, patterns_v, t0=0, t1=None):
        """Reconstructed packed part: K^, V^ [N, t1-t0, d] float32."""
        cfg = self.cfg
        t1 = self.t_quant if t1 is None else t1
        N, d, b, G = cfg.n_streams, cfg.head_dim, cfg.bits, cfg.group
        Gc = min(G, d)
        set_of = cfg.set_of()
        K = np.empty((N, t1 - t0, d), np.float32)
        V = np.empty((N, t1 - t0, d), np.float32)
        wpt = d * b // 32
        for s in range(N):
            ck = unpack_k(self.k_codes[s, :self.t_quant], self.t_quant, d, b) if self.t_quant else np.zeros((0, d), np.uint8)
            cv = unpack_v(self.v_codes[s, :self.t_quant * wpt], self.t_quant, d, b) if self.t_quant else np.zeros((0, d), np.uint8)
            if t1 > t0:
                kfull = dequant(0, ck, self.k_scale[s, :self.t_quant // G], self.k_zero[s, :self.t_quant // G],
                                self.k_idx[s, :self.t_quant].astype(np.int32), patterns_k[set_of[s]], G)
                vfull = dequant(1, cv, self.v_scale[s, :self.t_quant // 16], self.v_zero[s, :self.t_quant // 16],
                                self.v_idx[s, :self.t_quant].astype(np.int32), patterns_v[set_of[s]], G,
                                thresholded=cfg.v_rho > 0)
                K[s], V[s] = kfull[t0:t1], vfull[t0:t1]
        return K, V

    def materialize(self, patterns_k, patterns_v):
        """K^, V^ over packed part followed by the tail: [N, t_quant+t_tail, d] float32."""
        K, V = self.dequantize(patterns_k, patterns_v)
        tk = self.tail("k").view(np.float16).astype(np.float32)
        tv = self.tail("v").view(np.float16).astype(np.float32)
        return np.concatenate([K, tk], axis=1), np.concatenate([V, tv], axis=1)


def decode_attention(cache: Cache, q_u16, patterns_k, patterns_v, softmax_scale,
                     prefix: Cache | None = None, prefix_patterns_k=None, prefix_patterns_v=None):
    """softmax(scale * q.K^) V^ over [shared prefix | packed | tail] (Sec. 3.4 fused kernels' result).

    prefix: a cache with n_seq == 1 whose streams (one per KV head) come first
    in every sequence's context.
    """
    cfg = cache.cfg
    K, V = cache.materialize(patterns_k, patterns_v)
    d = cfg.head_dim
    K = K.reshape(cfg.n_seq, cfg.n_kv_heads, -1, d)
    V = V.reshape(cfg.n_seq, cfg.n_kv_heads, -1, d)
    if prefix is not None:
        pk, pv = prefix.materialize(prefix_patterns_k, prefix_patterns_v)
        pk = np.broadcast_to(pk[None], (cfg.n_seq,) + pk.shape)
        pv = np.broadcast_to(pv[None], (cfg.n_seq,) + pv.shape)
        K = np.concatenate([pk, K], axis=2)
        V = np.concatenate([pv, V], axis=2)
    return attend(q_u16, K, V, softmax_scale)


def decode_attention_ragged(caches, q_u16, patterns_k, patterns_v, softmax_scale,
                            prefix: Cache | None = None, prefix_patterns_k=None, prefix_patterns_v=None):
    """A batch whose sequences are filled to different lengths.  The attention of Sec. 3.4 is defined per
    sequence, so this is decode_attention applied to every sequence on its own: caches[i] is sequence i's cache
    (n_seq == 1, one pattern set per KV head), q_u16[i] its query heads."""
    outs, lses = [], []
    for i, c in enumerate(caches):
        assert c.cfg.n_seq == 1
        o, l = decode_attention(c, q_u16[i:i + 1], patterns_k, patterns_v, softmax_scale, prefix=prefix,
                                prefix_patterns_k=prefix_patterns_k, prefix_patterns_v=prefix_patterns_v)
        outs.append(o)
        lses.append(l)
    return np.concatenate(outs), np.concatenate(lses)
