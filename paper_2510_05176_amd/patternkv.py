"""ctypes binding of libpatternkv.so (the C ABI of include/patternkv.h).

Argument marshalling only: every step of the hot path runs in the HIP kernels of the
library.  PyTorch is used for device memory and the current stream.  There is no CPU
fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, asdict, replace

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpatternkv.so")

if not os.path.exists(_LIB_PATH):
    raise ImportError(
        f"{_LIB_PATH} is missing: build it with `python -m paper_2510_05176_amd.build` "
        "(hipcc, gfx950). There is no fallback path.")
_lib = C.CDLL(_LIB_PATH)

PK_OK = 0
METRIC_L2, METRIC_MINMAX = 0, 1
NO_PATTERN = 255   # v_idx of a token the adaptive threshold sent to raw quantization
OP_MINE, OP_APPEND, OP_DECODE = 0, 1, 2


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_seq", "n_kv_heads", "n_q_heads", "head_dim", "n_patterns", "seqs_per_set",
        "bits", "group", "recent", "flush", "t_capacity", "metric")] + [("v_rho", C.c_float), ("page_tokens", C.c_int32),
                                                                          ("n_pages", C.c_int32)]


class _Layout(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "k_codes", "k_scale", "k_zero", "k_idx", "v_codes", "v_scale", "v_zero", "v_idx",
        "tail_k", "tail_v", "total")] + [("align", C.c_uint32)]


class _Cache(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "k_codes", "k_scale", "k_zero", "k_idx", "v_codes", "v_scale", "v_zero", "v_idx",
        "tail_k", "tail_v", "page_table")]


class _State(C.Structure):
    _fields_ = [("t_quant", C.c_int32), ("t_tail", C.c_int32), ("tail_start", C.c_int32)]


ABI_VERSION = 5          # PK_ABI_VERSION of include/patternkv.h this binding's structs are laid out for

_lib.pk_abi_version.restype = C.c_uint32
if int(_lib.pk_abi_version()) != ABI_VERSION:
    raise ImportError(f"libpatternkv.so has ABI {int(_lib.pk_abi_version())}, this binding needs {ABI_VERSION}: rebuild")
_lib.pk_status_string.restype = C.c_char_p
_lib.pk_status_string.argtypes = [C.c_int]
_lib.pk_cache_layout.restype = C.c_int
_lib.pk_cache_layout.argtypes = [C.POINTER(_Config), C.POINTER(_Layout)]
_lib.pk_decode_plan.restype = C.c_int
_lib.pk_decode_plan.argtypes = [C.POINTER(_Config), C.c_int64, C.c_int64, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                C.POINTER(C.c_size_t)]
_lib.pk_workspace_bytes.restype = C.c_size_t
_lib.pk_workspace_bytes.argtypes = [C.POINTER(_Config), C.c_int, C.c_int64, C.c_int64]
_lib.pk_mine_patterns.restype = C.c_int
_lib.pk_mine_patterns.argtypes = [C.POINTER(_Config), C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                  C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                  C.c_void_p]
_lib.pk_quantize_append.restype = C.c_int
_lib.pk_quantize_append.argtypes = [C.POINTER(_Config), C.POINTER(_Cache), C.POINTER(_State), C.c_void_p,
                                    C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_size_t, C.c_void_p]
_lib.pk_quantize_append_ragged.restype = C.c_int
_lib.pk_quantize_append_ragged.argtypes = [C.POINTER(_Config), C.POINTER(_Cache), C.POINTER(_State), C.c_void_p, C.c_void_p,
                                           C.POINTER(C.c_int32), C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_size_t, C.c_void_p]
_lib.pk_decode_attention.restype = C.c_int
_lib.pk_decode_attention.argtypes = [C.POINTER(_Config), C.POINTER(_Cache), C.POINTER(_State),
                                     C.POINTER(_Config), C.POINTER(_Cache), C.POINTER(_State), C.c_void_p,
                                     C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_size_t, C.c_void_p]
_lib.pk_decode_attention_ragged.restype = C.c_int
_lib.pk_decode_attention_ragged.argtypes = [C.POINTER(_Config), C.POINTER(_Cache), C.POINTER(_State), C.c_void_p,
                                            C.POINTER(_Config), C.POINTER(_Cache), C.POINTER(_State), C.c_void_p,
                                            C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_size_t, C.c_void_p]
_lib.pk_decode_attention_noalloc.restype = C.c_int
_lib.pk_decode_attention_noalloc.argtypes = [C.POINTER(_Config), C.POINTER(_Cache), C.POINTER(_State),
                                             C.POINTER(_Config), C.POINTER(_Cache), C.POINTER(_State), C.c_void_p,
                                             C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
NOALLOC_SCRATCH_BYTES = 32 << 20   # PK_NOALLOC_SCRATCH_BYTES
_lib.pk_window_pattern.restype = C.c_int
_lib.pk_window_pattern.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
_lib.pk_dequantize.restype = C.c_int
_lib.pk_dequantize.argtypes = [C.POINTER(_Config), C.POINTER(_Cache), C.POINTER(_State), C.c_void_p,
                               C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]


class PkError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {_lib.pk_status_string(status).decode()} (status {status})")


def _check(status: int, where: str):
    if status != PK_OK:
        raise PkError(status, where)


def pk_abi_version() -> int:
    return int(_lib.pk_abi_version())


def pk_status_string(status: int) -> str:
    return _lib.pk_status_string(int(status)).decode()


@dataclass
class Config:
    n_seq: int = 1
    n_kv_heads: int = 1
    n_q_heads: int = 1
    head_dim: int = 128
    n_patterns: int = 16
    seqs_per_set: int = 0
    bits: int = 2
    group: int = 64
    recent: int = 0
    flush: int = 64
    t_capacity: int = 0
    metric: int = METRIC_L2
    v_rho: float = 0.0      # adaptive threshold on V (0 = off); see include/patternkv.h
    page_tokens: int = 0    # > 0: the packed arrays are a pool of n_pages pages of this many tokens (all KV heads)
    n_pages: int = 0

    def c(self) -> _Config:
        return _Config(**asdict(self))

    @property
    def n_streams(self) -> int:
        return self.n_seq * self.n_kv_heads

    @property
    def n_sets(self) -> int:
        if self.seqs_per_set == 0:
            return self.n_kv_heads
        return -(-self.n_seq // self.seqs_per_set) * self.n_kv_heads


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to the library must be contiguous"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def pk_cache_layout(cfg: Config) -> dict:
    lay = _Layout()
    c = cfg.c()
    _check(_lib.pk_cache_layout(C.byref(c), C.byref(lay)), "pk_cache_layout")
    return {n: int(getattr(lay, n)) for n, _ in _Layout._fields_}


def pk_decode_plan(cfg: Config, own_packed: int, prefix_packed: int = 0):
    """(split length in tokens, partial slots per stream, workspace bytes in use) of a decode over that many packed tokens."""
    c = cfg.c()
    split, slots, need = C.c_int32(0), C.c_int32(0), C.c_size_t(0)
    st = _lib.pk_decode_plan(C.byref(c), own_packed, prefix_packed, C.byref(split), C.byref(slots), C.byref(need))
    _check(st, "pk_decode_plan")
    return int(split.value), int(slots.value), int(need.value)


def pk_workspace_bytes(cfg: Config, op: int, a: int, b: int = 0) -> int:
    c = cfg.c()
    return int(_lib.pk_workspace_bytes(C.byref(c), op, a, b))


_ARRAYS = ("k_codes", "k_scale", "k_zero", "k_idx", "v_codes", "v_scale", "v_zero", "v_idx", "tail_k", "tail_v")


class Cache:
    """Device memory of one cache (torch uint8 tensors sized by pk_cache_layout) plus its host state."""

    def __init__(self, cfg: Config, device="cuda"):
        self.cfg = cfg
        lay = pk_cache_layout(cfg)
        self.bytes = {n: lay[n] for n in _ARRAYS}
        self.buf = {n: torch.zeros(max(lay[n], 16), dtype=torch.uint8, device=device) for n in _ARRAYS}
        self.state = _State(0, 0, 0)
        # paged: physical page of every logical page, int32 [n_seq, t_capacity / page_tokens]; the caller fills it
        self.page_table = None
        if cfg.page_tokens > 0:
            self.page_table = torch.zeros((cfg.n_seq, cfg.t_capacity // cfg.page_tokens), dtype=torch.int32, device=device)

    def c(self) -> _Cache:
        if self.page_table is not None:
            assert self.page_table.dtype == torch.int32 and self.page_table.is_contiguous()
            assert tuple(self.page_table.shape) == (self.cfg.n_seq, self.cfg.t_capacity // self.cfg.page_tokens)
        return _Cache(**{n: self.buf[n].data_ptr() for n in _ARRAYS},
                      page_table=None if self.page_table is None else self.page_table.data_ptr())

    @property
    def t_quant(self):
        return int(self.state.t_quant)

    @property
    def t_tail(self):
        return int(self.state.t_tail)

    @property
    def tail_start(self):
        return int(self.state.tail_start)

    def array(self, name):
        """Raw bytes of one cache array (uint8 tensor of the layout's size)."""
        return self.buf[name][: self.bytes[name]]

    def sequence(self, i: int) -> "Cache":
        """The part of sequence i as a cache of its own (n_seq = 1, one pattern set per KV head) over the same
        memory, with a fill state of its own: the arrays are laid out stream by stream."""
        return self.sequences(i, 1)

    def sequences(self, first: int, count: int) -> "Cache":
        """Sequences [first, first + count) as a cache of their own (one pattern set per KV head, shared by them).
        A paged cache shares its page pool with the view; only the tails and the page table rows are the view's."""
        sub = Cache.__new__(Cache)
        sub.cfg = replace(self.cfg, n_seq=count, seqs_per_set=0)
        sub.state = _State(0, 0, 0)
        paged = self.page_table is not None
        sub.page_table = self.page_table[first:first + count] if paged else None
        per = {n: self.bytes[n] // self.cfg.n_seq for n in _ARRAYS}
        sub.bytes, sub.buf = {}, {}
        for n in _ARRAYS:
            if paged and not n.startswith("tail"):
                sub.bytes[n], sub.buf[n] = self.bytes[n], self.buf[n]
            else:
                sub.bytes[n], sub.buf[n] = per[n] * count, self.buf[n][first * per[n]:(first + count) * per[n]]
        return sub


def pk_mine_patterns(cfg: Config, x: torch.Tensor, iters: int, patterns: torch.Tensor | None = None,
                     init_given: bool = False, assign: torch.Tensor | None = None,
                     inertia: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    """x [n_sets, T, d] fp16 (sets may be strided, rows contiguous) -> patterns [n_sets, P, d] fp16."""
    assert x.dtype == torch.float16 and x.dim() == 3 and x.stride(2) == 1 and (x.shape[1] == 1 or x.stride(1) == x.shape[2])
    n_sets, T, d = x.shape
    if patterns is None:
        patterns = torch.empty((n_sets, cfg.n_patterns, d), dtype=torch.float16, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(pk_workspace_bytes(cfg, OP_MINE, T, n_sets), 16), dtype=torch.uint8, device=x.device)
    c = cfg.c()
    set_stride = x.stride(0) if n_sets > 1 else T * d
    st = _lib.pk_mine_patterns(C.byref(c), C.c_void_p(x.data_ptr()), set_stride, n_sets, T, iters,
                               1 if init_given else 0, _ptr(patterns), _ptr(assign), _ptr(inertia),
                               _ptr(workspace), workspace.numel(), _stream())
    _check(st, "pk_mine_patterns")
    return patterns


def pk_window_pattern(x: torch.Tensor, out: torch.Tensor | None = None):
    """x [n_sets, n, d] fp16 (windows may be strided, rows contiguous) -> [n_sets, d] fp16: per-channel
    Chebyshev centre of every window (the decode-stage pattern).  `out` may be a strided view, e.g. one row of
    every set of a table [n_sets, P, d]."""
    assert x.dtype == torch.float16 and x.dim() == 3 and x.stride(2) == 1 and (x.shape[1] == 1 or x.stride(1) == x.shape[2])
    n_sets, n, d = x.shape
    if out is None:
        out = torch.empty((n_sets, d), dtype=torch.float16, device=x.device)
    assert out.dtype == torch.float16 and out.shape == (n_sets, d) and out.stride(1) == 1
    st = _lib.pk_window_pattern(C.c_void_p(x.data_ptr()), x.stride(0) if n_sets > 1 else n * d, n_sets, n, d,
                                C.c_void_p(out.data_ptr()), out.stride(0) if n_sets > 1 else d, _stream())
    _check(st, "pk_window_pattern")
    return out


def pk_quantize_append(cfg: Config, cache: Cache, k_new: torch.Tensor, v_new: torch.Tensor,
                       patterns_k: torch.Tensor, patterns_v: torch.Tensor, workspace: torch.Tensor | None = None):
    """k_new, v_new [n_seq, n_kv_heads, n_new, d] fp16 (token rows contiguous, streams may be strided)."""
    assert k_new.dtype == torch.float16 and v_new.dtype == torch.float16 and k_new.shape == v_new.shape
    n_seq, hkv, n_new, d = k_new.shape

    def stream_stride(t):
        # elements between consecutive (sequence, head) streams; strides of size-1 dimensions carry no meaning
        assert n_new <= 1 or t.stride(2) == d
        assert d == 1 or t.stride(3) == 1
        if hkv > 1:
            ss = t.stride(1)
            assert n_seq == 1 or t.stride(0) == hkv * ss
        elif n_seq > 1:
            ss = t.stride(0)
        else:
            ss = n_new * d
        return ss

    ss = stream_stride(k_new)
    assert stream_stride(v_new) == ss
    cc, kc = cfg.c(), cache.c()
    st = _lib.pk_quantize_append(C.byref(cc), C.byref(kc), C.byref(cache.state), C.c_void_p(k_new.data_ptr()),
                                 C.c_void_p(v_new.data_ptr()), n_new, ss, _ptr(patterns_k),
                                 _ptr(patterns_v), _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                 _stream())
    _check(st, "pk_quantize_append")


def pk_quantize_append_ragged(cfg: Config, cache: Cache, states: list, k_new: torch.Tensor, v_new: torch.Tensor, n_new: list,
                              patterns_k: torch.Tensor, patterns_v: torch.Tensor, seq_states_out: torch.Tensor | None = None,
                              workspace: torch.Tensor | None = None):
    """One append for sequences at different fill: states = one [t_quant, t_tail, tail_start] per sequence (updated in
    place), n_new = new vectors per sequence; k_new, v_new [n_seq, n_kv_heads, n_max, d] fp16, contiguous."""
    assert k_new.dtype == torch.float16 and v_new.dtype == torch.float16 and k_new.shape == v_new.shape
    assert k_new.is_contiguous() and v_new.is_contiguous()
    n_seq, hkv, n_max, d = k_new.shape
    assert n_seq == cfg.n_seq and len(states) == n_seq and len(n_new) == n_seq and max(n_new) <= n_max
    if seq_states_out is not None:
        assert seq_states_out.dtype == torch.int32 and tuple(seq_states_out.shape) == (n_seq, 4) and seq_states_out.is_contiguous()
    if workspace is None:
        workspace = torch.empty(max(pk_workspace_bytes(cfg, OP_APPEND, 0, 0), 16), dtype=torch.uint8, device=k_new.device)
    st_arr = (_State * n_seq)(*[_State(int(s[0]), int(s[1]), int(s[2])) for s in states])
    nn_arr = (C.c_int32 * n_seq)(*[int(n) for n in n_new])
    cc, kc = cfg.c(), cache.c()
    st = _lib.pk_quantize_append_ragged(C.byref(cc), C.byref(kc), st_arr, C.c_void_p(k_new.data_ptr()),
                                        C.c_void_p(v_new.data_ptr()), nn_arr, n_max * d, _ptr(patterns_k), _ptr(patterns_v),
                                        _ptr(seq_states_out), _ptr(workspace), workspace.numel(), _stream())
    _check(st, "pk_quantize_append_ragged")
    for i in range(n_seq):
        states[i][0], states[i][1], states[i][2] = st_arr[i].t_quant, st_arr[i].t_tail, st_arr[i].tail_start


def pk_decode_attention(cfg: Config, cache: Cache, q: torch.Tensor, softmax_scale: float,
                        patterns_k: torch.Tensor, patterns_v: torch.Tensor, out: torch.Tensor | None = None,
                        lse: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                        prefix: Cache | None = None):
    """q [n_seq, n_q_heads, d] fp16 -> out [n_seq, n_q_heads, d] fp32."""
    assert q.dtype == torch.float16
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    if workspace is None:
        a = cache.t_quant + cache.t_tail
        b = 0 if prefix is None else prefix.t_quant + prefix.t_tail
        workspace = torch.empty(max(pk_workspace_bytes(cfg, OP_DECODE, a, b), 16), dtype=torch.uint8, device=q.device)
    cc, kc = cfg.c(), cache.c()
    if prefix is not None:
        pc, pkc = prefix.cfg.c(), prefix.c()
        pargs = (C.byref(pc), C.byref(pkc), C.byref(prefix.state))
    else:
        pargs = (None, None, None)
    st = _lib.pk_decode_attention(C.byref(cc), C.byref(kc), C.byref(cache.state), *pargs, _ptr(q),
                                  C.c_float(softmax_scale), _ptr(patterns_k), _ptr(patterns_v), _ptr(out),
                                  _ptr(lse), _ptr(workspace), workspace.numel(), _stream())
    _check(st, "pk_decode_attention")
    return out


def pk_decode_attention_noalloc(cfg: Config, cache: Cache, q: torch.Tensor, softmax_scale: float,
                                patterns_k: torch.Tensor, patterns_v: torch.Tensor, out: torch.Tensor,
                                lse: torch.Tensor | None = None, prefix: Cache | None = None):
    """pk_decode_attention with the partial results in the library's fixed scratch array: nothing is allocated,
    here or in the library, so `out` [n_seq, n_q_heads, d] fp32 must be passed in."""
    assert q.dtype == torch.float16 and out.dtype == torch.float32 and out.shape == q.shape
    cc, kc = cfg.c(), cache.c()
    if prefix is not None:
        pc, pkc = prefix.cfg.c(), prefix.c()
        pargs = (C.byref(pc), C.byref(pkc), C.byref(prefix.state))
    else:
        pargs = (None, None, None)
    st = _lib.pk_decode_attention_noalloc(C.byref(cc), C.byref(kc), C.byref(cache.state), *pargs, _ptr(q),
                                          C.c_float(softmax_scale), _ptr(patterns_k), _ptr(patterns_v), _ptr(out),
                                          _ptr(lse), _stream())
    _check(st, "pk_decode_attention_noalloc")
    return out


def pk_decode_attention_ragged(cfg: Config, cache: Cache, seq_states: torch.Tensor, bound_t_quant: int, bound_t_tail: int,
                               q: torch.Tensor, softmax_scale: float, patterns_k: torch.Tensor, patterns_v: torch.Tensor,
                               out: torch.Tensor | None = None, lse: torch.Tensor | None = None,
                               workspace: torch.Tensor | None = None, prefix: Cache | None = None):
    """Decode over sequences filled to different lengths.  seq_states: device int32 [n_seq, 4] holding t_quant,
    t_tail, tail_start of every sequence's own cache (and an unused word); bound_*: host upper bounds."""
    assert q.dtype == torch.float16 and seq_states.dtype == torch.int32 and seq_states.is_contiguous()
    assert tuple(seq_states.shape) == (cfg.n_seq, 4)
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    if workspace is None:
        b = 0 if prefix is None else prefix.t_quant + prefix.t_tail
        workspace = torch.empty(max(pk_workspace_bytes(cfg, OP_DECODE, bound_t_quant + bound_t_tail, b), 16),
                                dtype=torch.uint8, device=q.device)
    cc, kc = cfg.c(), cache.c()
    bound = _State(bound_t_quant, bound_t_tail, 0)
    if prefix is not None:
        pc, pkc = prefix.cfg.c(), prefix.c()
        pargs = (C.byref(pc), C.byref(pkc), C.byref(prefix.state))
    else:
        pargs = (None, None, None)
    st = _lib.pk_decode_attention_ragged(C.byref(cc), C.byref(kc), C.byref(bound), _ptr(seq_states), *pargs, _ptr(q),
                                         C.c_float(softmax_scale), _ptr(patterns_k), _ptr(patterns_v), _ptr(out),
                                         _ptr(lse), _ptr(workspace), workspace.numel(), _stream())
    _check(st, "pk_decode_attention_ragged")
    return out


def pk_dequantize(cfg: Config, cache: Cache, patterns_k: torch.Tensor, patterns_v: torch.Tensor,
                  t0: int = 0, t1: int | None = None):
    """Reconstructed K^, V^ of packed tokens [t0, t1): two [N, t1-t0, d] fp32 tensors."""
    t1 = cache.t_quant if t1 is None else t1
    dev = patterns_k.device
    k = torch.empty((cfg.n_streams, t1 - t0, cfg.head_dim), dtype=torch.float32, device=dev)
    v = torch.empty_like(k)
    cc, kc = cfg.c(), cache.c()
    st = _lib.pk_dequantize(C.byref(cc), C.byref(kc), C.byref(cache.state), _ptr(patterns_k), _ptr(patterns_v),
                            t0, t1, _ptr(k), _ptr(v), _stream())
    _check(st, "pk_dequantize")
    return k, v
