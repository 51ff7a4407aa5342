"""ctypes front end of the CPU oracle (oracle/fx_oracle.cpp).  Test infrastructure only.

Every tensor is a numpy array; bf16 tensors travel as their uint16 bit patterns.  The geometry of a
problem is an `OracleLayout`: the same strided description of a ragged KV cache the paper's method
works on (logical blocks of g_j tokens per KV head, Sec. 2.1 and Sec. 5.3), written independently of
the HIP library's header.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfx_oracle.so")
_lib = None


class _CLayout(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("seq_len", ctypes.c_void_p),
        ("seq_base", ctypes.c_void_p),
        ("kv_head_stride", ctypes.c_int64),
        ("token_stride", ctypes.c_int64),
        ("sum_base", ctypes.c_void_p),
        ("gran", ctypes.c_void_p),
    ]


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _build

            _build.build()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.fxo_select.restype = ctypes.c_int
        _lib.fxo_layer_step.restype = ctypes.c_int
        _lib.fxo_token_weights.restype = ctypes.c_int64
    return _lib


def default_threads() -> int:
    return max(1, len(os.sched_getaffinity(0)))


@dataclass
class OracleLayout:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: np.ndarray  # int32 [batch]
    seq_base: np.ndarray  # int64 [batch]   element offsets into K and V
    kv_head_stride: int
    token_stride: int
    sum_base: np.ndarray  # int64 [batch * n_kv_heads]   block offsets into the summaries
    gran: np.ndarray  # int32 [n_kv_heads]

    def __post_init__(self):
        self.seq_len = np.ascontiguousarray(self.seq_len, dtype=np.int32)
        self.seq_base = np.ascontiguousarray(self.seq_base, dtype=np.int64)
        self.sum_base = np.ascontiguousarray(self.sum_base, dtype=np.int64).reshape(-1)
        self.gran = np.ascontiguousarray(self.gran, dtype=np.int32)
        assert self.sum_base.size == self.batch * self.n_kv_heads
        assert self.gran.size == self.n_kv_heads

    @property
    def batch(self) -> int:
        return int(self.seq_len.size)

    def n_blocks(self, b: int, j: int) -> int:
        g = int(self.gran[j])
        return (int(self.seq_len[b]) + g - 1) // g

    def max_blocks(self) -> int:
        return max(self.n_blocks(b, j) for b in range(self.batch) for j in range(self.n_kv_heads))

    def total_summary_blocks(self) -> int:
        return max(
            int(self.sum_base[b * self.n_kv_heads + j]) + self.n_blocks(b, j)
            for b in range(self.batch)
            for j in range(self.n_kv_heads)
        )

    def _c(self) -> _CLayout:
        return _CLayout(
            self.batch,
            self.n_q_heads,
            self.n_kv_heads,
            self.head_dim,
            self.seq_len.ctypes.data,
            self.seq_base.ctypes.data,
            self.kv_head_stride,
            self.token_stride,
            self.sum_base.ctypes.data,
            self.gran.ctypes.data,
        )


def _u16(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _ptr(a):
    return ctypes.c_void_p(None if a is None else a.ctypes.data)


def summarize(L: OracleLayout, K: np.ndarray, threads: int = 1) -> np.ndarray:
    """Min/max summaries, uint16 [total_blocks, 2, d] (row 0 = min, row 1 = max)."""
    K = _u16(K)
    S = np.zeros((L.total_summary_blocks(), 2, L.head_dim), dtype=np.uint16)
    c = L._c()
    _load().fxo_summarize(ctypes.byref(c), _ptr(K), _ptr(S), ctypes.c_int(threads))
    return S


def scores(L: OracleLayout, q, S, sink_tokens: int, window_tokens: int, threads: int = 1) -> np.ndarray:
    """fp64 [batch, Hq, max_blocks]; NaN outside each head's candidate range."""
    q, S = _u16(q), _u16(S)
    nb = L.max_blocks()
    out = np.full((L.batch, L.n_q_heads, nb), np.nan, dtype=np.float64)
    c = L._c()
    _load().fxo_scores(
        ctypes.byref(c), _ptr(q), _ptr(S), ctypes.c_int(sink_tokens), ctypes.c_int(window_tokens), _ptr(out),
        ctypes.c_int64(nb), ctypes.c_int(threads),
    )
    return out


def select(L: OracleLayout, q, S, *, budget_frac=None, budget_blocks=None, sink_tokens: int, window_tokens: int,
           k_max: int, threads: int = 1):
    """Returns (idx int32 [batch,Hq,k_max], cnt int32 [batch,Hq], tie_gap f64 [batch,Hq], kth_score f64)."""
    assert (budget_frac is None) != (budget_blocks is None)
    q, S = _u16(q), _u16(S)
    bf = None if budget_frac is None else np.ascontiguousarray(
        np.broadcast_to(np.asarray(budget_frac, dtype=np.float32), (L.batch, L.n_q_heads)))
    bb = None if budget_blocks is None else np.ascontiguousarray(
        np.broadcast_to(np.asarray(budget_blocks, dtype=np.int32), (L.batch, L.n_q_heads)))
    idx = np.empty((L.batch, L.n_q_heads, k_max), dtype=np.int32)
    cnt = np.empty((L.batch, L.n_q_heads), dtype=np.int32)
    gap = np.empty((L.batch, L.n_q_heads), dtype=np.float64)
    kth = np.empty((L.batch, L.n_q_heads), dtype=np.float64)
    c = L._c()
    rc = _load().fxo_select(
        ctypes.byref(c), _ptr(q), _ptr(S), _ptr(bf), _ptr(bb), ctypes.c_int(sink_tokens),
        ctypes.c_int(window_tokens), ctypes.c_int(k_max), _ptr(idx), _ptr(cnt), _ptr(gap), _ptr(kth),
        ctypes.c_int(threads),
    )
    if rc != 0:
        raise ValueError("k_max is smaller than a head's block budget")
    return idx, cnt, gap, kth


def sparse_attention(L: OracleLayout, q, K, V, idx, cnt, *, sink_tokens: int, window_tokens: int, mode: str = "two_pass",
                     chunk_tokens: int = 0, threads: int = 1, return_lse: bool = False, group_union: bool = False):
    q, K, V = _u16(q), _u16(K), _u16(V)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    cnt = np.ascontiguousarray(cnt, dtype=np.int32)
    k_max = idx.shape[-1]
    out = np.empty((L.batch, L.n_q_heads, L.head_dim), dtype=np.float64)
    lse = np.empty((L.batch, L.n_q_heads), dtype=np.float64) if return_lse else None
    m = {"two_pass": 0, "chunked": 1}[mode]
    if m == 1:
        assert chunk_tokens > 0
    c = L._c()
    _load().fxo_sparse_attention(
        ctypes.byref(c), _ptr(q), _ptr(K), _ptr(V), _ptr(idx), _ptr(cnt), ctypes.c_int(k_max),
        ctypes.c_int(sink_tokens), ctypes.c_int(window_tokens), ctypes.c_int(m), ctypes.c_int64(chunk_tokens),
        ctypes.c_int(1 if group_union else 0), _ptr(out), _ptr(lse), ctypes.c_int(threads),
    )
    return (out, lse) if return_lse else out


def dense_attention(L: OracleLayout, q, K, V, threads: int = 1, return_lse: bool = False):
    q, K, V = _u16(q), _u16(K), _u16(V)
    out = np.empty((L.batch, L.n_q_heads, L.head_dim), dtype=np.float64)
    lse = np.empty((L.batch, L.n_q_heads), dtype=np.float64) if return_lse else None
    c = L._c()
    _load().fxo_dense_attention(ctypes.byref(c), _ptr(q), _ptr(K), _ptr(V), _ptr(out), _ptr(lse), ctypes.c_int(threads))
    return (out, lse) if return_lse else out


def token_weights(L: OracleLayout, q, K, V, idx, cnt, *, sink_tokens: int, window_tokens: int, b: int, h: int,
                  group_union: bool = False):
    """Token set of head (b, h) and its softmax weights (two-pass)."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    cnt = np.ascontiguousarray(cnt, dtype=np.int32)
    cap = int(L.seq_len[b])
    tokens = np.empty(cap, dtype=np.int64)
    w = np.empty(cap, dtype=np.float64)
    c = L._c()
    n = _load().fxo_token_weights(
        ctypes.byref(c), _ptr(q), _ptr(K), _ptr(V), _ptr(idx), _ptr(cnt), ctypes.c_int(idx.shape[-1]),
        ctypes.c_int(sink_tokens), ctypes.c_int(window_tokens), ctypes.c_int(b), ctypes.c_int(h),
        ctypes.c_int(1 if group_union else 0), ctypes.c_int64(cap), _ptr(tokens), _ptr(w),
    )
    return tokens[:n].copy(), w[:n].copy()


def layer_step(L: OracleLayout, q, K, V, S, *, budget_frac=None, budget_blocks=None, sink_tokens: int,
               window_tokens: int, k_max: int, threads: int = 1):
    """Selection + sparse attention, the unit the benchmark's cpu_baseline leg times."""
    assert (budget_frac is None) != (budget_blocks is None)
    q, K, V, S = _u16(q), _u16(K), _u16(V), _u16(S)
    bf = None if budget_frac is None else np.ascontiguousarray(
        np.broadcast_to(np.asarray(budget_frac, dtype=np.float32), (L.batch, L.n_q_heads)))
    bb = None if budget_blocks is None else np.ascontiguousarray(
        np.broadcast_to(np.asarray(budget_blocks, dtype=np.int32), (L.batch, L.n_q_heads)))
    idx = np.empty((L.batch, L.n_q_heads, k_max), dtype=np.int32)
    cnt = np.empty((L.batch, L.n_q_heads), dtype=np.int32)
    out = np.empty((L.batch, L.n_q_heads, L.head_dim), dtype=np.float64)
    c = L._c()
    rc = _load().fxo_layer_step(
        ctypes.byref(c), _ptr(q), _ptr(K), _ptr(V), _ptr(S), _ptr(bf), _ptr(bb), ctypes.c_int(sink_tokens),
        ctypes.c_int(window_tokens), ctypes.c_int(k_max), _ptr(idx), _ptr(cnt), _ptr(out), ctypes.c_int(threads),
    )
    if rc != 0:
        raise ValueError("k_max is smaller than a head's block budget")
    return idx, cnt, out
