"""Python binding of libfluxion.so (the HIP C-ABI library declared in include/fluxion.h).

Argument marshalling only: every step of the path runs in the library's kernels.  PyTorch supplies
device memory and the current HIP stream.  There is no CPU fallback: if the built library is missing
or a call fails, this module raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FLUXION_LIB", os.path.join(_HERE, "libfluxion.so"))  # override: development builds

EXPORTS = (
    "fx_status_string", "fx_summarize", "fx_select_workspace_bytes", "fx_select", "fx_decode_workspace_bytes",
    "fx_sparse_decode", "fx_profile_enable", "fx_profile_read", "fx_probe_read", "fx_probe_read_streaming", "fx_probe_copy", "fx_select_workspace_view", "fx_choose_granularity",
    "fx_coarsen_summaries", "fx_summarize_append", "fx_sparse_decode_union", "fx_sparse_decode_static",
)

FX_OK, FX_ERR_INVALID_ARG, FX_ERR_UNSUPPORTED, FX_ERR_WORKSPACE_TOO_SMALL, FX_ERR_HIP, FX_ERR_SCRATCH_LIMIT = range(6)


class FluxionError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (fx_status {status})")


class _CLayout(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("max_seq_len", ctypes.c_int32),
        ("seq_len", ctypes.c_void_p),
        ("seq_base", ctypes.c_void_p),
        ("kv_head_stride", ctypes.c_int64),
        ("token_stride", ctypes.c_int64),
        ("sum_base", ctypes.c_void_p),
        ("gran", ctypes.c_void_p),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (run paper_2605_07719_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_07719_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        L.fx_status_string.restype = ctypes.c_char_p
        L.fx_status_string.argtypes = [ctypes.c_int]
        L.fx_select_workspace_bytes.restype = ctypes.c_size_t
        L.fx_select_workspace_bytes.argtypes = [ctypes.c_void_p]
        L.fx_decode_workspace_bytes.restype = ctypes.c_size_t
        L.fx_decode_workspace_bytes.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        L.fx_summarize.restype = ctypes.c_int
        L.fx_summarize.argtypes = [ctypes.c_void_p] * 4
        L.fx_select.restype = ctypes.c_int
        L.fx_select.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int32] * 3 + [ctypes.c_void_p] * 3 + [
            ctypes.c_size_t, ctypes.c_void_p]
        for fn in (L.fx_sparse_decode, L.fx_sparse_decode_union):
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_int32] * 3 + [ctypes.c_void_p] * 2 + [
                ctypes.c_size_t, ctypes.c_void_p]
        L.fx_sparse_decode_static.restype = ctypes.c_int
        L.fx_sparse_decode_static.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_int32] * 3 + [ctypes.c_void_p] * 2
        L.fx_summarize_append.restype = ctypes.c_int
        L.fx_summarize_append.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int32, ctypes.c_void_p]
        L.fx_profile_enable.restype = ctypes.c_int
        L.fx_profile_enable.argtypes = [ctypes.c_int]
        L.fx_profile_read.restype = ctypes.c_int
        L.fx_profile_read.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.fx_probe_read.restype = ctypes.c_int
        L.fx_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        L.fx_probe_read_streaming.restype = ctypes.c_int
        L.fx_probe_read_streaming.argtypes = L.fx_probe_read.argtypes
        L.fx_probe_copy.restype = ctypes.c_int
        L.fx_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().fx_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != FX_OK:
        raise FluxionError(status, where)


def _dptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


@dataclass
class Layout:
    """fx_layout with its device arrays kept alive.  `gran` stays on the host."""

    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    max_seq_len: int
    seq_len: torch.Tensor  # int32 [batch], device
    seq_base: torch.Tensor  # int64 [batch], device
    kv_head_stride: int
    token_stride: int
    sum_base: torch.Tensor  # int64 [batch * n_kv_heads], device
    gran: np.ndarray  # int32 [n_kv_heads], host

    def __post_init__(self):
        self.gran = np.ascontiguousarray(self.gran, dtype=np.int32)
        assert self.seq_len.dtype == torch.int32 and self.seq_base.dtype == torch.int64
        assert self.sum_base.dtype == torch.int64

    @property
    def batch(self) -> int:
        return int(self.seq_len.numel())

    def c_struct(self) -> _CLayout:
        return _CLayout(
            self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.max_seq_len,
            self.seq_len.data_ptr(), self.seq_base.data_ptr(), self.kv_head_stride, self.token_stride,
            self.sum_base.data_ptr(), self.gran.ctypes.data,
        )

    @staticmethod
    def from_host(n_q_heads, n_kv_heads, head_dim, seq_len: Sequence[int], seq_base: Sequence[int],
                  kv_head_stride: int, token_stride: int, sum_base: Sequence[int], gran: Sequence[int],
                  device="cuda", max_seq_len: Optional[int] = None) -> "Layout":
        seq_len = np.asarray(seq_len, dtype=np.int32)
        return Layout(
            n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=head_dim,
            max_seq_len=int(seq_len.max()) if max_seq_len is None else int(max_seq_len),
            seq_len=torch.from_numpy(seq_len).to(device),
            seq_base=torch.from_numpy(np.asarray(seq_base, dtype=np.int64)).to(device),
            kv_head_stride=int(kv_head_stride), token_stride=int(token_stride),
            sum_base=torch.from_numpy(np.asarray(sum_base, dtype=np.int64).reshape(-1)).to(device),
            gran=np.asarray(gran, dtype=np.int32),
        )


def select_workspace_bytes(layout: Layout) -> int:
    c = layout.c_struct()
    return int(lib().fx_select_workspace_bytes(ctypes.byref(c)))


def choose_granularity(n_q_heads: int, n_kv_heads: int, bgt0, slope, l_cpu: int, streaming=None,
                       candidates=(16, 32, 64, 128)):
    """fx_choose_granularity: (gran int32 [Hkv], budget float32 [Hq], volume float64 [Hkv])."""
    bgt0 = np.ascontiguousarray(bgt0, dtype=np.float32)
    slope = np.ascontiguousarray(slope, dtype=np.float32)
    assert bgt0.shape == (n_q_heads,) and slope.shape == (n_q_heads,)
    st = None if streaming is None else np.ascontiguousarray(streaming, dtype=np.uint8)
    cand = np.ascontiguousarray(candidates, dtype=np.int32)
    gran = np.zeros(n_kv_heads, dtype=np.int32)
    budget = np.zeros(n_q_heads, dtype=np.float32)
    volume = np.zeros(n_kv_heads, dtype=np.float64)
    fn = lib().fx_choose_granularity
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                   ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    _check(fn(n_q_heads, n_kv_heads, bgt0.ctypes.data, slope.ctypes.data, None if st is None else st.ctypes.data,
              int(l_cpu), cand.ctypes.data, int(cand.size), gran.ctypes.data, budget.ctypes.data,
              volume.ctypes.data), "fx_choose_granularity")
    return gran, budget, volume


def coarsen_summaries(fine: Layout, fine_summaries: torch.Tensor, coarse: Layout, coarse_summaries: torch.Tensor,
                      stream=None) -> None:
    """fx_coarsen_summaries: summaries at coarse.gran from summaries at fine.gran (exact)."""
    cf, cc = fine.c_struct(), coarse.c_struct()
    fn = lib().fx_coarsen_summaries
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_void_p] * 5
    _check(fn(ctypes.byref(cf), _dptr(fine_summaries), ctypes.byref(cc), _dptr(coarse_summaries), _stream(stream)),
           "fx_coarsen_summaries")


def select_workspace_view(layout: Layout) -> dict:
    """fx_select_workspace_view: byte offsets of the approximate scores and their error magnitudes."""
    c = layout.c_struct()
    a, m = ctypes.c_size_t(), ctypes.c_size_t()
    stride, mstride, gamma = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_float()
    fn = lib().fx_select_workspace_view
    fn.restype = ctypes.c_int
    _check(fn(ctypes.byref(c), ctypes.byref(a), ctypes.byref(m), ctypes.byref(stride), ctypes.byref(mstride),
              ctypes.byref(gamma)), "fx_select_workspace_view")
    return {"approx_offset": a.value, "mag_offset": m.value, "row_stride": stride.value,
            "mag_stride": mstride.value, "gamma": gamma.value}


def decode_workspace_bytes(layout: Layout, k_max: int, sink_tokens: int, window_tokens: int) -> int:
    c = layout.c_struct()
    return int(lib().fx_decode_workspace_bytes(ctypes.byref(c), k_max, sink_tokens, window_tokens))


def summarize(layout: Layout, K: torch.Tensor, summaries: torch.Tensor, stream=None) -> None:
    """fx_summarize: per-block min/max rows of K into `summaries` (bf16 [total_blocks, 2, d])."""
    c = layout.c_struct()
    _check(lib().fx_summarize(ctypes.byref(c), _dptr(K), _dptr(summaries), _stream(stream)), "fx_summarize")


def select(layout: Layout, q: torch.Tensor, summaries: torch.Tensor, *, budget_frac: Optional[torch.Tensor] = None,
           budget_blocks: Optional[torch.Tensor] = None, sink_tokens: int, window_tokens: int, k_max: int,
           idx: torch.Tensor, cnt: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    """fx_select: block scores and per-head top-k into idx (int32 [batch,Hq,k_max]) and cnt (int32 [batch,Hq])."""
    c = layout.c_struct()
    _check(
        lib().fx_select(
            ctypes.byref(c), _dptr(q), _dptr(summaries), _dptr(budget_frac), _dptr(budget_blocks), sink_tokens,
            window_tokens, k_max, _dptr(idx), _dptr(cnt), _dptr(workspace),
            workspace.numel() * workspace.element_size(), _stream(stream),
        ),
        "fx_select",
    )


def summarize_append(layout: Layout, K: torch.Tensor, summaries: torch.Tensor, prev_len: torch.Tensor,
                     max_new_tokens: int, stream=None) -> None:
    """fx_summarize_append: redo only the summary blocks that hold tokens at or after prev_len[b]."""
    assert prev_len.dtype == torch.int32
    c = layout.c_struct()
    _check(lib().fx_summarize_append(ctypes.byref(c), _dptr(K), _dptr(summaries), _dptr(prev_len), max_new_tokens,
                                     _stream(stream)), "fx_summarize_append")


def sparse_decode(layout: Layout, q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, idx: torch.Tensor,
                  cnt: torch.Tensor, *, k_max: int, sink_tokens: int, window_tokens: int, out: torch.Tensor,
                  workspace: torch.Tensor, stream=None, group_union: bool = False) -> None:
    """fx_sparse_decode (or fx_sparse_decode_union): split-K sparse attention + merge into out
    (float32 [batch,Hq,d])."""
    c = layout.c_struct()
    fn = lib().fx_sparse_decode_union if group_union else lib().fx_sparse_decode
    _check(
        fn(
            ctypes.byref(c), _dptr(q), _dptr(K), _dptr(V), _dptr(idx), _dptr(cnt), k_max, sink_tokens,
            window_tokens, _dptr(out), _dptr(workspace), workspace.numel() * workspace.element_size(),
            _stream(stream),
        ),
        "fx_sparse_decode",
    )


def sparse_decode_static(layout: Layout, q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, idx: torch.Tensor,
                         cnt: torch.Tensor, *, k_max: int, sink_tokens: int, window_tokens: int, out: torch.Tensor,
                         stream=None) -> None:
    """fx_sparse_decode_static: fx_sparse_decode with the scratch taken from the library's built-in buffer
    (for callers that cannot allocate a workspace)."""
    c = layout.c_struct()
    _check(
        lib().fx_sparse_decode_static(
            ctypes.byref(c), _dptr(q), _dptr(K), _dptr(V), _dptr(idx), _dptr(cnt), k_max, sink_tokens,
            window_tokens, _dptr(out), _stream(stream),
        ),
        "fx_sparse_decode_static",
    )


PROFILE_SLOTS = ("score", "topk", "plan", "attend", "merge")


def profile_enable(enable: bool) -> None:
    """fx_profile_enable: bracket every kernel of fx_select / fx_sparse_decode with HIP events."""
    _check(lib().fx_profile_enable(1 if enable else 0), "fx_profile_enable")


def profile_read() -> dict:
    """fx_profile_read: milliseconds per kernel of the most recent calls (waits for them)."""
    ms = (ctypes.c_float * len(PROFILE_SLOTS))()
    _check(lib().fx_profile_read(ms, len(PROFILE_SLOTS)), "fx_profile_read")
    return {name: float(ms[i]) for i, name in enumerate(PROFILE_SLOTS)}


def probe_read(src: torch.Tensor, sink: torch.Tensor, wg_per_cu: int = 8, stream=None) -> None:
    """fx_probe_read: plain streaming read of the whole tensor (measurement aid)."""
    _check(lib().fx_probe_read(_dptr(src), src.numel() * src.element_size(), _dptr(sink), wg_per_cu, _stream(stream)),
           "fx_probe_read")


def probe_read_streaming(src: torch.Tensor, sink: torch.Tensor, wg_per_cu: int = 8, stream=None) -> None:
    """fx_probe_read_streaming: the same read with non-temporal loads (measurement aid)."""
    _check(lib().fx_probe_read_streaming(_dptr(src), src.numel() * src.element_size(), _dptr(sink), wg_per_cu,
                                         _stream(stream)), "fx_probe_read_streaming")


def probe_copy(dst: torch.Tensor, src: torch.Tensor, wg_per_cu: int = 8, stream=None) -> None:
    """fx_probe_copy: plain copy src -> dst (measurement aid)."""
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= n
    _check(lib().fx_probe_copy(_dptr(dst), _dptr(src), n, wg_per_cu, _stream(stream)), "fx_probe_copy")
