"""Glue and comparison rules around the CPU oracle.  Test infrastructure only (like the rest of oracle/).

Turns a synthetic workload (any object with the fields the generators use; the package that defines it is
not imported here) into what the oracle wants, and states the comparison rule for selected block sets.
"""
from __future__ import annotations

import numpy as np

from . import fx_oracle as O

NEAR_TIE = 1e-5  # relative gap between the k-th and (k+1)-th score below which a head counts as a near tie


def layout_for(wl, pl) -> O.OracleLayout:
    """Oracle layout of workload `wl` placed as `pl` says (sequence lengths, offsets, strides, block sizes)."""
    return O.OracleLayout(
        n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim, seq_len=pl.seq_len,
        seq_base=pl.seq_base, kv_head_stride=pl.kv_head_stride, token_stride=pl.token_stride,
        sum_base=pl.sum_base.reshape(-1), gran=pl.gran,
    )


def bf16_tensor_bits(t) -> np.ndarray:
    """torch bf16 tensor (any device) -> host uint16 bit patterns."""
    import torch

    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f64(u16: np.ndarray) -> np.ndarray:
    return (u16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def compare_selection(idx_g, cnt_g, idx_o, cnt_o, gap, kth, scores):
    """Index-exact comparison with the near-tie rule: a head whose k-th and (k+1)-th oracle scores differ
    by less than 1e-5 relative may differ from the oracle, but only in blocks whose score lies within that
    band of the k-th score.  Returns (n_exempt_heads, n_heads_that_differ); raises on a real mismatch."""
    B, H = cnt_o.shape
    exempt = differ = 0
    for b in range(B):
        for h in range(H):
            assert cnt_g[b, h] == cnt_o[b, h], (b, h, cnt_g[b, h], cnt_o[b, h])
            k = int(cnt_o[b, h])
            row_g, row_o = idx_g[b, h], idx_o[b, h]
            assert (row_g[k:] == -1).all(), (b, h)
            assert (np.diff(row_g[:k]) > 0).all(), (b, h, "not ascending / duplicates")
            near = gap[b, h] < NEAR_TIE
            exempt += int(near)
            if np.array_equal(row_g[:k], row_o[:k]):
                continue
            differ += 1
            assert near, (b, h, "selection differs without a near tie", gap[b, h])
            sym = np.setxor1d(row_g[:k], row_o[:k])
            s = scores[b, h, sym]
            band = NEAR_TIE * np.maximum(np.abs(s), abs(kth[b, h]))
            assert (np.abs(s - kth[b, h]) <= band).all(), (b, h, "difference outside the near-tie band")
    return exempt, differ
