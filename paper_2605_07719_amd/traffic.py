"""Algorithmic byte counts of the hot path (host arithmetic for reporting; no kernels here).

The model follows the paper's own accounting of data movement: Sec. 3.3 counts the selected KV tokens
of a layer as tokens x KV heads x head_dim x 2 bytes x 2 (K and V); Eq. 3 (Sec. 5.3) counts, per group,
the block metadata read by selection (two vectors per block: minimum and maximum) plus the selected KV.
"""
from __future__ import annotations

import numpy as np

BF16 = 2


def paper_selected_kv_bytes(context: int, budget: float, n_kv_heads: int, head_dim: int, n_layers: int = 1) -> dict:
    """Sec. 3.3 arithmetic: tokens kept per layer and the K+V bytes they occupy."""
    tokens = budget * context
    per_layer = tokens * n_kv_heads * head_dim * BF16 * 2
    return {"tokens": tokens, "bytes_per_layer": per_layer, "bytes_all_layers": per_layer * n_layers}


def _geometry(N: int, g: int, sink: int, window: int):
    nb = -(-N // g)
    n_sink = -(-sink // g)
    w0 = max(N - window, 0) // g
    return nb, n_sink, w0


def select_bytes(seq_len, gran, n_q_heads, head_dim, sink_tokens, window_tokens, cnt) -> int:
    """Bytes fx_select must move: the candidate summaries once per (sequence, KV head), q, and the
    index lists it writes."""
    total = 0
    group = n_q_heads // len(gran)
    for b, N in enumerate(seq_len):
        for j, g in enumerate(gran):
            nb, n_sink, w0 = _geometry(int(N), int(g), sink_tokens, window_tokens)
            total += max(w0 - n_sink, 0) * 2 * head_dim * BF16
        total += n_q_heads * head_dim * BF16
    total += int(np.asarray(cnt).sum()) * 4 + int(np.asarray(cnt).size) * 4
    return int(total)


def decode_bytes(seq_len, gran, n_q_heads, head_dim, sink_tokens, window_tokens, idx, cnt) -> dict:
    """Bytes fx_sparse_decode must move.
    unique: K+V rows of the blocks some head of the group attends to, counted once per group
            (what the kernel has to read from HBM) + q + index lists + output;
    summed: the same counted once per head (the upper bound Eq. 3 uses)."""
    idx = np.asarray(idx)
    cnt = np.asarray(cnt)
    n_kv = len(gran)
    group = n_q_heads // n_kv
    unique_tokens = 0
    summed_tokens = 0
    for b, N in enumerate(seq_len):
        N = int(N)
        for j, g in enumerate(gran):
            g = int(g)
            nb, n_sink, w0 = _geometry(N, g, sink_tokens, window_tokens)
            if nb == 0:
                continue
            keep_always = np.zeros(nb, dtype=bool)
            keep_always[: min(n_sink, nb)] = True
            keep_always[min(w0, nb):] = True
            tokens_of = np.full(nb, g, dtype=np.int64)
            tokens_of[-1] = N - (nb - 1) * g
            union = keep_always.copy()
            for r in range(group):
                h = j * group + r
                sel = idx[b, h, : cnt[b, h]]
                sel = sel[(sel >= 0) & (sel < nb)]
                mine = keep_always.copy()
                mine[sel] = True
                union |= mine
                summed_tokens += int(tokens_of[mine].sum())
            unique_tokens += int(tokens_of[union].sum())
    row = head_dim * BF16 * 2  # one K row + one V row
    small = len(seq_len) * n_q_heads * head_dim * (BF16 + 4) + int(cnt.sum()) * 4 + int(cnt.size) * 4
    return {
        "unique_kv_bytes": unique_tokens * row,
        "summed_kv_bytes": summed_tokens * row,
        "unique_tokens": unique_tokens,
        "small_bytes": small,
        "unique_bytes": unique_tokens * row + small,
    }


def summarize_bytes(seq_len, gran, head_dim) -> int:
    """fx_summarize reads every key once and writes two rows per block."""
    total = 0
    for N in seq_len:
        for g in gran:
            total += int(N) * head_dim * BF16 + (-(-int(N) // int(g))) * 2 * head_dim * BF16
    return int(total)
