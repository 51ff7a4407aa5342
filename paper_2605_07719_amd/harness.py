"""Device buffers for one layer of a synthetic workload plus thin wrappers over the binding.

Used by the GPU tests, the smoke check and the benchmark.  Holds no arithmetic of the method: it only
allocates what the C ABI wants (index lists, counts, output, workspaces) and forwards to the binding.
"""
from __future__ import annotations

import numpy as np

from . import workloads as W


class GpuProblem:
    """Device copy of one layer of a workload plus the output/scratch buffers the C ABI wants."""

    def __init__(self, wl, tensors, k_max=None, device="cuda"):
        import torch

        from . import fluxion as F

        self.F = F
        self.wl = wl
        self.device = torch.device(device)
        pl = W.placement(wl)
        self.pl = pl
        self.layout = F.Layout.from_host(
            wl.n_q_heads, wl.n_kv_heads, wl.head_dim, pl.seq_len, pl.seq_base, pl.kv_head_stride, pl.token_stride,
            pl.sum_base.reshape(-1), pl.gran, device=device,
        )
        self.q = tensors.q.to(self.device)
        self.K = tensors.K.to(self.device)
        self.V = tensors.V.to(self.device)
        self.k_max = int(k_max if k_max is not None else max(1, int(pl.n_blocks.max())))
        self.S = torch.zeros((max(pl.total_blocks, 1), 2, wl.head_dim), dtype=torch.bfloat16, device=self.device)
        self.idx = torch.full((wl.batch, wl.n_q_heads, self.k_max), -7, dtype=torch.int32, device=self.device)
        self.cnt = torch.full((wl.batch, wl.n_q_heads), -7, dtype=torch.int32, device=self.device)
        self.out = torch.full((wl.batch, wl.n_q_heads, wl.head_dim), float("nan"), dtype=torch.float32,
                              device=self.device)
        self.ws_select = torch.empty(F.select_workspace_bytes(self.layout), dtype=torch.uint8, device=self.device)
        self.ws_decode = torch.empty(
            F.decode_workspace_bytes(self.layout, self.k_max, wl.sink_tokens, wl.window_tokens), dtype=torch.uint8,
            device=self.device)

    def summarize(self):
        self.F.summarize(self.layout, self.K, self.S)
        return self.S

    def select(self, budget_frac=None, budget_blocks=None):
        import torch

        wl = self.wl
        if budget_frac is None and budget_blocks is None:
            budget_frac, budget_blocks = wl.budget_frac, wl.budget_blocks
        bf = bb = None
        if budget_frac is not None:
            bf = torch.from_numpy(np.broadcast_to(
                np.asarray(budget_frac, dtype=np.float32), (wl.batch, wl.n_q_heads)).copy()).to(self.device)
        else:
            bb = torch.from_numpy(np.broadcast_to(
                np.asarray(budget_blocks, dtype=np.int32), (wl.batch, wl.n_q_heads)).copy()).to(self.device)
        self.F.select(self.layout, self.q, self.S, budget_frac=bf, budget_blocks=bb, sink_tokens=wl.sink_tokens,
                      window_tokens=wl.window_tokens, k_max=self.k_max, idx=self.idx, cnt=self.cnt,
                      workspace=self.ws_select)
        return self.idx, self.cnt

    def decode(self, idx=None, cnt=None, group_union=False):
        import torch

        wl = self.wl
        if idx is not None:
            self.idx.copy_(torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)))
            self.cnt.copy_(torch.from_numpy(np.ascontiguousarray(cnt, dtype=np.int32)))
        self.F.sparse_decode(self.layout, self.q, self.K, self.V, self.idx, self.cnt, k_max=self.k_max,
                             sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens, out=self.out,
                             workspace=self.ws_decode, group_union=group_union)
        return self.out


class SummaryPyramid:
    """Summaries of one layer's keys at every candidate block size, resident in one device buffer, so that a
    decode step may use a different block size per KV head (chosen per step by fx_choose_granularity) by
    pointing each (sequence, KV head) at the level it wants: only offsets change, no summary is rebuilt."""

    def __init__(self, wl, levels=(16, 32, 64, 128), device="cuda"):
        import torch

        from . import fluxion as F

        self.F, self.wl, self.device = F, wl, torch.device(device)
        self.pyr = W.pyramid(wl, levels)
        self.S = torch.empty((self.pyr.total_blocks, 2, wl.head_dim), dtype=torch.bfloat16, device=self.device)
        self.level_layout = {}
        for g in self.pyr.levels:
            pl = self.pyr.placements[g]
            self.level_layout[g] = F.Layout.from_host(
                wl.n_q_heads, wl.n_kv_heads, wl.head_dim, pl.seq_len, pl.seq_base, pl.kv_head_stride,
                pl.token_stride, pl.sum_base.reshape(-1), pl.gran, device=device)

    def level_view(self, g):
        lo = self.pyr.level_base[g]
        return self.S[lo : lo + self.pyr.placements[g].total_blocks]

    def build(self, K):
        """fx_summarize at the finest block size, every coarser level from the finest by fx_coarsen_summaries."""
        fine = self.pyr.levels[0]
        self.F.summarize(self.level_layout[fine], K, self.level_view(fine))
        for g in self.pyr.levels[1:]:
            self.F.coarsen_summaries(self.level_layout[fine], self.level_view(fine), self.level_layout[g],
                                     self.level_view(g))

    def layout(self, gran):
        """fx_layout of a step whose KV head j uses block size gran[j] (each a level of the pyramid)."""
        pl = self.pyr.placements[self.pyr.levels[0]]
        return self.F.Layout.from_host(
            self.wl.n_q_heads, self.wl.n_kv_heads, self.wl.head_dim, pl.seq_len, pl.seq_base, pl.kv_head_stride,
            pl.token_stride, self.pyr.sum_base(gran).reshape(-1), np.asarray(gran, dtype=np.int32),
            device=str(self.device))
