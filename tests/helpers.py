"""Glue shared by the tests: turn a synthetic workload into what the oracle wants."""
import numpy as np

from oracle import fx_oracle as O
from paper_2605_07719_amd import workloads as W


def oracle_layout(wl: W.Workload) -> O.OracleLayout:
    pl = W.placement(wl)
    return O.OracleLayout(
        n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim, seq_len=pl.seq_len,
        seq_base=pl.seq_base, kv_head_stride=pl.kv_head_stride, token_stride=pl.token_stride,
        sum_base=pl.sum_base.reshape(-1), gran=pl.gran,
    )


def host_arrays(t: W.LayerTensors):
    return W.to_u16(t.q), W.to_u16(t.K), W.to_u16(t.V)


def bf16_bits_to_f64(u16: np.ndarray) -> np.ndarray:
    return (u16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def geometry(N: int, g: int, sink: int, window: int):
    """(n_blocks, n_sink, w0): restated here from the reading of Sec. 2.2/3.2 so tests do not ask the
    oracle for it."""
    nb = -(-N // g)
    n_sink = -(-sink // g)
    w0 = max(N - window, 0) // g
    return nb, n_sink, w0


# ----------------------------------------------------------------------------------------------------
# GPU side: device buffers for a workload and thin wrappers over the binding (used by -m gpu tests).
# ----------------------------------------------------------------------------------------------------

class GpuProblem:
    """Device copy of one layer of a workload plus the output/scratch buffers the C ABI wants."""

    def __init__(self, wl, tensors, k_max=None, device="cuda"):
        import torch

        from paper_2605_07719_amd import fluxion as F

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

    def decode(self, idx=None, cnt=None):
        import torch

        wl = self.wl
        if idx is not None:
            self.idx.copy_(torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)))
            self.cnt.copy_(torch.from_numpy(np.ascontiguousarray(cnt, dtype=np.int32)))
        self.F.sparse_decode(self.layout, self.q, self.K, self.V, self.idx, self.cnt, k_max=self.k_max,
                             sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens, out=self.out,
                             workspace=self.ws_decode)
        return self.out


NEAR_TIE = 1e-5


def compare_selection(idx_g, cnt_g, idx_o, cnt_o, gap, kth, scores, n_sink_w0):
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
