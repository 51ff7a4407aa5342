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
