"""Glue shared by the tests: turn a synthetic workload into what the oracle wants."""
import numpy as np

from oracle import checks as C
from oracle import fx_oracle as O
from oracle.checks import NEAR_TIE, bf16_bits_to_f64  # noqa: F401  (re-exported for the tests)
from paper_2605_07719_amd import workloads as W
from paper_2605_07719_amd.harness import GpuProblem  # noqa: F401  (re-exported for the GPU tests)


def oracle_layout(wl: W.Workload) -> O.OracleLayout:
    return C.layout_for(wl, W.placement(wl))


def host_arrays(t: W.LayerTensors):
    return W.to_u16(t.q), W.to_u16(t.K), W.to_u16(t.V)


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


def compare_selection(idx_g, cnt_g, idx_o, cnt_o, gap, kth, scores, _unused=None):
    return C.compare_selection(idx_g, cnt_g, idx_o, cnt_o, gap, kth, scores)
