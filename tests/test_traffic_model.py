"""The byte model against the worked example the paper prints (Sec. 3.3) and against hand counts."""
import os

import numpy as np

from paper_2605_07719_amd import traffic as T

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_sec3_3_selected_kv_bytes.txt")


def read_golden():
    vals = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        vals[k] = float(v)
    return vals


def test_paper_worked_example():
    g = read_golden()
    r = T.paper_selected_kv_bytes(int(g["context_tokens"]), g["budget"], int(g["n_kv_heads"]), int(g["head_dim"]),
                                  int(g["n_layers"]))
    assert round(r["tokens"] / 1000, 1) == g["selected_tokens_k"]
    assert round(r["bytes_per_layer"] / 2**20, 1) == g["mib_per_layer"]
    assert round(r["bytes_all_layers"] / 2**20, 1) == g["mib_all_layers"]
    # the paper's two time estimates (it mixes MiB with decimal GB/s; both round to its figures)
    assert abs(r["bytes_all_layers"] / 2**20 / 1000 / g["pcie_gb_per_s"] * 1000 - g["pcie_ms"]) < 0.05
    assert round(r["bytes_all_layers"] / 2**20 / 1000 / g["dram_gb_per_s"] * 1000) == g["dram_ms"]


def test_decode_bytes_hand_count():
    # one sequence of 100 tokens, g=16 -> 7 blocks (last has 4 tokens); sink 16 -> block 0; window 20 ->
    # w0 = 80 // 16 = 5 -> blocks 5, 6.  Two heads in one group pick {2} and {2, 3}.
    idx = np.array([[[2, -1], [2, 3]]], dtype=np.int32)
    cnt = np.array([[1, 2]], dtype=np.int32)
    r = T.decode_bytes([100], [16], 2, 64, 16, 20, idx, cnt)
    always = 16 + 16 + 4
    assert r["unique_tokens"] == always + 32
    assert r["unique_kv_bytes"] == (always + 32) * 64 * 2 * 2
    assert r["summed_kv_bytes"] == ((always + 16) + (always + 32)) * 64 * 2 * 2


def test_select_and_summarize_bytes_hand_count():
    cnt = np.array([[1, 2]], dtype=np.int32)
    # candidates: blocks 1..4 -> 4 blocks * 2 rows * 64 * 2 B; q: 2 heads * 64 * 2 B; lists: 3 + 2 ints
    assert T.select_bytes([100], [16], 2, 64, 16, 20, cnt) == 4 * 2 * 64 * 2 + 2 * 64 * 2 + 5 * 4
    assert T.summarize_bytes([100], [16], 64) == 100 * 64 * 2 + 7 * 2 * 64 * 2
