"""Host-side bookkeeping that needs no GPU: the summary pyramid's offsets, the seeded head properties, and the
rule that ties bench.py's counter-derived traffic figure to the kernel sources it was measured on."""
import importlib
import os
import sys

import numpy as np

from oracle import selector as OS
from paper_2605_07719_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pyramid_levels_tile_the_buffer_without_overlap():
    wl = W.Workload(name="p", n_q_heads=8, n_kv_heads=4, head_dim=64, seq_len=[1000, 37, 4096], gran=[16] * 4,
                    sink_tokens=64, window_tokens=256)
    pyr = W.pyramid(wl)
    assert pyr.levels == [16, 32, 64, 128]
    end = 0
    for g in pyr.levels:
        pl = pyr.placements[g]
        assert pyr.level_base[g] == end                       # levels follow each other
        assert pl.n_blocks.tolist() == [[-(-n // g)] * 4 for n in wl.seq_len]
        end += pl.total_blocks
    assert pyr.total_blocks == end
    # a mixed choice points every (sequence, KV head) inside its own level, at that level's own offset
    gran = [16, 128, 32, 64]
    base = pyr.sum_base(gran)
    for j, g in enumerate(gran):
        pl = pyr.placements[g]
        assert (base[:, j] == pyr.level_base[g] + pl.sum_base[:, j]).all()
        assert (base[:, j] + pl.n_blocks[:, j] <= pyr.level_base[g] + pl.total_blocks).all()


def test_head_properties_are_seeded_and_feed_the_selector():
    a = W.head_properties(32, seed=3, n_kv_heads=8)
    b = W.head_properties(32, seed=3, n_kv_heads=8)
    c = W.head_properties(32, seed=4, n_kv_heads=8)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert not np.array_equal(a[0], c[0])
    bgt0, slope, streaming = a
    assert bgt0.dtype == np.float32 and slope.dtype == np.float32 and streaming.dtype == np.uint8
    assert (bgt0 > 0).all() and (bgt0 < 0.1).all() and (slope >= 0).all()
    seen = set()
    for seed in range(8):   # over a few steps every candidate block size is chosen somewhere
        p = W.head_properties(32, seed=seed, n_kv_heads=8)
        seen.update(OS.choose(32, 8, p[0], p[1], 130000, p[2])[0])
    assert seen == {16, 32, 64, 128}


def test_traffic_figure_is_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    sys.path.insert(0, ROOT)
    bench = importlib.import_module("bench")
    prof = tmp_path / "profiles"
    prof.mkdir()
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    csrc = tmp_path / "paper_2605_07719_amd" / "csrc"
    csrc.mkdir(parents=True)
    (csrc / "a.hip").write_text("kernel v1")
    stamp = bench.csrc_hash()
    (prof / "traffic.txt").write_text(f"# csrc_sha16 {stamp}\nwl_a attend_kernel 12345\n")
    assert bench.profiled_traffic("wl_a") == 12345.0
    assert bench.profiled_traffic("wl_b") is None             # no figure for that workload
    (csrc / "a.hip").write_text("kernel v2")                    # the kernels changed: the figure is stale
    assert bench.csrc_hash() != stamp
    assert bench.profiled_traffic("wl_a") is None
    (prof / "traffic.txt").write_text("wl_a attend_kernel 12345\n")   # no stamp at all
    assert bench.profiled_traffic("wl_a") is None
