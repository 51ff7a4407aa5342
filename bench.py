#!/usr/bin/env python3
"""Benchmark of the block-sparse decode hot path on one MI355X.

A step is one decode layer-step: fx_select followed by fx_sparse_decode (plan + split-K attention +
merge) for the whole batch on one layer's KV cache, cycling through the resident layers so that no
step re-reads a cache-resident layer.  fx_summarize runs once per layer before the timed region
(it is a cache-build step, not a per-token step) and is reported separately.

Prints ONE JSON line.  `value` is microseconds per layer-step on the headline workload (the
Llama-3-8B-shaped 32-layer stack at 32K context, batch 1, budget 0.05).  `roofline` describes the
dominant kernel (split-K attention) at the point the HBM target is defined on: 128K context, batch 16,
budget 0.05 (`roofline.workload` names it; the same object for the latency-bound headline workload is
`roofline_32k`).  `workloads` carries the figures of every other configuration, each with a sampled
check against the oracle (near-tie heads, max abs error) and the oracle's own time on that sample.
`cpu_baseline` is the fp64 oracle timed on this machine's host cores on the headline workload.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X datasheet HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class LayerSet:
    """Resident layers of one workload on the GPU with everything fx_* needs."""

    def __init__(self, wl, n_layers, device="cuda"):
        import torch

        from paper_2605_07719_amd import fluxion as F
        from paper_2605_07719_amd import workloads as W

        self.torch, self.F, self.W = torch, F, W
        self.wl = wl
        self.pl = pl = W.placement(wl)
        self.layout = F.Layout.from_host(
            wl.n_q_heads, wl.n_kv_heads, wl.head_dim, pl.seq_len, pl.seq_base, pl.kv_head_stride, pl.token_stride,
            pl.sum_base.reshape(-1), pl.gran, device=device)
        self.layers = []
        t0 = time.time()
        for layer in range(n_layers):
            t = W.make_layer(wl, layer, device=device)
            S = torch.empty((pl.total_blocks, 2, wl.head_dim), dtype=torch.bfloat16, device=device)
            self.layers.append((t.q, t.K, t.V, S))
        torch.cuda.synchronize()
        log(f"[bench] {wl.name}: generated {n_layers} layer(s) in {time.time() - t0:.1f}s "
            f"({n_layers * 2 * pl.kv_head_stride * wl.n_kv_heads * 2 / 2**30:.1f} GiB K+V)")
        if wl.budget_frac is not None:
            self.k_max = int(max(1, np.ceil(wl.budget_frac.max() * pl.n_blocks.max())))
            self.bf = torch.from_numpy(np.ascontiguousarray(wl.budget_frac, dtype=np.float32)).to(device)
            self.bb = None
        else:
            self.k_max = int(max(1, wl.budget_blocks.max()))
            self.bf = None
            self.bb = torch.from_numpy(np.ascontiguousarray(wl.budget_blocks, dtype=np.int32)).to(device)
        self.k_max = min(self.k_max, int(pl.n_blocks.max()))
        B, Hq, d = wl.batch, wl.n_q_heads, wl.head_dim
        self.idx = torch.empty((B, Hq, self.k_max), dtype=torch.int32, device=device)
        self.cnt = torch.empty((B, Hq), dtype=torch.int32, device=device)
        self.out = torch.empty((B, Hq, d), dtype=torch.float32, device=device)
        self.ws_sel = torch.empty(F.select_workspace_bytes(self.layout), dtype=torch.uint8, device=device)
        self.ws_dec = torch.empty(F.decode_workspace_bytes(self.layout, self.k_max, wl.sink_tokens, wl.window_tokens),
                                  dtype=torch.uint8, device=device)

    def summarize_all(self):
        torch = self.torch
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        self.F.summarize(self.layout, self.layers[0][1], self.layers[0][3])  # warm-up (module load)
        torch.cuda.synchronize()
        ev0.record()
        for (_, K, _, S) in self.layers:
            self.F.summarize(self.layout, K, S)
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / len(self.layers)  # ms per layer

    def step(self, layer):
        q, K, V, S = self.layers[layer % len(self.layers)]
        wl, F = self.wl, self.F
        F.select(self.layout, q, S, budget_frac=self.bf, budget_blocks=self.bb, sink_tokens=wl.sink_tokens,
                 window_tokens=wl.window_tokens, k_max=self.k_max, idx=self.idx, cnt=self.cnt, workspace=self.ws_sel)
        F.sparse_decode(self.layout, q, K, V, self.idx, self.cnt, k_max=self.k_max, sink_tokens=wl.sink_tokens,
                        window_tokens=wl.window_tokens, out=self.out, workspace=self.ws_dec)


def measure(ls: LayerSet, steps: int, warmup: int, use_graph: bool) -> dict:
    import torch

    from paper_2605_07719_amd import traffic as T

    F, wl, pl = ls.F, ls.wl, ls.pl
    n_layers = len(ls.layers)
    sum_ms = ls.summarize_all()

    for s in range(warmup):
        ls.step(s)
    torch.cuda.synchronize()

    # ---- eager timing: K steps between two events on the launch stream ---------------------------
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record()
    for s in range(steps):
        ls.step(warmup + s)
    ev1.record()
    torch.cuda.synchronize()
    eager_ms = ev0.elapsed_time(ev1) / steps
    out_eager = ls.out.clone()

    # ---- the same K steps captured once into a HIP graph and replayed (launch overhead removed) ----
    graph_ms = None
    if use_graph:
        try:
            g = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    for s in range(steps):
                        ls.step(warmup + s)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g.replay()  # untimed replay
            torch.cuda.synchronize()
            reps = []
            for _ in range(3):
                ev0.record()
                g.replay()
                ev1.record()
                torch.cuda.synchronize()
                reps.append(ev0.elapsed_time(ev1) / steps)
                if not torch.equal(ls.out, out_eager):
                    raise RuntimeError("graph replay output differs from the eager output")
            graph_ms = float(np.median(reps))
        except Exception as e:  # report, fall back to the eager figure
            log(f"[bench] HIP graph path unavailable: {e!r}")
            graph_ms = None

    # ---- per-kernel durations with HIP events inside the library (separate pass over the same steps)
    F.profile_enable(True)
    acc = {k: 0.0 for k in F.PROFILE_SLOTS}
    for s in range(steps):
        ls.step(warmup + s)
        ms = F.profile_read()
        for k in acc:
            acc[k] += ms[k]
    F.profile_enable(False)
    kern_ms = {k: v / steps for k, v in acc.items()}

    # ---- algorithmic bytes, from the selections the timed steps actually made ---------------------
    dec_unique, dec_summed, sel_bytes = [], [], []
    for layer in range(min(n_layers, steps)):
        ls.step(layer)
        torch.cuda.synchronize()
        idx, cnt = ls.idx.cpu().numpy(), ls.cnt.cpu().numpy()
        d = T.decode_bytes(pl.seq_len, pl.gran, wl.n_q_heads, wl.head_dim, wl.sink_tokens, wl.window_tokens, idx, cnt)
        dec_unique.append(d["unique_bytes"])
        dec_summed.append(d["summed_kv_bytes"])
        sel_bytes.append(T.select_bytes(pl.seq_len, pl.gran, wl.n_q_heads, wl.head_dim, wl.sink_tokens,
                                        wl.window_tokens, cnt))
    unique = float(np.mean(dec_unique))
    step_ms = graph_ms if graph_ms is not None else eager_ms
    attend_gbps = unique / (kern_ms["attend"] * 1e-3) / 1e9
    decode_call_ms = kern_ms["plan"] + kern_ms["attend"] + kern_ms["merge"]  # the whole fx_sparse_decode call
    decode_gbps = unique / (decode_call_ms * 1e-3) / 1e9
    return {
        "workload": wl.name,
        "us_per_layer_step": step_ms * 1e3,
        "us_per_layer_step_eager": eager_ms * 1e3,
        "us_per_layer_step_graph": None if graph_ms is None else graph_ms * 1e3,
        "kernel_us": {k: v * 1e3 for k, v in kern_ms.items()},
        "decode_unique_bytes": unique,
        "decode_summed_kv_bytes": float(np.mean(dec_summed)),
        "select_bytes": float(np.mean(sel_bytes)),
        "attend_GBps": attend_gbps,
        "attend_frac_of_hbm_peak": attend_gbps / HBM_PEAK_GBPS,
        "decode_call_GBps": decode_gbps,
        "decode_call_frac_of_hbm_peak": decode_gbps / HBM_PEAK_GBPS,
        "step_GBps": (unique + float(np.mean(sel_bytes))) / (step_ms * 1e-3) / 1e9,
        "summarize_ms_per_layer": sum_ms,
        "summarize_GBps": T.summarize_bytes(pl.seq_len, pl.gran, wl.head_dim) / (sum_ms * 1e-3) / 1e9,
        "layers_resident": n_layers,
        "batch": wl.batch,
        "max_context": int(max(wl.seq_len)),
        "k_max": ls.k_max,
    }


def csrc_hash() -> str:
    """Hash of the kernel sources: the counter-derived traffic figures under profiles/ are valid for one build."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2605_07719_amd", "csrc")
    for name in sorted(os.listdir(d)):
        h.update(name.encode())
        h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def profiled_traffic(workload: str, kernel: str = "attend_kernel"):
    """HBM bytes per launch of the dominant kernel measured with rocprofv3 hardware counters (FETCH_SIZE and
    WRITE_SIZE runs, summarised under profiles/traffic.txt).  None if no figure for this workload is committed
    or if the kernel sources changed since the counters were read (the file records the hash of csrc/)."""
    path = os.path.join(ROOT, "profiles", "traffic.txt")
    value, stamp = None, None
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == "#" and f[1] == "csrc_sha16":
                stamp = f[2]
            if len(f) == 3 and f[0] == workload and f[1] == kernel:
                value = float(f[2])
    except OSError:
        return None
    return value if stamp == csrc_hash() else None


def stream_probe(n_bytes=4 << 30) -> dict:
    """Plain streaming read and plain copy of a buffer far larger than the caches: what this machine reaches
    with no arithmetic at all (context for the roofline fraction, and the known-size transfers that
    hardware-counter readings are scaled against)."""
    import torch

    from paper_2605_07719_amd import fluxion as F

    src = torch.empty(n_bytes, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty(n_bytes, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(reps):
            fn()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / reps

    read = {w: n_bytes / timed(lambda: F.probe_read(src, sink, w)) / 1e6 for w in (1, 2, 3)}
    read_nt = {w: n_bytes / timed(lambda: F.probe_read_streaming(src, sink, w)) / 1e6 for w in (1, 2, 3)}
    copy_ms = timed(lambda: F.probe_copy(dst, src, 4))
    return {"bytes": n_bytes, "read_GBps": max(max(read.values()), max(read_nt.values())),
            "plain_read_GBps_by_wg_per_cu": read, "non_temporal_read_GBps_by_wg_per_cu": read_nt,
            "copy_GBps_read_plus_write": 2 * n_bytes / copy_ms / 1e6}


def output_deviation(ls: LayerSet) -> dict:
    """The paper's output-aware criterion (Eq. 2) used as a report: ||o_h(sparse) - o_h|| / max_h' ||o_h'|| of
    the selected-block output against full attention (budget 1.0 through the same kernels), for each head
    attending to its own selection and for the group-union variant.  Layer 0, untimed."""
    import torch

    F, wl = ls.F, ls.wl
    q, K, V, S = ls.layers[0]
    pl = ls.pl
    k_all = int(pl.n_blocks.max())
    kw = dict(sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    idx = torch.empty((wl.batch, wl.n_q_heads, k_all), dtype=torch.int32, device=q.device)
    cnt = torch.empty((wl.batch, wl.n_q_heads), dtype=torch.int32, device=q.device)
    ws = torch.empty(F.decode_workspace_bytes(ls.layout, k_all, wl.sink_tokens, wl.window_tokens), dtype=torch.uint8,
                     device=q.device)
    outs = {}
    one = torch.ones((wl.batch, wl.n_q_heads), dtype=torch.float32, device=q.device)
    for name, bf, bb, union in (("dense", one, None, False), ("own", ls.bf, ls.bb, False), ("union", ls.bf, ls.bb, True)):
        out = torch.empty_like(ls.out)
        F.select(ls.layout, q, S, budget_frac=bf, budget_blocks=bb, k_max=k_all, idx=idx, cnt=cnt, workspace=ls.ws_sel,
                 **kw)
        F.sparse_decode(ls.layout, q, K, V, idx, cnt, k_max=k_all, out=out, workspace=ws, group_union=union, **kw)
        outs[name] = out.double()
    scale = outs["dense"].norm(dim=-1).amax(dim=-1, keepdim=True)      # max over heads, per sequence
    res = {}
    for name in ("own", "union"):
        dev = (outs[name] - outs["dense"]).norm(dim=-1) / scale
        res[name] = {"mean": float(dev.mean()), "max": float(dev.max())}
    return res


def union_step_times(ls: LayerSet, steps: int = 16) -> dict:
    """The layer-step with group-union attention on the selections of fx_select (every head of a group attends
    over the union of the group's selections): per-kernel HIP-event times and the attention kernel's rate."""
    import torch

    from paper_2605_07719_amd import fluxion as F

    wl = ls.wl

    def union_step(i):
        q, K, V, S = ls.layers[i % len(ls.layers)]
        F.select(ls.layout, q, S, budget_frac=ls.bf, budget_blocks=ls.bb, sink_tokens=wl.sink_tokens,
                 window_tokens=wl.window_tokens, k_max=ls.k_max, idx=ls.idx, cnt=ls.cnt, workspace=ls.ws_sel)
        F.sparse_decode(ls.layout, q, K, V, ls.idx, ls.cnt, k_max=ls.k_max, sink_tokens=wl.sink_tokens,
                        window_tokens=wl.window_tokens, out=ls.out, workspace=ls.ws_dec, group_union=True)

    for i in range(64):  # the GPU may have idled while the host worked: let the clocks come back up
        union_step(i)
    torch.cuda.synchronize()
    F.profile_enable(True)
    acc = {k: 0.0 for k in F.PROFILE_SLOTS}
    for i in range(steps):
        union_step(i)
        for k, v in F.profile_read().items():
            acc[k] += v / steps * 1e3
    F.profile_enable(False)
    return {"kernel_us": acc, "us_per_layer_step": sum(acc.values())}


def next_rows(ls: LayerSet, steps: int = 16) -> dict:
    """Timings of the widened entry points on the workload of `ls`: group-union attention, the summary pyramid,
    incremental summaries and the host-side granularity/budget selector."""
    import torch

    from paper_2605_07719_amd import fluxion as F
    from paper_2605_07719_amd import traffic as T
    from paper_2605_07719_amd import workloads as W

    wl, pl = ls.wl, ls.pl
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=steps):
        fn(0)
        torch.cuda.synchronize()
        ev0.record()
        for i in range(reps):
            fn(i)
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / reps * 1e3  # us

    out = {"workload": wl.name}
    uni = union_step_times(ls, steps)
    out["union_kernel_us"] = uni["kernel_us"]          # HIP events around each kernel, as in measure()
    out["union_us_per_layer_step"] = uni["us_per_layer_step"]

    # summary pyramid: coarse summaries at 4x the block size from the resident ones
    if all(int(g) * 4 <= 128 for g in pl.gran):
        wl_c = W.Workload(**{**wl.__dict__, "gran": [int(g) * 4 for g in pl.gran]})
        pl_c = W.placement(wl_c)
        lay_c = F.Layout.from_host(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, pl_c.seq_len, pl_c.seq_base,
                                   pl_c.kv_head_stride, pl_c.token_stride, pl_c.sum_base.reshape(-1), pl_c.gran,
                                   device="cuda")
        S_c = torch.empty((pl_c.total_blocks, 2, wl.head_dim), dtype=torch.bfloat16, device="cuda")
        us = timed(lambda i: F.coarsen_summaries(ls.layout, ls.layers[i % len(ls.layers)][3], lay_c, S_c))
        fine_bytes = pl.total_blocks * 2 * wl.head_dim * 2
        out["coarsen_x4_us"] = us
        out["coarsen_x4_GBps_on_fine_summaries"] = fine_bytes / (us * 1e-6) / 1e9

    # incremental summaries: one new token per sequence (the block holding it is re-summarised)
    prev = torch.from_numpy(np.maximum(np.asarray(pl.seq_len, dtype=np.int32) - 1, 0)).cuda()
    out["summarize_append_1_token_us"] = timed(
        lambda i: F.summarize_append(ls.layout, ls.layers[i % len(ls.layers)][1], ls.layers[i % len(ls.layers)][3],
                                     prev, 1))

    # host selector: Eq. 1 per head, Eq. 3 argmin per group
    rng = np.random.default_rng(0)
    bgt0 = rng.uniform(0.01, 0.2, wl.n_q_heads).astype(np.float32)
    slope = rng.uniform(0.0, 0.02, wl.n_q_heads).astype(np.float32)
    t0 = time.perf_counter()
    for _ in range(200):
        F.choose_granularity(wl.n_q_heads, wl.n_kv_heads, bgt0, slope, int(max(pl.seq_len)))
    out["choose_granularity_host_us"] = (time.perf_counter() - t0) / 200 * 1e6
    return out


def per_query_granularity(steps: int, warmup: int, n_layers: int = 4) -> dict:
    """Block size and budgets chosen per decode step (Sec. 5.2 Eq. 1, Sec. 5.3 Eq. 3) on the shape of the
    head-specific configuration (batch 4 x 128K, 32 q / 8 kv heads): the summaries of all four candidate block
    sizes stay resident (finest level by fx_summarize, the others by fx_coarsen_summaries); every step has its
    own seeded head properties, fx_choose_granularity turns them into gran[] / budget[] on the host, and the
    step's layout points each KV head at its level.  Reported next to the fixed settings (16, 0.05) and
    (32, 0.05) on the same tensors: step time, unique bytes, and the Eq. 2 output deviation from full attention."""
    import torch

    from dataclasses import replace

    from paper_2605_07719_amd import fluxion as F
    from paper_2605_07719_amd import traffic as T
    from paper_2605_07719_amd import workloads as W
    from paper_2605_07719_amd.harness import SummaryPyramid

    shape = W.head_specific(n_layers=n_layers)
    # queries near a past key and keys with outlier channels (as in the Llama-stack configuration): peaky attention,
    # so that the Eq. 2 deviation measures what the selection keeps rather than the averaging noise of N(0,1) data
    wl = replace(shape, name="per_query_granularity_131072x4", gran=[16] * shape.n_kv_heads,
                 budget_frac=np.full((shape.batch, shape.n_q_heads), 0.05, dtype=np.float32),
                 q_mode="near_key", outlier_channels=4, planted_density=0.0)
    B, Hq, Hkv, d = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    kw = dict(sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    l_cpu = int(max(wl.seq_len)) - wl.sink_tokens - wl.window_tokens
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    layers, build_ms = [], []
    for layer in range(n_layers):
        t = W.make_layer(wl, layer, device="cuda")
        pyr = SummaryPyramid(wl)
        if layer == 0:
            pyr.build(t.K)  # warm-up of the two kernels
        torch.cuda.synchronize()
        ev0.record()
        pyr.build(t.K)
        ev1.record()
        torch.cuda.synchronize()
        build_ms.append(ev0.elapsed_time(ev1))
        layers.append((t.q, t.K, t.V, pyr))
    nb16 = int(W.placement(wl).n_blocks.max())

    def tables(kind, layer):
        pyr = layers[layer][3]
        if kind == "per_step":
            bgt0, slope, streaming = W.head_properties(Hq, seed=layer, n_kv_heads=Hkv)
            gran, budget, _ = F.choose_granularity(Hq, Hkv, bgt0, slope, l_cpu, streaming)
        else:
            gran = np.full(Hkv, 16 if kind == "fixed_16_0.05" else 32, dtype=np.int32)
            budget = np.full(Hq, 1.0 if kind == "dense" else 0.05, dtype=np.float32)
        k_need = max(int(np.ceil(float(budget[h]) * (-(-int(max(wl.seq_len)) // int(gran[h // (Hq // Hkv)])))))
                     for h in range(Hq))
        return pyr.layout(gran), torch.from_numpy(np.tile(budget, (B, 1))).cuda(), gran, max(1, k_need)

    sizing = layers[0][3].level_layout[16]  # the finest level needs the largest workspaces
    out = torch.empty((B, Hq, d), dtype=torch.float32, device="cuda")
    ws_sel = torch.empty(F.select_workspace_bytes(sizing), dtype=torch.uint8, device="cuda")
    cnt = torch.empty((B, Hq), dtype=torch.int32, device="cuda")

    def run_setting(kind, layer_ids, n_steps, n_warm):
        tabs = [tables(kind, l) for l in layer_ids]
        k_max = min(nb16, max(tb[3] for tb in tabs))
        idx = torch.empty((B, Hq, k_max), dtype=torch.int32, device="cuda")
        ws_dec = torch.empty(F.decode_workspace_bytes(sizing, k_max, wl.sink_tokens, wl.window_tokens),
                             dtype=torch.uint8, device="cuda")

        def step(i):
            q, K, V, pyr = layers[layer_ids[i % len(layer_ids)]]
            layout, bf, _, _ = tabs[i % len(layer_ids)]
            F.select(layout, q, pyr.S, budget_frac=bf, k_max=k_max, idx=idx, cnt=cnt, workspace=ws_sel, **kw)
            F.sparse_decode(layout, q, K, V, idx, cnt, k_max=k_max, out=out, workspace=ws_dec, **kw)

        for i in range(n_warm):
            step(i)
        torch.cuda.synchronize()
        ev0.record()
        for i in range(n_steps):
            step(i)
        ev1.record()
        torch.cuda.synchronize()
        us = ev0.elapsed_time(ev1) / max(n_steps, 1) * 1e3
        F.profile_enable(True)
        acc = {k: 0.0 for k in F.PROFILE_SLOTS}
        for i in range(len(layer_ids)):
            step(i)
            for k, v in F.profile_read().items():
                acc[k] += v / len(layer_ids) * 1e3
        F.profile_enable(False)
        uniq = []
        for i in range(len(layer_ids)):
            step(i)
            torch.cuda.synchronize()
            gran = tabs[i][2]
            uniq.append(T.decode_bytes(wl.seq_len, gran, Hq, d, wl.sink_tokens, wl.window_tokens, idx.cpu().numpy(),
                                       cnt.cpu().numpy())["unique_bytes"])
        step(0)  # leave layer_ids[0]'s output in `out`
        torch.cuda.synchronize()
        return {"us_per_layer_step_eager": us, "kernel_us": acc, "decode_unique_bytes": float(np.mean(uniq)),
                "gran_per_layer": [tb[2].tolist() for tb in tabs], "k_max": k_max}, out.double().clone()

    ids = list(range(n_layers))
    _, dense = run_setting("dense", [0], 1, 0)
    scale = dense.norm(dim=-1).amax(dim=-1, keepdim=True)
    res = {"workload": wl.name, "layers_resident": n_layers,
           "pyramid_build_ms_per_layer": float(np.mean(build_ms)),
           "pyramid_levels": [16, 32, 64, 128], "settings": {}}
    for kind in ("per_step", "fixed_16_0.05", "fixed_32_0.05"):
        r, _ = run_setting(kind, ids, steps, warmup)
        _, o0 = run_setting(kind, [0], 1, 0)
        dev = (o0 - dense).norm(dim=-1) / scale
        r["eq2_deviation_layer0"] = {"mean": float(dev.mean()), "max": float(dev.max())}
        res["settings"][kind] = r
    t0 = time.perf_counter()
    for layer in range(64):
        bgt0, slope, streaming = W.head_properties(Hq, seed=layer % n_layers, n_kv_heads=Hkv)
        F.choose_granularity(Hq, Hkv, bgt0, slope, l_cpu, streaming)
    res["host_tables_us_per_step"] = (time.perf_counter() - t0) / 64 * 1e6
    return res


def sampled_oracle(ls: LayerSet, sample, seconds: float) -> dict:
    """Outside every timed region: the GPU's layer 0 step against the oracle on the sequences `sample` (all their
    heads), and the oracle's own time for the layer-step of those sequences on this machine's host cores.
    Returns (parity figures, cpu baseline); the baseline is scaled linearly from the sample's tokens to the
    workload's when the sample is not the whole batch."""
    import torch

    from oracle import checks as C
    from oracle import fx_oracle as O
    from paper_2605_07719_amd import workloads as W

    wl = ls.wl
    q, K, V, S = ls.layers[0]
    ls.step(0)
    torch.cuda.synchronize()
    idx_g, cnt_g = ls.idx[sample].cpu().numpy(), ls.cnt[sample].cpu().numpy()
    out_g = ls.out[sample].cpu().numpy().astype(np.float64)
    sub_wl, sub_t = W.subset(wl, W.LayerTensors(q=q, K=K, V=V), sample)
    L = C.layout_for(sub_wl, W.placement(sub_wl))
    qh, Kh, Vh = W.to_u16(sub_t.q), W.to_u16(sub_t.K), W.to_u16(sub_t.V)
    del sub_t
    threads = O.default_threads()
    So = O.summarize(L, Kh, threads=threads)
    k_max = int(max(1, L.max_blocks()))
    kw = dict(sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    bud = dict(budget_frac=sub_wl.budget_frac, budget_blocks=sub_wl.budget_blocks)

    # ---- parity figures -------------------------------------------------------------------------
    parity = {"sample": f"sequences {list(sample)} of layer 0, all {wl.n_q_heads} heads",
              "heads_checked": int(cnt_g.size)}
    pl, sub_pl = ls.pl, W.placement(sub_wl)
    S_gpu = W.to_u16(S)
    same_summaries = all(
        np.array_equal(
            C.bf16_bits_to_f64(S_gpu[int(pl.sum_base[b, j]): int(pl.sum_base[b, j]) + int(pl.n_blocks[b, j])]),
            C.bf16_bits_to_f64(So[int(sub_pl.sum_base[n, j]): int(sub_pl.sum_base[n, j]) + int(pl.n_blocks[b, j])]))
        for n, b in enumerate(sample) for j in range(wl.n_kv_heads))
    parity["summaries_equal"] = bool(same_summaries)
    idx_o, cnt_o, gap, kth = O.select(L, qh, So, k_max=k_max, threads=threads, **bud, **kw)
    sc = O.scores(L, qh, So, wl.sink_tokens, wl.window_tokens, threads=threads)
    try:
        exempt, differ = C.compare_selection(idx_g, cnt_g, idx_o[..., : idx_g.shape[-1]], cnt_o, gap, kth, sc)
        parity.update(selection_exact=True, exempt_near_tie_heads=int(exempt), heads_differing_inside_band=int(differ))
    except AssertionError as e:  # a real mismatch: report it, never hide it
        parity.update(selection_exact=False, selection_error=repr(e))
    own = O.sparse_attention(L, qh, Kh, Vh, idx_g, cnt_g, threads=threads, **kw)
    parity["max_abs_err"] = float(np.abs(out_g - own).max())
    parity["max_abs_err_basis"] = "oracle attention over the blocks the GPU selected; tolerance 5e-3"

    # ---- the oracle's own time -------------------------------------------------------------------
    O.layer_step(L, qh, Kh, Vh, So, k_max=k_max, threads=threads, **bud, **kw)  # warm-up
    times = []
    t_end = time.time() + seconds
    while time.time() < t_end or len(times) < 3:
        t0 = time.perf_counter()
        O.layer_step(L, qh, Kh, Vh, So, k_max=k_max, threads=threads, **bud, **kw)
        times.append(time.perf_counter() - t0)
    scale = float(wl.total_tokens) / float(sub_wl.total_tokens)
    whole = len(sample) == wl.batch
    base = {
        "value": float(np.median(times) * 1e6 * scale), "unit": "us per decode layer-step", "cores": threads,
        "kind": "oracle", "workload": wl.name,
        "sample": (f"{len(times)} layer-steps (selection + sparse attention, all {wl.n_q_heads} heads) of layer 0 of "
                   f"{wl.name}, " + ("whole batch" if whole else
                                     f"sequences {list(sample)} only ({sub_wl.total_tokens} of {wl.total_tokens} tokens), "
                                     f"median scaled linearly by {scale:.2f}") + "; median"),
    }
    return parity, base


def roofline_of(r: dict) -> dict:
    """The `roofline` object of one measured workload (dominant kernel: split-K attention)."""
    return {
        "bound": "hbm", "kernel": "attend_kernel (split-K sparse attention)", "workload": r["workload"],
        "achieved": r["attend_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": r["attend_frac_of_hbm_peak"],
        "traffic": profiled_traffic(r["workload"]),
        "bytes_per_launch": r["decode_unique_bytes"], "us_per_launch": r["kernel_us"]["attend"],
        "frac_whole_decode_call": r["decode_call_frac_of_hbm_peak"],
        "note": "frac = unique K/V bytes of the step / attend_kernel time / 8 TB/s (the figure the 70% target is "
                "judged on); frac_whole_decode_call divides the same bytes by plan + attend + merge",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--no-graph", action="store_true", help="time eager launches only")
    ap.add_argument("--no-extra", action="store_true", help="skip the 128K-context workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle (timing and sampled parity check)")
    ap.add_argument("--only", default="", help="run only this extra workload as the headline (debug/profiling)")
    ap.add_argument("--budget", type=float, default=0.05)
    ap.add_argument("--print-csrc-hash", action="store_true", help="print the hash profiles/traffic.txt is stamped with")
    args = ap.parse_args()
    if args.print_csrc_hash:
        print(csrc_hash())
        return
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2605_07719_amd import fluxion as F
    from paper_2605_07719_amd import workloads as W

    F.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    use_graph = not args.no_graph
    with_oracle = not args.no_cpu_baseline

    # name -> (workload, resident layers, sequences the oracle checks and is timed on)
    extras = {
        "hbm_stress": lambda: (W.hbm_stress(budget=args.budget, n_layers=4), 4, [0]),
        "hbm_stress_dense": lambda: (W.hbm_stress(budget=1.0, n_layers=2), 2, [0]),
        "hbm_stress_0.02": lambda: (W.hbm_stress(budget=0.02, n_layers=4), 4, [0]),
        "hbm_stress_0.1": lambda: (W.hbm_stress(budget=0.1, n_layers=4), 4, [0]),
        "head_specific": lambda: (W.head_specific(n_layers=4), 4, [0]),
        "qwen_ragged": lambda: (W.qwen_ragged(n_layers=4), 4, [0]),
        # every head of a 7-head group on every block: the arithmetic-heaviest case of the attention kernel
        "qwen_ragged_dense": lambda: (W.with_budget(W.qwen_ragged(n_layers=2), 1.0), 2, [0]),
    }

    def run(ls, sample, oracle_seconds):
        r = measure(ls, args.steps, args.warmup, use_graph)
        base = None
        if with_oracle:
            r["parity"], base = sampled_oracle(ls, sample, oracle_seconds)
        return r, base

    baselines = []
    nxt = pq = None
    if args.only:
        wl, nl, sample = extras[args.only]()
        head, base = run(LayerSet(wl, nl), sample, 3.0)
        head_wl = wl
    else:
        head_wl = W.llama_stack()
        head_ls = LayerSet(head_wl, head_wl.n_layers)
        head, base = run(head_ls, [0], 10.0)
        head["eq2_output_deviation"] = output_deviation(head_ls)
        del head_ls
        torch.cuda.empty_cache()
    log("[bench] headline:", json.dumps(head))

    others = []
    if not args.no_extra and not args.only:
        for name, mk in extras.items():
            wl, nl, sample = mk()
            wl.name = wl.name if not name.endswith("_dense") or "b1.0" in wl.name else wl.name + "_dense"
            ls = LayerSet(wl, nl)
            r, b = run(ls, sample, 2.0)
            log(f"[bench] {name}:", json.dumps(r))
            others.append(r)
            if b is not None:
                baselines.append(b)
            if name == "hbm_stress":
                nxt = next_rows(ls)
                log("[bench] widened entry points:", json.dumps(nxt))
            if name == "head_specific":
                del ls
                ls = None
                torch.cuda.empty_cache()
                pq = per_query_granularity(min(args.steps, 32), min(args.warmup, 8))
                log("[bench] per-query granularity:", json.dumps(pq))
                continue
            if name == "qwen_ragged":
                u = union_step_times(ls, min(args.steps, 16))
                u["attend_frac_of_hbm_peak"] = r["decode_unique_bytes"] / (u["kernel_us"]["attend"] * 1e-6) / 1e9 / HBM_PEAK_GBPS
                r["group_union"] = u  # same bytes as the per-head step: every head now works on every block of the union
            del ls
            torch.cuda.empty_cache()

    probe = stream_probe()
    log("[bench] stream probe:", json.dumps(probe))
    for r in [head] + others:
        r["attend_frac_of_stream_read"] = r["attend_GBps"] / probe["read_GBps"]
        r["attend_traffic_bytes"] = profiled_traffic(r["workload"])

    target = others[0] if others else head   # the 128K, batch 16, budget 0.05 point when it was run
    line = {
        "metric": "us per decode layer-step (fx_select + fx_sparse_decode)",
        "value": head["us_per_layer_step"],
        "unit": "us",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["us_per_layer_step"] / 1e3,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "storage_dtype": "bf16",
        "data": "synthetic",
        "timing": "hip_graph_replay" if head["us_per_layer_step_graph"] is not None else "eager",
        "config": {
            "workload": f"{head['workload']} (value, ms_per_step, detail, cpu_baseline); roofline measured on "
                        f"{target['workload']}",
            "batch": head["batch"], "context": head["max_context"],
            "layers_resident": head["layers_resident"], "n_q_heads": head_wl.n_q_heads,
            "n_kv_heads": head_wl.n_kv_heads, "head_dim": head_wl.head_dim, "block_size": head_wl.gran,
            "budget": "per-head table" if head_wl.budget_frac is None or np.ptp(head_wl.budget_frac) > 0
            else float(head_wl.budget_frac.flat[0]),
            "sink_tokens": head_wl.sink_tokens, "window_tokens": head_wl.window_tokens,
        },
        "detail": head,
        "roofline": roofline_of(target),
        "roofline_32k": roofline_of(head),
        "stream_probe": probe,
        "next_rows": nxt,
        "per_query_granularity": pq,
        "workloads": others,
        "cpu_baseline": base,
        "cpu_baseline_workloads": baselines,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
