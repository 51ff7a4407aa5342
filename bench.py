#!/usr/bin/env python3
"""Benchmark of the block-sparse decode hot path on one MI355X.

A step is one decode layer-step: fx_select followed by fx_sparse_decode (plan + split-K attention +
merge) for the whole batch on one layer's KV cache, cycling through the resident layers so that no
step re-reads a cache-resident layer.  fx_summarize runs once per layer before the timed region
(it is a cache-build step, not a per-token step) and is reported separately.

Prints ONE JSON line.  `value` is microseconds per layer-step on the headline workload (the
Llama-3-8B-shaped 32-layer stack at 32K context, batch 1, budget 0.05); `roofline` describes the
dominant kernel (split-K attention) on that workload; `workloads` carries the same figures for the
128K-context configurations; `cpu_baseline` is the fp64 oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
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
        "step_GBps": (unique + float(np.mean(sel_bytes))) / (step_ms * 1e-3) / 1e9,
        "summarize_ms_per_layer": sum_ms,
        "summarize_GBps": T.summarize_bytes(pl.seq_len, pl.gran, wl.head_dim) / (sum_ms * 1e-3) / 1e9,
        "layers_resident": n_layers,
        "batch": wl.batch,
        "max_context": int(max(wl.seq_len)),
        "k_max": ls.k_max,
    }


def profiled_traffic(workload: str, kernel: str = "attend_kernel"):
    """HBM bytes per launch of the dominant kernel measured with rocprofv3 hardware counters (FETCH_SIZE and
    WRITE_SIZE runs, summarised under profiles/); None if no profile of this workload is committed."""
    path = os.path.join(ROOT, "profiles", "traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == workload and f[1] == kernel:
                return float(f[2])
    except OSError:
        pass
    return None


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
    # group-union attention on the selections of fx_select (every head of a group attends over the union)
    def union_step(i):
        q, K, V, S = ls.layers[i % len(ls.layers)]
        F.select(ls.layout, q, S, budget_frac=ls.bf, budget_blocks=ls.bb, sink_tokens=wl.sink_tokens,
                 window_tokens=wl.window_tokens, k_max=ls.k_max, idx=ls.idx, cnt=ls.cnt, workspace=ls.ws_sel)
        F.sparse_decode(ls.layout, q, K, V, ls.idx, ls.cnt, k_max=ls.k_max, sink_tokens=wl.sink_tokens,
                        window_tokens=wl.window_tokens, out=ls.out, workspace=ls.ws_dec, group_union=True)
    for i in range(64):  # the GPU idled while the host counted bytes: let the clocks come back up
        union_step(i)
    torch.cuda.synchronize()
    F.profile_enable(True)
    acc = {k: 0.0 for k in F.PROFILE_SLOTS}
    for i in range(steps):
        union_step(i)
        for k, v in F.profile_read().items():
            acc[k] += v / steps * 1e3
    F.profile_enable(False)
    out["union_kernel_us"] = acc                      # HIP events around each kernel, as in measure()
    out["union_us_per_layer_step"] = sum(acc.values())

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


def cpu_baseline(wl, seconds=12.0) -> dict:
    """The oracle, as it stands, on this machine's host cores: selection + sparse attention of one layer-step."""
    import torch

    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import host_arrays, oracle_layout
    from oracle import fx_oracle as O
    from paper_2605_07719_amd import workloads as W

    t = W.make_layer(wl, 0, device="cpu")
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    threads = O.default_threads()
    S = O.summarize(L, K, threads=threads)
    k_max = int(max(1, L.max_blocks()))
    kw = dict(budget_frac=wl.budget_frac, budget_blocks=wl.budget_blocks, sink_tokens=wl.sink_tokens,
              window_tokens=wl.window_tokens, k_max=k_max, threads=threads)
    O.layer_step(L, q, K, V, S, **kw)  # warm-up
    times = []
    t_end = time.time() + seconds
    while time.time() < t_end or len(times) < 5:
        t0 = time.perf_counter()
        O.layer_step(L, q, K, V, S, **kw)
        times.append(time.perf_counter() - t0)
    return {
        "value": float(np.median(times) * 1e6), "unit": "us per decode layer-step", "cores": threads, "kind": "oracle",
        "sample": f"{len(times)} full layer-steps (selection + sparse attention, all {wl.n_q_heads} heads) of layer 0 "
                  f"of {wl.name}; median",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--no-graph", action="store_true", help="time eager launches only")
    ap.add_argument("--no-extra", action="store_true", help="skip the 128K-context workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", default="", help="run only this extra workload as the headline (debug/profiling)")
    ap.add_argument("--budget", type=float, default=0.05)
    args = ap.parse_args()
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

    extras = {
        "hbm_stress": lambda: (W.hbm_stress(budget=args.budget, n_layers=4), 4),
        "hbm_stress_dense": lambda: (W.hbm_stress(budget=1.0, n_layers=2), 2),
        "hbm_stress_0.02": lambda: (W.hbm_stress(budget=0.02, n_layers=4), 4),
        "hbm_stress_0.1": lambda: (W.hbm_stress(budget=0.1, n_layers=4), 4),
        "head_specific": lambda: (W.head_specific(n_layers=4), 4),
        "qwen_ragged": lambda: (W.qwen_ragged(n_layers=4), 4),
    }

    if args.only:
        wl, nl = extras[args.only]()
        head = measure(LayerSet(wl, nl), args.steps, args.warmup, use_graph)
        head_wl = wl
    else:
        head_wl = W.llama_stack()
        head_ls = LayerSet(head_wl, head_wl.n_layers)
        head = measure(head_ls, args.steps, args.warmup, use_graph)
        head["eq2_output_deviation"] = output_deviation(head_ls)
        del head_ls
        torch.cuda.empty_cache()
    log("[bench] headline:", json.dumps(head))

    others = []
    nxt = None
    if not args.no_extra and not args.only:
        for name, mk in extras.items():
            wl, nl = mk()
            ls = LayerSet(wl, nl)
            r = measure(ls, max(8, args.steps // 4), max(4, args.warmup // 4), use_graph)
            log(f"[bench] {name}:", json.dumps(r))
            others.append(r)
            if name == "hbm_stress":
                nxt = next_rows(ls)
                log("[bench] widened entry points:", json.dumps(nxt))
            del ls
            torch.cuda.empty_cache()

    probe = stream_probe()
    log("[bench] stream probe:", json.dumps(probe))
    head["attend_frac_of_stream_read"] = head["attend_GBps"] / probe["read_GBps"]
    for r in others:
        r["attend_frac_of_stream_read"] = r["attend_GBps"] / probe["read_GBps"]
        r["attend_traffic_bytes"] = profiled_traffic(r["workload"])

    base = None
    if not args.no_cpu_baseline:
        base = cpu_baseline(head_wl)

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
            "workload": head["workload"], "batch": head["batch"], "context": head["max_context"],
            "layers_resident": head["layers_resident"], "n_q_heads": head_wl.n_q_heads,
            "n_kv_heads": head_wl.n_kv_heads, "head_dim": head_wl.head_dim, "block_size": head_wl.gran,
            "budget": "per-head table" if head_wl.budget_frac is None or np.ptp(head_wl.budget_frac) > 0
            else float(head_wl.budget_frac.flat[0]),
            "sink_tokens": head_wl.sink_tokens, "window_tokens": head_wl.window_tokens,
        },
        "detail": head,
        "roofline": {
            "bound": "hbm", "kernel": "attend_kernel (split-K sparse attention)",
            "achieved": head["attend_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": head["attend_frac_of_hbm_peak"], "traffic": profiled_traffic(head["workload"]),
            "bytes_per_launch": head["decode_unique_bytes"], "us_per_launch": head["kernel_us"]["attend"],
        },
        "roofline_128k": None if not others else {
            "bound": "hbm", "kernel": "attend_kernel (split-K sparse attention)", "workload": others[0]["workload"],
            "achieved": others[0]["attend_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": others[0]["attend_frac_of_hbm_peak"], "traffic": others[0]["attend_traffic_bytes"],
            "bytes_per_launch": others[0]["decode_unique_bytes"], "us_per_launch": others[0]["kernel_us"]["attend"],
        },
        "stream_probe": probe,
        "next_rows": nxt,
        "workloads": others,
        "cpu_baseline": base,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
