"""GPU parity at the full sizes of the named configurations, in the launch configuration bench.py times
(whole batch, one layer resident).  The GPU processes the whole batch; the oracle recomputes a sample of
sequences (all their heads) from a host copy of exactly those rows, and the two are compared on that
sample: summaries element by element, selections index-exact (near-tie rule), outputs within 5e-3."""
import numpy as np
import pytest
import torch

from helpers import GpuProblem, bf16_bits_to_f64, compare_selection
from oracle import fx_oracle as O
from paper_2605_07719_amd import workloads as W
from test_gpu_parity import TOL, oracle_on, run_oracle

pytestmark = pytest.mark.gpu


def check_sample(wl, sample, label):
    print(f"case={label} workload={wl.name} batch={wl.batch} sample={sample}", flush=True)
    t = W.make_layer(wl, 0, device="cuda")
    pl = W.placement(wl)
    if wl.budget_frac is not None:
        k_max = int(min(pl.n_blocks.max(), np.ceil(wl.budget_frac.max() * pl.n_blocks.max())))
    else:
        k_max = int(wl.budget_blocks.max())
    gp = GpuProblem(wl, t, k_max=max(k_max, 1))
    gp.summarize()
    idx, cnt = gp.select()
    out = gp.decode()
    torch.cuda.synchronize()
    print("  gpu done", flush=True)

    sub_wl, sub_t = W.subset(wl, t, sample)
    ref = run_oracle(sub_wl, sub_t)
    print("  oracle done", flush=True)
    sub_pl = W.placement(sub_wl)

    S_gpu = W.to_u16(gp.S)
    for n, b in enumerate(sample):
        for j in range(wl.n_kv_heads):
            nb = int(pl.n_blocks[b, j])
            a = S_gpu[int(pl.sum_base[b, j]) : int(pl.sum_base[b, j]) + nb]
            r = ref["S"][int(sub_pl.sum_base[n, j]) : int(sub_pl.sum_base[n, j]) + nb]
            assert np.array_equal(bf16_bits_to_f64(a), bf16_bits_to_f64(r)), (b, j)

    exempt, differ = compare_selection(idx[sample].cpu().numpy(), cnt[sample].cpu().numpy(), ref["idx"], ref["cnt"],
                                       ref["gap"], ref["kth"], ref["scores"], None)
    # Every head is compared: with the oracle's output where the selections agree, and in any case with the oracle's
    # attention over the blocks the GPU itself selected (heads that legitimately differ inside the near-tie band
    # attend to other blocks than the oracle's).
    out_s = out[sample].cpu().numpy().astype(np.float64)
    own = oracle_on(ref, sub_wl, idx[sample], cnt[sample])
    err_own = np.abs(out_s - own).max()
    same = np.array([[np.array_equal(idx[b, h, : ref["cnt"][n, h]].cpu().numpy(), ref["idx"][n, h, : ref["cnt"][n, h]])
                      for h in range(wl.n_q_heads)] for n, b in enumerate(sample)])
    err_same = np.abs(out_s - ref["out"])[same].max()
    print(f"  heads {same.size}, near-tie heads {exempt}, differing inside the band {differ}, "
          f"max abs err {err_same:.3e} (oracle selection), {err_own:.3e} (own selection, all heads)", flush=True)
    assert err_same < TOL and err_own < TOL
    del gp, t
    torch.cuda.empty_cache()


def test_llama_stack_32k_full_layer():
    wl = W.llama_stack(n_layers=1)
    check_sample(wl, [0], "config2")


def test_head_specific_128k_batch4():
    wl = W.head_specific(n_layers=1)
    check_sample(wl, [0, 3], "config3")


def test_qwen_ragged_batch16():
    wl = W.qwen_ragged(n_layers=1)
    lens = np.asarray(wl.seq_len)
    check_sample(wl, [int(lens.argmin()), int(lens.argmax())], "config4")


@pytest.mark.parametrize("budget", [0.02, 0.05, 0.1, 1.0])
def test_hbm_stress_128k_batch16(budget):
    """Every point of the budget sweep; the sampled sequences differ per point (first/last, middle ones, one for
    the dense point whose oracle pass is the longest)."""
    wl = W.hbm_stress(budget=budget, n_layers=1)
    sample = {0.02: [3, 12], 0.05: [0, 15], 0.1: [7, 8], 1.0: [5]}[budget]
    check_sample(wl, sample, f"config5_b{budget}")


def test_per_step_granularity_128k_batch4():
    """The head-specific shape (batch 4 x 128K) with block sizes and budgets chosen per step by
    fx_choose_granularity from seeded head properties, read from a resident four-level summary pyramid:
    the whole batch on the GPU, one sampled sequence (all heads) against the oracle run with the oracle
    selector's tables."""
    from dataclasses import replace

    from oracle import selector as OS
    from paper_2605_07719_amd import fluxion as F
    from paper_2605_07719_amd.harness import SummaryPyramid

    shape = W.head_specific(n_layers=1)
    wl = replace(shape, name="per_query_granularity", gran=[16] * shape.n_kv_heads)
    Hq, Hkv = wl.n_q_heads, wl.n_kv_heads
    l_cpu = int(max(wl.seq_len)) - wl.sink_tokens - wl.window_tokens
    bgt0, slope, streaming = W.head_properties(Hq, seed=0, n_kv_heads=Hkv)
    gran, budget, _ = F.choose_granularity(Hq, Hkv, bgt0, slope, l_cpu, streaming)
    o_gran, o_budget, _ = OS.choose(Hq, Hkv, bgt0, slope, l_cpu, streaming)
    assert gran.tolist() == o_gran and len(set(o_gran)) >= 3
    print(f"case=per_step_granularity gran={o_gran} streaming={int(streaming.sum())}", flush=True)
    wl_step = replace(wl, gran=o_gran, budget_frac=np.tile(np.asarray(o_budget, np.float32), (wl.batch, 1)))

    t = W.make_layer(wl, 0, device="cuda")
    pyr = SummaryPyramid(wl)
    pyr.build(t.K)
    layout = pyr.layout(gran)
    pl = W.placement(wl_step)
    k_max = int(max(1, np.ceil(float(np.max(budget)) * pl.n_blocks.max())))
    gp = GpuProblem(wl, t, k_max=k_max)          # buffers and workspaces sized at the finest level
    bf = torch.from_numpy(np.tile(budget, (wl.batch, 1))).cuda()
    kw = dict(sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    F.select(layout, gp.q, pyr.S, budget_frac=bf, k_max=k_max, idx=gp.idx, cnt=gp.cnt, workspace=gp.ws_select, **kw)
    F.sparse_decode(layout, gp.q, gp.K, gp.V, gp.idx, gp.cnt, k_max=k_max, out=gp.out, workspace=gp.ws_decode, **kw)
    torch.cuda.synchronize()
    print("  gpu done", flush=True)

    sample = [2]
    sub_wl, sub_t = W.subset(wl_step, t, sample)
    ref = run_oracle(sub_wl, sub_t)
    print("  oracle done", flush=True)
    sub_pl = W.placement(sub_wl)
    S_all, base = W.to_u16(pyr.S), pyr.pyr.sum_base(o_gran)
    for n, b in enumerate(sample):
        for j in range(Hkv):
            nb = int(pl.n_blocks[b, j])
            r = ref["S"][int(sub_pl.sum_base[n, j]) : int(sub_pl.sum_base[n, j]) + nb]
            assert np.array_equal(bf16_bits_to_f64(S_all[base[b, j] : base[b, j] + nb]), bf16_bits_to_f64(r)), (b, j)
    exempt, differ = compare_selection(gp.idx[sample].cpu().numpy(), gp.cnt[sample].cpu().numpy(),
                                       ref["idx"][..., :k_max], ref["cnt"], ref["gap"], ref["kth"], ref["scores"], None)
    own = oracle_on(ref, sub_wl, gp.idx[sample], gp.cnt[sample])
    err = np.abs(gp.out[sample].cpu().numpy().astype(np.float64) - own).max()
    print(f"  near-tie heads {exempt}, differing inside the band {differ}, max abs err {err:.3e}", flush=True)
    assert err < TOL
