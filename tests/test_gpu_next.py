"""GPU parity of the extensions around the hot path: summary pyramid, host selector feeding the kernels,
incremental summaries, group-union attention, streaming groups.  Same bar as test_gpu_parity.py."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from helpers import GpuProblem, bf16_bits_to_f64, compare_selection, host_arrays, oracle_layout
from oracle import fx_oracle as O
from oracle import selector as OS
from paper_2605_07719_amd import fluxion as F
from paper_2605_07719_amd import workloads as W
from test_gpu_parity import THREADS, TOL, run_oracle

pytestmark = pytest.mark.gpu


def base_workload(seed=21, **kw):
    args = dict(name="n", n_q_heads=8, n_kv_heads=2, head_dim=128, seq_len=[6000, 3333, 4100], gran=[16, 16],
                sink_tokens=64, window_tokens=256, budget_frac=np.full((3, 8), 0.08, dtype=np.float32), seed=seed)
    args.update(kw)
    return W.Workload(**args)


@pytest.mark.parametrize("coarse", [[32, 48], [16, 128], [64, 64]])
def test_summary_pyramid_equals_direct_summaries(coarse):
    wl = base_workload()
    t = W.make_layer(wl)
    gp = GpuProblem(wl, t)
    gp.summarize()
    wl_c = replace(wl, gran=coarse)
    gc = GpuProblem(wl_c, t)
    F.coarsen_summaries(gp.layout, gp.S, gc.layout, gc.S)
    torch.cuda.synchronize()
    _, K, _ = host_arrays(t)
    ref = O.summarize(oracle_layout(wl_c), K, threads=THREADS)
    assert np.array_equal(bf16_bits_to_f64(W.to_u16(gc.S)), bf16_bits_to_f64(ref))


def test_selector_tables_drive_the_kernels():
    """Head properties -> fx_choose_granularity -> gran[]/budget[] -> pyramid -> fx_select -> fx_sparse_decode,
    against the oracle run with the oracle selector's tables."""
    rng = np.random.default_rng(3)
    Hq, Hkv = 8, 2
    bgt0 = rng.uniform(0.01, 0.05, Hq).astype(np.float32)
    slope = np.concatenate([rng.uniform(0.0, 0.004, 4), rng.uniform(0.01, 0.03, 4)]).astype(np.float32)
    streaming = np.array([0, 1, 0, 0, 0, 0, 1, 0], dtype=np.uint8)
    wl16 = base_workload(seed=22)
    l_cpu = max(wl16.seq_len) - wl16.sink_tokens - wl16.window_tokens
    gran, budget, vol = F.choose_granularity(Hq, Hkv, bgt0, slope, l_cpu, streaming)
    o_gran, o_budget, _ = OS.choose(Hq, Hkv, bgt0, slope, l_cpu, streaming)
    assert gran.tolist() == o_gran and gran[0] > gran[1]          # flat heads go coarse, steep heads stay fine
    wl = replace(wl16, gran=gran.tolist(), budget_frac=np.tile(budget, (wl16.batch, 1)))
    t = W.make_layer(wl)
    fine = GpuProblem(wl16, t)
    fine.summarize()
    gp = GpuProblem(wl, t)
    F.coarsen_summaries(fine.layout, fine.S, gp.layout, gp.S)
    idx, cnt = gp.select()
    out = gp.decode()
    torch.cuda.synchronize()
    ref = run_oracle(replace(wl, budget_frac=np.tile(np.asarray(o_budget, np.float32), (wl.batch, 1))), t)
    compare_selection(idx.cpu().numpy(), cnt.cpu().numpy(), ref["idx"][..., : gp.k_max], ref["cnt"], ref["gap"],
                      ref["kth"], ref["scores"], None)
    assert (cnt[:, streaming.astype(bool)] == 0).all()
    assert np.abs(out.cpu().numpy().astype(np.float64) - ref["out"]).max() < TOL


def test_incremental_summaries_match_a_full_rebuild():
    wl_new = base_workload(seed=23, seq_len=[6000, 3333, 4100], gran=[16, 48])
    prev = np.array([5990, 3333 - 130, 4095], dtype=np.int32)      # +10, +130 (several blocks), +5 tokens
    wl_old = replace(wl_new, seq_len=prev.tolist())
    t = W.make_layer(wl_new)
    gp_new = GpuProblem(wl_new, t)
    # the old state: same cache rows, shorter lengths, summaries at the new cache's block offsets
    pl = W.placement(wl_new)
    old_layout = F.Layout.from_host(wl_new.n_q_heads, wl_new.n_kv_heads, wl_new.head_dim, prev, pl.seq_base,
                                    pl.kv_head_stride, pl.token_stride, pl.sum_base.reshape(-1), pl.gran,
                                    max_seq_len=int(pl.seq_len.max()))
    gp_new.S.fill_(float("nan"))
    F.summarize(old_layout, gp_new.K, gp_new.S)
    F.summarize_append(gp_new.layout, gp_new.K, gp_new.S, torch.from_numpy(prev).cuda(), 130)
    torch.cuda.synchronize()
    _, K, _ = host_arrays(t)
    ref = O.summarize(oracle_layout(wl_new), K, threads=THREADS)
    assert np.array_equal(bf16_bits_to_f64(W.to_u16(gp_new.S)), bf16_bits_to_f64(ref))
    del wl_old


@pytest.mark.parametrize("case", ["one_token_each", "from_empty", "nothing_new"])
def test_incremental_summaries_edge_cases(case):
    """Decode steady state (one token per sequence, also one that opens a new block), a cache built from empty
    by the append call alone, and an append of nothing."""
    new = np.array([4097, 3201, 4100], dtype=np.int32)            # 4097: its last token opens a new block
    prev, bound = {
        "one_token_each": (new - 1, 1),
        "from_empty": (np.zeros(3, dtype=np.int32), int(new.max())),
        "nothing_new": (new.copy(), 1),
    }[case]
    wl = base_workload(seed=26, seq_len=new.tolist(), gran=[32, 80])
    t = W.make_layer(wl)
    gp = GpuProblem(wl, t)
    pl = W.placement(wl)
    old_layout = F.Layout.from_host(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, prev, pl.seq_base, pl.kv_head_stride,
                                    pl.token_stride, pl.sum_base.reshape(-1), pl.gran,
                                    max_seq_len=int(pl.seq_len.max()))
    _, K, _ = host_arrays(t)
    ref_new = O.summarize(oracle_layout(wl), K, threads=THREADS)
    if case == "nothing_new":
        F.summarize(gp.layout, gp.K, gp.S)
        torch.cuda.synchronize()
        before = gp.S.clone()
    else:
        gp.S.fill_(float("nan"))
        if case != "from_empty":
            F.summarize(old_layout, gp.K, gp.S)
    F.summarize_append(gp.layout, gp.K, gp.S, torch.from_numpy(prev).cuda(), bound)
    torch.cuda.synchronize()
    assert np.array_equal(bf16_bits_to_f64(W.to_u16(gp.S)), bf16_bits_to_f64(ref_new))
    if case == "nothing_new":
        assert np.array_equal(W.to_u16(gp.S), W.to_u16(before))


def test_group_union_attention():
    wl = base_workload(seed=24, n_q_heads=14, n_kv_heads=2, gran=[32, 16], seq_len=[5000, 2100],
                       budget_frac=np.tile(np.array([0.02, 0.1, 0.0, 0.05, 0.3, 0.01, 0.07] * 2, np.float32), (2, 1)))
    t = W.make_layer(wl)
    ref = run_oracle(wl, t)
    kw = dict(sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    uni = O.sparse_attention(ref["L"], ref["q"], ref["K"], ref["V"], ref["idx"], ref["cnt"], group_union=True,
                             threads=THREADS, **kw)
    dense = O.dense_attention(ref["L"], ref["q"], ref["K"], ref["V"], threads=THREADS)
    gp = GpuProblem(wl, t, k_max=ref["k_max"])
    gp.idx.copy_(torch.from_numpy(ref["idx"]))
    gp.cnt.copy_(torch.from_numpy(ref["cnt"]))
    F.sparse_decode(gp.layout, gp.q, gp.K, gp.V, gp.idx, gp.cnt, k_max=gp.k_max, out=gp.out, workspace=gp.ws_decode,
                    group_union=True, **kw)
    out = gp.out.cpu().numpy().astype(np.float64)
    assert np.abs(out - uni).max() < TOL
    # Eq. 2 style deviation from full attention: the union variant sees a superset of every head's tokens
    scale = np.linalg.norm(dense, axis=-1).max()
    dev_own = np.linalg.norm(ref["out"] - dense, axis=-1) / scale
    dev_uni = np.linalg.norm(uni - dense, axis=-1) / scale
    print(f"  Eq.2 deviation: own mean {dev_own.mean():.4f} max {dev_own.max():.4f}; "
          f"union mean {dev_uni.mean():.4f} max {dev_uni.max():.4f}", flush=True)
    assert dev_uni.mean() < dev_own.mean()


def test_streaming_groups_are_skipped_and_still_correct():
    """KV head 0 of every sequence is a group of streaming heads (budget 0).  Its summaries are poisoned with NaN
    and its part of the score workspace with a marker: the selection and the outputs must not be affected, and
    the marker must survive fx_select (the score stage never visited the group, so it had no reason to read its
    summaries), while the other group's scores were written."""
    bud = np.full((3, 8), 0.1, dtype=np.float32)
    bud[:, :4] = 0.0
    wl = base_workload(seed=25, budget_frac=bud)
    t = W.make_layer(wl)
    ref = run_oracle(wl, t)
    gp = GpuProblem(wl, t, k_max=ref["k_max"])
    gp.summarize()
    pl = gp.pl
    for b in range(wl.batch):                                      # the streaming group's summary rows -> NaN
        lo = int(pl.sum_base[b, 0])
        gp.S[lo : lo + int(pl.n_blocks[b, 0])] = float("nan")
    gp.ws_select.fill_(0xFF)                                       # stale workspace must not matter
    idx, cnt = gp.select()
    torch.cuda.synchronize()
    assert int(cnt[:, :4].abs().sum()) == 0
    compare_selection(idx.cpu().numpy(), cnt.cpu().numpy(), ref["idx"], ref["cnt"], ref["gap"], ref["kth"],
                      ref["scores"], None)
    v = F.select_workspace_view(gp.layout)
    G, n_tiles = wl.group, v["mag_stride"]
    raw = gp.ws_select.cpu().numpy()
    approx = raw[v["approx_offset"] : v["approx_offset"] + 4 * wl.batch * wl.n_q_heads * n_tiles * 16]
    approx = approx.reshape(wl.batch, wl.n_kv_heads, n_tiles * G * 16 * 4)
    assert (approx[:, 0] == 0xFF).all()                            # streaming group: never written
    assert not (approx[:, 1] == 0xFF).all()                        # the selecting group: scored
    mags = raw[v["mag_offset"] : v["mag_offset"] + 4 * wl.batch * wl.n_q_heads * n_tiles]
    mags = mags.reshape(wl.batch, wl.n_q_heads, n_tiles * 4)
    assert (mags[:, :4] == 0xFF).all() and not (mags[:, 4:] == 0xFF).all()
    out = gp.decode().cpu().numpy().astype(np.float64)
    assert np.isfinite(out).all()
    assert np.abs(out - ref["out"]).max() < TOL


def test_per_step_granularity_from_a_resident_pyramid():
    """Sec. 5.2 / 5.3: the block size of a group and the budgets of its heads are chosen per decode step.  The
    summaries of all four candidate block sizes stay resident (built once: finest level by fx_summarize, the
    others by fx_coarsen_summaries); every step draws new head properties, fx_choose_granularity turns them
    into gran[] / budget[], and the step's layout points each KV head at its level.  Each step is compared with
    the oracle run at the block sizes and budgets of the oracle's own selector."""
    from paper_2605_07719_amd.harness import SummaryPyramid

    wl = base_workload(seed=27, n_q_heads=8, n_kv_heads=4, seq_len=[9000, 4111, 6500], gran=[16] * 4)
    t = W.make_layer(wl)
    gp = GpuProblem(wl, t)                       # q/K/V on the device, buffers sized for the finest level
    pyr = SummaryPyramid(wl)
    pyr.build(gp.K)
    l_cpu = max(wl.seq_len) - wl.sink_tokens - wl.window_tokens
    kw = dict(sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    seen = set()
    for step in range(4):
        bgt0, slope, streaming = W.head_properties(wl.n_q_heads, seed=step, streaming_frac=0.2, n_kv_heads=wl.n_kv_heads)
        gran, budget, _ = F.choose_granularity(wl.n_q_heads, wl.n_kv_heads, bgt0, slope, l_cpu, streaming)
        o_gran, o_budget, _ = OS.choose(wl.n_q_heads, wl.n_kv_heads, bgt0, slope, l_cpu, streaming)
        assert gran.tolist() == o_gran
        seen.update(o_gran)
        layout = pyr.layout(gran)
        bf = torch.from_numpy(np.tile(budget, (wl.batch, 1))).cuda()
        F.select(layout, gp.q, pyr.S, budget_frac=bf, k_max=gp.k_max, idx=gp.idx, cnt=gp.cnt, workspace=gp.ws_select,
                 **kw)
        F.sparse_decode(layout, gp.q, gp.K, gp.V, gp.idx, gp.cnt, k_max=gp.k_max, out=gp.out, workspace=gp.ws_decode,
                        **kw)
        torch.cuda.synchronize()
        wl_s = replace(wl, gran=o_gran, budget_frac=np.tile(np.asarray(o_budget, np.float32), (wl.batch, 1)))
        ref = run_oracle(wl_s, t)
        # the level each KV head reads equals the oracle's summaries at that block size
        S_all, pl_s = W.to_u16(pyr.S), W.placement(wl_s)
        base = pyr.pyr.sum_base(o_gran)
        for b in range(wl.batch):
            for j in range(wl.n_kv_heads):
                nb = int(pl_s.n_blocks[b, j])
                assert np.array_equal(bf16_bits_to_f64(S_all[base[b, j] : base[b, j] + nb]),
                                      bf16_bits_to_f64(ref["S"][int(pl_s.sum_base[b, j]) : int(pl_s.sum_base[b, j]) + nb]))
        exempt, differ = compare_selection(gp.idx.cpu().numpy(), gp.cnt.cpu().numpy(), ref["idx"][..., : gp.k_max],
                                           ref["cnt"], ref["gap"], ref["kth"], ref["scores"], None)
        own = O.sparse_attention(ref["L"], ref["q"], ref["K"], ref["V"], gp.idx.cpu().numpy(), gp.cnt.cpu().numpy(),
                                 threads=THREADS, **kw)
        err = np.abs(gp.out.cpu().numpy().astype(np.float64) - own).max()
        print(f"  step {step}: gran {o_gran}, streaming heads {int(streaming.sum())}, near-tie heads {exempt}, "
              f"max abs err {err:.3e}", flush=True)
        assert err < TOL
        assert (gp.cnt[:, streaming.astype(bool)] == 0).all()
    assert len(seen) >= 2                          # the steps really used different block sizes
