"""Pins for the oracle's attention arithmetic (App. A.1: s = q K^T / sqrt(D), O = softmax(s) V) and for
the fusion of partial results (Sec. 2.2, Sec. 4 step 4).  None of these re-call the oracle's own code:
they use a library softmax-attention, closed forms, or a compacted problem."""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from helpers import bf16_bits_to_f64, f32_to_bf16_bits, geometry, host_arrays, oracle_layout
from oracle import fx_oracle as O
from paper_2605_07719_amd import workloads as W


def small_workload(seed=3, token_major=False):
    wl = W.Workload(
        name="small", n_q_heads=6, n_kv_heads=2, head_dim=64, seq_len=[300, 77, 513], gran=[16, 32],
        sink_tokens=20, window_tokens=40, seed=seed,
    )
    t = W.make_layer(wl)
    return wl, t


def torch_dense(wl, t):
    """Library route: fp64 torch.softmax(q K^T / sqrt(d)) V per sequence and head."""
    pl = W.placement(wl)
    out = np.zeros((wl.batch, wl.n_q_heads, wl.head_dim))
    lse = np.zeros((wl.batch, wl.n_q_heads))
    for b in range(wl.batch):
        lo, n = int(pl.tok_off[b]), int(pl.seq_len[b])
        for h in range(wl.n_q_heads):
            j = h // wl.group
            k = t.K[j, lo : lo + n].double()
            v = t.V[j, lo : lo + n].double()
            s = (k @ t.q[b, h].double()) / np.sqrt(wl.head_dim)
            out[b, h] = (torch.softmax(s, dim=0) @ v).numpy()
            lse[b, h] = logsumexp(s.numpy())
    return out, lse


def test_dense_matches_library_softmax_attention():
    wl, t = small_workload()
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    out, lse = O.dense_attention(L, q, K, V, return_lse=True)
    ref, ref_lse = torch_dense(wl, t)
    assert np.abs(out - ref).max() < 1e-12
    assert np.abs(lse - ref_lse).max() < 1e-11


def test_dense_with_token_major_strides():
    """Same numbers through a [token][kv_head][d] placement: pins the use of seq_base and both strides."""
    wl, t = small_workload(seed=5)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    ref = O.dense_attention(L, q, K, V)
    Hkv, T, d = K.shape
    K2 = np.ascontiguousarray(K.transpose(1, 0, 2))  # [T, Hkv, d]
    V2 = np.ascontiguousarray(V.transpose(1, 0, 2))
    pl = W.placement(wl)
    L2 = O.OracleLayout(
        n_q_heads=wl.n_q_heads, n_kv_heads=Hkv, head_dim=d, seq_len=pl.seq_len, seq_base=pl.tok_off * Hkv * d,
        kv_head_stride=d, token_stride=Hkv * d, sum_base=pl.sum_base.reshape(-1), gran=pl.gran,
    )
    out = O.dense_attention(L2, q, K2, V2)
    assert np.array_equal(out, ref)


def test_two_token_closed_form():
    """d=4, q=(2,0,0,0), k1=(1.5,0,0,0), k2=0: logits (1.5, 0) after the 1/sqrt(4) scale, so the first
    weight is the logistic function of 1.5."""
    d = 4
    q = f32_to_bf16_bits(np.array([[[2.0, 0, 0, 0]]], dtype=np.float32))
    K = f32_to_bf16_bits(np.array([[[1.5, 0, 0, 0], [0, 0, 0, 0]]], dtype=np.float32))
    V = f32_to_bf16_bits(np.array([[[1.0, 0, 0, 0], [0, 1.0, 0, 0]]], dtype=np.float32))
    L = O.OracleLayout(1, 1, d, [2], [0], 2 * d, d, [0], [16])
    out = O.dense_attention(L, q, K, V)[0, 0]
    w1 = 1.0 / (1.0 + np.exp(-1.5))
    assert np.allclose(out, [w1, 1.0 - w1, 0.0, 0.0], atol=1e-15)


def test_uniform_keys_give_mean_of_values():
    rng = np.random.default_rng(0)
    d, N = 64, 200
    q = f32_to_bf16_bits(rng.standard_normal((1, 1, d)).astype(np.float32))
    row = f32_to_bf16_bits(rng.standard_normal(d).astype(np.float32))
    K = np.broadcast_to(row, (1, N, d)).copy()
    V = f32_to_bf16_bits(rng.standard_normal((1, N, d)).astype(np.float32))
    L = O.OracleLayout(1, 1, d, [N], [0], N * d, d, [0], [16])
    out = O.dense_attention(L, q, K, V)[0, 0]
    assert np.abs(out - bf16_bits_to_f64(V[0]).mean(axis=0)).max() < 1e-13


def test_dominant_key_returns_its_value():
    d, N = 64, 50
    rng = np.random.default_rng(1)
    qf = np.zeros((1, 1, d), dtype=np.float32)
    qf[0, 0, 3] = 64.0
    Kf = np.zeros((1, N, d), dtype=np.float32)
    Kf[0, 17, 3] = 64.0  # logit 64*64/8 = 512 against 0 elsewhere
    V = f32_to_bf16_bits(rng.standard_normal((1, N, d)).astype(np.float32))
    L = O.OracleLayout(1, 1, d, [N], [0], N * d, d, [0], [16])
    out = O.dense_attention(L, f32_to_bf16_bits(qf), f32_to_bf16_bits(Kf), V)[0, 0]
    assert np.abs(out - bf16_bits_to_f64(V[0, 17])).max() < 1e-13


def full_selection(wl, L):
    """idx/cnt that select every candidate block of every head, built from the geometry alone."""
    kmax = L.max_blocks()
    idx = -np.ones((wl.batch, wl.n_q_heads, kmax), dtype=np.int32)
    cnt = np.zeros((wl.batch, wl.n_q_heads), dtype=np.int32)
    for b in range(wl.batch):
        for h in range(wl.n_q_heads):
            g = wl.gran[h // wl.group]
            nb, n_sink, w0 = geometry(wl.seq_len[b], g, wl.sink_tokens, wl.window_tokens)
            c = np.arange(n_sink, max(w0, n_sink), dtype=np.int32)
            idx[b, h, : c.size] = c
            cnt[b, h] = c.size
    return idx, cnt


def test_all_candidates_selected_equals_dense():
    wl, t = small_workload(seed=7)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    idx, cnt = full_selection(wl, L)
    sparse = O.sparse_attention(L, q, K, V, idx, cnt, sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    dense = O.dense_attention(L, q, K, V)
    assert np.abs(sparse - dense).max() < 1e-12


def test_budget_one_through_select_equals_dense():
    wl, t = small_workload(seed=8)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    S = O.summarize(L, K)
    idx, cnt, _, _ = O.select(L, q, S, budget_frac=1.0, sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens,
                              k_max=L.max_blocks())
    ref_idx, ref_cnt = full_selection(wl, L)
    assert np.array_equal(cnt, ref_cnt) and np.array_equal(idx, ref_idx)
    sparse = O.sparse_attention(L, q, K, V, idx, cnt, sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    assert np.abs(sparse - O.dense_attention(L, q, K, V)).max() < 1e-12


def test_budget_zero_is_dense_over_sink_and_window_tokens():
    """Streaming head (Sec. 3.2): with nothing selected the output is attention over the retained tokens,
    checked by running the library route on a problem that holds only those tokens."""
    wl, t = small_workload(seed=9)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    idx = -np.ones((wl.batch, wl.n_q_heads, 4), dtype=np.int32)
    cnt = np.zeros((wl.batch, wl.n_q_heads), dtype=np.int32)
    out = O.sparse_attention(L, q, K, V, idx, cnt, sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    pl = W.placement(wl)
    for b in range(wl.batch):
        for h in range(wl.n_q_heads):
            j = h // wl.group
            g = wl.gran[j]
            N = wl.seq_len[b]
            nb, n_sink, w0 = geometry(N, g, wl.sink_tokens, wl.window_tokens)
            keep = [tk for tk in range(N) if (tk // g) < n_sink or (tk // g) >= w0]
            rows = np.asarray(keep) + int(pl.tok_off[b])
            k = torch.from_numpy(bf16_bits_to_f64(K[j, rows]))
            v = torch.from_numpy(bf16_bits_to_f64(V[j, rows]))
            s = (k @ torch.from_numpy(bf16_bits_to_f64(q[b, h]))) / np.sqrt(wl.head_dim)
            ref = (torch.softmax(s, 0) @ v).numpy()
            assert np.abs(out[b, h] - ref).max() < 1e-12


def test_weights_sum_to_one_and_token_set():
    wl, t = small_workload(seed=10)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    S = O.summarize(L, K)
    idx, cnt, _, _ = O.select(L, q, S, budget_frac=0.3, sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens,
                              k_max=L.max_blocks())
    for b in range(wl.batch):
        for h in range(wl.n_q_heads):
            g = wl.gran[h // wl.group]
            N = wl.seq_len[b]
            nb, n_sink, w0 = geometry(N, g, wl.sink_tokens, wl.window_tokens)
            tokens, w = O.token_weights(L, q, K, V, idx, cnt, sink_tokens=wl.sink_tokens,
                                        window_tokens=wl.window_tokens, b=b, h=h)
            assert abs(w.sum() - 1.0) < 1e-12 and (w > 0).all()
            blocks = set(idx[b, h, : cnt[b, h]].tolist()) | {i for i in range(nb) if i < n_sink or i >= w0}
            expect = [tk for tk in range(N) if tk // g in blocks]
            assert tokens.tolist() == expect


@pytest.mark.parametrize("chunk", [1, 7, 16, 33, 10**6])
def test_chunked_merge_equals_two_pass(chunk):
    """Any split of the token list into partial (m, l, acc) results fuses to the single-pass result."""
    wl, t = small_workload(seed=11)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    S = O.summarize(L, K)
    idx, cnt, _, _ = O.select(L, q, S, budget_frac=0.25, sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens,
                              k_max=L.max_blocks())
    kw = dict(sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    a = O.sparse_attention(L, q, K, V, idx, cnt, mode="two_pass", **kw)
    c = O.sparse_attention(L, q, K, V, idx, cnt, mode="chunked", chunk_tokens=chunk, **kw)
    assert np.abs(a - c).max() < 1e-12


def test_chunked_merge_survives_large_logit_spread():
    """Outlier channels make logits span tens of units; the merge must still agree (max-subtraction)."""
    wl = W.llama_stack(context=2048, n_layers=1)
    t = W.make_layer(wl)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    S = O.summarize(L, K)
    idx, cnt, _, _ = O.select(L, q, S, budget_frac=0.2, sink_tokens=32, window_tokens=256, k_max=64)
    kw = dict(sink_tokens=32, window_tokens=256)
    a = O.sparse_attention(L, q, K, V, idx, cnt, **kw)
    c = O.sparse_attention(L, q, K, V, idx, cnt, mode="chunked", chunk_tokens=32, **kw)
    assert np.abs(a - c).max() < 1e-12


def test_group_union_token_set_and_special_cases():
    """Union variant: the token set is the set-union of the group's selections (restated here); with one
    head per group it is the head's own set; if one head of a group selects everything the whole group is
    dense."""
    wl, t = small_workload(seed=12)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    S = O.summarize(L, K)
    kw = dict(sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    bud = np.tile(np.array([0.1, 0.3, 0.0, 0.2, 1.0, 0.05], dtype=np.float32), (wl.batch, 1))
    idx, cnt, _, _ = O.select(L, q, S, budget_frac=bud, k_max=L.max_blocks(), **kw)
    G = wl.group
    for b in range(wl.batch):
        for h in range(wl.n_q_heads):
            j = h // G
            g = wl.gran[j]
            N = wl.seq_len[b]
            nb, n_sink, w0 = geometry(N, g, wl.sink_tokens, wl.window_tokens)
            blocks = {i for i in range(nb) if i < n_sink or i >= w0}
            for hh in range(j * G, (j + 1) * G):
                blocks |= set(idx[b, hh, : cnt[b, hh]].tolist())
            tokens, w = O.token_weights(L, q, K, V, idx, cnt, b=b, h=h, group_union=True, **kw)
            assert tokens.tolist() == [tk for tk in range(N) if tk // g in blocks]
            assert abs(w.sum() - 1) < 1e-12
    uni = O.sparse_attention(L, q, K, V, idx, cnt, group_union=True, **kw)
    dense = O.dense_attention(L, q, K, V)
    assert np.abs(uni[:, 3:] - dense[:, 3:]).max() < 1e-12      # heads 3-5 share a group with a dense head
    own = O.sparse_attention(L, q, K, V, idx, cnt, **kw)
    assert np.abs(uni[:, :3] - own[:, :3]).max() > 1e-6          # heads 0-2 really see more tokens
    # G = 1: union == own
    wl1 = W.Workload(name="mha", n_q_heads=3, n_kv_heads=3, head_dim=64, seq_len=[400], gran=[16, 16, 32],
                     sink_tokens=16, window_tokens=32, seed=1)
    t1 = W.make_layer(wl1)
    L1 = oracle_layout(wl1)
    q1, K1, V1 = host_arrays(t1)
    i1, c1, _, _ = O.select(L1, q1, O.summarize(L1, K1), budget_frac=0.2, sink_tokens=16, window_tokens=32, k_max=32)
    a = O.sparse_attention(L1, q1, K1, V1, i1, c1, sink_tokens=16, window_tokens=32, group_union=True)
    c = O.sparse_attention(L1, q1, K1, V1, i1, c1, sink_tokens=16, window_tokens=32)
    assert np.array_equal(a, c)


def test_layer_step_is_select_followed_by_sparse_attention():
    """The wrapper the benchmark's cpu_baseline leg times must be exactly the two pinned routines chained:
    same index lists, same counts, same output bits, for fractional and for integer budgets, with threads."""
    wl = W.Workload(
        name="step", n_q_heads=6, n_kv_heads=2, head_dim=64, seq_len=[900, 333, 1500], gran=[16, 32],
        sink_tokens=20, window_tokens=70, seed=12,
        budget_frac=np.array([[0.0, 0.05, 0.3, 1.0, 0.11, 0.5]] * 3, dtype=np.float32),
    )
    t = W.make_layer(wl)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    S = O.summarize(L, K)
    k_max = L.max_blocks()
    kw = dict(sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens)
    for budgets in (dict(budget_frac=wl.budget_frac), dict(budget_blocks=np.array([[0, 3, 1, 40, 7, 2]] * 3, np.int32))):
        idx, cnt, _, _ = O.select(L, q, S, k_max=k_max, **budgets, **kw)
        out = O.sparse_attention(L, q, K, V, idx, cnt, **kw)
        for threads in (1, 3):
            idx2, cnt2, out2 = O.layer_step(L, q, K, V, S, k_max=k_max, threads=threads, **budgets, **kw)
            assert np.array_equal(idx2, idx) and np.array_equal(cnt2, cnt)
            assert np.array_equal(out2, out)
    with pytest.raises(ValueError):
        O.layer_step(L, q, K, V, S, k_max=2, budget_frac=wl.budget_frac, **kw)
