"""Pins for the oracle's block metadata, block scores and top-k (Sec. 2.1) and for the budget/geometry
readings.  Checks are invariants, brute force on tiny inputs, library routines (numpy min/max, argsort),
and the figures the configuration list fixes (candidate and block counts)."""
import itertools
import math

import numpy as np
import pytest

from helpers import bf16_bits_to_f64, f32_to_bf16_bits, geometry, host_arrays, oracle_layout
from oracle import fx_oracle as O
from paper_2605_07719_amd import workloads as W


def make(seed, seq_len, gran, hq=4, hkv=2, d=64, sink=16, window=48):
    wl = W.Workload(name="s", n_q_heads=hq, n_kv_heads=hkv, head_dim=d, seq_len=seq_len, gran=gran,
                    sink_tokens=sink, window_tokens=window, seed=seed)
    return wl, W.make_layer(wl)


# ------------------------------------------------------------------ summaries

def test_summaries_are_elementwise_min_max_of_block_keys():
    wl, t = make(1, [256, 100, 37], [16, 32])
    L = oracle_layout(wl)
    _, K, _ = host_arrays(t)
    S = O.summarize(L, K)
    Kf = bf16_bits_to_f64(K)
    Sf = bf16_bits_to_f64(S)
    pl = W.placement(wl)
    for b in range(wl.batch):
        for j in range(wl.n_kv_heads):
            g = wl.gran[j]
            N = wl.seq_len[b]
            for i in range(-(-N // g)):
                rows = Kf[j, pl.tok_off[b] + i * g : pl.tok_off[b] + min((i + 1) * g, N)]
                blk = int(pl.sum_base[b, j]) + i
                assert np.array_equal(Sf[blk, 0], rows.min(axis=0))  # library min: bracket and attained
                assert np.array_equal(Sf[blk, 1], rows.max(axis=0))
    assert S.shape[0] == pl.total_blocks


def test_coarsening_identity():
    """A block of 2g tokens is two blocks of g tokens: its summary is the min of mins / max of maxes."""
    for N in (512, 500):
        wl16, t = make(2, [N], [16], hq=2, hkv=1)
        wl32 = W.Workload(**{**wl16.__dict__, "gran": [32]})
        _, K, _ = host_arrays(t)
        S16 = bf16_bits_to_f64(O.summarize(oracle_layout(wl16), K))
        S32 = bf16_bits_to_f64(O.summarize(oracle_layout(wl32), K))
        for i in range(S32.shape[0]):
            kids = S16[2 * i : 2 * i + 2]
            assert np.array_equal(S32[i, 0], kids[:, 0].min(axis=0))
            assert np.array_equal(S32[i, 1], kids[:, 1].max(axis=0))


# ------------------------------------------------------------------ scores

def test_score_is_the_box_maximum_brute_force():
    """sum_c max(q_c mn_c, q_c mx_c) is the maximum of q.x over the box [mn, mx]; with d = 8 all 256
    corners can be enumerated."""
    d = 8
    wl, t = make(3, [160], [16], hq=2, hkv=1, d=d, sink=16, window=16)
    L = oracle_layout(wl)
    q, K, _ = host_arrays(t)
    S = O.summarize(L, K)
    sc = O.scores(L, q, S, 16, 16)
    qf, Sf = bf16_bits_to_f64(q), bf16_bits_to_f64(S)
    nb, n_sink, w0 = geometry(160, 16, 16, 16)
    assert (n_sink, w0) == (1, 9)
    for h in range(2):
        for i in range(nb):
            if not (n_sink <= i < w0):
                assert np.isnan(sc[0, h, i])
                continue
            best = max(
                sum(qf[0, h, c] * Sf[i, pick[c], c] for c in range(d)) for pick in itertools.product((0, 1), repeat=d)
            )
            assert abs(sc[0, h, i] - best) < 1e-12


def test_score_upper_bounds_every_logit_in_the_block():
    wl, t = make(4, [640, 333], [16, 64], hq=4, hkv=2)
    L = oracle_layout(wl)
    q, K, _ = host_arrays(t)
    S = O.summarize(L, K)
    sc = O.scores(L, q, S, wl.sink_tokens, wl.window_tokens)
    qf, Kf = bf16_bits_to_f64(q), bf16_bits_to_f64(K)
    pl = W.placement(wl)
    checked = 0
    for b in range(wl.batch):
        for h in range(wl.n_q_heads):
            j = h // wl.group
            g = wl.gran[j]
            nb, n_sink, w0 = geometry(wl.seq_len[b], g, wl.sink_tokens, wl.window_tokens)
            for i in range(n_sink, w0):
                rows = Kf[j, pl.tok_off[b] + i * g : pl.tok_off[b] + (i + 1) * g]
                assert sc[b, h, i] >= (rows @ qf[b, h]).max() - 1e-9
                checked += 1
    assert checked > 50


def test_single_token_blocks_score_is_the_dot_product_and_topk_is_exact_topk():
    wl, t = make(5, [200], [1], hq=2, hkv=1, sink=4, window=10)
    L = oracle_layout(wl)
    q, K, _ = host_arrays(t)
    S = O.summarize(L, K)
    assert np.array_equal(S[:, 0], K[0]) and np.array_equal(S[:, 1], K[0])
    sc = O.scores(L, q, S, 4, 10)
    qf, Kf = bf16_bits_to_f64(q), bf16_bits_to_f64(K)
    dots = Kf[0] @ qf[0].T  # [N, Hq]
    assert np.abs(sc[0, :, 4:190] - dots[4:190].T).max() < 1e-12
    idx, cnt, _, _ = O.select(L, q, S, budget_blocks=20, sink_tokens=4, window_tokens=10, k_max=20)
    for h in range(2):
        best = np.sort(np.argsort(-dots[4:190, h], kind="stable")[:20] + 4)
        assert np.array_equal(idx[0, h], best)


# ------------------------------------------------------------------ top-k

def rank_count_select(s, k, lo):
    """selected(i) <=> #{j : s_j > s_i or (s_j == s_i and j < i)} < k."""
    n = s.size
    chosen = []
    for i in range(n):
        rank = sum(1 for jj in range(n) if s[jj] > s[i] or (s[jj] == s[i] and jj < i))
        if rank < k:
            chosen.append(i + lo)
    return chosen


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_topk_against_rank_counting(seed):
    wl, t = make(20 + seed, [1000, 260], [16, 32], hq=4, hkv=2)
    L = oracle_layout(wl)
    q, K, _ = host_arrays(t)
    S = O.summarize(L, K)
    sc = O.scores(L, q, S, wl.sink_tokens, wl.window_tokens)
    bud = np.random.default_rng(seed).integers(0, 9, size=(2, 4)).astype(np.int32)
    idx, cnt, gap, kth = O.select(L, q, S, budget_blocks=bud, sink_tokens=wl.sink_tokens,
                                  window_tokens=wl.window_tokens, k_max=8)
    for b in range(2):
        for h in range(4):
            g = wl.gran[h // wl.group]
            nb, n_sink, w0 = geometry(wl.seq_len[b], g, wl.sink_tokens, wl.window_tokens)
            k = min(int(bud[b, h]), w0 - n_sink)
            want = rank_count_select(sc[b, h, n_sink:w0], k, n_sink)
            assert cnt[b, h] == k
            assert idx[b, h, :k].tolist() == want
            assert (idx[b, h, k:] == -1).all()
            srt = np.sort(sc[b, h, n_sink:w0])[::-1]
            if 0 < k < srt.size:
                assert kth[b, h] == srt[k - 1]
                assert math.isclose(gap[b, h], abs(srt[k - 1] - srt[k]) / max(abs(srt[k - 1]), abs(srt[k])))
            else:
                assert np.isinf(gap[b, h])


def test_exact_ties_go_to_the_lower_index():
    """Blocks 5, 9 and 12 hold identical keys, hence identical summaries and scores; they are made the
    strongest candidates.  With k = 2 the two lower indices must win, with k = 1 only block 5."""
    wl, t = make(30, [400], [16], hq=2, hkv=1, sink=16, window=32)
    L = oracle_layout(wl)
    q, K, _ = host_arrays(t)
    qf = bf16_bits_to_f64(q)
    boost = f32_to_bf16_bits((8.0 * np.sign(qf[0, 0])).astype(np.float32))  # aligned with head 0's query
    for blk in (5, 9, 12):
        K[0, blk * 16 : blk * 16 + 16] = boost
    S = O.summarize(L, K)
    sc = O.scores(L, q, S, 16, 32)
    assert sc[0, 0, 5] == sc[0, 0, 9] == sc[0, 0, 12] == np.nanmax(sc[0, 0])
    for k, want in ((1, [5]), (2, [5, 9]), (3, [5, 9, 12])):
        idx, cnt, gap, _ = O.select(L, q, S, budget_blocks=k, sink_tokens=16, window_tokens=32, k_max=4)
        assert idx[0, 0, :k].tolist() == want
        if k < 3:
            assert gap[0, 0] == 0.0


def test_candidate_counts_of_the_named_configurations():
    """Figures the configuration list fixes: tiny = 123 candidates, 8 + 1 + 4 = 13 blocks per head;
    Llama stack at 32K, g=32 = 1015 candidates and ceil(0.05 * 1015) = 51 blocks; 128K, g=32 with 64 sink
    and 256 window tokens = 4086 candidates and 82 / 205 / 409 / 4086 blocks for 0.02 / 0.05 / 0.1 / 1."""
    wl = W.tiny()
    t = W.make_layer(wl)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    S = O.summarize(L, K)
    sc = O.scores(L, q, S, wl.sink_tokens, wl.window_tokens)
    assert np.isfinite(sc[0, 0]).sum() == 123
    idx, cnt, _, _ = O.select(L, q, S, budget_blocks=wl.budget_blocks, sink_tokens=16, window_tokens=64, k_max=8)
    tokens, _ = O.token_weights(L, q, K, V, idx, cnt, sink_tokens=16, window_tokens=64, b=0, h=0)
    assert tokens.size == 13 * 16

    # only the counts matter below, so K is a tiny random cache reused through a fake geometry
    for N, sink, window, frac, n_cand, k in (
        (32768, 32, 256, 0.05, 1015, 51),
        (131072, 64, 256, 0.02, 4086, 82),
        (131072, 64, 256, 0.05, 4086, 205),
        (131072, 64, 256, 0.1, 4086, 409),
        (131072, 64, 256, 1.0, 4086, 4086),
    ):
        d = 8
        rng = np.random.default_rng(0)
        K = f32_to_bf16_bits(rng.standard_normal((1, N, d)).astype(np.float32))
        q = f32_to_bf16_bits(rng.standard_normal((1, 1, d)).astype(np.float32))
        L = O.OracleLayout(1, 1, d, [N], [0], N * d, d, [0], [32])
        S = O.summarize(L, K)
        idx, cnt, _, _ = O.select(L, q, S, budget_frac=np.float32(frac), sink_tokens=sink, window_tokens=window,
                                  k_max=n_cand)
        assert cnt[0, 0] == k
        assert np.isfinite(O.scores(L, q, S, sink, window)).sum() == n_cand


def test_sink_and_window_round_outward_to_whole_blocks():
    """Token counts worked out by hand from the reading taken for sink / window given in tokens: N = 1000,
    g = 48 (21 blocks, the last one holds 40 tokens), sink 100 tokens -> blocks 0..2 (144 tokens), window 300
    tokens -> blocks floor(700 / 48) = 14 .. 20 (tokens 672 .. 999: 328 tokens), candidates 3 .. 13 (11 blocks);
    a budget of 0.3 keeps ceil(3.3) = 4 of them; a head with budget 0 attends to 144 + 328 = 472 tokens."""
    wl, t = make(44, [1000], [48], hq=2, hkv=1, sink=100, window=300)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    S = O.summarize(L, K)
    assert S.shape[0] == 21
    sc = O.scores(L, q, S, 100, 300)
    assert np.flatnonzero(np.isfinite(sc[0, 0])).tolist() == list(range(3, 14))
    idx, cnt, _, _ = O.select(L, q, S, budget_frac=np.array([[0.3, 0.0]], np.float32), sink_tokens=100,
                              window_tokens=300, k_max=11)
    assert cnt.tolist() == [[4, 0]]
    assert all(3 <= i <= 13 for i in idx[0, 0, :4])
    tok0, _ = O.token_weights(L, q, K, V, idx, cnt, sink_tokens=100, window_tokens=300, b=0, h=0)
    tok1, _ = O.token_weights(L, q, K, V, idx, cnt, sink_tokens=100, window_tokens=300, b=0, h=1)
    assert tok1.tolist() == list(range(0, 144)) + list(range(672, 1000))
    assert tok0.size == 472 + 4 * 48


def test_short_context_has_no_candidates_and_is_dense():
    wl, t = make(40, [40, 16, 100], [16, 32], sink=32, window=64)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    S = O.summarize(L, K)
    idx, cnt, _, _ = O.select(L, q, S, budget_frac=0.5, sink_tokens=32, window_tokens=64, k_max=4)
    assert (cnt[:2] == 0).all()
    out = O.sparse_attention(L, q, K, V, idx, cnt, sink_tokens=32, window_tokens=64)
    dense = O.dense_attention(L, q, K, V)
    assert np.abs(out[:2] - dense[:2]).max() < 1e-12


def test_k_max_too_small_is_an_error():
    wl, t = make(41, [400], [16], hq=2, hkv=1)
    L = oracle_layout(wl)
    q, K, _ = host_arrays(t)
    S = O.summarize(L, K)
    with pytest.raises(ValueError):
        O.select(L, q, S, budget_frac=0.5, sink_tokens=16, window_tokens=48, k_max=3)


# ------------------------------------------------------------------ planted structure (config 1)

def test_tiny_config_finds_planted_blocks_and_tracks_dense():
    wl = W.tiny()
    t = W.make_layer(wl)
    L = oracle_layout(wl)
    q, K, V = host_arrays(t)
    S = O.summarize(L, K)
    idx, cnt, _, _ = O.select(L, q, S, budget_blocks=wl.budget_blocks, sink_tokens=16, window_tokens=64, k_max=8)
    for h in range(4):
        assert set(t.planted[0][h].tolist()) <= set(idx[0, h].tolist())
    sparse = O.sparse_attention(L, q, K, V, idx, cnt, sink_tokens=16, window_tokens=64)
    dense = O.dense_attention(L, q, K, V)
    none = O.sparse_attention(L, q, K, V, -np.ones_like(idx), np.zeros_like(cnt), sink_tokens=16, window_tokens=64)
    # Eq. 2 style deviation ||o_h(sparse) - o_h|| / max_h' ||o_h'||: keeping the selected blocks must bring
    # every head closer to full attention than keeping the retained tokens alone.
    scale = np.linalg.norm(dense, axis=-1).max()
    dev_sel = np.linalg.norm(sparse - dense, axis=-1) / scale
    dev_none = np.linalg.norm(none - dense, axis=-1) / scale
    assert (dev_sel < dev_none).all()
