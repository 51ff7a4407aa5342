"""Granularity-budget selector (Sec. 5.2 Eq. 1, Sec. 5.3 Eq. 3): pins for the oracle, then the library's
host function against the oracle.  No GPU involved: the selector is host control logic."""
import numpy as np
import pytest

from oracle import selector as OS
from paper_2605_07719_amd import fluxion as F
from paper_2605_07719_amd import traffic as T


# ---- pins of the oracle -------------------------------------------------------------------------------

def test_zero_slope_prefers_the_coarsest_block():
    """With k_h = 0 the KV term does not depend on blk and the metadata term 2L/blk falls with blk."""
    gran, budget, vol = OS.choose(4, 1, [0.05] * 4, [0.0] * 4, 100000)
    assert gran == [128] and budget == [0.05] * 4
    assert vol[0] == pytest.approx(2 * 100000 / 128 + 2 * 100000 * 0.2)


def test_two_candidate_crossover_closed_form():
    """V(16) - V(32) = 2L (1/32 - sum_h k_h): 32 wins exactly when the slopes sum to less than 1/32."""
    L = 50000
    for total_slope, want in ((1 / 32 - 1e-4, 32), (1 / 32 + 1e-4, 16)):
        slopes = [total_slope / 4] * 4
        gran, _, _ = OS.choose(4, 1, [0.0] * 4, slopes, L, candidates=(16, 32))
        assert gran == [want]


def test_hand_worked_group():
    # one group, two heads: bgt0 = (0.02, 0.01), k = (0.005, 0.01), L = 32000
    # blk 16: budgets .04, .05  -> V = 4000 + 64000 * .09 = 9760
    # blk 32: budgets .045, .06 -> V = 2000 + 64000 * .105 = 8720
    # blk 64: budgets .05, .07  -> V = 1000 + 64000 * .12 = 8680   <- minimum
    # blk 128: budgets .055, .08 -> V = 500 + 64000 * .135 = 9140
    gran, budget, vol = OS.choose(2, 1, [0.02, 0.01], [0.005, 0.01], 32000)
    assert gran == [64]
    assert budget == pytest.approx([0.05, 0.07])
    assert vol == pytest.approx([8680.0])


def test_streaming_heads_and_clipping():
    gran, budget, vol = OS.choose(4, 2, [0.5, 0.9, 0.1, 0.1], [0.1, 0.2, 0.0, 0.0], 1000,
                                  streaming=[0, 0, 1, 1])
    assert budget[2:] == [0.0, 0.0] and vol[1] == 0.0 and gran[1] == 16
    assert budget[1] == 1.0 and 0.0 <= budget[0] <= 1.0          # 0.9 + 0.2*log2(blk) clips to 1
    gran, budget, _ = OS.choose(2, 1, [-0.5, 0.01], [0.01, 0.0], 1000)
    assert budget[0] == 0.0                                        # negative budgets clip to 0


def test_volume_agrees_with_the_byte_model():
    """Eq. 3 counts keys; times d * 2 bytes it must equal what the byte model counts for the same
    selection: candidate summaries + per-head selected K and V (sink/window set to zero here)."""
    N, g, Hq, d = 4096, 32, 4, 128
    n_blocks = N // g
    budgets = [0.125, 0.25, 0.0625, 0.5]
    ks = [int(b * n_blocks) for b in budgets]
    idx = -np.ones((1, Hq, n_blocks), np.int32)
    cnt = np.array([ks], np.int32)
    for h, k in enumerate(ks):
        idx[0, h, :k] = np.arange(k)
    dec = T.decode_bytes([N], [g], Hq, d, 0, 0, idx, cnt)
    summaries = n_blocks * 2 * d * 2
    v = OS.group_volume(N, g, budgets)
    assert v * d * 2 == summaries + dec["summed_kv_bytes"]


# ---- the library's host function against the oracle ---------------------------------------------------

@pytest.mark.parametrize("seed", range(6))
def test_library_selector_matches_oracle(seed):
    rng = np.random.default_rng(seed)
    Hkv = int(rng.integers(1, 9))
    G = int(rng.choice([1, 2, 4, 7, 8]))
    Hq = Hkv * G
    bgt0 = rng.uniform(-0.02, 0.2, Hq).astype(np.float32)
    slope = rng.uniform(-0.005, 0.03, Hq).astype(np.float32)
    streaming = (rng.uniform(size=Hq) < 0.3).astype(np.uint8)
    L = int(rng.integers(1000, 200000))
    cands = (16, 32, 64, 128) if seed % 2 == 0 else (16, 48, 96)
    gran, budget, vol = F.choose_granularity(Hq, Hkv, bgt0, slope, L, streaming, cands)
    o_gran, o_budget, o_vol = OS.choose(Hq, Hkv, bgt0, slope, L, streaming, cands)
    assert gran.tolist() == o_gran
    assert np.array_equal(budget, np.asarray(o_budget, dtype=np.float32))
    assert np.allclose(vol, o_vol, rtol=1e-15, atol=0)


def test_library_selector_rejects_bad_arguments():
    with pytest.raises(F.FluxionError):
        F.choose_granularity(5, 2, np.zeros(5), np.zeros(5), 100)
    with pytest.raises(F.FluxionError):
        F.choose_granularity(4, 2, np.zeros(4), np.zeros(4), 100, candidates=(16, 0))
