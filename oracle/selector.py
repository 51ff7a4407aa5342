"""Oracle of the granularity-budget selector (test infrastructure only; plain Python, fp64).

Sec. 5.2, Eq. 1: a retrieval head's budget grows linearly in log2 of the block size,
    bgt_h(blk) = bgt0_h + k_h * log2(blk).
Sec. 5.3, Eq. 3: the data a GQA group touches at block size blk, in keys, is the block metadata (two
vectors per block) plus the selected KV (keys and values) summed over the group's heads,
    V(blk) = 2 * L_cpu / blk + 2 * L_cpu * sum_h bgt_h(blk),
and the group uses the candidate block size with the smallest V; each head's budget then follows from
Eq. 1 at that size.  Streaming heads (Sec. 3.2) take no part: budget 0, no contribution to V; a group of
streaming heads only is not scheduled (V = 0, first candidate kept).
Readings where the paper is silent: budgets are clipped to [0, 1]; ties in V keep the earlier candidate.
Parity pins: tests/test_selector.py (closed-form crossover, monotone special cases, hand-worked numbers,
agreement of V with the byte model's counts).
"""
import math


def head_budget(bgt0, slope, blk, streaming=False):
    if streaming:
        return 0.0
    return min(1.0, max(0.0, float(bgt0) + float(slope) * math.log2(blk)))


def group_volume(l_cpu, blk, budgets):
    return 2.0 * l_cpu / blk + 2.0 * l_cpu * sum(budgets)


def choose(n_q_heads, n_kv_heads, bgt0, slope, l_cpu, streaming=None, candidates=(16, 32, 64, 128)):
    G = n_q_heads // n_kv_heads
    streaming = [False] * n_q_heads if streaming is None else [bool(s) for s in streaming]
    gran, budget, volume = [], [0.0] * n_q_heads, []
    for j in range(n_kv_heads):
        heads = range(j * G, (j + 1) * G)
        if all(streaming[h] for h in heads):
            gran.append(candidates[0])
            volume.append(0.0)
            continue
        best = None
        for blk in candidates:
            v = group_volume(l_cpu, blk, [head_budget(bgt0[h], slope[h], blk, streaming[h]) for h in heads])
            if best is None or v < best[0]:
                best = (v, blk)
        gran.append(best[1])
        volume.append(best[0])
        for h in heads:
            budget[h] = head_budget(bgt0[h], slope[h], best[1], streaming[h])
    return gran, budget, volume
