"""Seeded synthetic inputs for the block-sparse decode path.

This module only fabricates tensors and the bookkeeping that says where they live (sequence lengths,
offsets, strides, block sizes, budgets).  It holds none of the method's arithmetic: no summaries, no
scores, no selection, no attention.  The HIP binding and the CPU oracle are both fed from here so that
they see the same bytes; neither is imported here.

The efficiency workloads of the paper (Sec. 7.1) are length-controlled benchmark inputs run through
Llama-3.1-8B-Instruct and Qwen2.5-7B-Instruct; neither the inputs nor the weights are available, so
the tensors below stand in for them: same shapes (32 q / 8 kv heads, head_dim 128, 32 layers; 28 q / 4
kv heads, 28 layers), contexts 32K-128K, batch 1-16, mixed lengths, and roughly Gaussian q.k (the
paper's App. A observes that q.k / (|q| sqrt(D)) is close to normal).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional

import numpy as np
import torch


@dataclass
class Workload:
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: List[int]  # tokens per sequence (ragged)
    gran: List[int]  # logical block size per KV head
    sink_tokens: int
    window_tokens: int
    n_layers: int = 1
    budget_frac: Optional[np.ndarray] = None  # float32 [batch, Hq], or None
    budget_blocks: Optional[np.ndarray] = None  # int32 [batch, Hq], or None
    outlier_channels: int = 0  # K channels per KV head multiplied by outlier_scale
    outlier_scale: float = 10.0
    planted_per_head: int = 0  # fixed number of hot blocks per (sequence, q head) ...
    planted_density: float = 0.0  # ... or a fraction of the interior blocks
    plant_margin_lo: int = 128  # hot blocks are drawn from tokens [margin_lo, N - margin_hi)
    plant_margin_hi: int = 512
    q_mode: str = "normal"  # "normal": q ~ N(0,1);  "near_key": q = 0.5 * k_t* + N(0,1)
    seed: int = 0
    notes: str = ""

    @property
    def batch(self) -> int:
        return len(self.seq_len)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seq_len))


@dataclass
class Placement:
    """Where a workload's tensors live: K and V are [Hkv, total_tokens, d] (head-major over the whole
    batch, each sequence's tokens contiguous), summaries are [total_blocks, 2, d]."""

    seq_len: np.ndarray  # int32 [batch]
    tok_off: np.ndarray  # int64 [batch]   first token row of each sequence
    seq_base: np.ndarray  # int64 [batch]   = tok_off * d (element offset)
    kv_head_stride: int  # = total_tokens * d
    token_stride: int  # = d
    n_blocks: np.ndarray  # int64 [batch, Hkv]
    sum_base: np.ndarray  # int64 [batch, Hkv]  running sum of n_blocks in (b, j) order
    total_blocks: int
    gran: np.ndarray  # int32 [Hkv]


def placement(wl: Workload) -> Placement:
    d = wl.head_dim
    seq_len = np.asarray(wl.seq_len, dtype=np.int32)
    tok_off = np.zeros(wl.batch, dtype=np.int64)
    tok_off[1:] = np.cumsum(seq_len.astype(np.int64))[:-1]
    gran = np.asarray(wl.gran, dtype=np.int32)
    assert gran.size == wl.n_kv_heads
    n_blocks = -(-seq_len.astype(np.int64)[:, None] // gran.astype(np.int64)[None, :])
    flat = n_blocks.reshape(-1)
    sum_base = np.zeros_like(flat)
    sum_base[1:] = np.cumsum(flat)[:-1]
    return Placement(
        seq_len=seq_len,
        tok_off=tok_off,
        seq_base=tok_off * d,
        kv_head_stride=int(wl.total_tokens) * d,
        token_stride=d,
        n_blocks=n_blocks,
        sum_base=sum_base.reshape(wl.batch, wl.n_kv_heads),
        total_blocks=int(flat.sum()),
        gran=gran,
    )


@dataclass
class LayerTensors:
    q: torch.Tensor  # bf16 [batch, Hq, d]
    K: torch.Tensor  # bf16 [Hkv, total_tokens, d]
    V: torch.Tensor  # bf16 [Hkv, total_tokens, d]
    planted: List[List[np.ndarray]] = field(default_factory=list)  # [batch][Hq] -> hot block indices


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_layer(wl: Workload, layer: int = 0, device="cpu") -> LayerTensors:
    """Fabricate q, K, V of one layer.  Deterministic in (wl.seed, layer, device type)."""
    dev = torch.device(device)
    pl = placement(wl)
    d, Hkv, Hq, G = wl.head_dim, wl.n_kv_heads, wl.n_q_heads, wl.group
    T = wl.total_tokens
    g_main = _gen(dev, (wl.seed * 1000003 + layer) * 8 + 1)
    g_cpu = _gen("cpu", (wl.seed * 1000003 + layer) * 8 + 2)  # small host-side draws (indices)

    K = torch.empty((Hkv, T, d), dtype=torch.bfloat16, device=dev)
    V = torch.empty((Hkv, T, d), dtype=torch.bfloat16, device=dev)
    for j in range(Hkv):  # per head: bounds the size of any temporary
        K[j].normal_(0.0, 1.0, generator=g_main)
        V[j].normal_(0.0, 1.0, generator=g_main)

    if wl.outlier_channels > 0:
        for j in range(Hkv):
            ch = torch.randperm(d, generator=g_cpu)[: wl.outlier_channels].to(dev)
            K[j][:, ch] = (K[j][:, ch].float() * wl.outlier_scale).to(torch.bfloat16)

    q32 = torch.empty((wl.batch, Hq, d), dtype=torch.float32, device=dev).normal_(0.0, 1.0, generator=g_main)
    if wl.q_mode == "near_key":
        for b in range(wl.batch):
            t_star = torch.randint(0, int(pl.seq_len[b]), (Hq,), generator=g_cpu)
            for h in range(Hq):
                row = int(pl.tok_off[b]) + int(t_star[h])
                q32[b, h] += 0.5 * K[h // G, row].float()
    elif wl.q_mode != "normal":
        raise ValueError(wl.q_mode)
    q = q32.to(torch.bfloat16)

    planted: List[List[np.ndarray]] = []
    if wl.planted_per_head > 0 or wl.planted_density > 0.0:
        qf = q.float()
        q_dir = qf / qf.norm(dim=-1, keepdim=True)
        for b in range(wl.batch):
            per_b: List[np.ndarray] = [np.zeros(0, dtype=np.int64) for _ in range(Hq)]
            N = int(pl.seq_len[b])
            for j in range(Hkv):
                g = int(pl.gran[j])
                lo = -(-wl.plant_margin_lo // g)
                hi = max((N - wl.plant_margin_hi) // g, lo)
                n_int = hi - lo
                n_plant = wl.planted_per_head if wl.planted_per_head > 0 else int(round(wl.planted_density * n_int))
                n_plant = min(n_plant, n_int // max(G, 1))
                if n_plant <= 0:
                    continue
                perm = torch.randperm(n_int, generator=g_cpu)[: n_plant * G].numpy() + lo
                for r in range(G):
                    h = j * G + r
                    blocks = np.sort(perm[r * n_plant : (r + 1) * n_plant]).astype(np.int64)
                    per_b[h] = blocks
                    rows = (torch.from_numpy(blocks)[:, None] * g + torch.arange(g)[None, :]).reshape(-1)
                    rows = (rows + int(pl.tok_off[b])).to(dev)
                    K[j, rows] = (K[j, rows].float() + 3.0 * q_dir[b, h][None, :]).to(torch.bfloat16)
            planted.append(per_b)
    return LayerTensors(q=q, K=K, V=V, planted=planted)


# ---------------------------------------------------------------------------------------------------
# The five named configurations.  `scale_context` shrinks the context (and nothing else) so the same
# recipe can be used for parity tests the oracle finishes in seconds.
# ---------------------------------------------------------------------------------------------------

def _head_budgets(n_q_heads: int, n_dense: int, mean: float, lo: float, hi: float, rng: np.random.Generator):
    """Log-uniform budgets in [lo, hi] rescaled to the requested mean, then `n_dense` heads set to 1.0."""
    b = np.exp(rng.uniform(np.log(lo), np.log(hi), size=n_q_heads))
    dense = rng.choice(n_q_heads, size=n_dense, replace=False) if n_dense > 0 else np.zeros(0, dtype=np.int64)
    sparse = np.setdiff1d(np.arange(n_q_heads), dense)
    b[sparse] *= mean / b[sparse].mean()
    b[dense] = 1.0
    return np.minimum(b, 1.0).astype(np.float32)


def tiny(seed: int = 0) -> Workload:
    """Config 1: 4 q heads on 1 KV head, d=64, 2048 tokens, g=16, top-8 + 1 sink block + 4 window blocks."""
    return Workload(
        name="tiny", n_q_heads=4, n_kv_heads=1, head_dim=64, seq_len=[2048], gran=[16], sink_tokens=16,
        window_tokens=64, budget_blocks=np.full((1, 4), 8, dtype=np.int32), planted_per_head=4,
        plant_margin_lo=16, plant_margin_hi=80, seed=seed,
    )


def llama_stack(context: int = 32768, n_layers: int = 32, budget: float = 0.05, seed: int = 0) -> Workload:
    """Config 2: Llama-3-8B-shaped stack, batch 1, g=32, uniform budget, 1 sink block + 8 window blocks."""
    return Workload(
        name=f"llama_stack_{context}", n_q_heads=32, n_kv_heads=8, head_dim=128, seq_len=[context], gran=[32] * 8,
        sink_tokens=32, window_tokens=256, n_layers=n_layers, budget_frac=np.full((1, 32), budget, dtype=np.float32),
        outlier_channels=4, q_mode="near_key", seed=seed,
    )


def head_specific(context: int = 131072, batch: int = 4, n_layers: int = 4, seed: int = 0) -> Workload:
    """Config 3: Llama-shaped layer, per-KV-head block size from {16,32,64}, log-uniform head budgets with
    mean 0.05 plus 2 dense heads, hot blocks at 0.5% density."""
    rng = np.random.default_rng(seed + 303)
    gran = rng.choice([16, 32, 64], size=8).tolist()
    bud = _head_budgets(32, 2, 0.05, 0.01, 0.2, rng)
    return Workload(
        name=f"head_specific_{context}x{batch}", n_q_heads=32, n_kv_heads=8, head_dim=128, seq_len=[context] * batch,
        gran=gran, sink_tokens=64, window_tokens=256, n_layers=n_layers,
        budget_frac=np.broadcast_to(bud, (batch, 32)).copy(), planted_density=0.005, seed=seed,
    )


def qwen_ragged(lo: int = 16384, hi: int = 65536, batch: int = 16, n_layers: int = 28, seed: int = 0) -> Workload:
    """Config 4: Qwen2.5-7B-shaped ragged batch (28 q / 4 kv, G=7), lengths uniform in [lo, hi], g=32."""
    rng = np.random.default_rng(seed + 404)
    lens = rng.integers(lo, hi + 1, size=batch).tolist()
    bud = _head_budgets(28, 2, 0.05, 0.01, 0.2, rng)
    return Workload(
        name=f"qwen_ragged_{lo}-{hi}x{batch}", n_q_heads=28, n_kv_heads=4, head_dim=128, seq_len=lens, gran=[32] * 4,
        sink_tokens=64, window_tokens=256, n_layers=n_layers, budget_frac=np.broadcast_to(bud, (batch, 28)).copy(),
        outlier_channels=4, q_mode="near_key", seed=seed,
    )


def hbm_stress(budget: float = 0.05, context: int = 131072, batch: int = 16, n_layers: int = 16, seed: int = 0) -> Workload:
    """Config 5: Llama shape, batch 16 x 128K, g=32, uniform budget from {0.02, 0.05, 0.1, 1.0}, hot blocks.
    32 layers of this shape are 256 GiB of K+V and do not fit one GPU; 16 layers (128 GiB) do."""
    return Workload(
        name=f"hbm_stress_{context}x{batch}_b{budget}", n_q_heads=32, n_kv_heads=8, head_dim=128,
        seq_len=[context] * batch, gran=[32] * 8, sink_tokens=64, window_tokens=256, n_layers=n_layers,
        budget_frac=np.full((batch, 32), budget, dtype=np.float32), planted_density=0.005, seed=seed,
    )


def with_budget(wl: Workload, budget: float) -> Workload:
    return replace(wl, budget_frac=np.full((wl.batch, wl.n_q_heads), budget, dtype=np.float32), budget_blocks=None)


def subset(wl: Workload, tensors: LayerTensors, seqs: List[int]):
    """A smaller workload holding only the chosen sequences, with copies of their q/K/V rows (used to
    hand the oracle a bounded slice of a large layer)."""
    pl = placement(wl)
    sub = replace(
        wl, name=wl.name + "_sub", seq_len=[int(pl.seq_len[b]) for b in seqs],
        budget_frac=None if wl.budget_frac is None else wl.budget_frac[seqs].copy(),
        budget_blocks=None if wl.budget_blocks is None else wl.budget_blocks[seqs].copy(),
    )
    rows = torch.cat([torch.arange(int(pl.tok_off[b]), int(pl.tok_off[b]) + int(pl.seq_len[b])) for b in seqs])
    rows = rows.to(tensors.K.device)
    t = LayerTensors(
        q=tensors.q[seqs].contiguous(), K=tensors.K[:, rows].contiguous(), V=tensors.V[:, rows].contiguous(),
        planted=[tensors.planted[b] for b in seqs] if tensors.planted else [],
    )
    return sub, t


def to_u16(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> host uint16 bit patterns."""
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


# ---------------------------------------------------------------------------------------------------
# Per-query granularity (Sec. 5.2, 5.3: the block size of a group is chosen per decode step from predicted
# head properties).  The head-property predictor needs trained weights and is not part of this build; the
# seeded draws below stand in for its outputs.  The summary pyramid keeps one set of summaries per candidate
# block size in one buffer, so that a step's mixed block sizes are just a table of offsets.
# ---------------------------------------------------------------------------------------------------

def head_properties(n_q_heads: int, seed: int, streaming_frac: float = 0.125, n_kv_heads: int = 1):
    """Stand-ins for the predictor's per-head outputs of one step: budget at block size 1 (`bgt0`), growth
    per log2 of the block size (`slope`), and the streaming flag (Sec. 3.2).  Half of the heads are flat
    (their budget hardly grows with the block size, so coarse blocks are cheap for them), half are steep;
    a per-group factor makes some GQA groups flat as a whole, so that all candidate block sizes occur."""
    rng = np.random.default_rng(seed + 707)
    bgt0 = np.exp(rng.uniform(np.log(0.005), np.log(0.08), size=n_q_heads))
    flat = rng.random(n_q_heads) < 0.5
    slope = np.where(flat, rng.uniform(0.0, 0.003, size=n_q_heads), rng.uniform(0.008, 0.03, size=n_q_heads))
    slope = slope * np.repeat(rng.choice([0.1, 0.35, 1.0], size=n_kv_heads), n_q_heads // n_kv_heads)
    streaming = rng.random(n_q_heads) < streaming_frac
    return bgt0.astype(np.float32), slope.astype(np.float32), streaming.astype(np.uint8)


@dataclass
class Pyramid:
    """Summaries of one layer at several block sizes in one [total_blocks, 2, d] buffer: level g occupies the
    blocks [level_base[g], level_base[g] + placements[g].total_blocks)."""

    levels: List[int]
    level_base: dict
    placements: dict  # block size -> Placement with that block size for every KV head
    total_blocks: int

    def sum_base(self, gran) -> np.ndarray:
        """int64 [batch, Hkv]: block offset of (b, j) inside the combined buffer when KV head j uses gran[j]."""
        cols = [self.level_base[int(g)] + self.placements[int(g)].sum_base[:, j] for j, g in enumerate(gran)]
        return np.stack(cols, axis=1).astype(np.int64)


def pyramid(wl: Workload, levels=(16, 32, 64, 128)) -> Pyramid:
    base, placements, off = {}, {}, 0
    for g in levels:
        pl = placement(replace(wl, gran=[int(g)] * wl.n_kv_heads))
        base[int(g)], placements[int(g)] = off, pl
        off += pl.total_blocks
    return Pyramid(levels=[int(g) for g in levels], level_base=base, placements=placements, total_blocks=off)
