"""The layer-step (fx_select + fx_sparse_decode) captured in a HIP graph: every replay must reproduce the
eager result bit for bit, with the program's own eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from helpers import GpuProblem
from paper_2605_07719_amd import workloads as W
from test_gpu_parity import TOL, run_oracle, small_cases

pytestmark = pytest.mark.gpu


def _graph_case(wl):
    layers = [W.make_layer(wl, layer) for layer in range(3)]
    refs = [run_oracle(wl, t) for t in layers]
    gps = [GpuProblem(wl, t, k_max=refs[0]["k_max"]) for t in layers]
    for gp in gps:
        gp.summarize()
    # share the selection/output/workspace buffers of problem 0 across the layers, as a decode loop would
    main = gps[0]

    def step(layer):
        gp = gps[layer]
        F = main.F
        bf = bfs[layer]
        F.select(gp.layout, gp.q, gp.S, budget_frac=bf, sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens,
                 k_max=main.k_max, idx=main.idx, cnt=main.cnt, workspace=main.ws_select)
        F.sparse_decode(gp.layout, gp.q, gp.K, gp.V, main.idx, main.cnt, k_max=main.k_max,
                        sink_tokens=wl.sink_tokens, window_tokens=wl.window_tokens, out=outs[layer],
                        workspace=main.ws_decode)

    bfs = [torch.from_numpy(wl.budget_frac.copy()).cuda() for _ in layers]
    outs = [torch.zeros_like(main.out) for _ in layers]
    for layer in range(3):          # eager pass (also warms up every kernel before capture)
        step(layer)
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    for layer in range(3):
        assert np.abs(eager[layer].cpu().numpy().astype(np.float64) - refs[layer]["out"]).max() < TOL

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for layer in range(3):
                step(layer)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for rep in range(4):
        for o in outs:
            o.fill_(float("nan"))                     # eager work between replays
        main.idx.fill_(-9)
        main.ws_decode.random_(0, 255)                # stale scratch must not matter
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for layer in range(3):
            assert torch.equal(outs[layer], eager[layer]), (rep, layer)
        step(rep % 3)                                  # an eager step between replays
        torch.cuda.synchronize()
        assert torch.equal(outs[rep % 3], eager[rep % 3])


def test_graph_replays_match_eager_and_oracle():
    _graph_case(small_cases()["d128_g4"])


def test_graph_replays_with_claimed_units():
    """A step large enough for the attention kernel's throughput regime (static shares plus units claimed from
    a counter that the plan kernel resets): replays must still reproduce the eager bits."""
    B = 8
    wl = W.Workload(name="graph_claimed", n_q_heads=8, n_kv_heads=4, head_dim=64, seq_len=[32768] * B,
                    gran=[16, 32, 16, 32], sink_tokens=64, window_tokens=256,
                    budget_frac=np.full((B, 8), 0.9, dtype=np.float32), seed=21)
    _graph_case(wl)


def test_stream_probes_run():
    """The measurement aids (plain read, non-temporal read, copy) accept a device buffer and complete."""
    from paper_2605_07719_amd import fluxion as F

    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    F.probe_read(src, sink, 2)
    F.probe_read_streaming(src, sink, 2)
    F.probe_copy(dst, src, 2)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
