"""MI355X-native block-sparse decode attention (summaries, block selection, split-K sparse attention).

`paper_2605_07719_amd.fluxion` is the binding over the HIP C-ABI library; `paper_2605_07719_amd.workloads`
fabricates seeded synthetic inputs.  Nothing here falls back to a CPU path: using the binding without
the built library raises.
"""
