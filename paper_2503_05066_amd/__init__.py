"""Capacity-aware MoE layer forward for MI355X (gfx950): HIP kernels behind a C ABI.

`paper_2503_05066_amd.synth` draws the seeded workloads; `paper_2503_05066_amd.capmoe`
is the thin binding to the shared library.  The library is loaded on first use, so
importing this package needs neither a GPU nor a built library.
"""
