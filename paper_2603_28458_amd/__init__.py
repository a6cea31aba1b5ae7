"""HISA hierarchical indexer for MI355X (gfx950): HIP kernels behind a C-ABI, with a thin binding.

`workloads` (seeded synthetic inputs) imports nothing native; the binding in `hisa` loads the
compiled library on first use and raises if it is missing.
"""
