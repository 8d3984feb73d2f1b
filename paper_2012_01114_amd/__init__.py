"""attnring: skip-aware multi-head self-attention for MI355X (gfx950).

`attnring` is the binding of the C-ABI library (include/attnring.h), `inputs`
the seeded synthetic workloads, `build` compiles the library in-tree.
"""
