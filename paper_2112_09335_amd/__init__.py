"""Community-blocked ADMM sweep for GCN training on MI355X (gfx950).

`synth` draws seeded inputs; `binding` is the ctypes layer over the C-ABI HIP library
(loaded on first use; it raises if the library has not been built).
"""
