"""SparseGemv hot path (2bit-CSR, INT4/FP16, N:4 sparsity) for MI355X / gfx950.

`synth` (input generators) is importable without the HIP library; everything in
`binding` needs the built `libegt.so` and raises if it is missing.
"""
