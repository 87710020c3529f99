"""Seeded synthetic inputs for the SparseGemv path.

This module only draws random numbers and casts them: it contains none of the
method's arithmetic (no pruning, no quantisation, no packing), so both the HIP
path and the CPU oracle can be fed from it without sharing logic.

Recipe (stands in for trained decoder weights and real activations):
  W = float16( standard_normal(float32) * 0.02 ),  x = float16( standard_normal(float32) )
drawn from numpy's Generator(PCG64(seed)).
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 1158200000
HEADLINE = 0                     # config id used for the headline workload

# decoder layer of a 7B-shaped model: (name, rows = out features, cols = in features)
LAYER_MATRICES = (
    ("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
    ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008),
)
N_LAYERS = 32


def seed_for(config: int, matrix_index: int = 0) -> int:
    return SEED_BASE + 100000 * config + matrix_index


def weights(rows: int, cols: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    w = rng.standard_normal((rows, cols), dtype=np.float32)
    w *= np.float32(0.02)
    return w.astype(np.float16)


def activations(cols: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed + 50000))
    return rng.standard_normal(cols, dtype=np.float32).astype(np.float16)


def activation_rows(m: int, cols: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed + 50000))
    return rng.standard_normal((m, cols), dtype=np.float32).astype(np.float16)


def sparse_layers(seed: int = SEED_BASE + 400000) -> np.ndarray:
    """Layer-adaptive mix of the 32-layer stack: the sorted ids of the 16 layers
    stored 2:4-sparse INT4; the other 16 are dense INT4."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return np.sort(rng.permutation(N_LAYERS)[: N_LAYERS // 2])


def layer_kinds(plan: str = "config4") -> list:
    """Per-layer storage of the 32-layer stack: "s24" (2:4 sparse INT4), "s14" (1:4 sparse
    INT4) or "d" (dense INT4).  "config4": the seeded half/half mix of 2:4 and dense;
    "mix3": a seeded three-way mix (11 x 2:4, 11 x 1:4, 10 x dense), the layer-adaptive
    setting with both sparsities in use."""
    if plan == "config4":
        sp = set(int(v) for v in sparse_layers())
        return ["s24" if l in sp else "d" for l in range(N_LAYERS)]
    if plan == "mix3":
        rng = np.random.Generator(np.random.PCG64(SEED_BASE + 410000))
        order = rng.permutation(N_LAYERS)
        kinds = [""] * N_LAYERS
        for pos, layer in enumerate(order):
            kinds[int(layer)] = "s24" if pos < 11 else ("s14" if pos < 22 else "d")
        return kinds
    raise ValueError(plan)
