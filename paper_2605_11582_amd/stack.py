"""The 7B-shaped decoder stack of linear layers as a sequence of GEMV launches.

32 layers x {q, k, v, o (4096x4096), gate, up (11008x4096), down (4096x11008)};
a seeded half of the layers is stored 2:4-sparse INT4 in 2bit-CSR, the other half
dense INT4 (the layer-adaptive mix of Sec. 3.2, with the layer choice drawn from a
seed instead of an importance score).  Every matrix gets its own seeded x of the
right length; outputs are not chained.  Only marshalling and bookkeeping live here:
all arithmetic runs in libegt.so.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import binding as B
from . import synth

GROUP = 128


@dataclass
class StackMatrix:
    layer: int
    name: str
    rows: int
    cols: int
    sparse: bool
    call: object = None            # pre-marshalled launch
    keep: tuple = ()               # device tensors kept alive
    nbytes: int = 0                # algorithmic bytes of one launch
    y: object = None


def algorithmic_bytes(rows: int, cols: int, sparse: bool) -> int:
    if sparse:
        slots = rows * cols // 2
        return slots // 2 + slots // 4 + 4 * rows * (cols // GROUP) + 4 * rows + 4 + 2 * cols + 2 * rows
    return rows * cols // 2 + 4 * rows * (cols // GROUP) + 2 * cols + 2 * rows


def pack_layer_matrix(layer: int, mi: int, sparse: bool):
    """Host-side compressed form of matrix `mi` of `layer` (distinct seeded weights)."""
    name, rows, cols = synth.LAYER_MATRICES[mi]
    seed = synth.seed_for(4, layer * len(synth.LAYER_MATRICES) + mi)
    w = synth.weights(rows, cols, seed)
    x = synth.activations(cols, seed)
    if sparse:
        p = B.pack_2bitcsr(w, B.prune_n4(w, 2), 2, GROUP, B.VAL_INT4)
        return w, x, p
    q, qp = B.quant_int4(w, GROUP)
    return w, x, (q, qp)


@dataclass
class LayerStack:
    matrices: list = field(default_factory=list)

    @property
    def nbytes(self) -> int:
        return sum(m.nbytes for m in self.matrices)

    def run(self, stream_ptr=None) -> None:
        """One decode step's worth of linear layers: 224 launches in sequence."""
        if stream_ptr is None:
            for m in self.matrices:
                m.call()
        else:
            for m in self.matrices:
                m.call(stream_ptr)

    @staticmethod
    def build(device="cuda:0", distinct_layers=None, progress=None) -> "LayerStack":
        """Uploads the whole stack.  `distinct_layers`: how many layers of each kind get
        their own seeded weights (None = all); the remaining layers reuse the packed
        bytes of an earlier layer of the same kind in freshly allocated device memory
        (same traffic, same launches; only the numbers repeat)."""
        import torch
        sparse_ids = set(int(v) for v in synth.sparse_layers())
        st = LayerStack()
        cache = {True: [], False: []}
        for layer in range(synth.N_LAYERS):
            sparse = layer in sparse_ids
            reuse = distinct_layers is not None and len(cache[sparse]) >= distinct_layers
            if reuse:
                host = cache[sparse][layer % len(cache[sparse])]
            else:
                host = [pack_layer_matrix(layer, mi, sparse) for mi in range(len(synth.LAYER_MATRICES))]
                cache[sparse].append(host)
            for mi, (name, rows, cols) in enumerate(synth.LAYER_MATRICES):
                _, x, packed = host[mi]
                xd = torch.from_numpy(x.view(np.int16)).to(device).view(torch.float16)
                y = torch.empty(rows, dtype=torch.float16, device=device)
                m = StackMatrix(layer, name, rows, cols, sparse, nbytes=algorithmic_bytes(rows, cols, sparse), y=y)
                if sparse:
                    pd = packed.to(device)
                    m.call = B.prepared_sparse_gemv(pd, xd, y)
                    m.keep = (pd, xd)
                else:
                    q, qp = packed
                    qd = torch.from_numpy(q).to(device)
                    qpd = torch.from_numpy(qp.view(np.int16)).to(device)
                    m.call = B.prepared_int4_gemv(qd, qpd, rows, cols, GROUP, xd, y)
                    m.keep = (qd, qpd, xd)
                st.matrices.append(m)
            if progress:
                progress(layer)
        return st
