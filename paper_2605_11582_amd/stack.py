"""The 7B-shaped decoder stack of linear layers as a sequence of GEMV launches.

32 layers x {q, k, v, o (4096x4096), gate, up (11008x4096), down (4096x11008)};
every layer is stored 2:4-sparse INT4, 1:4-sparse INT4 (both in 2bit-CSR) or dense
INT4 according to a seeded plan (the layer-adaptive mix of Sec. 3.2, with the layer
choice drawn from a seed instead of an importance score).  Every matrix gets its own
seeded x of the right length; outputs are not chained.  Only marshalling and
bookkeeping live here: all arithmetic runs in libegt.so.
"""
from __future__ import annotations

import os
from dataclasses import dataclass, field

import numpy as np

from . import binding as B
from . import synth

GROUP = 128
N_KEEP = {"s24": 2, "s14": 1}


@dataclass
class StackMatrix:
    layer: int
    name: str
    rows: int
    cols: int
    kind: str                      # "s24", "s14" or "d"
    call: object = None            # pre-marshalled launch
    keep: tuple = ()               # device tensors kept alive
    nbytes: int = 0                # algorithmic bytes of one launch
    y: object = None

    @property
    def sparse(self) -> bool:
        return self.kind != "d"


def algorithmic_bytes(rows: int, cols: int, kind) -> int:
    if kind is True:
        kind = "s24"
    elif kind is False:
        kind = "d"
    if kind != "d":
        slots = rows * N_KEEP[kind] * cols // 4
        return slots // 2 + slots // 4 + 4 * rows * (cols // GROUP) + 4 * rows + 4 + 2 * cols + 2 * rows
    return rows * cols // 2 + 4 * rows * (cols // GROUP) + 2 * cols + 2 * rows


def pack_layer_matrix(layer: int, mi: int, kind):
    """Host-side compressed form of matrix `mi` of `layer` (distinct seeded weights)."""
    if kind is True:
        kind = "s24"
    elif kind is False:
        kind = "d"
    name, rows, cols = synth.LAYER_MATRICES[mi]
    seed = synth.seed_for(4, layer * len(synth.LAYER_MATRICES) + mi)
    w = synth.weights(rows, cols, seed)
    x = synth.activations(cols, seed)
    if kind != "d":
        n = N_KEEP[kind]
        p = B.pack_2bitcsr(w, B.prune_n4(w, n), n, GROUP, B.VAL_INT4)
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

    def fuse(self) -> list:
        """Pre-marshalled launches with the q/k/v and the gate/up projections of every
        layer fused into one launch each: 4 launches per layer instead of 7."""
        calls = []
        nm = len(synth.LAYER_MATRICES)
        for l0 in range(0, len(self.matrices), nm):
            layer = self.matrices[l0:l0 + nm]
            by_name = {m.name: m for m in layer}
            for group in (("q", "k", "v"), ("o",), ("gate", "up"), ("down",)):
                ms = [by_name[n] for n in group]
                if len(ms) == 1:
                    calls.append(ms[0].call)
                elif ms[0].kind != "d":
                    calls.append(B.prepared_sparse_gemv_batch([m.keep[0] for m in ms], [m.keep[1] for m in ms],
                                                              [m.y for m in ms]))
                else:
                    calls.append(B.prepared_int4_gemv_batch([m.keep[0] for m in ms], [m.keep[1] for m in ms],
                                                            ms[0].rows, ms[0].cols, GROUP,
                                                            [m.keep[2] for m in ms], [m.y for m in ms]))
        return calls

    def _item(self, m):
        if m.kind != "d":
            return ("sparse", m.keep[0], m.keep[1], m.y)
        return ("dense", m.keep[0], m.keep[1], m.rows, m.cols, GROUP, m.keep[2], m.y)

    def per_layer(self) -> list:
        """One launch per decoder layer: its seven products, of three shapes, in one table."""
        nm = len(synth.LAYER_MATRICES)
        return [B.prepared_gemv_stack([self._item(m) for m in self.matrices[l0:l0 + nm]])
                for l0 in range(0, len(self.matrices), nm)]

    def one_launch(self):
        """The whole stack - 224 products of mixed storage forms - in a single launch."""
        return B.prepared_gemv_stack([self._item(m) for m in self.matrices])

    def verify_step(self, M: int, kind="s24"):
        """A verification step of M candidate tokens (Sec. 3.4) through the 2:4 (kind "s24"),
        the 1:4 ("s14") or all sparse (("s24", "s14"): one launch per form) layers of the
        stack: every such matrix times M token rows of its own.  Returns the pre-marshalled
        call and the algorithmic bytes of one call."""
        kinds = (kind,) if isinstance(kind, str) else tuple(kind)
        import torch
        items, nbytes = [], 0
        rows_of = {}                                   # seeded token rows, drawn once per row length
        for k, m in enumerate(self.matrices):
            if m.kind not in kinds:
                continue
            dev = m.y.device
            if m.cols not in rows_of:
                rows_of[m.cols] = synth.activation_rows(M, m.cols, synth.seed_for(4, 1000 + m.cols)).view(np.int16)
            X = torch.from_numpy(rows_of[m.cols]).to(dev).view(torch.float16)       # a device copy per matrix
            Y = torch.empty((M, m.rows), dtype=torch.float16, device=dev)
            items.append((m.keep[0], X, Y))
            nbytes += m.nbytes + (M - 1) * 2 * (m.cols + m.rows)
        return B.prepared_gemm_stack(items), nbytes

    @staticmethod
    def build(device="cuda:0", distinct_layers=None, progress=None, plan="config4", on_matrix=None) -> "LayerStack":
        """Uploads the whole stack.  `distinct_layers`: how many layers of each kind get
        their own seeded weights (None = all 32, the configuration as stated); the
        remaining layers reuse the packed bytes of an earlier layer of the same kind in
        freshly allocated device memory (same traffic, same launches; only the numbers
        repeat).  `on_matrix(layer, mi, kind, w, x, packed)` is called for every matrix
        with weights of its own while its host data is alive (the dense weights are not
        kept afterwards)."""
        import torch
        from concurrent.futures import ThreadPoolExecutor
        kinds = synth.layer_kinds(plan)
        st = LayerStack()
        cache = {"s24": [], "s14": [], "d": []}
        nm = len(synth.LAYER_MATRICES)
        # which layers get weights of their own is known up front, so their matrices are
        # drawn and packed by a few host threads ahead of the upload (numpy's generator and
        # the encoder both release the interpreter lock)
        own, count = [], {"s24": 0, "s14": 0, "d": 0}
        for layer in range(synth.N_LAYERS):
            if distinct_layers is None or count[kinds[layer]] < distinct_layers:
                own.append(layer)
                count[kinds[layer]] += 1
        pool = ThreadPoolExecutor(max_workers=max(1, min(6, (os.cpu_count() or 2) // 2)))
        pending, ahead = {}, 10                         # at most `ahead` matrices in flight
        todo = [(layer, mi) for layer in own for mi in range(nm)]

        def refill():
            while todo and len(pending) < ahead:
                key = todo.pop(0)
                pending[key] = pool.submit(pack_layer_matrix, key[0], key[1], kinds[key[0]])
        for layer in range(synth.N_LAYERS):
            kind = kinds[layer]
            if layer not in own:
                host = cache[kind][layer % len(cache[kind])]
            else:
                host = []
                for mi in range(nm):
                    refill()
                    w, x, packed = pending.pop((layer, mi)).result()
                    if on_matrix:
                        on_matrix(layer, mi, kind, w, x, packed)
                    host.append((None, x, packed))
                    del w
                if distinct_layers is not None:
                    cache[kind].append(host)
            for mi, (name, rows, cols) in enumerate(synth.LAYER_MATRICES):
                _, x, packed = host[mi]
                xd = torch.from_numpy(x.view(np.int16)).to(device).view(torch.float16)
                y = torch.empty(rows, dtype=torch.float16, device=device)
                m = StackMatrix(layer, name, rows, cols, kind, nbytes=algorithmic_bytes(rows, cols, kind), y=y)
                if kind != "d":
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
        pool.shutdown()
        return st
