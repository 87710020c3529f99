"""Config 4: the 32-layer 7B-shaped stack, 224 GEMV launches (16 layers 2:4-sparse INT4 in
2bit-CSR, 16 dense INT4), plain and replayed from a HIP graph; the three-way layer mix;
the trigger cost model on a measured M-sweep."""
import numpy as np
import pytest

from oracle import egt_oracle as O
from paper_2605_11582_amd import binding as B, stack as S, synth
import gpu_common as G

pytestmark = pytest.mark.gpu


def test_layer_plan():
    ids = synth.sparse_layers()
    assert len(ids) == 16 and len(set(ids.tolist())) == 16 and ids.min() >= 0 and ids.max() < 32
    total = sum(S.algorithmic_bytes(r, c, True) for _, r, c in synth.LAYER_MATRICES) * 16 + \
        sum(S.algorithmic_bytes(r, c, False) for _, r, c in synth.LAYER_MATRICES) * 16
    assert total == 3043344832                    # closed form of the byte model for this stack


def test_three_way_plan():
    kinds = synth.layer_kinds("mix3")
    assert sorted(set(kinds)) == ["d", "s14", "s24"]
    assert (kinds.count("s24"), kinds.count("s14"), kinds.count("d")) == (11, 11, 10)


class _OracleSamples:
    """Collects, while a stack is built, the oracle's result on sampled rows of every matrix
    that has weights of its own: the oracle prunes, quantises and packs those rows itself
    (bit-compared with the library's bytes) and multiplies them with x in float64."""

    def __init__(self, per_matrix=32):
        self.per_matrix = per_matrix
        self.ref = {}                                   # (layer, mi) -> (rows, y_ref, a_ref)

    def __call__(self, layer, mi, kind, w, x, packed):
        name, rows, cols = synth.LAYER_MATRICES[mi]
        pick = G.sample_rows(rows, self.per_matrix, layer * len(synth.LAYER_MATRICES) + mi)
        if kind != "d":
            n = S.N_KEEP[kind]
            o = O.pack_2bitcsr(w[pick], O.prune_n4_magnitude(w[pick], n), n, 128, O.VAL_INT4)
            sub = G.row_subset(packed, pick)
            for k in ("values", "idx", "qparams"):
                assert np.array_equal(o[k], sub[k]), (layer, name, k)
            y_ref, a_ref = O.gemv(o, x)
        else:
            oq, oqp = O.quant_int4_dense(w[pick], 128)
            assert np.array_equal(oq, packed[0][pick]) and np.array_equal(oqp, packed[1][pick]), (layer, name)
            y_ref, a_ref = O.int4_gemv(oq, oqp, 128, x)
        self.ref[(layer, mi)] = (pick, y_ref, a_ref)

    def check(self, outputs, what):
        nm = len(synth.LAYER_MATRICES)
        worst = 0.0
        for (layer, mi), (pick, y_ref, a_ref) in self.ref.items():
            worst = max(worst, G.assert_close(outputs[layer * nm + mi][pick], y_ref, a_ref,
                                              f"{what} layer {layer} {synth.LAYER_MATRICES[mi][0]}"))
        return worst


def _progress(layer):
    if layer % 4 == 3:
        print(f"  layer {layer} packed, checked and uploaded", flush=True)


def test_stack_parity_and_graph_replay():
    # config 4 as stated: all 32 layers carry their own seeded weights (224 distinct matrices);
    # the oracle re-encodes sampled rows of every one of them
    torch = G.torch_mod()
    print("building the 32-layer stack, every layer with its own weights", flush=True)
    samples = _OracleSamples()
    st = S.LayerStack.build("cuda:0", distinct_layers=None, progress=_progress, on_matrix=samples)
    assert len(st.matrices) == 224 and st.nbytes == 3043344832 and len(samples.ref) == 224
    sparse_ids = set(int(v) for v in synth.sparse_layers())
    assert [k != "d" for k in synth.layer_kinds("config4")] == [l in sparse_ids for l in range(32)]
    st.run()
    torch.cuda.synchronize()
    eager = [m.y.cpu().numpy().copy() for m in st.matrices]
    worst = samples.check(eager, "config 4")
    print(f"  224 matrices match the oracle on sampled rows (max err / bound {worst:.4f})", flush=True)
    # distinct seeds give distinct results: no layer repeats another layer's output
    nm = len(synth.LAYER_MATRICES)
    seen = set()
    for m_i in range(0, 224, nm):
        key = eager[m_i].tobytes()
        assert key not in seen
        seen.add(key)
    # fused launches (q/k/v and gate/up in one launch each): same bits as the separate launches
    fused = st.fuse()
    assert len(fused) == 32 * 4
    for m in st.matrices:
        m.y.fill_(3.0)
    for c in fused:
        c()
    torch.cuda.synchronize()
    for m_i, m in enumerate(st.matrices):
        assert np.array_equal(m.y.cpu().numpy().view(np.uint16), eager[m_i].view(np.uint16)), ("fused", m.layer, m.name)
    print("  fused launches match the separate ones", flush=True)
    # one launch per layer (seven products of three shapes), and the whole stack in one launch
    for what, launches in (("one launch per layer", st.per_layer()), ("one launch per stack", [st.one_launch()])):
        for m in st.matrices:
            m.y.fill_(3.0)
        for c in launches:
            c()
        torch.cuda.synchronize()
        outs = [m.y.cpu().numpy() for m in st.matrices]
        samples.check(outs, what)
        for m_i, m in enumerate(st.matrices):
            assert np.array_equal(outs[m_i].view(np.uint16), eager[m_i].view(np.uint16)), (what, m.layer, m.name)
        print(f"  {what}: {len(launches)} launches match the oracle and the separate launches bit for bit", flush=True)
    # HIP graph of the 224 launches: several replays, with eager work between them
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        st.run(side.cuda_stream)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            st.run(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        for m in st.matrices:
            m.y.fill_(7.0)                          # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for m_i, m in enumerate(st.matrices):
            assert np.array_equal(m.y.cpu().numpy().view(np.uint16), eager[m_i].view(np.uint16)), (rep, m.layer, m.name)
        print(f"  graph replay {rep} matches the eager run", flush=True)


def test_three_way_mix_stack_parity():
    # the layer-adaptive mix with both sparsities in use (2:4, 1:4 and dense layers, Sec. 3.2):
    # two layers of each kind carry their own weights and are checked against the oracle; the
    # other layers reuse those bytes in their own device memory and must reproduce the bits
    torch = G.torch_mod()
    samples = _OracleSamples(per_matrix=48)
    st = S.LayerStack.build("cuda:0", distinct_layers=2, progress=_progress, plan="mix3", on_matrix=samples)
    kinds = synth.layer_kinds("mix3")
    nm = len(synth.LAYER_MATRICES)
    assert len(st.matrices) == 224 and len(samples.ref) == 6 * nm
    assert sorted(set(kinds[l] for (l, _) in samples.ref)) == ["d", "s14", "s24"]
    assert st.nbytes == sum(S.algorithmic_bytes(r, c, kinds[l]) for l in range(32) for _, r, c in synth.LAYER_MATRICES)
    st.run()
    torch.cuda.synchronize()
    eager = [m.y.cpu().numpy().copy() for m in st.matrices]
    worst = samples.check(eager, "mix3")
    print(f"  {len(samples.ref)} matrices of the three kinds match the oracle (max err / bound {worst:.4f})", flush=True)
    own = {}                                            # kind -> layers with their own weights, in order
    for (l, _) in samples.ref:
        if l not in own.setdefault(kinds[l], []):
            own[kinds[l]].append(l)
    for m_i, m in enumerate(st.matrices):
        src_layer = own[m.kind][m.layer % len(own[m.kind])] if m.layer not in own[m.kind] else m.layer
        src = src_layer * nm + m_i % nm
        assert np.array_equal(eager[m_i].view(np.uint16), eager[src].view(np.uint16)), (m.layer, m.name)
    # fused launches on the mixed stack: q/k/v and gate/up of a 1:4 layer in one launch too
    fused = st.fuse()
    for m in st.matrices:
        m.y.fill_(3.0)
    for c in fused:
        c()
    torch.cuda.synchronize()
    for m_i, m in enumerate(st.matrices):
        assert np.array_equal(m.y.cpu().numpy().view(np.uint16), eager[m_i].view(np.uint16)), ("fused", m.layer, m.name)


def test_mixed_table_in_one_launch_small_shapes():
    # egt_gemv_stack_run on a table of small matrices of every storage form and of several
    # shapes (ragged row counts, one and several tiles per row, several rows per tile, an empty
    # matrix): element by element against the oracle and bit for bit against separate calls
    torch = G.torch_mod()
    specs = [("s24", 37, 4096), ("d", 50, 4096), ("s14", 45, 4096), ("s24", 21, 11008), ("d", 19, 11008),
             ("s14", 21, 11008), ("s24", 70, 2048), ("s24", 0, 4096), ("d", 33, 8192), ("s24", 300, 8192),
             ("s14", 19, 2048), ("d", 131, 1024), ("s24", 257, 1024), ("s24", 1003, 4096)]
    items, refs, singles = [], [], []
    for k, (kind, rows, cols) in enumerate(specs):
        w = synth.weights(rows, cols, 4400 + k)
        x = synth.activations(cols, 4400 + k)
        xd = G.to_dev(x.view(np.uint16)).view(torch.float16)
        ybuf = torch.full((rows + 128,), G.CANARY, dtype=torch.int16, device="cuda")
        y = ybuf[64:64 + rows].view(torch.float16)
        y1 = torch.empty(rows, dtype=torch.float16, device="cuda")
        if kind == "d":
            q, qp = B.quant_int4(w, 128)
            qd, qpd = G.to_dev(q), G.to_dev(qp)
            items.append(("dense", qd, qpd, rows, cols, 128, xd, y))
            oq, oqp = O.quant_int4_dense(w, 128)
            refs.append(O.int4_gemv(oq, oqp, 128, x))
            B.int4_gemv(qd, qpd, rows, cols, 128, xd, y1)
        else:
            n = S.N_KEEP[kind]
            mask = O.prune_n4_magnitude(w, n)
            p = B.pack_2bitcsr(w, mask, n, 128, 0).to("cuda")
            items.append(("sparse", p, xd, y))
            refs.append(O.gemv(O.pack_2bitcsr(w, mask, n, 128, 0), x))
            B.sparse_gemv(p, xd, y1)
        singles.append((ybuf, y1))
    call = B.prepared_gemv_stack(items)
    # two launches: 2:4 and dense matrices with 1, 2, 3, 4 and 6 tiles per row (twelve waves), the 1:4 matrices (four waves)
    assert call.plan.count == len(specs) and call.plan.nparts == 2
    assert [(q.count, q.mode, q.block_threads, q.forms) for q in call.plan.part] == [(11, 0, 768, 5), (3, 0, 256, 2)]
    for rep in range(2):
        call()
        torch.cuda.synchronize()
        for k, (kind, rows, cols) in enumerate(specs):
            ybuf, y1 = singles[k]
            host = ybuf.cpu().numpy().view(np.uint16)
            assert np.all(host[:64] == G.CANARY) and np.all(host[64 + rows:] == G.CANARY), ("write outside y", k)
            y = host[64:64 + rows].view(np.float16)
            G.assert_close(y, refs[k][0], refs[k][1], f"table item {k} {kind} {rows}x{cols}")
            assert np.array_equal(y.view(np.uint16), y1.cpu().numpy().view(np.uint16)), (k, kind, rows, cols)
            ybuf[64:64 + rows].fill_(0)
    # other wave counts: one tile per row everywhere -> 4 waves; four tiles per row -> 4 waves too
    small = B.prepared_gemv_stack([items[0], items[2]])
    assert small.plan.nparts == 2 and small.plan.part[0].block_threads == 256 and small.plan.part[1].block_threads == 256
    small()
    torch.cuda.synchronize()
    for k in (0, 2):
        y = items[k][-1].cpu().numpy()
        G.assert_close(y, refs[k][0], refs[k][1], f"4-wave table item {k}")


@pytest.mark.parametrize("seed", range(3))
def test_seeded_tables_equal_separate_calls(seed):
    # tables nobody picked by hand: random storage forms, shapes and order, with and without 1:4
    # members (one launch or two); every member bit for bit against its separate call
    torch = G.torch_mod()
    rng = np.random.default_rng(4900 + seed)
    kinds = ["s24", "d", "s14"] if seed != 1 else ["s24", "d"]
    colset = {"s24": [1024, 2048, 4096, 8192, 11008, 12288], "d": [1024, 2048, 4096, 8192, 11008], "s14": [2048, 4096, 8192, 11008]}
    items, singles = [], []
    for k in range(int(rng.integers(5, 12))):
        kind = kinds[int(rng.integers(len(kinds)))]
        cols = int(rng.choice(colset[kind]))
        rows = int(rng.choice([0, 1, 15, 64, 200, 777, 1500])) if k else 333
        print(f"  table {seed} item {k}: {kind} {rows}x{cols}", flush=True)
        w = synth.weights(rows, cols, 4900 + 50 * seed + k)
        xd = G.to_dev(synth.activations(cols, 4900 + k).view(np.uint16)).view(torch.float16)
        ybuf = torch.full((rows + 128,), G.CANARY, dtype=torch.int16, device="cuda")
        y = ybuf[64:64 + rows].view(torch.float16)
        y1 = torch.zeros(rows, dtype=torch.float16, device="cuda")
        if kind == "d":
            q, qp = B.quant_int4(w, 128)
            qd, qpd = G.to_dev(q), G.to_dev(qp)
            items.append(("dense", qd, qpd, rows, cols, 128, xd, y))
            B.int4_gemv(qd, qpd, rows, cols, 128, xd, y1)
        else:
            n = S.N_KEEP[kind]
            p = B.pack_2bitcsr(w, B.prune_n4(w, n), n, 128, 0).to("cuda")
            items.append(("sparse", p, xd, y))
            B.sparse_gemv(p, xd, y1)
        singles.append((ybuf, y1, rows))
    call = B.prepared_gemv_stack(items)
    has14 = any(it[0] == "sparse" and it[1].n_keep == 1 for it in items)
    others = any(not (it[0] == "sparse" and it[1].n_keep == 1) for it in items)
    assert call.plan.nparts == (2 if has14 and others else 1) and call.plan.count == len(items)
    for rep in range(2):
        call()
        torch.cuda.synchronize()
        for k, (ybuf, y1, rows) in enumerate(singles):
            host = ybuf.cpu().numpy().view(np.uint16)
            assert np.all(host[:64] == G.CANARY) and np.all(host[64 + rows:] == G.CANARY), ("write outside y", k)
            assert np.array_equal(host[64:64 + rows], y1.cpu().numpy().view(np.uint16)), (seed, k)
            ybuf[64:64 + rows].fill_(0)


def test_row_block_list_on_ragged_shapes():
    # the resident-workgroup form on a table with row counts that are
    # no multiple of a row block, one, two and six tiles per row, a matrix shorter than one row
    # block and an empty one: sampled rows against the oracle (which re-encodes them), all
    # rows bit for bit against the separate calls, and nothing written outside y
    torch = G.torch_mod()
    # (storage form, rows, columns, quantisation group)
    specs = [("s24", 11008, 4096, 128), ("d", 4099, 11008, 128), ("s24", 4097, 8192, 128), ("d", 1001, 4096, 128), ("s24", 0, 4096, 128),
             ("s24", 37, 4096, 128), ("d", 5, 4096, 128), ("s24", 145, 11008, 128),
             ("s24", 500, 4096, 64), ("s24", 300, 8192, 256), ("d", 200, 4096, 256), ("d", 100, 11008, 256), ("s24", 90, 12288, 4096)]
    items, checks = [], []
    for k, (kind, rows, cols, grp) in enumerate(specs):
        print(f"  packing {kind} {rows}x{cols} g={grp}", flush=True)
        w = synth.weights(rows, cols, 4700 + k)
        x = synth.activations(cols, 4700 + k)
        xd = G.to_dev(x.view(np.uint16)).view(torch.float16)
        ybuf = torch.full((rows + 128,), G.CANARY, dtype=torch.int16, device="cuda")
        y = ybuf[64:64 + rows].view(torch.float16)
        y1 = torch.empty(rows, dtype=torch.float16, device="cuda")
        pick = G.sample_rows(rows, 40, k) if rows else np.zeros(0, dtype=np.int64)
        if kind == "d":
            q, qp = B.quant_int4(w, grp)
            qd, qpd = G.to_dev(q), G.to_dev(qp)
            items.append(("dense", qd, qpd, rows, cols, grp, xd, y))
            oq, oqp = O.quant_int4_dense(w[pick], grp)
            assert np.array_equal(oq, q[pick]) and np.array_equal(oqp, qp[pick])
            ref = O.int4_gemv(oq, oqp, grp, x)
            B.int4_gemv(qd, qpd, rows, cols, grp, xd, y1)
        else:
            ph = B.pack_2bitcsr(w, B.prune_n4(w, 2), 2, grp, 0)
            if rows:
                o = O.pack_2bitcsr(w[pick], O.prune_n4_magnitude(w[pick], 2), 2, grp, 0)
                sub = G.row_subset(ph, pick)
                for name in ("values", "idx", "qparams"):
                    assert np.array_equal(o[name], sub[name]), name
                ref = O.gemv(o, x)
            else:
                ref = (np.zeros(0), np.zeros(0))
            p = ph.to("cuda")
            items.append(("sparse", p, xd, y))
            B.sparse_gemv(p, xd, y1)
        checks.append((ybuf, y1, pick, ref))
    call = B.prepared_gemv_stack(items, form=B.STACK_RESIDENT)
    assert (call.plan.mode, call.plan.block_threads) == (1, 768) and call.plan.nitems > 0
    for rep in range(3):
        call()
        torch.cuda.synchronize()
        for k, (kind, rows, cols, grp) in enumerate(specs):
            ybuf, y1, pick, ref = checks[k]
            host = ybuf.cpu().numpy().view(np.uint16)
            assert np.all(host[:64] == G.CANARY) and np.all(host[64 + rows:] == G.CANARY), ("write outside y", k)
            y = host[64:64 + rows].view(np.float16)
            if rows:
                G.assert_close(y[pick], ref[0], ref[1], f"row blocks item {k} {kind} {rows}x{cols}")
            assert np.array_equal(y.view(np.uint16), y1.cpu().numpy().view(np.uint16)), (k, kind, rows, cols)
            ybuf[64:64 + rows].fill_(0)
    # a broken row pointer gives NaN in that row and leaves the other rows alone
    p0 = items[0][1]
    rp = p0.row_ptr.view(torch.int32)
    saved = rp[[7, 4000]].clone()
    rp[7] += 8
    rp[4000] = 0
    call()
    torch.cuda.synchronize()
    y = checks[0][0].cpu().numpy().view(np.uint16)[64:64 + 11008].view(np.float16)
    good = checks[0][1].cpu().numpy()
    assert np.isnan(y[7]) and np.isnan(y[4000])
    keep = np.ones(11008, dtype=bool)
    keep[[7, 4000]] = False
    assert np.array_equal(y[keep].view(np.uint16), good[keep].view(np.uint16))
    rp[[7, 4000]] = saved


def test_row_block_list_on_1to4_shapes():
    # the same form for 1:4 matrices: rows of 16, 32, 64 and 86 chunks (four, two and one row per tile of 64
    # chunks, two tiles per row), row counts that are no multiple of a tile, a matrix shorter than one row
    # block and an empty one: sampled rows against the oracle, all rows bit for bit against the separate
    # calls, nothing written outside y, and NaN for a broken row pointer
    torch = G.torch_mod()
    # (rows, columns, quantisation group)
    specs = [(11008, 4096, 128), (4099, 11008, 128), (4097, 8192, 128), (1001, 2048, 128), (0, 4096, 128), (37, 4096, 128),
             (5, 2048, 128), (145, 11008, 128), (3, 4096, 128), (301, 16384, 256), (64, 12288, 512), (77, 4096, 4096), (130, 8192, 256)]
    items, checks = [], []
    for k, (rows, cols, grp) in enumerate(specs):
        print(f"  packing 1:4 {rows}x{cols} g={grp}", flush=True)
        w = synth.weights(rows, cols, 4900 + k)
        x = synth.activations(cols, 4900 + k)
        xd = G.to_dev(x.view(np.uint16)).view(torch.float16)
        ybuf = torch.full((rows + 128,), G.CANARY, dtype=torch.int16, device="cuda")
        y = ybuf[64:64 + rows].view(torch.float16)
        y1 = torch.empty(rows, dtype=torch.float16, device="cuda")
        pick = G.sample_rows(rows, 40, k) if rows else np.zeros(0, dtype=np.int64)
        ph = B.pack_2bitcsr(w, B.prune_n4(w, 1), 1, grp, 0)
        if rows:
            o = O.pack_2bitcsr(w[pick], O.prune_n4_magnitude(w[pick], 1), 1, grp, 0)
            sub = G.row_subset(ph, pick)
            for name in ("values", "idx", "qparams"):
                assert np.array_equal(o[name], sub[name]), name
            ref = O.gemv(o, x)
        else:
            ref = (np.zeros(0), np.zeros(0))
        pd = ph.to("cuda")
        items.append(("sparse", pd, xd, y))
        B.sparse_gemv(pd, xd, y1)
        checks.append((ybuf, y1, pick, ref))
    call = B.prepared_gemv_stack(items, form=B.STACK_RESIDENT)
    assert (call.plan.nparts, call.plan.mode, call.plan.block_threads, call.plan.forms) == (1, 1, 512, 2) and call.plan.nitems > 0
    for rep in range(3):
        call()
        torch.cuda.synchronize()
        for k, (rows, cols, grp) in enumerate(specs):
            ybuf, y1, pick, ref = checks[k]
            host = ybuf.cpu().numpy().view(np.uint16)
            assert np.all(host[:64] == G.CANARY) and np.all(host[64 + rows:] == G.CANARY), ("write outside y", k)
            y = host[64:64 + rows].view(np.float16)
            if rows:
                G.assert_close(y[pick], ref[0], ref[1], f"row blocks item {k} 1:4 {rows}x{cols} g={grp}")
            assert np.array_equal(y.view(np.uint16), y1.cpu().numpy().view(np.uint16)), (k, rows, cols)
            ybuf[64:64 + rows].fill_(0)
    p0 = items[0][1]
    rp = p0.row_ptr.view(torch.int32)
    saved = rp[[7, 4000]].clone()
    rp[7] += 8
    rp[4000] = 0
    call()
    torch.cuda.synchronize()
    y = checks[0][0].cpu().numpy().view(np.uint16)[64:64 + 11008].view(np.float16)
    good = checks[0][1].cpu().numpy()
    assert np.isnan(y[7]) and np.isnan(y[4000])
    keep = np.ones(11008, dtype=bool)
    keep[[7, 4000]] = False
    assert np.array_equal(y[keep].view(np.uint16), good[keep].view(np.uint16))
    rp[[7, 4000]] = saved


def test_trigger_model_on_a_measured_sweep():
    # Sec. 3.4: time one all-2:4 layer (q/k/v/o, gate/up, down) for M = 1..64 on the GPU, fit
    # the verification cost with the library and compare fit and trigger point with the
    # oracle on the very same measured points
    torch = G.torch_mod()
    shapes = ((4096, 4096, 4), (11008, 4096, 2), (4096, 11008, 1))
    sweep = (1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64)
    layer_us = {m: 0.0 for m in sweep}
    for rows, cols, reps in shapes:
        _, _, p = G.packed_full(rows, cols, 2, 128, 0, synth.seed_for(5, 7))
        pd = p.to("cuda:0")
        for M in sweep:
            X = G.to_dev(synth.activation_rows(M, cols, 5).view(np.uint16)).view(torch.float16)
            Y = torch.empty((M, rows), dtype=torch.float16, device="cuda:0")
            call = B.prepared_sparse_gemm_smallm(pd, X, Y)
            for _ in range(20):
                call()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(100):
                call()
            e1.record()
            torch.cuda.synchronize()
            layer_us[M] += reps * e0.elapsed_time(e1) * 10.0          # ms per 100 calls -> us per call
    print("  layer time by M (us):", {m: round(v, 1) for m, v in layer_us.items()}, flush=True)
    ms, ts = list(sweep[1:]), [layer_us[m] for m in sweep[1:]]
    a, b = B.fit_verify_cost(ms, ts)
    oa, ob = O.fit_verify_cost(ms, ts)
    assert a == pytest.approx(oa, rel=1e-9, abs=1e-9) and b == pytest.approx(ob, rel=1e-9, abs=1e-12)
    assert b > 0 and all(v > 0 for v in ts)             # more candidates cost more, as the paper observes
    assert layer_us[64] > layer_us[1]
    for cand, rem in (([64, 24, 9, 4, 2, 1], [6, 5, 4, 3, 2, 1]), ([48, 48, 12, 3], [4, 3, 2, 1]), ([64], [1])):
        got = B.trigger_depth(layer_us[1], a, b, cand, rem)
        want = O.trigger_depth(layer_us[1], oa, ob, cand, rem)
        assert got[0] == want[0] and got[1] == pytest.approx(want[1], rel=1e-9, abs=1e-9), (cand, rem)
        gains = [r * layer_us[1] - (a + b * c) for c, r in zip(cand, rem)]
        assert got[0] == (int(np.argmax(gains)) if max(gains) > 0 else -1)


def test_smallm_kernels_replay_in_a_hip_graph():
    # the several-token path, the K-split kernel with one and two token groups per pass
    # and its 1:4 form, captured together; every replay must reproduce the eager bits
    torch = G.torch_mod()
    cases = []
    for (rows, cols, n, M) in ((300, 4096, 2, 2), (300, 4096, 2, 12), (300, 4096, 2, 40), (200, 11008, 1, 20),
                               (90, 2048, 2, 64)):
        w = synth.weights(rows, cols, 9000 + rows + M)
        p = B.pack_2bitcsr(w, B.prune_n4(w, n), n, 128, B.VAL_INT4).to("cuda:0")
        X = G.to_dev(synth.activation_rows(M, cols, 9000 + M).view(np.uint16)).view(torch.float16)
        Y = torch.zeros((M, rows), dtype=torch.float16, device="cuda:0")
        cases.append((B.prepared_sparse_gemm_smallm(p, X, Y), Y))
    # and tables of several products in one launch (one and four token groups)
    for M in (9, 50):
        items = []
        for (rows, cols) in ((300, 4096), (70, 11008), (130, 2048)):
            w = synth.weights(rows, cols, 9100 + rows + M)
            p = B.pack_2bitcsr(w, B.prune_n4(w, 2), 2, 128, B.VAL_INT4).to("cuda:0")
            X = G.to_dev(synth.activation_rows(M, cols, 9100 + M).view(np.uint16)).view(torch.float16)
            items.append((p, X, torch.zeros((M, rows), dtype=torch.float16, device="cuda:0")))
        table = B.prepared_gemm_stack(items)
        cases += [(table if k == 0 else (lambda stream_ptr=None: None), it[2]) for k, it in enumerate(items)]
    for call, _ in cases:
        call()
    torch.cuda.synchronize()
    eager = [Y.cpu().numpy().copy() for _, Y in cases]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for call, _ in cases:
            call(side.cuda_stream)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            sp = torch.cuda.current_stream().cuda_stream
            for call, _ in cases:
                call(sp)
    for rep in range(3):
        for _, Y in cases:
            Y.fill_(5.0)                            # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, (_, Y) in enumerate(cases):
            assert np.array_equal(Y.cpu().numpy().view(np.uint16), eager[k].view(np.uint16)), (rep, k)


@pytest.mark.parametrize("M,n", [(2, 2), (5, 2), (16, 2), (17, 2), (32, 2), (33, 2), (40, 2), (64, 2),
                                 (3, 1), (16, 1), (20, 1), (32, 1)])
def test_gemm_stack_equals_the_oracle_and_the_separate_products(M, n):
    # a verification step through several layers in one launch: shapes with fewer row tiles than
    # workgroups, a ragged last tile, several rounds of row tiles, a row length that ends inside
    # a K-step, an empty matrix; Y buffers with and without 8-byte alignment, canaries around
    torch = G.torch_mod()
    print(f"case gemm stack M={M} n={n}", flush=True)
    if n == 2:
        shapes = [(300, 4096, 128), (70, 11008, 128), (16 * 96 * 8 + 40, 4096, 4096), (133, 8192, 64), (0, 4096, 128),
                  (21, 4160, 64), (50, 832, 64), (1700, 2048, 128)]
        shapes += [(40, 64, 64), (33, 320, 64), (18, 1280, 256)]     # rows shorter than a round of K-steps, and than a K-step
    else:                                             # 1:4: chunks of 128 columns, K-steps of 512
        shapes = [(300, 4096, 128), (70, 11008, 128), (16 * 96 * 4 + 40, 4096, 4096), (133, 8192, 256), (0, 4096, 128),
                  (21, 4224, 128), (50, 1664, 128), (1700, 2048, 128), (40, 128, 128), (33, 640, 128), (18, 1536, 512)]
    ps, os_, Xs = [], [], []
    for k, (rows, cols, g) in enumerate(shapes):
        w = synth.weights(rows, cols, 8800 + 7 * k + M)
        mask = O.prune_n4_magnitude(w, n)
        ps.append(B.pack_2bitcsr(w, mask, n, g, B.VAL_INT4))
        os_.append(O.pack_2bitcsr(w, mask, n, g, B.VAL_INT4) if 0 < rows <= 400 else None)
        Xs.append(synth.activation_rows(M, cols, 8800 + k))
    pds = [p.to("cuda:0") for p in ps]
    Xd = [G.to_dev(X.view(np.uint16)).view(torch.float16) for X in Xs]
    guards = [64, 3, 64, 1, 64, 64, 2, 64, 64, 5, 64]
    ybufs = [torch.full((2 * gd + M * p.rows,), G.CANARY, dtype=torch.int16, device="cuda:0") for gd, p in zip(guards, ps)]
    Yd = [yb[gd:gd + M * p.rows].view(torch.float16).view(M, p.rows) for yb, gd, p in zip(ybufs, guards, ps)]
    call = B.prepared_gemm_stack(list(zip(pds, Xd, Yd)))
    assert (call.plan.count, call.plan.M) == (len(shapes), M)
    # a row tile per wave: the workgroups of the launch cover the rows of every matrix
    assert call.plan.grid_x == sum(-(-p.rows // (16 * (call.plan.block_threads // 64))) for p in ps)
    first = {}
    for rep in range(2):
        call()
        torch.cuda.synchronize()
        for k, p in enumerate(ps):
            host = ybufs[k].cpu().numpy().view(np.uint16)
            gd = guards[k]
            assert np.all(host[:gd] == G.CANARY) and np.all(host[gd + M * p.rows:] == G.CANARY), ("write outside Y", k)
            if p.rows == 0:
                continue
            Y = host[gd:gd + M * p.rows].view(np.float16).reshape(M, p.rows)
            rows = G.sample_rows(p.rows, 400, 8800 + k) if p.rows > 400 else np.arange(p.rows)
            Y_ref, A_ref = O.gemm_smallm(G.row_subset(ps[k], rows) if p.rows > 400 else os_[k], Xs[k])
            G.assert_close(Y[:, rows], Y_ref, A_ref, f"gemm stack member {k}")
            if rep == 0:
                first[k] = Y.copy()
            else:
                assert np.array_equal(Y.view(np.uint16), first[k].view(np.uint16)), ("second run differs", k)
            ybufs[k][gd:gd + M * p.rows].fill_(0)
    # the same bits whatever else the table holds: two of the members, in the other order, as a table of their own
    Y2 = {k: torch.zeros((M, ps[k].rows), dtype=torch.float16, device="cuda:0") for k in (3, 0)}
    B.prepared_gemm_stack([(pds[k], Xd[k], Y2[k]) for k in (3, 0)])()
    torch.cuda.synchronize()
    for k in (3, 0):
        assert np.array_equal(Y2[k].cpu().numpy().view(np.uint16), first[k].view(np.uint16)), ("other table differs", k)


@pytest.mark.parametrize("seed", range(8))
def test_gemm_stack_seeded_sweep_of_shapes(seed):
    # seeded tables: row counts around the tile and workgroup sizes, row lengths that end anywhere inside a K-step or
    # a round, every group size the form takes, both storage forms, any number of tokens; every output against the oracle
    torch = G.torch_mod()
    rng = np.random.default_rng(9200 + seed)
    n = 2 if seed % 3 else 1
    chunk = 64 if n == 2 else 128
    M = int(rng.integers(2, 65 if n == 2 else 33))
    print(f"case gemm stack sweep seed={seed} n={n} M={M}", flush=True)
    ps, os_, Xs = [], [], []
    for k in range(6):
        rows = int(rng.choice([1, 15, 16, 17, 127, 128, 129, 200, int(rng.integers(1, 300))]))
        cols = chunk * int(rng.integers(1, 8192 // chunk + 1))
        groups = [g for g in (64, 128, 256, 512, 1024, 2048, 4096, 8192) if g >= (64 if n == 2 else 128) and cols % g == 0]
        g = int(rng.choice(groups))
        w = synth.weights(rows, cols, 9200 + 10 * seed + k)
        mask = O.prune_n4_magnitude(w, n)
        ps.append(B.pack_2bitcsr(w, mask, n, g, B.VAL_INT4))
        os_.append(O.pack_2bitcsr(w, mask, n, g, B.VAL_INT4))
        Xs.append(synth.activation_rows(M, cols, 9200 + 10 * seed + k))
        print(f"  member {k}: {rows} x {cols} g={g}", flush=True)
    pds = [p.to("cuda:0") for p in ps]
    Xd = [G.to_dev(X.view(np.uint16)).view(torch.float16) for X in Xs]
    ybufs = [torch.full((128 + M * p.rows,), G.CANARY, dtype=torch.int16, device="cuda:0") for p in ps]
    Yd = [yb[64:64 + M * p.rows].view(torch.float16).view(M, p.rows) for yb, p in zip(ybufs, ps)]
    B.prepared_gemm_stack(list(zip(pds, Xd, Yd)))()
    torch.cuda.synchronize()
    for k, p in enumerate(ps):
        host = ybufs[k].cpu().numpy().view(np.uint16)
        assert np.all(host[:64] == G.CANARY) and np.all(host[64 + M * p.rows:] == G.CANARY), ("write outside Y", k)
        Y = host[64:64 + M * p.rows].view(np.float16).reshape(M, p.rows)
        Y_ref, A_ref = O.gemm_smallm(os_[k], Xs[k])
        G.assert_close(Y, Y_ref, A_ref, f"sweep seed {seed} member {k}")


@pytest.mark.parametrize("M", [3, 16, 24, 50])
def test_gemm_stack_broken_row_ptr_yields_nan_for_every_token(M):
    # rows 7 and 40 of the second matrix point somewhere else: NaN for every token of those rows, the other
    # rows and the other matrices as before
    torch = G.torch_mod()
    print(f"case gemm stack broken row_ptr M={M}", flush=True)
    ps, Xd, goods = [], [], []
    for k, (rows, cols) in enumerate(((150, 4096), (200, 2048), (40, 11008))):
        w = synth.weights(rows, cols, 8900 + k)
        ps.append(B.pack_2bitcsr(w, B.prune_n4(w, 2), 2, 128, B.VAL_INT4))
        Xd.append(G.to_dev(synth.activation_rows(M, cols, 8900 + k).view(np.uint16)).view(torch.float16))

    def run():
        pds = [p.to("cuda:0") for p in ps]
        Ys = [torch.zeros((M, p.rows), dtype=torch.float16, device="cuda:0") for p in ps]
        B.prepared_gemm_stack(list(zip(pds, Xd, Ys)))()
        torch.cuda.synchronize()
        return [Y.cpu().numpy() for Y in Ys]
    goods = run()
    ps[1].row_ptr[7] += 8
    ps[1].row_ptr[40] = 0xFFFFFFF8
    Ys = run()
    assert np.all(np.isnan(Ys[1][:, 7])) and np.all(np.isnan(Ys[1][:, 40]))
    keep = np.ones(200, dtype=bool)
    keep[[7, 40]] = False
    assert np.array_equal(Ys[1][:, keep].view(np.uint16), goods[1][:, keep].view(np.uint16))
    for k in (0, 2):
        assert np.array_equal(Ys[k].view(np.uint16), goods[k].view(np.uint16)), k


def test_gemm_stack_rejects_what_it_does_not_run():
    torch = G.torch_mod()
    w = synth.weights(64, 4096, 1)
    X = torch.zeros((8, 4096), dtype=torch.float16, device="cuda:0")
    Y = torch.zeros((8, 64), dtype=torch.float16, device="cuda:0")
    for n, g, kind in ((1, 64, B.VAL_INT4), (2, 32, B.VAL_INT4), (2, 0, B.VAL_FP16)):
        p = B.pack_2bitcsr(w, B.prune_n4(w, n), n, g, kind).to("cuda:0")
        with pytest.raises(B.EgtError) as e:
            B.prepared_gemm_stack([(p, X, Y)])
        assert e.value.status == 6
    # the two storage forms in one table (the binding makes a table per form; here through the C ABI); 1:4 beyond 32 tokens
    p2 = B.pack_2bitcsr(w, B.prune_n4(w, 2), 2, 128, B.VAL_INT4).to("cuda:0")
    p1 = B.pack_2bitcsr(w, B.prune_n4(w, 1), 1, 128, B.VAL_INT4).to("cuda:0")
    import ctypes
    arr, views = (B.GemmItem * 2)(), [p2.view(), p1.view()]
    for k in range(2):
        arr[k].sparse, arr[k].X, arr[k].Y = ctypes.pointer(views[k]), X.data_ptr(), Y.data_ptr()
    assert B.lib().egt_gemm_stack_plan(arr, 2, 8, None, 0, ctypes.byref(B.GemmPlan())) == 6
    # ... and the binding's two tables give each member the bits of a table of its own
    Ya, Yb, Yc, Yd = (torch.zeros_like(Y) for _ in range(4))
    Xr = G.to_dev(synth.activation_rows(8, 4096, 77).view(np.uint16)).view(torch.float16)
    mixed = B.prepared_gemm_stack([(p2, Xr, Ya), (p1, Xr, Yb)])
    assert [pl.n_keep for pl in mixed.plans] == [2, 1]
    mixed()
    B.prepared_gemm_stack([(p2, Xr, Yc)])()
    B.prepared_gemm_stack([(p1, Xr, Yd)])()
    torch.cuda.synchronize()
    assert torch.equal(Ya.view(torch.int16), Yc.view(torch.int16)) and torch.equal(Yb.view(torch.int16), Yd.view(torch.int16))
    assert float(Ya.abs().max()) > 0 and float(Yb.abs().max()) > 0
    X40 = torch.zeros((40, 4096), dtype=torch.float16, device="cuda:0")
    with pytest.raises(B.EgtError) as e:
        B.prepared_gemm_stack([(p1, X40, torch.zeros((40, 64), dtype=torch.float16, device="cuda:0"))])
    assert e.value.status == 6


def test_two_streams_at_once_give_the_serial_results():
    # the library keeps no state between calls: products enqueued on two streams (default
    # priority) at the same time equal the ones computed one after the other, bit for bit
    torch = G.torch_mod()
    w = synth.weights(3000, 4096, 8800)
    p = B.pack_2bitcsr(w, B.prune_n4(w, 2), 2, 128, B.VAL_INT4).to("cuda")
    pf = B.pack_2bitcsr(w, B.prune_n4(w, 2), 2, 0, B.VAL_FP16).to("cuda")
    q, qp = B.quant_int4(w, 128)
    qd, qpd = G.to_dev(q), G.to_dev(qp)
    x = G.to_dev(synth.activations(4096, 8801).view(np.uint16)).view(torch.float16)
    X = G.to_dev(synth.activation_rows(16, 4096, 8802).view(np.uint16)).view(torch.float16)

    def work(tag, stream, out):
        for rep in range(8):
            B.sparse_gemv(p, x, out["a"], stream=stream)
            B.sparse_gemm_smallm(p, X, out["b"], stream=stream)
            B.sparse_gemv(pf, x, out["c"], stream=stream)
            B.int4_gemv(qd, qpd, 3000, 4096, 128, x, out["d"], stream=stream)
            B.sparse_gemm_smallm(pf, X[:3], out["e"], stream=stream)

    def outputs():
        return {"a": torch.empty(3000, dtype=torch.float16, device="cuda"),
                "b": torch.empty((16, 3000), dtype=torch.float16, device="cuda"),
                "c": torch.empty(3000, dtype=torch.float16, device="cuda"),
                "d": torch.empty(3000, dtype=torch.float16, device="cuda"),
                "e": torch.empty((3, 3000), dtype=torch.float16, device="cuda")}

    serial = outputs()
    work("serial", None, serial)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    o1, o2 = outputs(), outputs()
    print("case two streams", flush=True)
    work("s1", s1, o1)
    work("s2", s2, o2)
    s1.synchronize()
    s2.synchronize()
    for k in serial:
        assert torch.equal(serial[k], o1[k]) and torch.equal(serial[k], o2[k]), k
