"""Config 4: the 32-layer 7B-shaped stack, 224 GEMV launches (16 layers 2:4-sparse INT4 in
2bit-CSR, 16 dense INT4), plain and replayed from a HIP graph."""
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


def test_stack_parity_and_graph_replay():
    torch = G.torch_mod()
    print("building the stack (2 layers with their own weights, 30 reuse their bytes)", flush=True)
    st = S.LayerStack.build("cuda:0", distinct_layers=1, progress=lambda l: print(f"  layer {l} uploaded", flush=True) if l % 8 == 7 else None)
    assert len(st.matrices) == 224 and st.nbytes == 3043344832
    st.run()
    torch.cuda.synchronize()
    eager = [m.y.cpu().numpy().copy() for m in st.matrices]
    sparse_ids = set(int(v) for v in synth.sparse_layers())
    first = {True: min(sparse_ids), False: min(set(range(32)) - sparse_ids)}
    assert [k != "d" for k in synth.layer_kinds("config4")] == [l in sparse_ids for l in range(32)]
    nm = len(synth.LAYER_MATRICES)
    # the two layers with their own weights: the oracle packs sampled rows itself and multiplies
    for sparse, layer in first.items():
        for mi, (name, rows, cols) in enumerate(synth.LAYER_MATRICES):
            print(f"  oracle check layer {layer} ({'sparse' if sparse else 'dense'}) {name}", flush=True)
            w, x, packed = S.pack_layer_matrix(layer, mi, sparse)
            pick = G.sample_rows(rows, 48, layer * nm + mi)
            y = eager[layer * nm + mi]
            if sparse:
                o = O.pack_2bitcsr(w[pick], O.prune_n4_magnitude(w[pick], 2), 2, 128, O.VAL_INT4)
                sub = G.row_subset(packed, pick)
                for k in ("values", "idx", "qparams"):
                    assert np.array_equal(o[k], sub[k]), k
                y_ref, a_ref = O.gemv(o, x)
            else:
                oq, oqp = O.quant_int4_dense(w[pick], 128)
                assert np.array_equal(oq, packed[0][pick]) and np.array_equal(oqp, packed[1][pick])
                y_ref, a_ref = O.int4_gemv(oq, oqp, 128, x)
            G.assert_close(y[pick], y_ref, a_ref, f"layer {layer} {name}")
    # layers that reuse those bytes must reproduce the same outputs bit for bit
    for m_i, m in enumerate(st.matrices):
        src = first[m.sparse] * nm + m_i % nm
        assert np.array_equal(eager[m_i].view(np.uint16), eager[src].view(np.uint16)), (m.layer, m.name)
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
