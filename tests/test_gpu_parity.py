"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle."""
import numpy as np
import pytest

from oracle import egt_oracle as O
from paper_2605_11582_amd import binding as B, synth
import gpu_common as G

pytestmark = pytest.mark.gpu


def _small_case(rows, cols, n, g, kind, seed, drop=0.0):
    rng = np.random.default_rng(seed)
    w = synth.weights(rows, cols, seed)
    mask = O.prune_n4_magnitude(w, n)
    if drop:
        mask = (mask & (rng.random(mask.shape) >= drop)).astype(np.uint8)
    o = O.pack_2bitcsr(w, mask, n, g, kind)
    p = B.pack_2bitcsr(w, mask, n, g, kind)
    for k in ("row_ptr", "values", "idx"):
        assert np.array_equal(getattr(p, k), o[k])
    return p, o


# ---------------------------------------------------------------- element by element, small
@pytest.mark.parametrize("rows,cols,n,g,kind", [
    (37, 96, 2, 32, 0), (5, 32, 1, 16, 0), (64, 160, 3, 32, 0), (33, 128, 4, 64, 0),
    (19, 224, 2, 0, 1), (7, 64, 1, 0, 1), (130, 1056, 2, 96, 0), (3, 4128, 2, 4128, 0),
    (257, 1024, 2, 128, 0), (100, 1024, 1, 128, 0), (70, 2048, 2, 64, 0), (70, 2048, 2, 256, 0),
    (45, 4096, 2, 128, 0), (45, 4096, 2, 0, 1), (21, 11008, 2, 128, 0), (21, 11008, 1, 128, 0),
    (21, 11008, 2, 0, 1), (50, 320, 2, 64, 0),
    (45, 4096, 1, 128, 0), (33, 8192, 1, 256, 0), (19, 2048, 1, 128, 0), (30, 4096, 1, 0, 1),
    (21, 11008, 1, 0, 1), (130, 4096, 1, 256, 0), (9, 12288, 1, 128, 0), (41, 4160, 2, 64, 0),
    # narrow quantisation groups on the matrix-core paths
    (45, 4096, 2, 32, 0), (70, 1024, 2, 32, 0), (21, 11008, 2, 32, 0), (33, 2048, 2, 32, 0),
    (45, 4096, 1, 32, 0), (45, 4096, 1, 64, 0), (21, 11008, 1, 64, 0), (19, 2048, 1, 32, 0), (9, 12288, 1, 32, 0),
    # the widest rows the tuned kernels take, and wider ones (the generic kernels)
    (4, 32768, 2, 128, 0), (4, 32768, 1, 128, 0), (3, 32768, 2, 0, 1), (3, 32768, 1, 0, 1),
    (3, 40960, 2, 128, 0), (3, 36864, 1, 128, 0), (2, 65536, 2, 0, 1),
    # 1:4 with FP16 values: one, two and four load instructions per row, two phases, a partly filled one
    (70, 2048, 1, 0, 1), (133, 4096, 1, 0, 1), (40, 8192, 1, 0, 1), (37, 11008, 1, 0, 1), (18, 16384, 1, 0, 1), (9, 20608, 1, 0, 1),
    # the slot-by-slot kernel past the first 128 columns of its LDS layout: every kept count, with a word of
    # eight slots inside one quantisation group (16, 8, 32 columns) and across three (12 columns, 3 of 4 kept)
    (9, 4128, 2, 16, 0), (6, 4128, 3, 12, 0), (5, 4160, 4, 8, 0), (5, 4128, 1, 32, 0), (5, 4128, 1, 16, 0),
])
def test_sparse_gemv_small(rows, cols, n, g, kind):
    print(f"case sparse_gemv {rows}x{cols} n={n} g={g} kind={kind}", flush=True)
    p, o = _small_case(rows, cols, n, g, kind, seed=1000 + rows + cols + n, drop=0.1)
    x = synth.activations(cols, 77 + rows)
    y_ref, a_ref = O.gemv(o, x)
    y = G.run_sparse_gemv(p, x)
    G.assert_close(y, y_ref, a_ref, "sparse_gemv")


@pytest.mark.parametrize("rows,cols,n,g,M", [(70, 4096, 2, 64, 1), (70, 4096, 1, 32, 1), (300, 1024, 2, 128, 6)])
def test_row_group_sizes_run_on_the_ordinary_kernels(rows, cols, n, g, M):
    # rows quantised with group sizes of their own are stored at the finest granularity
    rng = np.random.default_rng(rows + cols + g)
    w = synth.weights(rows, cols, 6100 + g)
    mask = O.prune_n4_magnitude(w, n)
    rg = rng.choice([g, 2 * g, 4 * g, cols], size=rows)
    p = B.pack_2bitcsr(w, mask, n, g, 0, row_group=rg)
    o = O.pack_2bitcsr(w, mask, n, g, 0, row_group=rg)
    for k in ("values", "idx", "qparams"):
        assert np.array_equal(getattr(p, k), o[k]), k
    X = synth.activation_rows(M, cols, 6100 + g)
    Y_ref, A_ref = O.gemm_smallm(o, X)
    Y = G.run_sparse_gemm(p, X) if M > 1 else G.run_sparse_gemv(p, np.ascontiguousarray(X[0]))[None, :]
    G.assert_close(Y, Y_ref, A_ref, "row groups")


def test_config1_full_parity_and_determinism():
    seed = synth.seed_for(1)
    w = synth.weights(1024, 1024, seed)
    x = synth.activations(1024, seed)
    mask = B.prune_n4(w, 2)
    p = B.pack_2bitcsr(w, mask, 2, 128, 0)
    o = O.pack_2bitcsr(w, O.prune_n4_magnitude(w, 2), 2, 128, 0)
    for k in ("row_ptr", "values", "idx", "qparams"):
        assert np.array_equal(getattr(p, k), o[k])
    y_ref, a_ref = O.gemv(o, x)
    y = G.run_sparse_gemv(p, x)
    G.assert_close(y, y_ref, a_ref, "config 1")
    # no atomics anywhere: two runs give the same bits
    assert np.array_equal(y.view(np.uint16), G.run_sparse_gemv(p, x).view(np.uint16))


@pytest.mark.parametrize("kind,g", [(0, 128), (1, 0)])
def test_one_hot_x_returns_decoded_column_bit_exact(kind, g):
    p, o = _small_case(96, 4096, 2, g, kind, seed=4242)
    W = O.dense_from_packed(o)
    for j in (0, 5, 2049, 4095):
        e = np.zeros(4096, dtype=np.float16)
        e[j] = 1
        y = G.run_sparse_gemv(p, e)
        assert np.array_equal(y.view(np.uint16), W[:, j].astype(np.float16).view(np.uint16)), f"column {j}"


def test_zero_mask_and_empty_matrix():
    w = synth.weights(64, 4096, 9)
    x = synth.activations(4096, 9)
    for kind, g in [(0, 128), (1, 0)]:
        p = B.pack_2bitcsr(w, np.zeros_like(w, dtype=np.uint8), 2, g, kind)
        y = G.run_sparse_gemv(p, x)
        assert np.all(y.view(np.uint16) & 0x7FFF == 0)
    p0 = B.pack_2bitcsr(np.zeros((0, 4096), dtype=np.float16), np.zeros((0, 4096), dtype=np.uint8), 2, 128, 0)
    assert G.run_sparse_gemv(p0, x).size == 0


def test_broken_row_ptr_yields_nan_not_a_fault():
    p, o = _small_case(64, 4096, 2, 128, 0, seed=31)
    x = synth.activations(4096, 31)
    good = G.run_sparse_gemv(p, x)
    p.row_ptr[7] += 8
    p.row_ptr[40] = 0xFFFFFFF8
    torch = G.torch_mod()
    pd = p.to("cuda")
    y = torch.zeros(64, dtype=torch.float16, device="cuda")
    B.sparse_gemv(pd, G.to_dev(x.view(np.uint16)).view(torch.float16), y)
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    assert np.isnan(y[7]) and np.isnan(y[40])
    keep = np.ones(64, dtype=bool)
    keep[[7, 40]] = False
    assert np.array_equal(y[keep].view(np.uint16), good[keep].view(np.uint16))


@pytest.mark.parametrize("rows,cols,n,g,kind", [(1, 64, 2, 32, 0), (3, 128, 2, 64, 0), (2, 192, 2, 0, 1), (17, 64, 2, 64, 0),
                                                (1, 128, 1, 32, 0), (5, 384, 1, 128, 0), (16, 256, 1, 0, 1),
                                                (31, 4096, 2, 128, 0), (1, 4096, 2, 128, 0)])
@pytest.mark.parametrize("M", [2, 17, 64])
def test_smallm_tiny_matrices(rows, cols, n, g, kind, M):
    # fewer rows than a row tile, one or two chunks per row, every token count class
    print(f"case smallm tiny {rows}x{cols} n={n} g={g} kind={kind} M={M}", flush=True)
    p, o = _small_case(rows, cols, n, g, kind, seed=5100 + M + rows + cols)
    X = synth.activation_rows(M, cols, 5100 + M)
    Y_ref, A_ref = O.gemm_smallm(o, X)
    G.assert_close(G.run_sparse_gemm(p, X), Y_ref, A_ref, f"smallm tiny {rows}x{cols} M={M}")


@pytest.mark.parametrize("cols,n,M", [(4096, 2, 2), (4096, 2, 4), (4096, 2, 9), (4096, 2, 40), (1024, 2, 5),
                                      (4096, 1, 3), (11008, 1, 20)])
def test_broken_row_ptr_yields_nan_for_every_token(cols, n, M):
    # the several-token path, the K-split kernel (one and two token groups per pass) and 1:4
    p, o = _small_case(64, cols, n, 128, 0, seed=4300 + M)
    X = synth.activation_rows(M, cols, 4300 + M)
    good = G.run_sparse_gemm(p, X)
    p.row_ptr[7] += 8
    p.row_ptr[40] = 0xFFFFFFF8
    Y = G.run_sparse_gemm(p, X)
    assert np.all(np.isnan(Y[:, 7])) and np.all(np.isnan(Y[:, 40]))
    keep = np.ones(64, dtype=bool)
    keep[[7, 40]] = False
    assert np.array_equal(Y[:, keep].view(np.uint16), good[:, keep].view(np.uint16))


# ---------------------------------------------------------------- dense INT4
@pytest.mark.parametrize("rows,cols,g", [(37, 64, 8), (130, 1024, 128), (21, 11008, 128), (50, 4096, 64),
                                         (9, 4096, 4096), (66, 2048, 32), (33, 320, 64), (45, 4096, 128),
                                         (7, 512, 128), (70, 2048, 128), (33, 8192, 128), (19, 2176, 128),
                                         (1, 4096, 128), (131, 1024, 128),
                                         # other group sizes on the matrix-core path
                                         (70, 4096, 256), (33, 1024, 32), (20, 512, 64), (40, 1024, 512),
                                         (21, 11008, 256), (21, 11008, 64), (35, 2048, 2048), (18, 6144, 32),
                                         # groups that are a multiple of 4 but not of 8 columns
                                         (37, 96, 12), (9, 160, 20), (70, 64, 4), (5, 1092, 84)])
def test_int4_gemv_small(rows, cols, g):
    print(f"case int4_gemv {rows}x{cols} g={g}", flush=True)
    w = synth.weights(rows, cols, 500 + rows)
    x = synth.activations(cols, 500 + rows)
    q, qp = B.quant_int4(w, g)
    oq, oqp = O.quant_int4_dense(w, g)
    assert np.array_equal(q, oq) and np.array_equal(qp, oqp)
    y_ref, a_ref = O.int4_gemv(oq, oqp, g, x)
    G.assert_close(G.run_int4_gemv(q, qp, g, x), y_ref, a_ref, "int4_gemv")


@pytest.mark.parametrize("g", [128, 32, 64, 256])
def test_int4_one_hot_x_returns_decoded_column_bit_exact(g):
    w = synth.weights(64, 4096, 77)
    q, qp = B.quant_int4(w, g)
    Wd = O.dequant_int4_dense(q, qp, g)
    for j in (0, 1, 130, 4095):
        e = np.zeros(4096, dtype=np.float16)
        e[j] = 1
        y = G.run_int4_gemv(q, qp, g, e)
        assert np.array_equal(y.view(np.uint16), Wd[:, j].astype(np.float16).view(np.uint16)), f"column {j}"


def test_config2_dense_int4_full():
    seed = synth.seed_for(2)
    w = synth.weights(4096, 4096, seed)
    x = synth.activations(4096, seed)
    q, qp = B.quant_int4(w, 128)
    oq, oqp = O.quant_int4_dense(w, 128)
    assert np.array_equal(q, oq) and np.array_equal(qp, oqp)
    y_ref, a_ref = O.int4_gemv(oq, oqp, 128, x)
    G.assert_close(G.run_int4_gemv(q, qp, 128, x), y_ref, a_ref, "config 2")


# ---------------------------------------------------------------- full sizes, sampled rows
@pytest.mark.parametrize("name,rows,cols,kind,g,cfg", [
    ("headline", 11008, 4096, 0, 128, synth.HEADLINE), ("config3", 11008, 4096, 1, 0, 3),
    ("down", 4096, 11008, 0, 128, 5),
])
def test_full_size_sampled_rows(name, rows, cols, kind, g, cfg):
    print(f"case full-size {name}", flush=True)
    seed = synth.seed_for(cfg)
    w, mask, p = G.packed_full(rows, cols, 2, g, kind, seed)
    x = synth.activations(cols, seed)
    y = G.run_sparse_gemv(p, x)
    pick = G.sample_rows(rows, 192, seed)
    # the oracle packs the sampled rows on its own: bytes must match the library's rows
    o = O.pack_2bitcsr(w[pick], O.prune_n4_magnitude(w[pick], 2), 2, g, kind)
    sub = G.row_subset(p, pick)
    for k in ("values", "idx", "qparams"):
        assert (o[k] is None and sub[k] is None) or np.array_equal(o[k], sub[k]), k
    y_ref, a_ref = O.gemv(o, x)
    G.assert_close(y[pick], y_ref, a_ref, name)
    # property that holds at any size: every other row, decoded by the oracle from the
    # library's bytes in slabs, also agrees
    for r0 in range(0, rows, 2048):
        rr = np.arange(r0, min(rows, r0 + 2048))
        yr, ar = O.gemv(G.row_subset(p, rr), x)
        G.assert_close(y[rr], yr, ar, f"{name} rows {r0}..")


@pytest.mark.parametrize("kind", [0, 2])
def test_tall_matrix_sampled_rows(kind):
    # 65536 x 4096 (the launch-amortised row of the bench table), both nibble orders: sampled rows
    # against the oracle's own packing of them, and the last slab decoded from the library's bytes
    rows, cols = 65536, 4096
    print(f"case tall {rows}x{cols} kind={kind}", flush=True)
    seed = synth.seed_for(synth.HEADLINE, 7)
    w, mask, p = G.packed_full(rows, cols, 2, 128, kind, seed)
    x = synth.activations(cols, seed)
    y = G.run_sparse_gemv(p, x)
    pick = G.sample_rows(rows, 256, seed)
    o = O.pack_2bitcsr(w[pick], O.prune_n4_magnitude(w[pick], 2), 2, 128, kind)
    sub = G.row_subset(p, pick)
    for k in ("values", "idx", "qparams"):
        assert np.array_equal(o[k], sub[k]), k
    y_ref, a_ref = O.gemv(o, x)
    G.assert_close(y[pick], y_ref, a_ref, "tall, sampled")
    rr = np.arange(rows - 1024, rows)
    yr, ar = O.gemv(G.row_subset(p, rr), x)
    G.assert_close(y[rr], yr, ar, "tall, last rows")


# ---------------------------------------------------------------- paired nibble order
@pytest.mark.parametrize("rows,cols,n,g", [
    (257, 4096, 2, 128), (45, 4096, 2, 64), (21, 11008, 2, 128), (70, 1024, 2, 128), (70, 2048, 2, 256), (33, 8192, 2, 128),
    (4, 32768, 2, 128),                                    # the tuned M = 1 kernels
    (45, 4096, 2, 32), (37, 96, 2, 32), (45, 4096, 1, 128), (64, 160, 3, 32), (3, 40960, 2, 128),   # slot by slot
])
def test_paired_order_gives_the_bits_of_the_canonical_order(rows, cols, n, g):
    """The two nibble orders hold the same codes, the tuned kernels dequantise them to the same
    FP16 values and add in the same order: same bits where both run a tuned kernel, the
    oracle's tolerance everywhere."""
    print(f"case paired {rows}x{cols} n={n} g={g}", flush=True)
    rng = np.random.default_rng(rows + cols)
    w = synth.weights(rows, cols, 7300 + rows + cols + g)
    mask = O.prune_n4_magnitude(w, n)
    mask = (mask & (rng.random(mask.shape) >= 0.1)).astype(np.uint8)
    pp = B.pack_2bitcsr(w, mask, n, g, B.VAL_INT4_PAIRED)
    pc = B.pack_2bitcsr(w, mask, n, g, B.VAL_INT4)
    o = O.pack_2bitcsr(w, mask, n, g, O.VAL_INT4_PAIRED)
    assert np.array_equal(pp.values, o["values"]) and np.array_equal(pp.idx, o["idx"])
    x = synth.activations(cols, 7300 + rows)
    y_ref, a_ref = O.gemv(o, x)
    yp = G.run_sparse_gemv(pp, x)
    G.assert_close(yp, y_ref, a_ref, "paired order")
    tuned = n == 2 and g >= 64 and (cols in (1024, 2048) or (cols >= 4096 and cols % 64 == 0 and cols <= 32768))
    if tuned:
        assert np.array_equal(yp.view(np.uint16), G.run_sparse_gemv(pc, x).view(np.uint16))
    X = synth.activation_rows(3, cols, 7300 + cols)
    Y_ref, A_ref = O.gemm_smallm(o, X)
    G.assert_close(G.run_sparse_gemm(pp, X), Y_ref, A_ref, "paired order, three tokens")


def test_paired_order_full_size_and_in_other_entry_points():
    rows, cols = 11008, 4096
    seed = synth.seed_for(synth.HEADLINE)
    w = synth.weights(rows, cols, seed)
    mask = B.prune_n4(w, 2)
    pp = B.pack_2bitcsr(w, mask, 2, 128, B.VAL_INT4_PAIRED)
    pc = B.pack_2bitcsr(w, mask, 2, 128, B.VAL_INT4)
    x = synth.activations(cols, seed)
    yp = G.run_sparse_gemv(pp, x)
    assert np.array_equal(yp.view(np.uint16), G.run_sparse_gemv(pc, x).view(np.uint16))
    pick = G.sample_rows(rows, 128, seed)
    o = O.pack_2bitcsr(w[pick], O.prune_n4_magnitude(w[pick], 2), 2, 128, O.VAL_INT4_PAIRED)
    words = cols // 2 // 8 * 4                               # value bytes per row
    assert np.array_equal(np.concatenate([pp.values[r * words:(r + 1) * words] for r in pick]), o["values"])
    y_ref, a_ref = O.gemv(o, x)
    G.assert_close(yp[pick], y_ref, a_ref, "paired order, headline shape")
    # batched call: one launch per member; the workspace and table forms say so
    torch = G.torch_mod()
    pd = pp.to("cuda")
    xd = G.to_dev(x.view(np.uint16)).view(torch.float16)
    ys = [torch.zeros(rows, dtype=torch.float16, device="cuda") for _ in range(2)]
    B.prepared_sparse_gemv_batch([pd, pd], [xd, xd], ys)()
    torch.cuda.synchronize()
    assert np.array_equal(ys[1].cpu().numpy().view(np.uint16), yp.view(np.uint16))
    assert B.smallm_ws_bytes(pd, 64) == 0
    with pytest.raises(B.EgtError) as e:
        B.prepared_gemv_stack([("sparse", pd, xd, ys[0])])
    assert e.value.status == 6


# ---------------------------------------------------------------- rows of different lengths
def _ragged_case(rows, cols, g, kind, seed, choices=(1, 2), drop=0.0):
    rng = np.random.default_rng(seed)
    w = synth.weights(rows, cols, seed)
    nk = rng.choice(choices, size=rows).astype(np.int32)
    mask = np.zeros((rows, cols), dtype=np.uint8)
    for n in np.unique(nk):
        mask[nk == n] = B.prune_n4(np.ascontiguousarray(w[nk == n]), int(n))
    if drop:
        mask = (mask & (rng.random(mask.shape) >= drop)).astype(np.uint8)
    return w, mask, nk


@pytest.mark.parametrize("rows,cols,g,kind,choices", [
    (37, 96, 32, 0, (1, 2)), (64, 4096, 128, 0, (1, 2)), (130, 1056, 96, 0, (1, 2, 3, 4)), (45, 4096, 0, 1, (1, 2)),
    (21, 11008, 128, 0, (1, 2)), (9, 2112, 12, 0, (2, 4)), (3, 40960, 128, 0, (1, 2)), (1, 32, 32, 0, (1,)),
    # x at the 64 KB LDS limit of the one-token kernel; groups
    # of 20 columns (a word of eight slots then spans up to three groups at 1:4); the paired nibble order
    (5, 32768, 128, 0, (1, 2, 3, 4)), (40, 4160, 20, 0, (1, 2, 3, 4)), (33, 2048, 64, 2, (1, 2, 4)),
])
@pytest.mark.parametrize("M", [1, 5])
def test_ragged_rows_small(rows, cols, g, kind, choices, M):
    print(f"case ragged {rows}x{cols} g={g} kind={kind} rows keep {choices} M={M}", flush=True)
    w, mask, nk = _ragged_case(rows, cols, g, kind, 7000 + rows + cols, choices, drop=0.1)
    p = B.pack_2bitcsr_rows(w, mask, nk, g, kind)
    o = O.pack_2bitcsr_rows(w, mask, nk, g, kind)
    for k in ("row_ptr", "values", "idx"):
        assert np.array_equal(getattr(p, k), o[k]), k
    X = synth.activation_rows(M, cols, 7000 + rows)
    Y_ref, A_ref = O.gemm_rows(o, X)
    Y = G.run_sparse_gemm(p, X, ldx_pad=8, ldy_pad=3) if M > 1 else G.run_sparse_gemv(p, np.ascontiguousarray(X[0]))[None, :]
    G.assert_close(Y, Y_ref, A_ref, "ragged rows")


def test_ragged_rows_half_of_the_headline_matrix_at_one_in_four():
    """Sec. 3.2's adaptive N:4 inside one matrix: every second row class keeps 1 of 4."""
    rows, cols, g = 11008, 4096, 128
    seed = synth.seed_for(synth.HEADLINE)
    rng = np.random.default_rng(seed)
    w = synth.weights(rows, cols, seed)
    nk = rng.permutation(np.repeat([1, 2], rows // 2)).astype(np.int32)
    mask = np.zeros((rows, cols), dtype=np.uint8)
    for n in (1, 2):
        mask[nk == n] = B.prune_n4(np.ascontiguousarray(w[nk == n]), n)
    p = B.pack_2bitcsr_rows(w, mask, nk, g, 0)
    uniform = sum(B.sizes(rows, cols, 2, g, 0))
    saved = uniform - p.nbytes()
    print(f"ragged 50/50 1:4 and 2:4: {p.nbytes()} bytes against {uniform} for 2:4 throughout, {saved} saved", flush=True)
    assert saved == (rows // 2) * (cols // 4) * 6 // 8             # one slot (4 + 2 bits) per 4-group in half of the rows
    x = synth.activations(cols, seed)
    y = G.run_sparse_gemv(p, x)
    pick = G.sample_rows(rows, 192, seed)
    # sampled rows: the oracle packs them itself, its bytes must be the library's rows
    o = O.pack_2bitcsr_rows(w[pick], mask[pick], nk[pick], g, 0)
    for k, r in enumerate(pick):
        t0, t1 = int(p.row_ptr[r]), int(p.row_ptr[r + 1])
        u0, u1 = int(o["row_ptr"][k]), int(o["row_ptr"][k + 1])
        assert t1 - t0 == u1 - u0
        assert np.array_equal(p.values[t0 // 2:t1 // 2], o["values"][u0 // 2:u1 // 2])
        assert np.array_equal(p.idx[t0 // 8:t1 // 8], o["idx"][u0 // 8:u1 // 8])
    assert np.array_equal(p.qparams[pick], o["qparams"])
    y_ref, a_ref = O.gemv_rows(o, x)
    G.assert_close(y[pick], y_ref, a_ref, "ragged sampled rows")
    # every row, decoded by the oracle from the library's bytes
    y_all, a_all = O.gemv_rows(G.oracle_view(p), x)
    G.assert_close(y, y_all, a_all, "ragged all rows")


def test_ragged_broken_row_ptr_yields_nan_not_a_fault():
    w, mask, nk = _ragged_case(64, 1024, 128, 0, 7100)
    p = B.pack_2bitcsr_rows(w, mask, nk, 128, 0)
    x = synth.activations(1024, 71)
    good = G.run_sparse_gemv(p, x)
    torch = G.torch_mod()
    bad_rows = set()

    def run(q):
        y = torch.zeros(64, dtype=torch.float16, device="cuda")
        B.sparse_gemv(q.to("cuda"), G.to_dev(x.view(np.uint16)).view(torch.float16), y)
        torch.cuda.synchronize()
        return y.cpu().numpy()

    q = B.Packed(**{**p.__dict__, "row_ptr": p.row_ptr.copy()})
    q.row_ptr[7] += 4                       # rows 6 and 7 are not whole rows, row 7 not on an index word
    q.row_ptr[40] = 0xFFFFFFF8              # row 39 runs far past the buffers, row 40 has a negative length
    y = run(q)
    bad_rows = [6, 7, 39, 40]
    assert np.all(np.isnan(y[bad_rows]))
    keep = np.ones(64, dtype=bool)
    keep[bad_rows] = False
    assert np.array_equal(y[keep].view(np.uint16), good[keep].view(np.uint16))
    # a view that vouches for fewer slots than row_ptr walks: the rows beyond are not read
    q = B.Packed(**{**p.__dict__, "total_slots": int(p.row_ptr[50])})
    y = run(q)
    assert np.all(np.isnan(y[50:])) and np.array_equal(y[:50].view(np.uint16), good[:50].view(np.uint16))


# ---------------------------------------------------------------- small M
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 16, 33, 64])
def test_smallm_small_shapes(M):
    print(f"case smallm M={M}", flush=True)
    for rows, cols, n, g, kind in [(70, 1024, 2, 128, 0), (33, 96, 1, 32, 0), (40, 4096, 2, 0, 1), (18, 11008, 2, 128, 0)]:
        p, o = _small_case(rows, cols, n, g, kind, seed=900 + M + rows)
        X = synth.activation_rows(M, cols, 900 + M)
        Y_ref, A_ref = O.gemm_smallm(o, X)
        Y = G.run_sparse_gemm(p, X, ldx_pad=8 if M % 2 else 0, ldy_pad=6 if M % 2 else 0)
        G.assert_close(Y, Y_ref, A_ref, f"smallm {rows}x{cols} M={M}")


@pytest.mark.parametrize("rows,cols,n,g,kind,M", [
    (4200, 256, 2, 128, 0, 7),      # one K-step (one wave), several row tiles per workgroup, ragged last tile
    (5000, 768, 2, 64, 0, 16),      # three waves, groups of 64
    (5000, 768, 2, 256, 0, 40),     # two token groups per pass, second pass half empty
    (4130, 1280, 2, 128, 0, 17),    # five waves, M just past one token group
    (300, 8704, 2, 128, 0, 32),     # 34 K-steps: phases with idle waves at the end
    (300, 8704, 2, 128, 0, 9),
    (4100, 512, 2, 0, 1, 5),        # FP16 values
    (4100, 512, 2, 0, 1, 48),
    (13000, 256, 2, 128, 0, 3),     # more row tiles than three per workgroup on 256 workgroups: two rounds
    (20000, 512, 2, 128, 0, 40),    # rounds x passes: 1250 row tiles, three token groups, two per pass
    (17000, 640, 1, 128, 0, 20),    # the same at 1:4 (one token group per pass), partly filled last step
    (20000, 2304, 2, 0, 1, 9),      # rounds with FP16 values (tiles requested two phases ahead)
    (13000, 320, 2, 64, 0, 16),     # rounds with a partly filled last step
    (33000, 128, 2, 128, 0, 5),     # nine row tiles per workgroup: three rounds, one wave
    (4200, 512, 2, 32, 0, 6),       # groups of 32 columns: two {scale, zero} pairs per chunk
    (4200, 512, 2, 32, 0, 30),
    (50, 8704, 2, 32, 0, 16),
    (70, 4160, 2, 64, 0, 5),        # K not a multiple of the K-step: a partly filled last step
    (70, 4160, 2, 64, 0, 20),
    (40, 320, 2, 0, 1, 33),         # the same with FP16 values
    (4100, 6464, 2, 0, 1, 9),       # FP16 values, tiles requested two phases ahead: four phases of 8 waves,
    (4100, 2304, 2, 0, 1, 16),      #   a partly filled last step; two phases, the second with one wave
    (60, 11072, 2, 0, 1, 3),        # one tile per workgroup: three phases of 16 waves, the last partly filled
    (200, 4352, 2, 0, 1, 13),       # 17 steps on 16 waves
    (4200, 1024, 1, 128, 0, 6),     # 1:4: {value, 0} pairs, eight instructions per step
    (300, 4096, 1, 128, 0, 16),
    (300, 4096, 1, 256, 0, 40),     # 1:4 runs its token groups one after the other
    (60, 11008, 1, 128, 0, 4),      # 86 chunks: a half-filled last step
    (60, 11008, 1, 64, 0, 16),      # 1:4 with two and four {scale, zero} pairs per chunk
    (60, 2176, 1, 32, 0, 7),
    (4100, 640, 1, 0, 1, 12),       # 1:4, FP16 values, partly filled last step
    (90, 4096, 1, 0, 1, 64),
])
def test_smallm_tile_and_wave_shapes(rows, cols, n, g, kind, M):
    print(f"case smallm shapes {rows}x{cols} n={n} g={g} kind={kind} M={M}", flush=True)
    p, o = _small_case(rows, cols, n, g, kind, seed=1300 + M + rows)
    X = synth.activation_rows(M, cols, 1300 + M)
    Y_ref, A_ref = O.gemm_smallm(o, X)
    for pad in (0, 6, 7):        # 8-byte stores of four rows, the 2-byte fallback, odd strides
        Y = G.run_sparse_gemm(p, X, ldx_pad=pad, ldy_pad=pad)
        G.assert_close(Y, Y_ref, A_ref, f"smallm {rows}x{cols} M={M} pad={pad}")


@pytest.mark.parametrize("rows,cols,g,M", [
    (70, 4096, 128, 2), (70, 4096, 128, 3), (70, 4096, 128, 4),
    (33, 4096, 64, 2), (33, 4096, 256, 4), (19, 4096, 4096, 3),      # other group sizes
    (1000, 4096, 128, 4), (1003, 4096, 128, 2),                      # many workgroups, ragged rows
    (9000, 4096, 128, 2),                                            # more rows than the four-token form takes
    (300, 8192, 128, 2), (77, 4160, 64, 2), (1000, 6144, 256, 2),    # two tokens, two tiles per row (the second partly filled)
])
def test_few_tokens_on_the_row_per_wave_mapping(rows, cols, g, M):
    # M = 2..4 at 2:4 INT4 with K >= 4096 runs on the M = 1 kernel's mapping (the weights are
    # dequantised once and multiplied with one B operand per token)
    print(f"case few tokens {rows}x{cols} g={g} M={M}", flush=True)
    p, o = _small_case(rows, cols, 2, g, 0, seed=1700 + M + rows)
    X = synth.activation_rows(M, cols, 1700 + M)
    Y_ref, A_ref = O.gemm_smallm(o, X)
    for pad in (0, 8):
        Y = G.run_sparse_gemm(p, X, ldx_pad=pad, ldy_pad=pad // 2)
        G.assert_close(Y, Y_ref, A_ref, f"few tokens {rows}x{cols} M={M} pad={pad}")
    # token 0 alone is the M = 1 product: the same instructions in the same order
    y0 = G.run_sparse_gemv(p, np.ascontiguousarray(X[0]))
    assert np.array_equal(Y[0].view(np.uint16), y0.view(np.uint16))


@pytest.mark.parametrize("rows,cols,M", [(70, 4096, 2), (1003, 4096, 2), (9000, 4096, 2), (70, 4096, 3), (1003, 4096, 4),
                                         (9000, 4096, 3), (11008, 4096, 4),
                                         # two tokens, several tiles per row (the last one partly filled)
                                         (300, 11008, 2), (70, 8192, 2), (41, 4160, 2), (33, 16384, 2), (1030, 5120, 2)])
def test_few_tokens_with_fp16_values_on_the_row_per_wave_mapping(rows, cols, M):
    # FP16 values, M = 2..4: the M = 1 kernel's contiguous-kilobyte loads with one B operand per token
    print(f"case few tokens fp16 {rows}x{cols} M={M}", flush=True)
    p, o = _small_case(rows, cols, 2, 0, 1, seed=1900 + rows, drop=0.1)
    X = synth.activation_rows(M, cols, 1900 + rows)
    Y_ref, A_ref = O.gemm_smallm(o, X)
    for pad in (0, 8):
        Y = G.run_sparse_gemm(p, X, ldx_pad=pad, ldy_pad=pad // 2)
        G.assert_close(Y, Y_ref, A_ref, f"few tokens fp16 {rows} M={M} pad={pad}")
    for m in range(M):            # each token alone is the M = 1 product: same instructions, same order
        y1 = G.run_sparse_gemv(p, np.ascontiguousarray(X[m]))
        assert np.array_equal(Y[m].view(np.uint16), y1.view(np.uint16))
    Y6 = G.run_sparse_gemm(p, X, ldx_pad=6)          # token rows not 16-byte aligned: the K-split kernel
    G.assert_close(Y6, Y_ref, A_ref, "few tokens fp16, unaligned rows of X")


@pytest.mark.parametrize("rows,cols", [(11008, 4096), (4096, 11008)])
@pytest.mark.parametrize("M", [2, 4, 16, 24, 64])
def test_config5_smallm_full_size(rows, cols, M):
    print(f"case config5 {rows}x{cols} M={M}", flush=True)
    seed = synth.seed_for(5, 0 if rows == 11008 else 1)
    w, mask, p = G.packed_full(rows, cols, 2, 128, 0, seed)
    X = synth.activation_rows(M, cols, seed + M)
    Y = G.run_sparse_gemm(p, X)
    pick = G.sample_rows(rows, 96, seed + M)
    o = O.pack_2bitcsr(w[pick], O.prune_n4_magnitude(w[pick], 2), 2, 128, 0)
    sub = G.row_subset(p, pick)
    for k in ("values", "idx", "qparams"):
        assert np.array_equal(o[k], sub[k]), k
    Y_ref, A_ref = O.gemm_smallm(o, X)
    G.assert_close(Y[:, pick], Y_ref, A_ref, f"config 5 M={M}")
    # M-row product equals M independent GEMVs on the same device path (within tolerance)
    y0 = G.run_sparse_gemv(p, np.ascontiguousarray(X[0]))
    G.assert_close(y0[pick], Y_ref[0], A_ref[0], "row 0 as a GEMV")


@pytest.mark.parametrize("rows,cols,M", [(4096, 11008, 64), (4096, 11008, 17), (2000, 8192, 33), (500, 12288, 40), (16, 8192, 64),
                                         (11008, 4096, 64), (11008, 4096, 49), (4096, 11008, 32), (9000, 2048, 64), (8193, 1536, 33)])
def test_smallm_split_over_k_with_a_workspace(rows, cols, M):
    # K split over workgroups, FP32 partial sums through a caller-provided workspace: sampled
    # rows against the oracle, every output close to the one-launch kernel's (same products,
    # another order of the FP32 additions), identical bits on a second run, a canary behind the
    # bytes the library said it needs, nothing written outside Y
    torch = G.torch_mod()
    print(f"case smallm split {rows}x{cols} M={M}", flush=True)
    w, mask, p = G.packed_full(rows, cols, 2, 128, 0, 5200 + rows + cols)
    X = synth.activation_rows(M, cols, 5200 + M)
    pd = p.to("cuda")
    need = B.smallm_ws_bytes(pd, M)
    assert need >= 2 * 4 * M * rows                      # at least two slices of FP32 partial sums
    ws = torch.full((need + 4096,), 0x5A, dtype=torch.uint8, device="cuda")
    Xd = G.to_dev(X.view(np.uint16)).view(torch.float16)
    Ybuf = torch.full((M + 2, rows + 8), G.CANARY, dtype=torch.int16, device="cuda")
    Y = Ybuf[1:M + 1, :rows].view(torch.float16)
    B.sparse_gemm_smallm_ws(pd, Xd, Y, ws[:need])
    torch.cuda.synchronize()
    host = Ybuf.cpu().numpy().view(np.uint16)
    assert np.all(host[0] == G.CANARY) and np.all(host[M + 1] == G.CANARY) and np.all(host[:, rows:] == G.CANARY)
    assert torch.all(ws[need:] == 0x5A)
    got = host[1:M + 1, :rows].view(np.float16)
    pick = G.sample_rows(rows, 24, M)
    o = O.pack_2bitcsr(w[pick], O.prune_n4_magnitude(w[pick], 2), 2, 128, 0)
    Y_ref, A_ref = O.gemm_smallm(o, X)
    G.assert_close(got[:, pick], Y_ref, A_ref, "split over K")
    one = G.run_sparse_gemm(p, X)
    diff = np.abs(got.astype(np.float64) - one.astype(np.float64))
    assert np.all(diff <= 2e-3 * np.maximum(1.0, np.abs(one.astype(np.float64))))
    first = got.copy()
    ws.fill_(0x33)                                       # whatever the workspace holds before the call
    Ybuf.fill_(G.CANARY)
    B.sparse_gemm_smallm_ws(pd, Xd, Y, ws[:need])
    torch.cuda.synchronize()
    again = Ybuf.cpu().numpy().view(np.uint16)[1:M + 1, :rows]
    assert np.array_equal(again, first.view(np.uint16))
    # a broken row pointer: NaN for every token of that row, the other rows untouched
    rp = pd.row_ptr.view(torch.int32)
    keep_rp = rp[3].clone()
    rp[3] += 8
    B.sparse_gemm_smallm_ws(pd, Xd, Y, ws[:need])
    torch.cuda.synchronize()
    bad = Ybuf.cpu().numpy().view(np.uint16)[1:M + 1, :rows].view(np.float16)
    assert np.all(np.isnan(bad[:, 3]))
    others = np.ones(rows, dtype=bool)
    others[3] = False
    assert np.array_equal(bad[:, others].view(np.uint16), first[:, others].view(np.uint16))
    rp[3] = keep_rp
    # too small a workspace is refused on the host
    with pytest.raises(B.EgtError) as e:
        v = pd.view()
        B._check(B.lib().egt_sparse_gemm_smallm_ws(__import__("ctypes").byref(v), Xd.data_ptr(), cols, Y.data_ptr(), Y.stride(0), M,
                                                   ws.data_ptr(), need - 1, None))
    assert e.value.status == 2


@pytest.mark.parametrize("rows,cols,M,ldx_pad,ldy_pad", [(2000, 8192, 40, 8, 3), (1000, 8192, 64, 16, 1), (8200, 1536, 33, 8, 4)])
def test_smallm_split_with_strided_x_and_y(rows, cols, M, ldx_pad, ldy_pad):
    # token rows of X and Y that do not follow each other: X rows on 16-byte boundaries (the
    # form with X held in LDS), Y rows that do not allow 8-byte stores
    torch = G.torch_mod()
    print(f"case smallm split strided {rows}x{cols} M={M}", flush=True)
    p, o = _small_case(rows, cols, 2, 128, 0, seed=5300 + rows)
    X = synth.activation_rows(M, cols, 5300 + M)
    pd = p.to("cuda")
    need = B.smallm_ws_bytes(pd, M, cols + ldx_pad)
    assert need > 0
    ws = torch.full((need + 1024,), 0x5A, dtype=torch.uint8, device="cuda")
    Xbuf = torch.full((M, cols + ldx_pad), float("nan"), dtype=torch.float16, device="cuda")
    Xbuf[:, :cols] = G.to_dev(X.view(np.uint16)).view(torch.float16)
    Ybuf = torch.full((M + 2, rows + ldy_pad), G.CANARY, dtype=torch.int16, device="cuda")
    Y = Ybuf[1:M + 1, :rows].view(torch.float16)
    B.sparse_gemm_smallm_ws(pd, Xbuf[:, :cols], Y, ws[:need])
    torch.cuda.synchronize()
    host = Ybuf.cpu().numpy().view(np.uint16)
    assert np.all(host[0] == G.CANARY) and np.all(host[M + 1] == G.CANARY) and np.all(host[:, rows:] == G.CANARY)
    assert torch.all(ws[need:] == 0x5A)
    Y_ref, A_ref = O.gemm_smallm(o, X)
    G.assert_close(host[1:M + 1, :rows].view(np.float16), Y_ref, A_ref, "split, strided")
    # X rows that are not on 16-byte boundaries: the split form does not apply, the call still computes the product
    Xodd = torch.zeros((M, cols + 2), dtype=torch.float16, device="cuda")
    Xodd[:, :cols] = Xbuf[:, :cols]
    assert B.smallm_ws_bytes(pd, M, cols + 2) == 0
    Ybuf.fill_(G.CANARY)
    B.sparse_gemm_smallm_ws(pd, Xodd[:, :cols], Y, None)
    torch.cuda.synchronize()
    G.assert_close(Ybuf.cpu().numpy().view(np.uint16)[1:M + 1, :rows].view(np.float16), Y_ref, A_ref, "one launch, odd ldx")


def test_smallm_workspace_not_needed_where_the_split_does_not_pay():
    torch = G.torch_mod()
    for rows, cols, n, g, kind, M in ((11008, 4096, 2, 128, 0, 32), (4096, 4096, 2, 128, 0, 64), (4096, 11008, 2, 128, 0, 16), (300, 8192, 1, 128, 0, 40),
                                      (300, 8192, 2, 0, 1, 40), (300, 8192, 2, 32, 0, 40)):
        p = B.Packed(rows, cols, n, g, kind, None, None, None, None)
        assert B.smallm_ws_bytes(p, M) == 0
    # the workspace call is then the one-launch call
    p, o = _small_case(300, 8192, 2, 32, 0, seed=77)
    X = synth.activation_rows(40, 8192, 78)
    pd = p.to("cuda")
    Xd = G.to_dev(X.view(np.uint16)).view(torch.float16)
    Y1 = torch.zeros((40, 300), dtype=torch.float16, device="cuda")
    Y2 = torch.zeros((40, 300), dtype=torch.float16, device="cuda")
    B.sparse_gemm_smallm(pd, Xd, Y1)
    B.sparse_gemm_smallm_ws(pd, Xd, Y2, None)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)


# ---------------------------------------------------------------- measurement aid
def test_stream_read_folds_every_word_once():
    torch = G.torch_mod()
    rng = np.random.default_rng(3)
    for nbytes in (16, 4096 + 16, 1 << 20, (1 << 20) + 48):
        data = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
        src = torch.from_numpy(data).cuda()
        sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
        B.stream_read(src, nbytes, sink)
        torch.cuda.synchronize()
        got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
        want = np.bitwise_xor.reduce(data.view(np.uint32))
        assert got == want, nbytes


# ---------------------------------------------------------------- batched launches
@pytest.mark.parametrize("rows,cols,n,g,kind,count", [(70, 4096, 2, 128, 0, 3), (33, 11008, 2, 128, 0, 2),
                                                      (40, 4096, 1, 128, 0, 4), (21, 4096, 2, 0, 1, 2),
                                                      (19, 96, 3, 32, 0, 3)])
def test_sparse_gemv_batch_equals_separate_calls(rows, cols, n, g, kind, count):
    torch = G.torch_mod()
    ps, xs, refs = [], [], []
    for k in range(count):
        p, o = _small_case(rows, cols, n, g, kind, seed=7000 + 13 * k + rows)
        x = synth.activations(cols, 7000 + k)
        ps.append(p); xs.append(x); refs.append(O.gemv(o, x))
    pds = [p.to("cuda") for p in ps]
    xds = [G.to_dev(x.view(np.uint16)).view(torch.float16) for x in xs]
    ys = [torch.full((rows,), 9.0, dtype=torch.float16, device="cuda") for _ in range(count)]
    B.sparse_gemv_batch(pds, xds, ys)
    torch.cuda.synchronize()
    for k in range(count):
        y = ys[k].cpu().numpy()
        G.assert_close(y, refs[k][0], refs[k][1], f"batch member {k}")
        assert np.array_equal(y.view(np.uint16), G.run_sparse_gemv(ps[k], xs[k]).view(np.uint16))


@pytest.mark.parametrize("rows,cols,n,g,kind,M,count,shared", [
    (70, 4096, 2, 128, 0, 16, 3, True), (33, 11008, 2, 128, 0, 7, 2, False), (300, 4096, 2, 128, 0, 33, 3, True),
    (4100, 1024, 2, 64, 0, 5, 4, False), (40, 4096, 1, 128, 0, 16, 2, True), (21, 4096, 2, 0, 1, 8, 2, False),
    (50, 4096, 2, 32, 0, 64, 2, True),
    # no batched kernel: two tokens on the M = 1 kernel's mapping, the paired nibble order, a slot-by-slot shape, one token
    (70, 4096, 2, 128, 0, 2, 3, True), (37, 4096, 2, 128, 2, 16, 2, False), (19, 96, 3, 32, 0, 5, 3, True), (45, 4096, 2, 128, 0, 1, 2, False),
])
def test_sparse_gemm_batch_equals_separate_calls(rows, cols, n, g, kind, M, count, shared):
    torch = G.torch_mod()
    print(f"case gemm batch {rows}x{cols} n={n} g={g} kind={kind} M={M} x{count} shared={shared}", flush=True)
    ps, Xs, refs = [], [], []
    for k in range(count):
        p, o = _small_case(rows, cols, n, g, kind, seed=7300 + 13 * k + rows)
        X = synth.activation_rows(M, cols, 7300 + (0 if shared else k))
        ps.append(p); Xs.append(X); refs.append(O.gemm_smallm(o, X))
    pds = [p.to("cuda") for p in ps]
    xbuf = [G.to_dev(X.view(np.uint16)).view(torch.float16) for X in (Xs[:1] if shared else Xs)]
    Xd = [xbuf[0] if shared else xbuf[k] for k in range(count)]
    ybufs = [torch.full((M + 2, rows + 8), G.CANARY, dtype=torch.int16, device="cuda") for _ in range(count)]
    Yd = [yb[1:M + 1, :rows].view(torch.float16) for yb in ybufs]
    for rep in range(2):
        B.sparse_gemm_smallm_batch(pds, Xd, Yd)
        torch.cuda.synchronize()
        for k in range(count):
            host = ybufs[k].cpu().numpy().view(np.uint16)
            assert np.all(host[0] == G.CANARY) and np.all(host[M + 1] == G.CANARY) and np.all(host[:, rows:] == G.CANARY), ("write outside Y", k)
            Y = host[1:M + 1, :rows].view(np.float16)
            G.assert_close(Y, refs[k][0], refs[k][1], f"gemm batch member {k}")
            assert np.array_equal(Y.view(np.uint16), G.run_sparse_gemm(ps[k], Xs[k]).view(np.uint16)), k
            ybufs[k][1:M + 1, :rows].fill_(0)


@pytest.mark.parametrize("M", [1, 3, 16, 40])
def test_fused_projections_equal_the_separate_products(M):
    # q/k/v packed as one matrix (concat_rows): every output has the bits of the separate product
    torch = G.torch_mod()
    rows, cols = (300, 70, 133), 4096
    ps, os_ = [], []
    for k, r in enumerate(rows):
        p, o = _small_case(r, cols, 2, 128, 0, seed=7600 + k)
        ps.append(p); os_.append(o)
    fused = B.concat_rows(ps)
    X = synth.activation_rows(M, cols, 7600 + M)
    Yf = G.run_sparse_gemm(fused, X) if M > 1 else G.run_sparse_gemv(fused, X[0])[None, :]
    at = 0
    for k, r in enumerate(rows):
        Y_ref, A_ref = O.gemm_smallm(os_[k], X)
        G.assert_close(Yf[:, at:at + r], Y_ref, A_ref, f"fused member {k}")
        Yk = G.run_sparse_gemm(ps[k], X) if M > 1 else G.run_sparse_gemv(ps[k], X[0])[None, :]
        assert np.array_equal(np.ascontiguousarray(Yf[:, at:at + r]).view(np.uint16), Yk.view(np.uint16)), k
        at += r


@pytest.mark.parametrize("rows,cols,g,count", [(50, 4096, 128, 3), (21, 11008, 128, 2), (30, 320, 64, 2),
                                               (40, 4096, 64, 4), (40, 4096, 256, 2)])
def test_int4_gemv_batch_equals_separate_calls(rows, cols, g, count):
    torch = G.torch_mod()
    qs, qps, xs = [], [], []
    for k in range(count):
        w = synth.weights(rows, cols, 8000 + k + rows)
        q, qp = B.quant_int4(w, g)
        qs.append(q); qps.append(qp); xs.append(synth.activations(cols, 8000 + k))
    qd = [G.to_dev(q) for q in qs]
    qpd = [G.to_dev(qp) for qp in qps]
    xd = [G.to_dev(x.view(np.uint16)).view(torch.float16) for x in xs]
    ys = [torch.full((rows,), 9.0, dtype=torch.float16, device="cuda") for _ in range(count)]
    B.int4_gemv_batch(qd, qpd, rows, cols, g, xd, ys)
    torch.cuda.synchronize()
    for k in range(count):
        y_ref, a_ref = O.int4_gemv(*O.quant_int4_dense(synth.weights(rows, cols, 8000 + k + rows), g), g, xs[k])
        y = ys[k].cpu().numpy()
        G.assert_close(y, y_ref, a_ref, f"batch member {k}")
        assert np.array_equal(y.view(np.uint16), G.run_int4_gemv(qs[k], qps[k], g, xs[k]).view(np.uint16))


# ---------------------------------------------------------------- seeded sweep over shapes
def _random_sparse_case(rng):
    big = rng.random() < 0.1
    rows = int(rng.integers(4000, 5200)) if big else int(rng.integers(1, 400))
    cols = 32 * int(rng.integers(1, 41 if big else 361))
    if rng.random() < 0.3:
        cols = int(rng.choice([4096, 11008, 8192, 1024, 2048, 4160, 12288]))
    if big and cols > 2048:
        cols = 1024
    n = int(rng.choice([1, 2, 2, 2, 1, 3, 4]))
    kind = int(rng.random() < 0.25)
    g = 0 if kind else int(rng.choice([g for g in (32, 64, 128, 256, 512, cols, 96, 16) if cols % g == 0]))
    M = 1 if rng.random() < 0.35 else int(rng.choice([2, 3, 4, 5, 7, 8, 15, 16, 17, 31, 32, 33, 48, 57, 63, 64]))
    if big and M > 20:
        M = int(rng.integers(2, 20))
    return rows, cols, n, g, kind, M, int(rng.choice([0, 0, 2, 6, 7, 8])), 0.3 if rng.random() < 0.3 else 0.0


@pytest.mark.parametrize("block", range(4))
def test_seeded_sweep_of_sparse_shapes(block):
    # shapes nobody picked by hand: every kernel form and the dispatch between them
    rng = np.random.default_rng(4400 + block)
    for case in range(25):
        rows, cols, n, g, kind, M, pad, drop = _random_sparse_case(rng)
        what = f"sweep {block}/{case}: {rows}x{cols} n={n} g={g} kind={kind} M={M} pad={pad} drop={drop}"
        print("case " + what, flush=True)
        p, o = _small_case(rows, cols, n, g, kind, seed=4400 + 100 * block + case, drop=drop)
        if M == 1:
            x = synth.activations(cols, 4400 + case)
            y_ref, a_ref = O.gemv(o, x)
            G.assert_close(G.run_sparse_gemv(p, x), y_ref, a_ref, what)
        else:
            X = synth.activation_rows(M, cols, 4400 + case)
            Y_ref, A_ref = O.gemm_smallm(o, X)
            G.assert_close(G.run_sparse_gemm(p, X, ldx_pad=pad, ldy_pad=pad), Y_ref, A_ref, what)


def test_seeded_sweep_of_row_lengths_nibble_orders_and_narrow_groups():
    # the same for what the sweep above leaves out: rows of different lengths, the paired nibble
    # order, quantisation groups down to four columns
    rng = np.random.default_rng(4700)
    for case in range(36):
        rows = int(rng.integers(1, 300))
        cols = 32 * int(rng.integers(1, 300))
        if rng.random() < 0.3:
            cols = int(rng.choice([4096, 11008, 8192, 1024, 2048, 4160, 12288, 16384]))
        kind = int(rng.choice([0, 0, 1, 2]))
        g = 0 if kind == 1 else int(rng.choice([g for g in (4, 8, 12, 16, 20, 24, 32, 64, 96, 128, 256, 512, cols) if cols % g == 0]))
        ragged = rng.random() < 0.5
        M = 1 if rng.random() < 0.5 else int(rng.choice([2, 3, 4, 5, 8, 16, 17, 33, 64]))
        w = synth.weights(rows, cols, 4700 + case)
        if ragged:
            choices = [(1, 2), (1, 2, 3, 4), (2, 4), (3,), (1,)][int(rng.integers(0, 5))]
            nk = rng.choice(choices, size=rows).astype(np.int32)
            mask = np.zeros((rows, cols), dtype=np.uint8)
            for n in np.unique(nk):
                mask[nk == n] = B.prune_n4(np.ascontiguousarray(w[nk == n]), int(n))
        else:
            n = int(rng.choice([1, 2, 2, 3, 4]))
            mask = B.prune_n4(w, n)
        if rng.random() < 0.3:
            mask = (mask & (rng.random(mask.shape) >= 0.3)).astype(np.uint8)
        what = f"sweep {case}: {rows}x{cols} kind={kind} g={g} M={M} " + (f"rows keep {choices}" if ragged else f"n={n}")
        print("case " + what, flush=True)
        if ragged:
            p, o = B.pack_2bitcsr_rows(w, mask, nk, g, kind), O.pack_2bitcsr_rows(w, mask, nk, g, kind)
        else:
            p, o = B.pack_2bitcsr(w, mask, n, g, kind), O.pack_2bitcsr(w, mask, n, g, kind)
        for k in ("values", "idx", "qparams", "row_ptr"):
            assert (getattr(p, k) is None and o[k] is None) or np.array_equal(getattr(p, k), o[k]), what + " " + k
        if M == 1:
            x = synth.activations(cols, 4700 + case)
            y_ref, a_ref = (O.gemv_rows if ragged else O.gemv)(o, x)
            G.assert_close(G.run_sparse_gemv(p, x), y_ref, a_ref, what)
        else:
            X = synth.activation_rows(M, cols, 4700 + case)
            Y_ref, A_ref = (O.gemm_rows if ragged else O.gemm_smallm)(o, X)
            G.assert_close(G.run_sparse_gemm(p, X), Y_ref, A_ref, what)


@pytest.mark.parametrize("block", range(2))
def test_seeded_sweep_of_the_workspace_form(block):
    # the workspace entry point on shapes nobody picked by hand: whichever form the library
    # chooses (X held in LDS, X fetched per workgroup, or no split), the product must be the
    # oracle's, nothing may be written past the bytes it asked for, and a second run must
    # give the same bits
    torch = G.torch_mod()
    rng = np.random.default_rng(4800 + block)
    for case in range(10):
        cols = int(rng.choice([512, 1024, 1536, 2048, 4096, 4352, 8192, 11008, 12288]))
        rows = int(rng.choice([5, 16, 130, 1000, 2001, 4096, 8200, 9001]))
        if rows * cols > 40_000_000:
            rows = 40_000_000 // cols
        M = int(rng.integers(17, 65))
        g = int(rng.choice([64, 128, 256]))
        if cols % g:
            g = 128 if cols % 128 == 0 else 64
        pad = int(rng.choice([0, 8, 24]))
        what = f"workspace sweep {block}/{case}: {rows}x{cols} g={g} M={M} ldx=+{pad}"
        print("case " + what, flush=True)
        p, o = _small_case(rows, cols, 2, g, 0, seed=4800 + 100 * block + case)
        X = synth.activation_rows(M, cols, 4800 + case)
        pd = p.to("cuda")
        need = B.smallm_ws_bytes(pd, M, cols + pad)
        ws = torch.full((need + 512,), 0x5A, dtype=torch.uint8, device="cuda")
        Xbuf = torch.zeros((M, cols + pad), dtype=torch.float16, device="cuda")
        Xbuf[:, :cols] = G.to_dev(X.view(np.uint16)).view(torch.float16)
        Ybuf = torch.full((M + 2, rows + 5), G.CANARY, dtype=torch.int16, device="cuda")
        Y = Ybuf[1:M + 1, :rows].view(torch.float16)
        outs = []
        for rep in range(2):
            B.sparse_gemm_smallm_ws(pd, Xbuf[:, :cols], Y, ws[:need] if need else None)
            torch.cuda.synchronize()
            host = Ybuf.cpu().numpy().view(np.uint16)
            assert np.all(host[0] == G.CANARY) and np.all(host[M + 1] == G.CANARY) and np.all(host[:, rows:] == G.CANARY), what
            assert torch.all(ws[need:] == 0x5A), what
            outs.append(host[1:M + 1, :rows].copy())
            ws[:need].fill_(0x77)
        assert np.array_equal(outs[0], outs[1]), what
        Y_ref, A_ref = O.gemm_smallm(o, X)
        G.assert_close(outs[0].view(np.float16), Y_ref, A_ref, what)


def test_seeded_sweep_of_dense_shapes():
    rng = np.random.default_rng(4500)
    for case in range(40):
        rows = int(rng.integers(1, 400))
        cols = 8 * int(rng.integers(1, 1500))
        if rng.random() < 0.4:
            cols = int(rng.choice([4096, 11008, 8192, 1024, 2048, 4160, 12288, 512]))
        g = int(rng.choice([g for g in (8, 16, 32, 64, 128, 256, 512, cols, 96) if cols % g == 0]))
        print(f"case dense sweep {case}: {rows}x{cols} g={g}", flush=True)
        w = synth.weights(rows, cols, 4500 + case)
        x = synth.activations(cols, 4500 + case)
        q, qp = B.quant_int4(w, g)
        oq, oqp = O.quant_int4_dense(w, g)
        assert np.array_equal(q, oq) and np.array_equal(qp, oqp)
        y_ref, a_ref = O.int4_gemv(oq, oqp, g, x)
        G.assert_close(G.run_int4_gemv(q, qp, g, x), y_ref, a_ref, f"dense sweep {rows}x{cols} g={g}")
