"""Host half of the C ABI against the oracle: bit-exact packing, error codes,
symbol export.  Runs without a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import egt_oracle as O
from paper_2605_11582_amd import binding as B, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _same_packed(p, o):
    assert (p.rows, p.cols, p.n_keep, p.group, p.val_kind) == (o["rows"], o["cols"], o["n_keep"], o["group"], o["val_kind"])
    assert np.array_equal(p.row_ptr, o["row_ptr"])
    assert np.array_equal(p.idx, o["idx"])
    assert np.array_equal(p.values, o["values"])
    if o["qparams"] is None:
        assert p.qparams is None
    else:
        assert np.array_equal(p.qparams, o["qparams"])


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "egt.h")).read()
    declared = set(re.findall(r"\b(egt_[a-z0-9_]+)\s*\(", text))
    assert declared == set(B.SYMBOLS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(L, name) is not None


def test_library_packs_the_handworked_rows():
    # the hand-worked fixtures pin the library directly, not only through the oracle
    from helpers import read_fixture
    fx = read_fixture("handworked_1x32.txt")
    w = np.array([float(v) for v in fx["w"]], dtype=np.float16)[None, :]
    mask = np.array([int(v) for v in fx["mask"]], dtype=np.uint8)[None, :]
    p = B.pack_2bitcsr(w, mask, 2, 32, B.VAL_INT4)
    assert p.idx.tolist() == [int(v, 16) for v in fx["idx_words"]]
    assert p.values.tolist() == [int(v, 16) for v in fx["value_bytes"]]
    assert np.asarray(p.qparams).reshape(-1).tolist() == [int(v, 16) for v in fx["qparams"]]
    pf = B.pack_2bitcsr(w, mask, 2, 0, B.VAL_FP16)
    assert np.asarray(pf.values).view(np.uint16).tolist() == [int(v, 16) for v in fx["fp16_bits"]]
    fq = read_fixture("handworked_quantiser.txt")
    w = np.zeros((1, 32), dtype=np.float16)
    mask = np.zeros((1, 32), dtype=np.uint8)
    w[0, :4] = [float(v) for v in fq["row_w"]]
    mask[0, :4] = [int(v) for v in fq["row_mask"]]
    p = B.pack_2bitcsr(w, mask, 2, 32, B.VAL_INT4)
    assert np.asarray(p.qparams).reshape(-1).tolist() == [int(v, 16) for v in fq["row_qparams"]]
    assert p.values.tolist() == [int(v, 16) for v in fq["row_value_bytes"]]
    assert p.idx.tolist() == [int(v, 16) for v in fq["row_idx_words"]]
    # the quantiser cases as one-group rows: kept values vmin and vmax (and a zero)
    for name in ("all_positive", "all_negative", "rounded_scale_up", "rounded_scale_dn"):
        vmin, vmax, bits, zero = fq[name]
        w = np.zeros((1, 32), dtype=np.float16)
        mask = np.zeros((1, 32), dtype=np.uint8)
        w[0, 0], w[0, 4] = float(vmin), float(vmax)
        mask[0, 0] = mask[0, 4] = 1
        qp = np.asarray(B.pack_2bitcsr(w, mask, 2, 32, B.VAL_INT4).qparams).reshape(-1)
        assert int(qp[0]) == int(bits, 16), name
        assert float(qp[1:2].view(np.float16)[0]) == float(zero), name


def test_status_strings():
    assert B.status_str(0) == "ok"
    assert len({B.status_str(i) for i in range(8)}) == 8


def test_sizes_match_oracle_and_reject_bad_shapes():
    for args in [(11008, 4096, 2, 128, 0), (4096, 11008, 1, 128, 0), (11008, 4096, 2, 0, 1), (8, 32, 3, 16, 0), (0, 32, 2, 32, 0)]:
        assert B.sizes(*args) == O.buffer_sizes(*args)
    for bad in [(8, 48, 2, 16, 0), (8, 64, 5, 32, 0), (8, 64, 0, 32, 0), (8, 64, 2, 48, 0), (8, 64, 2, 6, 0),
                (8, 64, 2, 32, 1), (8, 64, 2, 0, 0), (8, 64, 2, 32, 7), (-1, 64, 2, 32, 0)]:
        with pytest.raises(B.EgtError) as e:
            B.sizes(*bad)
        assert e.value.status == 2
        with pytest.raises(ValueError):
            O.check_shape(*bad)


@pytest.mark.parametrize("n", [1, 2, 3, 4])
def test_prune_matches_oracle(n):
    w = synth.weights(64, 256, 123 + n)
    w[0, :16] = np.float16(0.25)
    w[1, :8] = [0.0, -0.0, 0.5, -0.5, -0.0, 0.0, 0.0, -0.0]
    assert np.array_equal(B.prune_n4(w, n), O.prune_n4_magnitude(w, n))


@pytest.mark.parametrize("n", [1, 2, 3])
def test_importance_prune_matches_oracle(n):
    rng = np.random.default_rng(300 + n)
    w = synth.weights(200, 256, 300 + n)
    w[0, :16] = np.float16(0.25)                              # ties inside groups
    w[1, :8] = [0.0, -0.0, 0.5, -0.5, -0.0, 0.0, 0.0, -0.0]
    norm = np.abs(rng.standard_normal(256)).astype(np.float32) * 3
    norm[5] = 0.0
    grad = np.abs(rng.standard_normal((200, 256))).astype(np.float32) * 0.01
    assert np.array_equal(B.prune_n4_importance(w, norm, grad, n), O.prune_n4_importance(w, norm, grad, n))
    assert np.array_equal(B.prune_n4_importance(w, norm, None, n), O.prune_n4_importance(w, norm, None, n))
    # constant statistics reduce to magnitude pruning
    assert np.array_equal(B.prune_n4_importance(w, np.full(256, 2.0, np.float32), None, n), B.prune_n4(w, n))


def test_importance_prune_rejects_bad_statistics():
    w = synth.weights(8, 32, 1)
    norm = np.ones(32, np.float32)
    for bad in (-1.0, np.nan, np.inf):
        nb = norm.copy()
        nb[7] = bad
        with pytest.raises(B.EgtError) as e:
            B.prune_n4_importance(w, nb, None, 2)
        assert e.value.status == 4
    g = np.zeros((8, 32), np.float32)
    g[3, 3] = -0.5
    with pytest.raises(B.EgtError) as e:
        B.prune_n4_importance(w, norm, g, 2)
    assert e.value.status == 4
    wn = w.copy()
    wn[2, 2] = np.float16(np.inf)
    with pytest.raises(B.EgtError) as e:
        B.prune_n4_importance(wn, norm, None, 2)
    assert e.value.status == 4
    with pytest.raises(B.EgtError) as e:
        B.prune_n4_importance(w, norm, None, 5)
    assert e.value.status == 2


@pytest.mark.parametrize("n,g,kind", [(2, 128, 0), (1, 128, 0), (2, 0, 1), (1, 0, 1), (3, 64, 0), (4, 32, 0), (2, 4, 0)])
def test_pack_bit_exact_config_like(n, g, kind):
    w = synth.weights(96, 512, 777 + 10 * n + kind)
    mask = O.prune_n4_magnitude(w, n)
    mask[5, 16:20] = 0                       # under-full groups and an empty row
    mask[6, :] = 0
    _same_packed(B.pack_2bitcsr(w, mask, n, g, kind), O.pack_2bitcsr(w, mask, n, g, kind))


@pytest.mark.parametrize("n,g", [(2, 32), (1, 64), (2, 128)])
def test_pack_with_row_groups_bit_exact(n, g):
    rng = np.random.default_rng(600 + n + g)
    w = synth.weights(150, 1024, 600 + n + g)
    mask = O.prune_n4_magnitude(w, n)
    mask[3, 64:192] = 0
    rg = rng.choice([g, 2 * g, 4 * g, 1024], size=150)
    _same_packed(B.pack_2bitcsr(w, mask, n, g, 0, row_group=rg), O.pack_2bitcsr(w, mask, n, g, 0, row_group=rg))
    # every row at the stored granularity = the plain encoder
    a, b = B.pack_2bitcsr(w, mask, n, g, 0, row_group=np.full(150, g)), B.pack_2bitcsr(w, mask, n, g, 0)
    for k in ("row_ptr", "values", "idx", "qparams"):
        assert np.array_equal(getattr(a, k), getattr(b, k)), k
    for bad in (g + 4, 3 * g if 1024 % (3 * g) else 5 * g, 0, -g):
        rb = rg.copy()
        rb[17] = bad
        with pytest.raises(B.EgtError) as e:
            B.pack_2bitcsr(w, mask, n, g, 0, row_group=rb)
        assert e.value.status == 2
    with pytest.raises(B.EgtError) as e:                   # FP16 values have no groups
        B.pack_2bitcsr(w, mask, n, 0, 1, row_group=np.full(150, 64))
    assert e.value.status == 2


def test_pack_bit_exact_config1():
    seed = synth.seed_for(1)
    w = synth.weights(1024, 1024, seed)
    mask = B.prune_n4(w, 2)
    assert np.array_equal(mask, O.prune_n4_magnitude(w, 2))
    _same_packed(B.pack_2bitcsr(w, mask, 2, 128, 0), O.pack_2bitcsr(w, mask, 2, 128, 0))


def test_pack_handles_wide_value_ranges_and_subnormals():
    rng = np.random.default_rng(9)
    # exponents all over the binary16 range, including subnormals and exact ties
    bits = rng.integers(0, 0x7C00, size=(32, 256)).astype(np.uint16) | (rng.integers(0, 2, size=(32, 256)).astype(np.uint16) << 15)
    w = bits.view(np.float16)
    mask = O.prune_n4_magnitude(w, 2)
    _same_packed(B.pack_2bitcsr(w, mask, 2, 32, 0), O.pack_2bitcsr(w, mask, 2, 32, 0))
    small = (rng.integers(0, 64, size=(16, 128)).astype(np.uint16)).view(np.float16)   # subnormals only
    m2 = O.prune_n4_magnitude(small, 2)
    _same_packed(B.pack_2bitcsr(small, m2, 2, 64, 0), O.pack_2bitcsr(small, m2, 2, 64, 0))
    # half-integer multiples of the scale: ties must go to even on both sides
    grid = (0.5 * rng.integers(-14, 17, size=(16, 128))).astype(np.float16)
    grid[:, 0], grid[:, 1] = -7.0, 8.0
    m3 = np.ones_like(grid, dtype=np.uint8)
    _same_packed(B.pack_2bitcsr(grid, m3, 4, 128, 0), O.pack_2bitcsr(grid, m3, 4, 128, 0))


@settings(max_examples=60, deadline=None)
@given(rows=st.integers(0, 9), kb=st.integers(1, 6), n=st.integers(1, 4), kind=st.integers(0, 1),
       gsel=st.integers(0, 3), seed=st.integers(0, 2 ** 31), drop=st.floats(0, 0.5))
def test_pack_bit_exact_random(rows, kb, n, kind, gsel, seed, drop):
    cols = 32 * kb
    groups = [g for g in (4, 8, 16, 32, 64, 96, 128, 192) if cols % g == 0]
    g = 0 if kind == 1 else groups[gsel % len(groups)]
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((rows, cols)) * rng.choice([1e-4, 0.02, 3.0, 500.0])).astype(np.float16)
    mask = O.prune_n4_magnitude(w, n) if rows else np.zeros((0, cols), dtype=np.uint8)
    mask = mask & (rng.random(mask.shape) >= drop)          # random under-full groups
    _same_packed(B.pack_2bitcsr(w, mask.astype(np.uint8), n, g, kind), O.pack_2bitcsr(w, mask, n, g, kind))


def test_pack_errors_leave_outputs_untouched():
    w = synth.weights(8, 64, 5)
    mask = O.prune_n4_magnitude(w, 2)
    bad = mask.copy()
    bad[7, 60:64] = [1, 1, 1, 0]
    with pytest.raises(B.EgtError) as e:
        B.pack_2bitcsr(w, bad, 2, 32, 0)
    assert e.value.status == 3
    w2 = w.copy()
    r, c = np.argwhere(mask == 1)[-1]
    w2[r, c] = np.float16(np.nan)
    with pytest.raises(B.EgtError) as e:
        B.pack_2bitcsr(w2, mask, 2, 32, 0)
    assert e.value.status == 4
    w2[r, c] = w[r, c]
    r, c = np.argwhere(mask == 0)[0]
    w2[r, c] = np.float16(np.inf)            # a pruned entry is never looked at
    B.pack_2bitcsr(w2, mask, 2, 32, 0)
    # direct call with canary buffers: nothing is written on error
    b = B.sizes(8, 64, 2, 32, 0)
    bufs = [np.full(n, 0xA5, dtype=np.uint8) for n in b]
    v = B.View(0, 0, 0, 0, 0, *[x.ctypes.data for x in bufs])
    st_ = B.lib().egt_pack_2bitcsr(w.ctypes.data, 64, bad.ctypes.data, 64, 8, 64, 2, 32, 0, ctypes.byref(v))
    assert st_ == 3 and all(np.all(x == 0xA5) for x in bufs)
    assert B.lib().egt_pack_2bitcsr(None, 64, bad.ctypes.data, 64, 8, 64, 2, 32, 0, ctypes.byref(v)) == 1
    assert B.lib().egt_pack_2bitcsr(w.ctypes.data, 32, bad.ctypes.data, 64, 8, 64, 2, 32, 0, ctypes.byref(v)) == 2


def test_pack_reports_the_first_offending_group_whatever_the_thread_timing():
    # several errors in one matrix: the one of the first offending 4-group in row-major order
    # is returned, every time; a group with both faults reports the mask
    w = synth.weights(600, 64, 6)
    mask = O.prune_n4_magnitude(w, 2)
    overfull = mask.copy()
    overfull[500, 8:12] = 1                    # EGT_ERR_MASK late in the matrix
    wn = w.copy()
    r, c = 20, int(np.argwhere(mask[20] == 1)[3][0])
    wn[r, c] = np.float16(np.inf)              # EGT_ERR_NONFINITE early
    for _ in range(20):
        with pytest.raises(B.EgtError) as e:
            B.pack_2bitcsr(wn, overfull, 2, 32, 0)
        assert e.value.status == 4
    overfull2 = mask.copy()
    overfull2[3, 0:4] = 1
    for _ in range(20):
        with pytest.raises(B.EgtError) as e:
            B.pack_2bitcsr(wn, overfull2, 2, 32, 0)
        assert e.value.status == 3
    both = mask.copy()
    both[r, 4 * (c // 4):4 * (c // 4) + 4] = 1
    with pytest.raises(B.EgtError) as e:
        B.pack_2bitcsr(wn, both, 2, 32, 0)
    assert e.value.status == 3


def test_strided_inputs():
    big = synth.weights(16, 256, 11)
    w = big[:, 64:192]                         # row stride 256, 128 columns
    mask_big = np.zeros((16, 200), dtype=np.uint8)
    mask_big[:, :128] = O.prune_n4_magnitude(np.ascontiguousarray(w), 2)
    mask = mask_big[:, :128]
    p = B.pack_2bitcsr(w, mask, 2, 64, 0)
    _same_packed(p, O.pack_2bitcsr(np.ascontiguousarray(w), np.ascontiguousarray(mask), 2, 64, 0))


@pytest.mark.parametrize("n,g,kind", [(2, 64, 0), (1, 32, 0), (2, 0, 1), (3, 16, 0)])
def test_unpack_matches_oracle_decode(n, g, kind):
    w = synth.weights(40, 256, 31 + n)
    mask = O.prune_n4_magnitude(w, n)
    mask[3, 8:12] = 0
    p = B.pack_2bitcsr(w, mask, n, g, kind)
    o = O.pack_2bitcsr(w, mask, n, g, kind)
    wd, md = B.unpack_2bitcsr(p)
    assert np.array_equal(md, O.mask_from_packed(o))
    assert np.array_equal(wd.view(np.uint16), O.dense_from_packed(o).astype(np.float16).view(np.uint16))
    if kind == 1:                              # FP16 values: pack(unpack(P)) == P byte for byte
        p2 = B.pack_2bitcsr(wd, md, n, g, kind)
        assert np.array_equal(p2.values, p.values) and np.array_equal(p2.idx, p.idx)


def test_unpack_rejects_broken_buffers():
    w = synth.weights(8, 64, 77)
    p = B.pack_2bitcsr(w, O.prune_n4_magnitude(w, 2), 2, 32, 0)
    good = p.row_ptr.copy()
    p.row_ptr[3] += 8
    with pytest.raises(B.EgtError) as e:
        B.unpack_2bitcsr(p)
    assert e.value.status == 5
    p.row_ptr[:] = good
    p.idx[0] = 0x0000                          # offsets 0,0: not ascending
    with pytest.raises(B.EgtError) as e:
        B.unpack_2bitcsr(p)
    assert e.value.status == 5


# ----------------------------------------------------------------- paired nibble order
def test_library_packs_the_handworked_row_in_the_paired_order():
    from helpers import read_fixture
    fx = read_fixture("handworked_1x32.txt")
    w = np.array([float(v) for v in fx["w"]], dtype=np.float16)[None, :]
    mask = np.array([int(v) for v in fx["mask"]], dtype=np.uint8)[None, :]
    p = B.pack_2bitcsr(w, mask, 2, 32, B.VAL_INT4_PAIRED)
    assert p.values.tolist() == [int(v, 16) for v in fx["value_bytes_paired"]]
    assert p.idx.tolist() == [int(v, 16) for v in fx["idx_words"]]
    assert np.asarray(p.qparams).reshape(-1).tolist() == [int(v, 16) for v in fx["qparams"]]


@pytest.mark.parametrize("n,g,drop", [(2, 128, False), (2, 32, True), (1, 64, True), (3, 16, False)])
def test_paired_pack_bit_exact_and_round_trip(n, g, drop):
    w = synth.weights(33, 512, 700 + n + g)
    mask = O.prune_n4_magnitude(w, n)
    if drop:
        mask[np.random.default_rng(g).random(mask.shape) < 0.1] = 0
    p = B.pack_2bitcsr(w, mask, n, g, B.VAL_INT4_PAIRED)
    _same_packed(p, O.pack_2bitcsr(w, mask, n, g, O.VAL_INT4_PAIRED))
    assert B.sizes(33, 512, n, g, B.VAL_INT4_PAIRED) == B.sizes(33, 512, n, g, B.VAL_INT4)
    wd, md = B.unpack_2bitcsr(p)
    wc, mc = B.unpack_2bitcsr(B.pack_2bitcsr(w, mask, n, g, B.VAL_INT4))
    assert np.array_equal(wd.view(np.uint16), wc.view(np.uint16)) and np.array_equal(md, mc)
    nk = np.random.default_rng(n).choice([1, 2], size=33).astype(np.int32)
    mr = np.zeros_like(mask)
    for k in (1, 2):
        mr[nk == k] = O.prune_n4_magnitude(w[nk == k], k)
    pr = B.pack_2bitcsr_rows(w, mr, nk, g, B.VAL_INT4_PAIRED)
    orr = O.pack_2bitcsr_rows(w, mr, nk, g, O.VAL_INT4_PAIRED)
    assert np.array_equal(pr.values, orr["values"]) and np.array_equal(pr.idx, orr["idx"])
    assert L_status_of_fp16_group_rule() == 2


def L_status_of_fp16_group_rule():
    # the paired order follows the INT4 shape rules: a group size is required
    out = (ctypes.c_size_t * 4)()
    return B.lib().egt_2bitcsr_sizes(8, 64, 2, 0, B.VAL_INT4_PAIRED, out)


# ----------------------------------------------------------------- rows of different lengths
def _mixed(R, K, seed, choices=(1, 2), drop=False):
    rng = np.random.default_rng(seed)
    w = synth.weights(R, K, seed)
    nk = rng.choice(choices, size=R).astype(np.int32)
    mask = np.zeros((R, K), dtype=np.uint8)
    for n in np.unique(nk):
        mask[nk == n] = O.prune_n4_magnitude(w[nk == n], int(n))
    if drop:                                   # some groups keep fewer than their row allows: padding slots
        mask[rng.random((R, K)) < 0.1] = 0
    return w, mask, nk


def _same_ragged(p, o):
    assert (p.rows, p.cols, p.n_keep, p.group, p.val_kind, p.total_slots) == \
        (o["rows"], o["cols"], 0, o["group"], o["val_kind"], o["total_slots"])
    for key in ("row_ptr", "idx", "values"):
        assert np.array_equal(getattr(p, key), o[key]), key
    assert (p.qparams is None) if o["qparams"] is None else np.array_equal(p.qparams, o["qparams"])


def test_library_packs_the_handworked_ragged_matrix():
    from helpers import read_fixture
    fx, fx1 = read_fixture("handworked_ragged_2x32.txt"), read_fixture("handworked_1x32.txt")
    w = np.array([[float(v) for v in fx["w0"]], [float(v) for v in fx1["w"]]], dtype=np.float16)
    mask = np.array([[int(v) for v in fx["mask0"]], [int(v) for v in fx1["mask"]]], dtype=np.uint8)
    p = B.pack_2bitcsr_rows(w, mask, [1, 2], 32, B.VAL_INT4)
    assert p.n_keep == 0 and p.total_slots == 24
    assert p.row_ptr.tolist() == [int(v) for v in fx["row_ptr"]]
    assert p.idx.tolist() == [int(v, 16) for v in fx["idx_words"]]
    assert p.values.tolist() == [int(v, 16) for v in fx["value_bytes"]]
    assert np.asarray(p.qparams).reshape(-1).tolist() == [int(v, 16) for v in fx["qparams"]]
    assert list(B.sizes_rows(2, 32, [1, 2], 32, B.VAL_INT4)) == [int(v) for v in fx["sizes"]]
    pf = B.pack_2bitcsr_rows(w, mask, [1, 2], 0, B.VAL_FP16)
    assert np.asarray(pf.values).view(np.uint16).tolist()[:8] == [int(v, 16) for v in fx["fp16_bits0"]]


@pytest.mark.parametrize("choices,g,kind,drop", [((1, 2), 128, 0, False), ((1, 2), 32, 0, True), ((1, 2, 3, 4), 16, 0, True),
                                                 ((1, 2), 0, 1, True), ((2, 4), 12, 0, False)])
def test_ragged_pack_bit_exact_and_round_trip(choices, g, kind, drop):
    R, K = 37, 384
    w, mask, nk = _mixed(R, K, 400 + g, choices, drop)
    p = B.pack_2bitcsr_rows(w, mask, nk, g, kind)
    o = O.pack_2bitcsr_rows(w, mask, nk, g, kind)
    _same_ragged(p, o)
    assert B.sizes_rows(R, K, nk, g, kind) == O.buffer_sizes_rows(K, nk, g, kind) == \
        (p.row_ptr.nbytes, p.values.nbytes, p.idx.nbytes, 0 if p.qparams is None else p.qparams.nbytes)
    wd, md = B.unpack_2bitcsr(p)
    assert np.array_equal(md, O.mask_from_packed_rows(o))
    assert np.array_equal(wd.view(np.uint16), O.dense_from_packed_rows(o).astype(np.float16).view(np.uint16))


def test_ragged_pack_of_equal_rows_is_the_uniform_pack():
    w, mask, _ = _mixed(16, 128, 410, choices=(2,))
    p = B.pack_2bitcsr_rows(w, mask, [2] * 16, 64, 0)
    u = B.pack_2bitcsr(w, mask, 2, 64, 0)
    for key in ("row_ptr", "values", "idx", "qparams"):
        assert np.array_equal(getattr(p, key), getattr(u, key))
    assert p.total_slots == 16 * 64


def test_ragged_pack_and_unpack_errors():
    w, mask, nk = _mixed(8, 64, 420)
    for bad in ([0] + [1] * 7, [5] + [1] * 7):
        with pytest.raises(B.EgtError) as e:
            B.sizes_rows(8, 64, bad, 32, 0)
        assert e.value.status == 2
    with pytest.raises(ValueError):
        B.sizes_rows(8, 64, [1, 2], 32, 0)
    full = O.prune_n4_magnitude(w, 2)
    one = np.array([2, 2, 2, 1, 2, 2, 2, 2], dtype=np.int32)
    with pytest.raises(B.EgtError) as e:        # a 2:4 mask in a row that keeps one entry per 4-group
        B.pack_2bitcsr_rows(w, full, one, 32, 0)
    assert e.value.status == 3
    L = B.lib()
    assert L.egt_pack_2bitcsr_rows(16, 64, 16, 64, 8, 64, None, 32, 0, ctypes.byref(B.View())) == 1
    assert L.egt_2bitcsr_sizes_rows(8, 64, None, 32, 0, (ctypes.c_size_t * 4)()) == 1
    p = B.pack_2bitcsr_rows(w, mask, nk, 32, 0)
    good = p.row_ptr.copy()
    p.row_ptr[3] += 8                           # rows 2 and 3 are no longer whole rows
    with pytest.raises(B.EgtError) as e:
        B.unpack_2bitcsr(p)
    assert e.value.status == 5
    p.row_ptr[:] = good
    p.total_slots += 8                          # the running sum does not end where the view says
    with pytest.raises(B.EgtError) as e:
        B.unpack_2bitcsr(p)
    assert e.value.status == 5


def test_device_entry_points_check_a_ragged_view_without_a_gpu():
    L = B.lib()
    ok = B.View(0, 64, 0, 32, 0, 16, 16, 16, 16, 0)                  # no rows: nothing runs
    assert L.egt_sparse_gemv(ctypes.byref(ok), 16, 16, None) == 0
    odd = B.View(8, 64, 0, 32, 0, 16, 16, 16, 16, 132)               # not whole index words
    assert L.egt_sparse_gemv(ctypes.byref(odd), 16, 16, None) == 2
    big = B.View(8, 64, 0, 32, 0, 16, 16, 16, 16, 8 * 64 + 8)        # more slots than the matrix has entries
    assert L.egt_sparse_gemv(ctypes.byref(big), 16, 16, None) == 2
    items = _fake_items([B.View(64, 4096, 0, 128, 0, 16, 16, 16, 16, 64 * 1024)])
    plan = B.StackPlan()
    assert L.egt_gemv_stack_plan(items, 1, B.STACK_AUTO, None, 0, ctypes.byref(plan)) == 6   # no table form for ragged rows


@pytest.mark.parametrize("g,cols", [(8, 512), (32, 512), (128, 512), (4, 64), (12, 96), (20, 160)])
def test_quant_int4_dense_bit_exact(g, cols):
    w = synth.weights(48, cols, 55 + g)
    q, qp = B.quant_int4(w, g)
    oq, oqp = O.quant_int4_dense(w, g)
    assert np.array_equal(q, oq) and np.array_equal(qp, oqp)


def test_device_entry_points_reject_bad_arguments_without_a_gpu():
    L = B.lib()
    v = B.View(8, 64, 2, 32, 0, 16, 16, 16, 16)          # fake non-null aligned pointers, never used
    assert L.egt_sparse_gemv(None, 16, 16, None) == 1
    assert L.egt_sparse_gemv(ctypes.byref(v), None, 16, None) == 1
    assert L.egt_sparse_gemm_smallm(ctypes.byref(v), 16, 64, 16, 8, 0, None) == 2
    assert L.egt_sparse_gemm_smallm(ctypes.byref(v), 16, 64, 16, 8, 65, None) == 2
    assert L.egt_sparse_gemm_smallm(ctypes.byref(v), 16, 32, 16, 8, 2, None) == 2
    assert L.egt_sparse_gemm_smallm(ctypes.byref(v), 16, 64, 16, 4, 2, None) == 2
    v2 = B.View(8, 48, 2, 16, 0, 16, 16, 16, 16)
    assert L.egt_sparse_gemv(ctypes.byref(v2), 16, 16, None) == 2
    v3 = B.View(8, 64, 2, 32, 0, 16, 16, 16, None)
    assert L.egt_sparse_gemv(ctypes.byref(v3), 16, 16, None) == 1
    v4 = B.View(8, 64, 2, 32, 0, 16, 24, 16, 16)         # misaligned values pointer
    assert L.egt_sparse_gemv(ctypes.byref(v4), 16, 16, None) == 5
    assert L.egt_int4_gemv(None, 16, 8, 64, 32, 16, 16, None) == 1
    assert L.egt_int4_gemv(16, 16, 8, 64, 12, 16, 16, None) == 2       # 64 % 12 != 0
    assert L.egt_int4_gemv(16, 16, 8, 60, 6, 16, 16, None) == 2        # group % 4 != 0
    assert L.egt_int4_gemv(16, 16, 0, 60, 12, 16, 16, None) == 0       # group % 4 == 0 is accepted (empty matrix)
    assert L.egt_stream_read(16, 24, 16, None) == 2
    views = (B.View * 2)(v, B.View(8, 64, 2, 16, 0, 16, 16, 16, 16))       # second view differs in group size
    ptrs = (ctypes.c_void_p * 2)(16, 16)
    assert L.egt_sparse_gemv_batch(views, ptrs, ptrs, 2, None) == 2
    assert L.egt_sparse_gemv_batch(views, ptrs, ptrs, 5, None) == 2
    assert L.egt_sparse_gemv_batch(None, ptrs, ptrs, 1, None) == 1
    assert L.egt_int4_gemv_batch(ptrs, ptrs, 8, 64, 32, ptrs, ptrs, 0, None) == 2
    assert L.egt_sparse_gemm_smallm_batch(views, ptrs, 64, ptrs, 8, 4, 2, None) == 2      # members of different group size
    same = (B.View * 2)(v, v)
    assert L.egt_sparse_gemm_smallm_batch(same, ptrs, 64, ptrs, 8, 4, 0, None) == 2       # count
    assert L.egt_sparse_gemm_smallm_batch(same, ptrs, 64, ptrs, 8, 65, 2, None) == 2      # M
    assert L.egt_sparse_gemm_smallm_batch(same, ptrs, 32, ptrs, 8, 4, 2, None) == 2       # ldx < cols
    assert L.egt_sparse_gemm_smallm_batch(same, ptrs, 64, ptrs, 4, 4, 2, None) == 2       # ldy < rows
    assert L.egt_sparse_gemm_smallm_batch(None, ptrs, 64, ptrs, 8, 4, 2, None) == 1
    nulls = (ctypes.c_void_p * 2)(16, None)
    assert L.egt_sparse_gemm_smallm_batch(same, nulls, 64, ptrs, 8, 4, 2, None) == 1
    odd = (ctypes.c_void_p * 2)(16, 24)
    assert L.egt_sparse_gemm_smallm_batch(same, odd, 64, ptrs, 8, 4, 2, None) == 5        # X off a 16-byte boundary
    assert L.egt_stream_read(None, 32, 16, None) == 1


@pytest.mark.parametrize("n,g,kind", [(2, 128, 0), (1, 64, 0), (2, 0, 1), (3, 32, 2)])
def test_concat_rows_equals_packing_the_stacked_matrix(n, g, kind):
    # q/k/v as one matrix: concatenating three packed matrices gives the bytes of packing their rows stacked
    ws = [synth.weights(r, 256, 8800 + k) for k, r in enumerate((37, 16, 50))]
    masks = [B.prune_n4(w, n) for w in ws]
    fused = B.concat_rows([B.pack_2bitcsr(w, m, n, g, kind) for w, m in zip(ws, masks)])
    whole = B.pack_2bitcsr(np.concatenate(ws), np.concatenate(masks), n, g, kind)
    assert (fused.rows, fused.cols, fused.n_keep, fused.group, fused.val_kind) == (103, 256, n, g, kind)
    for name in ("row_ptr", "values", "idx", "qparams"):
        a, b = getattr(fused, name), getattr(whole, name)
        assert (a is None and b is None) or np.array_equal(a, b), name
    with pytest.raises(ValueError):
        B.concat_rows([B.pack_2bitcsr(ws[0], masks[0], n, g, kind), B.pack_2bitcsr(synth.weights(8, 128, 1), B.prune_n4(synth.weights(8, 128, 1), n), n, g, kind)])


def _fake_items(views, dense=()):
    """Items over fake, aligned, never dereferenced device pointers."""
    n = len(views) + len(dense)
    items = (B.GemvItem * n)()
    for k, v in enumerate(views):
        items[k].sparse = ctypes.pointer(v)
    for k, (rows, cols, group) in enumerate(dense, start=len(views)):
        items[k].q, items[k].qparams, items[k].rows, items[k].cols, items[k].group = 16, 16, rows, cols, group
    for it in items:
        it.x, it.y = 16, 16
    return items


def test_stack_plan_checks_items_and_reports_the_launch_shape():
    L = B.lib()
    # (25 MB of 2:4 and dense matrices: below the 32 MB from which a table is streamed)
    view = B.View(2048, 4096, 2, 128, 0, 16, 16, 16, 16)          # fake aligned device pointers, never used
    down = B.View(2048, 11008, 2, 128, 0, 16, 16, 16, 16)
    one4 = B.View(2048, 11008, 1, 128, 0, 16, 16, 16, 16)
    items = _fake_items([view, down, one4], [(2048, 11008, 128)])
    plan = B.StackPlan()
    assert L.egt_gemv_stack_plan(items, 4, 0, None, 0, ctypes.byref(plan)) == 0          # size query
    # two launches: the 2:4 and dense matrices (tiles per row 1, 3 and 6: six waves), and the 1:4
    # matrix by itself (two tiles per row: four waves; 1376 pieces of x: 8 per thread)
    assert (plan.count, plan.nparts, plan.table_bytes) == (4, 2, 4 * B.STACK_ENTRY_BYTES)
    a, b = plan.part[0], plan.part[1]
    assert (a.count, a.mode, a.block_threads, a.forms, a.table_bytes) == (3, 0, 384, 5, 3 * B.STACK_ENTRY_BYTES)
    assert (b.count, b.mode, b.block_threads, b.forms, b.x_pieces, b.table_bytes) == (1, 0, 256, 2, 8, B.STACK_ENTRY_BYTES)
    assert a.grid_x >= 128 and 0 < a.lds_bytes <= 65536 and 0 < b.lds_bytes <= 65536
    # asked for, both parts walk lists of row blocks: 12 waves for the one, 8 for the 1:4 matrix (two tiles per row)
    res = B.StackPlan()
    assert L.egt_gemv_stack_plan(items, 4, B.STACK_RESIDENT, None, 0, ctypes.byref(res)) == 0
    assert [(res.part[p].mode, res.part[p].block_threads, res.part[p].forms) for p in range(2)] == [(1, 768, 5), (1, 512, 2)]
    table = np.full(4 * B.STACK_ENTRY_BYTES, 0xA5, dtype=np.uint8)
    assert L.egt_gemv_stack_plan(items, 4, 0, table.ctypes.data, table.nbytes - 1, ctypes.byref(plan)) == 2
    assert np.all(table == 0xA5)
    assert L.egt_gemv_stack_plan(items, 4, 0, table.ctypes.data, table.nbytes, ctypes.byref(plan)) == 0
    assert not np.all(table == 0xA5)
    # errors leave table and plan untouched
    table[:] = 0xA5
    plan2 = B.StackPlan(-1)
    bad = B.View(2048, 4096, 2, 0, 1, 16, 16, 16, None)                # FP16 values: no multi-matrix form
    items[1].sparse = ctypes.pointer(bad)
    assert L.egt_gemv_stack_plan(items, 4, 0, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 6
    assert np.all(table == 0xA5) and plan2.count == -1
    items[1].sparse = ctypes.pointer(down)
    items[3].group = 96                                                # 11008 % 96 != 0
    assert L.egt_gemv_stack_plan(items, 4, 0, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 2
    items[3].group = 64                                                # dense groups below 128: not in this form
    assert L.egt_gemv_stack_plan(items, 4, 0, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 6
    items[3].group = 128
    items[2].x = 24
    assert L.egt_gemv_stack_plan(items, 4, 0, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 5
    items[2].x = None
    assert L.egt_gemv_stack_plan(items, 4, 0, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 1
    items[2].x = 16
    assert L.egt_gemv_stack_plan(items, 0, 0, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 2
    assert L.egt_gemv_stack_plan(None, 4, 0, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 1
    wide = B.View(64, 16384, 2, 128, 0, 16, 16, 16, 16)                # four tiles per row beside three: twelve waves
    items[0].sparse = ctypes.pointer(wide)
    assert L.egt_gemv_stack_plan(items, 4, 0, None, 0, ctypes.byref(plan2)) == 0 and plan2.block_threads == 768
    # the run call checks the plan before anything is launched
    assert L.egt_gemv_stack_run(None, ctypes.byref(plan), None) == 1
    assert L.egt_gemv_stack_run(24, ctypes.byref(plan), None) == 5
    for field, value in (("count", 0), ("block_threads", 100), ("block_threads", 2048), ("lds_bytes", 1 << 20), ("x_pieces", 3),
                         ("forms", 0), ("forms", 8), ("forms", 3), ("mode", 2)):
        for part in range(plan.nparts):
            broken = B.StackPlan.from_buffer_copy(plan)
            setattr(broken.part[part], field, value)
            assert L.egt_gemv_stack_run(16, ctypes.byref(broken), None) == 2, (field, part)
    empty = B.StackPlan.from_buffer_copy(plan)
    for part in range(empty.nparts):
        empty.part[part].grid_x = 0
    assert L.egt_gemv_stack_run(16, ctypes.byref(empty), None) == 0       # all matrices empty: nothing to launch


def test_gemm_stack_plan_checks_items_and_reports_the_launch_shape():
    L = B.lib()
    views = [B.View(4096, 4096, 2, 128, 0, 16, 16, 16, 16), B.View(4096, 11008, 2, 128, 0, 16, 16, 16, 16),
             B.View(0, 4096, 2, 128, 0, None, None, None, None)]
    items = (B.GemmItem * 3)()
    for k, v in enumerate(views):
        items[k].sparse, items[k].X, items[k].Y = ctypes.pointer(v), 16, 16
    plan = B.GemmPlan()
    assert L.egt_gemm_stack_plan(items, 3, 16, None, 0, ctypes.byref(plan)) == 0
    # up to 16 tokens: workgroups of 8 waves that own a row tile each (the tallest matrix has 256 tiles);
    # two regions of four K-steps of eight pairs of token rows of 1056 bytes
    # (the launch: 32 workgroups for each of the two matrices with rows, named in a list behind the descriptors)
    assert (plan.count, plan.M, plan.grid_x, plan.block_threads, plan.lds_bytes, plan.table_bytes) == \
        (3, 16, 64, 512, 2 * 4 * 8 * 1056, 3 * B.STACK_ENTRY_BYTES + 4 * 64)
    wide = B.GemmPlan()
    assert L.egt_gemm_stack_plan(items, 3, 17, None, 0, ctypes.byref(wide)) == 0
    # up to 32 tokens: two token groups, rounds of two K-steps; beyond: four groups, 16 waves
    assert (wide.grid_x, wide.block_threads, wide.lds_bytes) == (64, 512, 2 * 2 * 2 * 8 * 1056)
    assert L.egt_gemm_stack_plan(items, 3, 33, None, 0, ctypes.byref(wide)) == 0
    assert (wide.grid_x, wide.block_threads, wide.lds_bytes) == (32, 1024, 2 * 4 * 2 * 8 * 1056)
    table = np.full(3 * B.STACK_ENTRY_BYTES + 4 * 64, 0xA5, dtype=np.uint8)
    assert L.egt_gemm_stack_plan(items, 3, 16, table.ctypes.data, table.nbytes - 1, ctypes.byref(plan)) == 2
    assert np.all(table == 0xA5)
    assert L.egt_gemm_stack_plan(items, 3, 16, table.ctypes.data, table.nbytes, ctypes.byref(plan)) == 0
    assert not np.all(table == 0xA5)
    # the descriptors stand in the order of falling row length (11008 columns = 172 chunks first; geometry behind six
    # pointers: rows, tokens, chunks), the list names matrix and place for every workgroup
    geom = table[:3 * B.STACK_ENTRY_BYTES].reshape(3, B.STACK_ENTRY_BYTES)[:, 48:60].copy().view(np.int32)
    assert geom.tolist() == [[4096, 16, 172], [4096, 16, 64], [0, 16, 64]]
    wgs = table[3 * B.STACK_ENTRY_BYTES:].view(np.uint32)
    assert np.array_equal(wgs >> 16, np.repeat([0, 1], 32)) and np.array_equal(wgs & 0xFFFF, np.tile(np.arange(32), 2))
    # errors leave table and plan untouched
    table[:] = 0xA5
    plan2 = B.GemmPlan(-1)
    for M in (1, 65):
        assert L.egt_gemm_stack_plan(items, 3, M, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 2
    assert L.egt_gemm_stack_plan(items, 0, 16, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 2
    assert L.egt_gemm_stack_plan(None, 3, 16, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 1
    items[1].X = None
    assert L.egt_gemm_stack_plan(items, 3, 16, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 1
    items[1].X = 24
    assert L.egt_gemm_stack_plan(items, 3, 16, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 5
    items[1].X = 16
    # (1:4 beside 2:4, 1:4 with groups below 128, 2:4 with groups below 64, FP16 values)
    for bad in (B.View(64, 4096, 1, 128, 0, 16, 16, 16, 16), B.View(64, 4096, 2, 32, 0, 16, 16, 16, 16),
                B.View(64, 4096, 2, 0, 1, 16, 16, 16, None)):
        items[0].sparse = ctypes.pointer(bad)
        assert L.egt_gemm_stack_plan(items, 3, 17, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 6
    assert np.all(table == 0xA5) and plan2.count == -1
    short = B.View(64, 64, 2, 64, 0, 16, 16, 16, 16)        # a single chunk of 64 columns
    items[0].sparse = ctypes.pointer(short)
    assert L.egt_gemm_stack_plan(items, 3, 17, table.ctypes.data, table.nbytes, ctypes.byref(plan2)) == 0
    assert not np.all(table == 0xA5) and plan2.count == 3
    # a table of 1:4 matrices: rounds of two K-steps of 512 columns, sixteen token rows of 1040 bytes per K-step
    one4 = (B.GemmItem * 2)()
    v14 = [B.View(4096, 4096, 1, 128, 0, 16, 16, 16, 16), B.View(11008, 4096, 1, 256, 0, 16, 16, 16, 16)]
    for k, v in enumerate(v14):
        one4[k].sparse, one4[k].X, one4[k].Y = ctypes.pointer(v), 16, 16
    p14 = B.GemmPlan()
    assert L.egt_gemm_stack_plan(one4, 2, 16, None, 0, ctypes.byref(p14)) == 0
    assert (p14.n_keep, p14.grid_x, p14.block_threads, p14.lds_bytes) == (1, 32 + 86, 512, 2 * 2 * 16 * 1040)
    assert L.egt_gemm_stack_plan(one4, 2, 32, None, 0, ctypes.byref(p14)) == 0
    assert (p14.n_keep, p14.grid_x, p14.block_threads, p14.lds_bytes) == (1, 16 + 43, 1024, 2 * 2 * 2 * 16 * 1040)
    assert L.egt_gemm_stack_plan(one4, 2, 33, None, 0, ctypes.byref(p14)) == 6
    v14[1].group_size = 64
    assert L.egt_gemm_stack_plan(one4, 2, 16, None, 0, ctypes.byref(p14)) == 6
    assert plan.n_keep == 2
    # the run call checks the plan before anything is launched
    assert L.egt_gemm_stack_run(None, ctypes.byref(plan), None) == 1
    assert L.egt_gemm_stack_run(24, ctypes.byref(plan), None) == 5
    for field, value in (("count", 0), ("M", 1), ("M", 40), ("n_keep", 0), ("n_keep", 3), ("grid_x", -1), ("grid_x", 1 << 21), ("block_threads", 256), ("lds_bytes", 1024),
                         ("table_bytes", 160)):
        broken = B.GemmPlan.from_buffer_copy(plan)
        setattr(broken, field, value)
        assert L.egt_gemm_stack_run(16, ctypes.byref(broken), None) == 2, field


def test_stack_plan_cuts_a_large_table_into_row_blocks():
    # three decoder layers of 2:4 and dense INT4 matrices (more than 256 MB): resident
    # workgroups walk a list of row blocks; the list covers every row of every matrix exactly once
    L = B.lib()
    layer = [B.View(r, c, 2, 128, 0, 16, 16, 16, 16) for (_, r, c) in synth.LAYER_MATRICES]
    dense = [(r, c, 128) for (_, r, c) in synth.LAYER_MATRICES]
    items = _fake_items(layer + layer, dense)
    plan = B.StackPlan()
    assert L.egt_gemv_stack_plan(items, 21, B.STACK_AUTO, None, 0, ctypes.byref(plan)) == 0
    assert (plan.mode, plan.block_threads, plan.forms) == (1, 768, 5)      # tiles per row 1, 2, 3, 6: twelve waves
    assert plan.grid_x == 512 and plan.nitems >= plan.grid_x               # 300 MB: two spans per compute unit
    first_bytes = (4 * (plan.grid_x + 1) + 15) // 16 * 16
    assert plan.table_bytes == 21 * B.STACK_ENTRY_BYTES + first_bytes + 16 * plan.nitems
    table = np.zeros(plan.table_bytes, dtype=np.uint8)
    assert L.egt_gemv_stack_plan(items, 21, B.STACK_AUTO, table.ctypes.data, table.nbytes, ctypes.byref(plan)) == 0
    off = 21 * B.STACK_ENTRY_BYTES
    first = table[off:off + 4 * (plan.grid_x + 1)].view(np.uint32)
    work = table[off + first_bytes:].view(np.uint32).reshape(-1, 4)
    assert first[0] == 0 and first[-1] == plan.nitems and np.all(np.diff(first.astype(np.int64)) >= 0)
    rows = [r for (_, r, _) in synth.LAYER_MATRICES] * 3
    cols = [c for (_, _, c) in synth.LAYER_MATRICES] * 3
    row_bytes = [c // 4 + c // 8 + 4 * (c // 128) if k < 14 else c // 2 + 4 * (c // 128) for k, c in enumerate(cols)]
    covered = [np.zeros(r, dtype=np.int32) for r in rows]
    per_block = np.zeros(plan.grid_x, dtype=np.int64)
    for b in range(plan.grid_x):
        for m, r0, n, _ in work[first[b]:first[b + 1]]:
            desc = table[m * B.STACK_ENTRY_BYTES:(m + 1) * B.STACK_ENTRY_BYTES].view(np.int32)
            item_rows = int(desc[21])                   # six pointers, form, rows, nchunks, phases, gshift, groups, 3 extents, item_rows
            assert 0 < n <= item_rows <= 2048 and 16 * int(desc[15]) * item_rows <= 24 * 1024
            covered[m][r0:r0 + n] += 1
            per_block[b] += int(n) * row_bytes[m]
    assert all(np.all(c == 1) for c in covered)         # every row of every matrix exactly once
    # every workgroup streams the same number of bytes, to within one row, and a contiguous stretch
    assert per_block.max() - per_block.min() <= 2 * max(row_bytes)
    flat = [(int(m), int(r0)) for m, r0, _, _ in work]
    assert flat == sorted(flat)
    # a table of 1:4 matrices: workgroups of eight waves; an item starts on a tile (two rows of 4096 columns, four
    # of 2048) and every row is covered exactly once
    shapes14 = [(4097, 4096), (1001, 2048), (4099, 11008), (11008, 4096), (130, 8192)]
    it14 = _fake_items([B.View(r, c, 1, 128, 0, 16, 16, 16, 16) for (r, c) in shapes14])
    p14 = B.StackPlan()
    assert L.egt_gemv_stack_plan(it14, 5, B.STACK_RESIDENT, None, 0, ctypes.byref(p14)) == 0       # (21 MB: asked for)
    assert (p14.nparts, p14.mode, p14.block_threads, p14.forms) == (1, 1, 512, 2)
    t14 = np.zeros(p14.table_bytes, dtype=np.uint8)
    assert L.egt_gemv_stack_plan(it14, 5, B.STACK_RESIDENT, t14.ctypes.data, t14.nbytes, ctypes.byref(p14)) == 0
    off14 = 5 * B.STACK_ENTRY_BYTES
    fb14 = (4 * (p14.grid_x + 1) + 15) // 16 * 16
    first14 = t14[off14:off14 + 4 * (p14.grid_x + 1)].view(np.uint32)
    work14 = t14[off14 + fb14:].view(np.uint32).reshape(-1, 4)
    assert first14[0] == 0 and first14[-1] == p14.nitems == len(work14)
    cov14 = [np.zeros(r, dtype=np.int32) for (r, _) in shapes14]
    for m, r0, n, _ in work14:
        desc = t14[m * B.STACK_ENTRY_BYTES:(m + 1) * B.STACK_ENTRY_BYTES].view(np.int32)
        rpt = {4096: 2, 2048: 4}.get(shapes14[m][1], 1)
        assert int(desc[22]) == {4096: 5, 2048: 4}.get(shapes14[m][1], -1)          # log2(chunks per row) where a tile holds several rows
        assert r0 % rpt == 0 and 0 < n <= int(desc[21]) and int(desc[21]) % rpt == 0
        assert 16 * int(desc[15]) * -(-int(n) // rpt) <= 24 * 1024                  # the item's partial sums fit their LDS share
        cov14[m][r0:r0 + n] += 1
    assert all(np.all(c == 1) for c in cov14)
    # a smaller table keeps the short-lived workgroups unless the caller asks otherwise
    one = _fake_items(layer[:4])
    assert L.egt_gemv_stack_plan(one, 4, B.STACK_AUTO, None, 0, ctypes.byref(plan)) == 0 and plan.mode == 0
    assert L.egt_gemv_stack_plan(one, 4, B.STACK_RESIDENT, None, 0, ctypes.byref(plan)) == 0 and plan.mode == 1
    assert L.egt_gemv_stack_plan(items, 21, B.STACK_GRID, None, 0, ctypes.byref(plan)) == 0 and plan.mode == 0
    assert L.egt_gemv_stack_plan(items, 21, 3, None, 0, ctypes.byref(plan)) == 2
    narrow = _fake_items([B.View(4096, 1024, 2, 128, 0, 16, 16, 16, 16)])      # several rows per tile: no resident form
    assert L.egt_gemv_stack_plan(narrow, 1, B.STACK_RESIDENT, None, 0, ctypes.byref(plan)) == 6
    # inconsistent mode-1 plans are refused
    assert L.egt_gemv_stack_plan(items, 21, B.STACK_AUTO, None, 0, ctypes.byref(plan)) == 0
    for field, value in (("nitems", 0), ("grid_x", plan.nitems + 1), ("table_bytes", 5), ("part_offset", 1 << 20), ("forms", 7)):
        broken = B.StackPlan.from_buffer_copy(plan)
        setattr(broken.part[0], field, value)
        assert L.egt_gemv_stack_run(16, ctypes.byref(broken), None) == 2, field
    for field, value in (("nparts", 0), ("nparts", 3), ("count", 20), ("table_bytes", plan.table_bytes + 16)):
        broken = B.StackPlan.from_buffer_copy(plan)
        setattr(broken, field, value)
        assert L.egt_gemv_stack_run(16, ctypes.byref(broken), None) == 2, field


def test_smallm_workspace_size_query():
    L = B.lib()
    out = ctypes.c_size_t(7)
    down = B.View(4096, 11008, 2, 128, 0, 16, 16, 16, 16)
    # 64 tokens, K = 11008: X held in LDS, 43 steps in 11 slices, 16 x 16 FP32 sums per (slice, row tile, token group)
    assert L.egt_sparse_gemm_smallm_ws_bytes(ctypes.byref(down), 11008, 64, ctypes.byref(out)) == 0 and out.value == 11 * 256 * 4 * 1024
    # 17..32 tokens there: four slices of K, X fetched per workgroup, partial sums per token and row
    assert L.egt_sparse_gemm_smallm_ws_bytes(ctypes.byref(down), 11008, 32, ctypes.byref(out)) == 0 and out.value == 4 * 4 * 32 * 4096
    assert L.egt_sparse_gemm_smallm_ws_bytes(ctypes.byref(down), 11008, 16, ctypes.byref(out)) == 0 and out.value == 0
    gate = B.View(11008, 4096, 2, 128, 0, 16, 16, 16, 16)
    assert L.egt_sparse_gemm_smallm_ws_bytes(ctypes.byref(gate), 4096, 64, ctypes.byref(out)) == 0 and out.value == 4 * 688 * 4 * 1024
    assert L.egt_sparse_gemm_smallm_ws_bytes(ctypes.byref(gate), 4096, 32, ctypes.byref(out)) == 0 and out.value == 0
    assert L.egt_sparse_gemm_smallm_ws_bytes(ctypes.byref(gate), 4100, 64, ctypes.byref(out)) == 0 and out.value == 0   # rows of X not on 16 bytes
    square = B.View(4096, 4096, 2, 128, 0, 16, 16, 16, 16)
    assert L.egt_sparse_gemm_smallm_ws_bytes(ctypes.byref(square), 4096, 64, ctypes.byref(out)) == 0 and out.value == 0
    assert L.egt_sparse_gemm_smallm_ws_bytes(ctypes.byref(down), 11008, 65, ctypes.byref(out)) == 2
    assert L.egt_sparse_gemm_smallm_ws_bytes(ctypes.byref(down), 100, 64, ctypes.byref(out)) == 2
    assert L.egt_sparse_gemm_smallm_ws_bytes(ctypes.byref(down), 11008, 64, None) == 1
    assert L.egt_sparse_gemm_smallm_ws_bytes(None, 11008, 64, ctypes.byref(out)) == 1
    # the device call checks its arguments before anything is launched
    assert L.egt_sparse_gemm_smallm_ws(ctypes.byref(down), 16, 11008, 16, 4096, 64, None, 0, None) == 1
    assert L.egt_sparse_gemm_smallm_ws(ctypes.byref(down), 16, 11008, 16, 4096, 64, 16, 100, None) == 2
    assert L.egt_sparse_gemm_smallm_ws(ctypes.byref(down), 16, 11008, 16, 4096, 64, 24, 1 << 30, None) == 5
    assert L.egt_sparse_gemm_smallm_ws(ctypes.byref(down), 16, 11008, 16, 100, 64, 16, 1 << 30, None) == 2


def test_trigger_cost_model():
    # exact line is recovered; noisy points match the oracle's least squares
    m = [1, 2, 4, 8, 16, 32, 64]
    a, b = B.fit_verify_cost(m, [3.0 + 0.25 * v for v in m])
    assert a == pytest.approx(3.0) and b == pytest.approx(0.25)
    rng = np.random.default_rng(4)
    t = [5.0 + 0.4 * v + rng.normal(0, 0.3) for v in m]
    assert B.fit_verify_cost(m, t) == pytest.approx(O.fit_verify_cost(m, t))
    with pytest.raises(B.EgtError):
        B.fit_verify_cost([4, 4], [1.0, 2.0])
    # trie wide at the top, narrow at the bottom: candidates shrink with depth
    cand = [64, 24, 9, 4, 2, 1]
    rem = [6, 5, 4, 3, 2, 1]
    for t_ar, aa, bb in [(10.0, 8.0, 0.5), (10.0, 8.0, 2.0), (1.0, 50.0, 1.0), (10.0, 0.0, 0.0)]:
        assert B.trigger_depth(t_ar, aa, bb, cand, rem) == pytest.approx(O.trigger_depth(t_ar, aa, bb, cand, rem))
    # closed form: with a flat verification cost (b = 0) the earliest depth wins;
    # when verifying never pays, the answer is "never" (-1)
    assert B.trigger_depth(10.0, 8.0, 0.0, cand, rem)[0] == 0
    assert B.trigger_depth(1.0, 50.0, 1.0, cand, rem) == (-1, 0.0)
    # brute force over all depths
    gains = [r * 10.0 - (8.0 + 2.0 * c) for c, r in zip(cand, rem)]
    assert B.trigger_depth(10.0, 8.0, 2.0, cand, rem)[0] == int(np.argmax(gains))
