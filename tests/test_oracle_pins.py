"""Pins for the CPU oracle: hand-worked bytes, closed forms, invariants, brute
force, textbook reductions.  None of these re-uses the oracle's own formulas."""
import itertools

import numpy as np
import pytest
import scipy.sparse

from oracle import egt_oracle as O
from paper_2605_11582_amd import synth
from helpers import read_fixture


def _rand_w(R, K, seed, scale=0.02):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((R, K)) * scale).astype(np.float16)


def _rand_x(K, seed):
    return np.random.default_rng(seed).standard_normal(K).astype(np.float16)


# ----------------------------------------------------------------- fixture
def _fixture():
    fx = read_fixture("handworked_1x32.txt")
    w = np.array([float(v) for v in fx["w"]], dtype=np.float16)[None, :]
    mask = np.array([int(v) for v in fx["mask"]], dtype=np.uint8)[None, :]
    return fx, w, mask


def test_handworked_int4_bytes():
    fx, w, mask = _fixture()
    p = O.pack_2bitcsr(w, mask, 2, 32, O.VAL_INT4)
    assert [int(v, 16) for v in fx["idx_words"]] == p["idx"].tolist()
    assert [int(v, 16) for v in fx["value_bytes"]] == p["values"].tolist()
    assert [int(v, 16) for v in fx["qparams"]] == p["qparams"].reshape(-1).tolist()
    assert [int(v) for v in fx["row_ptr"]] == p["row_ptr"].tolist()
    col, w_hat, q = O.decode_2bitcsr(p)
    assert [int(v) for v in fx["offs"]] == (col[0] % 4).tolist()
    assert [int(v) for v in fx["q"]] == q[0].tolist()
    x = np.arange(1, 33).astype(np.float16)
    y, a = O.gemv(p, x)
    assert y[0] == float(fx["y"][0]) and a[0] == float(fx["abs_sum"][0])


def test_handworked_fp16_bytes():
    fx, w, mask = _fixture()
    p = O.pack_2bitcsr(w, mask, 2, 0, O.VAL_FP16)
    assert [int(v, 16) for v in fx["fp16_bits"]] == p["values"].view(np.uint16).tolist()
    assert [int(v, 16) for v in fx["idx_words"]] == p["idx"].tolist()
    assert p["qparams"] is None
    y, _ = O.gemv(p, np.arange(1, 33).astype(np.float16))
    assert y[0] == float(fx["y_fp16"][0])


def test_handworked_quantiser_cases():
    fx = read_fixture("handworked_quantiser.txt")
    for name in ("all_positive", "all_negative", "rounded_scale_up", "rounded_scale_dn", "nothing_kept"):
        vmin, vmax, bits, zero = fx[name]
        s16, z = O.quant_params(np.array([float(vmin)]), np.array([float(vmax)]))
        assert int(s16.view(np.uint16)[0]) == int(bits, 16), name
        assert float(z[0]) == float(zero), name
    # an entry the mask drops does not widen the range of its group
    w = np.zeros((1, 32), dtype=np.float16)
    mask = np.zeros((1, 32), dtype=np.uint8)
    w[0, :4] = [float(v) for v in fx["row_w"]]
    mask[0, :4] = [int(v) for v in fx["row_mask"]]
    p = O.pack_2bitcsr(w, mask, 2, 32, O.VAL_INT4)
    assert p["qparams"].reshape(-1).tolist() == [int(v, 16) for v in fx["row_qparams"]]
    assert p["values"].tolist() == [int(v, 16) for v in fx["row_value_bytes"]]
    assert p["idx"].tolist() == [int(v, 16) for v in fx["row_idx_words"]]


# ----------------------------------------------------------------- trigger cost model
def test_fit_of_an_exact_line_and_against_polyfit():
    m = [1, 2, 4, 8, 16, 32, 64]
    a, b = O.fit_verify_cost(m, [3.0 + 0.25 * v for v in m])
    assert a == pytest.approx(3.0) and b == pytest.approx(0.25)
    t = [34.0, 38.5, 45.0, 49.5, 55.0, 71.0, 115.0]
    slope, icpt = np.polyfit(np.array(m, dtype=np.float64), np.array(t), 1)     # library least squares
    a, b = O.fit_verify_cost(m, t)
    assert a == pytest.approx(icpt) and b == pytest.approx(slope)


def test_trigger_depth_worked_by_hand():
    # t_ar = 10, a = 8, b = 2: gains per depth are
    #   6*10-(8+2*64) = -76, 5*10-(8+48) = -6, 4*10-(8+18) = 14, 3*10-(8+8) = 14, 2*10-(8+4) = 8, 10-(8+2) = 0
    # the largest gain, 14, is reached first at depth 2
    cand, rem = [64, 24, 9, 4, 2, 1], [6, 5, 4, 3, 2, 1]
    assert O.trigger_depth(10.0, 8.0, 2.0, cand, rem) == (2, 14.0)
    # a flat cost (b = 0): the depth with the most tokens left wins, gain 60 - 8
    assert O.trigger_depth(10.0, 8.0, 0.0, cand, rem) == (0, 52.0)
    # verification dearer than everything it saves: never trigger
    assert O.trigger_depth(1.0, 50.0, 1.0, cand, rem) == (-1, 0.0)


# ----------------------------------------------------------------- size model
def test_size_ratio_30_percent():
    # the paper's figure: index + weights = 30 % of the original CSR
    m = O.size_model(11008, 4096, 2, value_bits=4, csr_index_bits=16)
    assert m["ratio"] == pytest.approx(6 / 20) and m["ratio"] == pytest.approx(0.30)
    assert O.size_model(64, 64, 2, 16, 32)["ratio"] == pytest.approx(18 / 48)       # 37.5 %
    assert O.size_model(64, 64, 2, 16, 16)["ratio"] == pytest.approx(18 / 32)       # 56.25 %
    # INT4 + 2 bit + group-128 parameters against FP16 + int32 CSR: 6.5 / 48
    m = O.size_model(128, 1024, 2, 4, 32, group=128, csr_value_bits=16)
    assert m["ratio"] == pytest.approx(6.5 / 48)
    # 1:4 has the same per-non-zero ratio
    assert O.size_model(64, 64, 1, 4, 16)["ratio"] == pytest.approx(0.30)


def test_buffer_sizes_closed_form():
    assert O.buffer_sizes(11008, 4096, 2, 128, O.VAL_INT4) == (44036, 11272192, 5636096, 1409024)
    assert O.buffer_sizes(11008, 4096, 2, 0, O.VAL_FP16) == (44036, 45088768, 5636096, 0)
    assert O.buffer_sizes(4096, 11008, 1, 128, O.VAL_INT4) == (16388, 4096 * 2752 // 2, 4096 * 2752 // 4, 4096 * 86 * 4)
    w = _rand_w(8, 64, 1)
    for n, kind, g in [(2, O.VAL_INT4, 32), (1, O.VAL_INT4, 16), (2, O.VAL_FP16, 0), (4, O.VAL_INT4, 64)]:
        p = O.pack_2bitcsr(w, O.prune_n4_magnitude(w, n), n, g, kind)
        sizes = O.buffer_sizes(8, 64, n, g, kind)
        got = (p["row_ptr"].nbytes, p["values"].nbytes, p["idx"].nbytes,
               0 if p["qparams"] is None else p["qparams"].nbytes)
        assert got == sizes


# ----------------------------------------------------------------- pruning
@pytest.mark.parametrize("n", [1, 2, 3])
def test_prune_is_top_n_by_sort(n):
    w = _rand_w(16, 64, 7)
    w[0, :8] = np.float16(0.5)                 # ties -> lower column wins
    w[1, 4:8] = [0.0, -0.0, 0.25, -0.25]
    mask = O.prune_n4_magnitude(w, n)
    assert np.all(mask.reshape(16, 16, 4).sum(axis=2) == n)
    for r in range(16):
        for c in range(16):
            grp = np.abs(w[r, 4 * c:4 * c + 4].astype(np.float64))
            order = sorted(range(4), key=lambda j: (-grp[j], j))
            expect = np.zeros(4, dtype=np.uint8)
            expect[order[:n]] = 1
            assert np.array_equal(mask[r, 4 * c:4 * c + 4], expect)


def test_prune_equals_eq3_ranking_with_constant_statistics():
    # Eq. (3) with a constant activation norm and gradient ranks like |w|
    w = _rand_w(8, 32, 3)
    score = O.importance_eq3(w, np.full(32, 1.7), np.full((8, 32), 0.3))
    mask = O.prune_n4_magnitude(w, 2)
    s = score.reshape(8, 8, 4)
    top2 = np.argsort(-s, axis=2, kind="stable")[:, :, :2]
    expect = np.zeros_like(s, dtype=np.uint8)
    np.put_along_axis(expect, top2, 1, axis=2)
    assert np.array_equal(mask, expect.reshape(8, 32))


@pytest.mark.parametrize("n", [1, 2, 3])
def test_importance_pruning_is_top_n_of_eq3_by_exact_arithmetic(n):
    # brute force with exact rationals: score = |w| * norm + |w| * grad, largest n per
    # 4-group, ties to the lower column.  Inputs are small dyadic numbers so the float64
    # evaluation in the oracle is exact and must agree with the rational one.
    from fractions import Fraction
    rng = np.random.default_rng(40 + n)
    w = (rng.integers(-8, 9, size=(6, 16)) / 8.0).astype(np.float16)      # many ties, zeros
    norm = rng.integers(0, 5, size=16) / 4.0
    grad = rng.integers(0, 3, size=(6, 16)) / 2.0
    mask = O.prune_n4_importance(w, norm, grad, n)
    for r in range(6):
        for c in range(0, 16, 4):
            sc = [abs(Fraction(float(w[r, c + j]))) * Fraction(float(norm[c + j])) +
                  abs(Fraction(float(w[r, c + j]))) * Fraction(float(grad[r, c + j])) for j in range(4)]
            order = sorted(range(4), key=lambda j: (-sc[j], j))
            expect = np.zeros(4, dtype=np.uint8)
            expect[order[:n]] = 1
            assert np.array_equal(mask[r, c:c + 4], expect), (r, c)


def test_importance_pruning_special_cases():
    w = _rand_w(8, 32, 5)
    # constant statistics: the magnitude mask
    assert np.array_equal(O.prune_n4_importance(w, np.full(32, 0.75), None, 2), O.prune_n4_magnitude(w, 2))
    # all scores zero: the lower columns win
    m = O.prune_n4_importance(w, np.zeros(32), None, 2)
    assert np.array_equal(m.reshape(8, 8, 4), np.broadcast_to(np.array([1, 1, 0, 0], np.uint8), (8, 8, 4)))
    # a huge activation norm on column 4c+3 forces that column in (unless its weight is 0)
    norm = np.ones(32)
    norm[3::4] = 1e6
    m = O.prune_n4_importance(w, norm, None, 1)
    nz = np.asarray(w, dtype=np.float16)[:, 3::4] != 0
    assert np.all(m[:, 3::4][nz] == 1)
    # the gradient term alone can decide: zero norms, gradient only on column 4c+2
    grad = np.zeros((8, 32))
    grad[:, 2::4] = 1.0
    m = O.prune_n4_importance(w, np.zeros(32), grad, 1)
    nz = np.asarray(w, dtype=np.float16)[:, 2::4] != 0
    assert np.all(m[:, 2::4][nz] == 1)


def test_row_groups_reduce_to_separate_packs_of_each_class():
    # rows quantised with their own group size = the rows of a pack with that group size,
    # its parameters repeated down to the stored granularity; decode sees no difference
    rng = np.random.default_rng(77)
    R, K, g = 12, 256, 32
    w = _rand_w(R, K, 77)
    mask = O.prune_n4_magnitude(w, 2)
    rg = rng.choice([32, 64, 128, 256], size=R)
    p = O.pack_2bitcsr(w, mask, 2, g, 0, row_group=rg)
    assert p["qparams"].shape == (R, K // g, 2) and p["group"] == g
    W = O.dense_from_packed(p)
    for gr in (32, 64, 128, 256):
        sel = np.nonzero(rg == gr)[0]
        if len(sel) == 0:
            continue
        ref = O.pack_2bitcsr(w[sel], mask[sel], 2, gr, 0)
        assert np.array_equal(np.repeat(ref["qparams"], gr // g, axis=1), p["qparams"][sel])
        assert np.array_equal(O.dense_from_packed(ref), W[sel])
    # a coarser group can only widen the range: its scale is at least the finer group's
    fine = O.pack_2bitcsr(w, mask, 2, g, 0)
    s_f = fine["qparams"][:, :, 0].view(np.float16).astype(np.float64)
    s_c = p["qparams"][:, :, 0].view(np.float16).astype(np.float64)
    assert np.all(s_c >= s_f)
    with pytest.raises(ValueError):
        O.pack_2bitcsr(w, mask, 2, g, 0, row_group=np.full(R, 48))


# ----------------------------------------------------------------- structure
@pytest.mark.parametrize("n,kind,g", [(2, 0, 32), (1, 0, 32), (2, 1, 0), (3, 0, 16), (4, 0, 64)])
def test_structure_invariants(n, kind, g):
    R, K = 12, 128
    w = _rand_w(R, K, 11 + n)
    p = O.pack_2bitcsr(w, O.prune_n4_magnitude(w, n), n, g, kind)
    S = n * K // 4
    assert np.all(np.diff(p["row_ptr"].astype(np.int64)) == S)
    assert p["row_ptr"][-1] == n * R * K // 4
    # decode the index words by hand: 8 fields of 2 bits, low bits first
    fields = np.array([[(int(wd) >> (2 * k)) & 3 for k in range(8)] for wd in p["idx"]]).reshape(R, K // 4, n)
    assert np.all(np.diff(fields, axis=2) > 0) if n > 1 else True
    assert fields.min() >= 0 and fields.max() <= 3
    if kind == 0:
        assert p["values"].size == R * S // 2
        z = p["qparams"][:, :, 1].view(np.float16).astype(np.float64)
        assert np.all(z == np.rint(z)) and z.min() >= 0 and z.max() <= 15


def test_overfull_group_is_an_error():
    w = _rand_w(2, 32, 5)
    mask = O.prune_n4_magnitude(w, 2)
    mask[1, 4:8] = [1, 1, 1, 0]
    with pytest.raises(ValueError):
        O.pack_2bitcsr(w, mask, 2, 32, O.VAL_INT4)


def test_nonfinite_kept_weight_is_an_error():
    w = _rand_w(2, 32, 5)
    mask = O.prune_n4_magnitude(w, 2)
    r, c = np.argwhere(mask == 1)[3]
    w[r, c] = np.float16(np.inf)
    with pytest.raises(FloatingPointError):
        O.pack_2bitcsr(w, mask, 2, 32, O.VAL_INT4)


# ----------------------------------------------------------------- round trips
def test_fp16_round_trip_returns_original_bits():
    w = _rand_w(16, 96, 21)
    mask = O.prune_n4_magnitude(w, 2)
    p = O.pack_2bitcsr(w, mask, 2, 0, O.VAL_FP16)
    W = O.dense_from_packed(p)
    assert np.array_equal(W, np.where(mask == 1, w.astype(np.float64), 0.0))
    assert np.array_equal(O.mask_from_packed(p), mask)


def test_padding_slots_and_fp16_idempotence():
    w = _rand_w(16, 128, 22)
    mask = O.prune_n4_magnitude(w, 2)
    mask[3, 8:12] = [0, 0, 1, 0]             # an under-full group: padded with offset 0
    mask[4, :] = 0                            # an empty row: every group padded with 0,1
    for kind, g in [(O.VAL_INT4, 64), (O.VAL_FP16, 0)]:
        p = O.pack_2bitcsr(w, mask, 2, g, kind)
        W1, m1 = O.dense_from_packed(p), O.mask_from_packed(p)
        assert np.all(m1 >= mask) and np.all(m1.reshape(16, 32, 4).sum(axis=2) == 2)
        assert np.all(W1[(m1 == 1) & (mask == 0)] == 0)          # padding decodes to exact zero
        assert m1[3, 8:12].tolist() == [1, 0, 1, 0]
        assert np.array_equal(m1[4], np.tile([1, 1, 0, 0], 32))
    # FP16 values: decoding and packing again reproduces every buffer byte for byte
    p = O.pack_2bitcsr(w, mask, 2, 0, O.VAL_FP16)
    p2 = O.pack_2bitcsr(O.dense_from_packed(p).astype(np.float16), O.mask_from_packed(p), 2, 0, O.VAL_FP16)
    for k in ("row_ptr", "values", "idx"):
        assert np.array_equal(p[k], p2[k])


def test_lossless_grid_round_trip():
    # weights exactly on an fp16-exact grid s0*{-z..15-z} survive quantisation
    rng = np.random.default_rng(5)
    s0, z0 = 0.125, 6
    codes = rng.integers(0, 16, size=(8, 64))
    codes[:, 0], codes[:, 1] = 0, 15         # make every group span the full range
    codes[:, 32], codes[:, 33] = 0, 15
    w = (s0 * (codes - z0)).astype(np.float16)
    mask = np.ones_like(codes, dtype=np.uint8)
    p = O.pack_2bitcsr(w, mask, 4, 32, O.VAL_INT4)
    assert np.array_equal(O.dense_from_packed(p), w.astype(np.float64))
    assert np.all(p["qparams"][:, :, 0].view(np.float16) == np.float16(s0))
    assert np.all(p["qparams"][:, :, 1].view(np.float16) == np.float16(z0))


# ----------------------------------------------------------------- quantiser bounds
def test_quantiser_error_bounds():
    w = _rand_w(32, 256, 31)
    n, g = 2, 128
    mask = O.prune_n4_magnitude(w, n)
    p = O.pack_2bitcsr(w, mask, n, g, O.VAL_INT4)
    col, w_hat, q = O.decode_2bitcsr(p)
    assert q.min() >= 0 and q.max() <= 15
    s = p["qparams"][:, :, 0].view(np.float16).astype(np.float64)
    z = p["qparams"][:, :, 1].view(np.float16).astype(np.float64)
    rows = np.arange(32)[:, None]
    v = w.astype(np.float64)[rows, col]
    s_slot, z_slot = s[rows, col // g], z[rows, col // g]
    unclamped = np.rint(v / s_slot) + z_slot
    inside = (unclamped >= 0) & (unclamped <= 15)
    err = np.abs(v - w_hat)
    assert np.all(err[inside] <= s_slot[inside] / 2 + 1e-12)
    assert np.all(err <= 1.5 * s_slot + 1e-12)
    # extremes land on code 0 / 15 (within one step after the scale is rounded)
    for r in range(32):
        for G in range(2):
            sel = (col[r] // g) == G
            assert q[r][sel].min() <= 1 and q[r][sel].max() >= 14


def test_all_zero_group_and_zero_mask():
    w = np.zeros((4, 64), dtype=np.float16)
    p = O.pack_2bitcsr(w, np.zeros((4, 64), dtype=np.uint8), 2, 32, O.VAL_INT4)
    assert np.all(p["qparams"][:, :, 0].view(np.float16) == 1.0)
    assert np.all(p["qparams"][:, :, 1] == 0) and np.all(p["values"] == 0)
    y, a = O.gemv(p, _rand_x(64, 1))
    assert np.all(y == 0) and np.all(a == 0)
    # a non-zero matrix under an all-zero mask also multiplies to exactly zero
    w2 = _rand_w(4, 64, 9)
    for kind, g in [(0, 32), (1, 0)]:
        p2 = O.pack_2bitcsr(w2, np.zeros((4, 64), dtype=np.uint8), 2, g, kind)
        y, _ = O.gemv(p2, _rand_x(64, 2))
        assert np.all(y == 0)


# ----------------------------------------------------------------- the product
def _python_loops_gemv(p, x):
    """Decode and multiply with nothing but Python integers and floats."""
    R, K, n, g = p["rows"], p["cols"], p["n_keep"], p["group"]
    S = n * K // 4
    xs = [float(v) for v in x]
    ys = []
    for r in range(R):
        acc = 0.0
        for j in range(S):
            t = int(p["row_ptr"][r]) + j
            off = (int(p["idx"][t // 8]) >> (2 * (t % 8))) & 3
            c = 4 * (j // n) + off
            if p["val_kind"] == O.VAL_FP16:
                wv = float(p["values"].view(np.float16)[t])
            else:
                byte = int(p["values"][t // 2])
                qv = (byte >> 4) if t % 2 else (byte & 15)
                s = float(p["qparams"][r, c // g, 0:1].view(np.float16)[0])
                z = float(p["qparams"][r, c // g, 1:2].view(np.float16)[0])
                wv = s * (qv - z)
            acc += wv * xs[c]
        ys.append(acc)
    return np.array(ys)


@pytest.mark.parametrize("n,kind,g", [(2, 0, 32), (1, 0, 16), (2, 1, 0), (1, 1, 0)])
def test_gemv_against_python_loops_and_dense_matmul(n, kind, g):
    R, K = 8, 32
    w = _rand_w(R, K, 40 + n)
    x = _rand_x(K, 41)
    p = O.pack_2bitcsr(w, O.prune_n4_magnitude(w, n), n, g, kind)
    y, a = O.gemv(p, x)
    np.testing.assert_allclose(y, _python_loops_gemv(p, x), rtol=0, atol=1e-12)
    W = O.dense_from_packed(p)
    np.testing.assert_allclose(y, W @ x.astype(np.float64), rtol=0, atol=1e-12)
    np.testing.assert_allclose(a, np.abs(W) @ np.abs(x.astype(np.float64)), rtol=0, atol=1e-12)


def test_gemv_config1_against_scipy_csr():
    seed = synth.seed_for(1)
    w = synth.weights(1024, 1024, seed)
    x = synth.activations(1024, seed)
    p = O.pack_2bitcsr(w, O.prune_n4_magnitude(w, 2), 2, 128, O.VAL_INT4)
    y, _ = O.gemv(p, x)
    W = O.dense_from_packed(p)
    assert (W != 0).sum() <= 1024 * 512
    y_csr = scipy.sparse.csr_matrix(W) @ x.astype(np.float64)
    np.testing.assert_allclose(y, y_csr, rtol=0, atol=1e-10)


def test_special_inputs():
    R, K = 16, 64
    w = _rand_w(R, K, 50)
    p = O.pack_2bitcsr(w, O.prune_n4_magnitude(w, 2), 2, 32, O.VAL_INT4)
    W = O.dense_from_packed(p)
    for j in (0, 17, 63):                      # one-hot x picks column j
        e = np.zeros(K, dtype=np.float16)
        e[j] = 1
        assert np.array_equal(O.gemv(p, e)[0], W[:, j])
    y1, _ = O.gemv(p, np.ones(K, dtype=np.float16))
    np.testing.assert_allclose(y1, W.sum(axis=1), atol=1e-12)
    x = _rand_x(K, 51)
    assert np.array_equal(O.gemv(p, (2 * x).astype(np.float16))[0], 2 * O.gemv(p, x)[0])


def test_smallm_equals_independent_gemvs():
    R, K, M = 16, 64, 5
    w = _rand_w(R, K, 60)
    X = np.random.default_rng(61).standard_normal((M, K)).astype(np.float16)
    p = O.pack_2bitcsr(w, O.prune_n4_magnitude(w, 2), 2, 32, O.VAL_INT4)
    Y, A = O.gemm_smallm(p, X)
    assert Y.shape == (M, R)
    for m in range(M):
        y, a = O.gemv(p, X[m])
        assert np.array_equal(Y[m], y) and np.array_equal(A[m], a)
    np.testing.assert_allclose(Y, X.astype(np.float64) @ O.dense_from_packed(p).T, atol=1e-12)


def test_full_mask_sparse_path_equals_dense_int4_path():
    # n_keep = 4 keeps everything: 2bit-CSR and the dense INT4 format hold the same codes
    R, K, g = 8, 128, 64
    w = _rand_w(R, K, 70)
    x = _rand_x(K, 71)
    p = O.pack_2bitcsr(w, np.ones((R, K), dtype=np.uint8), 4, g, O.VAL_INT4)
    qb, qp = O.quant_int4_dense(w, g)
    assert np.array_equal(qb.reshape(-1), p["values"])
    assert np.array_equal(qp, p["qparams"])
    y_s, a_s = O.gemv(p, x)
    y_d, a_d = O.int4_gemv(qb, qp, g, x)
    np.testing.assert_allclose(y_s, y_d, atol=1e-12)
    np.testing.assert_allclose(a_s, a_d, atol=1e-12)
    # dense path against its own brute force from the nibbles
    q = np.array([[(int(qb[r, c // 2]) >> (4 * (c % 2))) & 15 for c in range(K)] for r in range(R)], dtype=np.float64)
    s = qp[:, :, 0].view(np.float16).astype(np.float64)
    z = qp[:, :, 1].view(np.float16).astype(np.float64)
    Wd = np.array([[s[r, c // g] * (q[r, c] - z[r, c // g]) for c in range(K)] for r in range(R)])
    np.testing.assert_allclose(y_d, Wd @ x.astype(np.float64), atol=1e-12)
    # and the quantised matrix stays within half a step of the original
    assert np.all(np.abs(Wd - w.astype(np.float64)) <= 0.5 * np.repeat(s, g, axis=1) * 1.0001 + 1e-12)


def test_single_rounding_of_scale():
    # (xmax-xmin)/15 chosen so that rounding through float32 first would differ
    # from one direct float64 -> float16 rounding (a double-rounding trap).
    target = np.float64(1.0) + 2.0 ** -11 + 2.0 ** -30    # just above an fp16 tie
    assert np.float16(target) != np.float16(np.float32(target))
    s16, z = O.quant_params(np.array([0.0]), np.array([15.0 * target]))
    assert s16[0] == np.float16(1.0) + np.float16(2.0 ** -10)


def test_synth_is_seeded():
    a = synth.weights(4, 32, synth.seed_for(1))
    b = synth.weights(4, 32, synth.seed_for(1))
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    assert abs(float(synth.weights(256, 256, 3).astype(np.float64).std()) - 0.02) < 0.001
    assert len(synth.sparse_layers()) == 16


# ----------------------------------------------------------------- rows of different lengths
def _ragged_fixture():
    fx1, w1, mask1 = _fixture()
    fx = read_fixture("handworked_ragged_2x32.txt")
    w0 = np.array([float(v) for v in fx["w0"]], dtype=np.float16)[None, :]
    mask0 = np.array([int(v) for v in fx["mask0"]], dtype=np.uint8)[None, :]
    return fx, fx1, np.concatenate([w0, w1]), np.concatenate([mask0, mask1])


def test_handworked_ragged_bytes():
    fx, fx1, w, mask = _ragged_fixture()
    p = O.pack_2bitcsr_rows(w, mask, [1, 2], 32, O.VAL_INT4)
    assert p["n_keep"] == 0 and p["total_slots"] == 24
    assert [int(v) for v in fx["row_ptr"]] == p["row_ptr"].tolist()
    assert [int(v, 16) for v in fx["idx_words"]] == p["idx"].tolist()
    assert [int(v, 16) for v in fx["value_bytes"]] == p["values"].tolist()
    assert [int(v, 16) for v in fx["qparams"]] == p["qparams"].reshape(-1).tolist()
    assert [int(v) for v in fx["sizes"]] == list(O.buffer_sizes_rows(32, [1, 2], 32, O.VAL_INT4))
    col, w_hat = O.decode_row(p, 0)
    assert [int(v) for v in fx["cols0"]] == col.tolist()
    assert [0.5 * (int(q) - 4) for q in fx["q0"]] == w_hat.tolist()
    x = np.arange(1, 33).astype(np.float16)
    y, a = O.gemv_rows(p, x)
    assert y.tolist() == [float(v) for v in fx["y"]] and a.tolist() == [float(v) for v in fx["abs_sum"]]
    # FP16 values: raw bits of the kept weights, +0.0 in the padding slot
    pf = O.pack_2bitcsr_rows(w, mask, [1, 2], 0, O.VAL_FP16)
    bits = pf["values"].view(np.uint16).tolist()
    assert bits == [int(v, 16) for v in fx["fp16_bits0"]] + [int(v, 16) for v in fx1["fp16_bits"]]
    assert pf["idx"].tolist() == p["idx"].tolist() and pf["qparams"] is None
    yf, _ = O.gemv_rows(pf, x)
    assert yf.tolist() == [float(fx["y"][0]), float(fx1["y_fp16"][0])]


@pytest.mark.parametrize("n,kind,g", [(1, 0, 32), (2, 0, 16), (3, 0, 64), (2, 1, 0), (4, 1, 0)])
def test_equal_rows_reduce_to_the_uniform_format(n, kind, g):
    R, K = 6, 64
    w = _rand_w(R, K, 90 + n)
    mask = O.prune_n4_magnitude(w, n)
    u = O.pack_2bitcsr(w, mask, n, g, kind)
    p = O.pack_2bitcsr_rows(w, mask, [n] * R, g, kind)
    for key in ("row_ptr", "values", "idx"):
        assert np.array_equal(u[key], p[key]), key
    if kind == O.VAL_INT4:
        assert np.array_equal(u["qparams"], p["qparams"])
    x = _rand_x(K, 91)
    assert np.array_equal(O.gemv(u, x)[0], O.gemv_rows(p, x)[0])
    assert np.array_equal(O.dense_from_packed(u), O.dense_from_packed_rows(p))


def _mixed_case(R, K, seed, choices=(1, 2)):
    rng = np.random.default_rng(seed)
    w = _rand_w(R, K, seed + 1)
    nk = rng.choice(choices, size=R)
    mask = np.zeros((R, K), dtype=np.uint8)
    for n in np.unique(nk):
        sel = nk == n
        mask[sel] = O.prune_n4_magnitude(w[sel], int(n))
    return w, mask, nk


def test_ragged_fp16_is_the_masked_matrix_and_its_csr_product():
    R, K = 24, 96
    w, mask, nk = _mixed_case(R, K, 100, choices=(1, 2, 3, 4))
    p = O.pack_2bitcsr_rows(w, mask, nk, 0, O.VAL_FP16)
    want = np.where(mask != 0, w.astype(np.float64), 0.0)
    assert np.array_equal(O.dense_from_packed_rows(p), want)          # decode(encode) = the kept entries
    assert np.array_equal(O.mask_from_packed_rows(p), mask)           # top-n masks are full: no padding
    assert np.array_equal(np.diff(p["row_ptr"].astype(np.int64)), nk * (K // 4))
    X = np.stack([_rand_x(K, 101 + m) for m in range(3)])
    Y, A = O.gemm_rows(p, X)
    csr = scipy.sparse.csr_matrix(want)
    assert csr.nnz <= int(nk.sum()) * (K // 4)
    for m in range(3):
        np.testing.assert_allclose(Y[m], csr @ X[m].astype(np.float64), rtol=0, atol=1e-12)
        np.testing.assert_allclose(A[m], abs(csr) @ np.abs(X[m].astype(np.float64)), rtol=0, atol=1e-12)


def test_ragged_int4_rows_against_brute_force_bit_reading():
    """Every slot of every row read with Python integer arithmetic straight from the buffers."""
    R, K, g = 10, 64, 16
    w, mask, nk = _mixed_case(R, K, 110)
    p = O.pack_2bitcsr_rows(w, mask, nk, g, O.VAL_INT4)
    x = _rand_x(K, 111).astype(np.float64)
    idx, vals, qp, row_ptr = p["idx"].tolist(), p["values"].tolist(), p["qparams"], p["row_ptr"].tolist()
    y = []
    for r in range(R):
        acc, t, n = 0.0, row_ptr[r], int(nk[r])
        assert row_ptr[r + 1] - row_ptr[r] == n * K // 4
        for c4 in range(K // 4):
            prev = -1
            for _ in range(n):
                off = (idx[t // 8] >> (2 * (t % 8))) & 3
                assert off > prev
                prev = off
                q = (vals[t // 2] >> (4 * (t % 2))) & 15
                c = 4 * c4 + off
                s = float(qp[r, c // g, 0:1].view(np.float16)[0])
                z = float(qp[r, c // g, 1:2].view(np.float16)[0])
                acc += s * (q - z) * x[c]
                t += 1
        assert t == row_ptr[r + 1]
        y.append(acc)
    np.testing.assert_allclose(O.gemv_rows(p, x.astype(np.float16))[0], np.array(y), rtol=0, atol=1e-12)
    # a 1:4 row is quantised from its own kept values: the same bytes as packing it alone
    r1 = int(np.nonzero(nk == 1)[0][0])
    alone = O.pack_2bitcsr(w[r1:r1 + 1], mask[r1:r1 + 1], 1, g, O.VAL_INT4)
    t0 = row_ptr[r1]
    assert np.array_equal(p["values"][t0 // 2: t0 // 2 + K // 8], alone["values"])
    assert np.array_equal(p["qparams"][r1], alone["qparams"][0])


def test_ragged_sizes_and_bytes_saved():
    # half of the rows at 1:4 instead of 2:4: a quarter fewer value and index bytes
    R, K, g = 64, 256, 128
    nk = np.array([1, 2] * (R // 2))
    b_mixed = O.buffer_sizes_rows(K, nk, g, O.VAL_INT4)
    b_24 = O.buffer_sizes(R, K, 2, g, O.VAL_INT4)
    assert b_mixed[0] == b_24[0] and b_mixed[3] == b_24[3]
    assert 4 * (b_mixed[1] + b_mixed[2]) == 3 * (b_24[1] + b_24[2])
    w, mask, _ = _mixed_case(R, K, 120)
    mask = np.zeros_like(mask)
    p = O.pack_2bitcsr_rows(w, mask, nk, g, O.VAL_INT4)
    assert (p["row_ptr"].nbytes, p["values"].nbytes, p["idx"].nbytes, p["qparams"].nbytes) == b_mixed
    assert not O.dense_from_packed_rows(p).any()                      # an empty mask: all padding, all zero


def test_ragged_errors():
    w, mask, nk = _mixed_case(4, 32, 130)
    for bad in ([0, 1, 2, 1], [1, 2, 5, 1], [1, 2]):
        with pytest.raises(ValueError):
            O.pack_2bitcsr_rows(w, mask, bad, 32, O.VAL_INT4)
    full = O.prune_n4_magnitude(w, 2)
    with pytest.raises(ValueError):                                    # a 2:4 mask in a 1:4 row
        O.pack_2bitcsr_rows(w, full, [2, 2, 1, 2], 32, O.VAL_INT4)
    p = O.pack_2bitcsr_rows(w, mask, nk, 32, O.VAL_INT4)
    p["row_ptr"] = p["row_ptr"].copy()
    p["row_ptr"][1] += 4
    with pytest.raises(ValueError):
        O.decode_row(p, 1)


# ----------------------------------------------------------------- paired nibble order
def test_handworked_paired_bytes_and_the_mask_property():
    fx, w, mask = _fixture()
    p = O.pack_2bitcsr(w, mask, 2, 32, O.VAL_INT4_PAIRED)
    c = O.pack_2bitcsr(w, mask, 2, 32, O.VAL_INT4)
    assert [int(v, 16) for v in fx["value_bytes_paired"]] == p["values"].tolist()
    assert np.array_equal(p["idx"], c["idx"]) and np.array_equal(p["qparams"], c["qparams"]) and np.array_equal(p["row_ptr"], c["row_ptr"])
    # what the order is for: two masks on the word and on the word >> 8 give the slot pairs (2j, 2j+1)
    q = [int(v) for v in fx["q"]]
    for wi, word in enumerate(p["values"].view("<u4").tolist()):
        pairs = [word & 0x000F000F, (word & 0x00F000F0) >> 4, (word >> 8) & 0x000F000F, ((word >> 8) & 0x00F000F0) >> 4]
        for j, pr in enumerate(pairs):
            assert (pr & 0xF, pr >> 16) == (q[8 * wi + 2 * j], q[8 * wi + 2 * j + 1])
    col_p, w_p, q_p = O.decode_2bitcsr(p)
    col_c, w_c, q_c = O.decode_2bitcsr(c)
    assert np.array_equal(col_p, col_c) and np.array_equal(w_p, w_c) and np.array_equal(q_p, q_c)
    x = np.arange(1, 33).astype(np.float16)
    assert O.gemv(p, x)[0][0] == float(fx["y"][0])


@pytest.mark.parametrize("n,g", [(2, 128), (1, 32), (3, 16), (4, 64)])
def test_paired_order_is_a_permutation_of_the_canonical_codes(n, g):
    R, K = 12, 256
    w = _rand_w(R, K, 140 + n)
    mask = O.prune_n4_magnitude(w, n)
    mask[2, 8:16] = 0
    p = O.pack_2bitcsr(w, mask, n, g, O.VAL_INT4_PAIRED)
    c = O.pack_2bitcsr(w, mask, n, g, O.VAL_INT4)
    assert O.buffer_sizes(R, K, n, g, O.VAL_INT4_PAIRED) == O.buffer_sizes(R, K, n, g, O.VAL_INT4)
    # nibble k of every word of the canonical bytes is slot k; of the paired bytes slot (0,2,4,6,1,3,5,7)[k]
    nib = lambda b: np.stack([b & 15, b >> 4], axis=1).reshape(-1, 8)
    assert np.array_equal(nib(p["values"]), nib(c["values"])[:, [0, 2, 4, 6, 1, 3, 5, 7]])
    assert np.array_equal(O.dense_from_packed(p), O.dense_from_packed(c))
    x = _rand_x(K, 141)
    assert np.array_equal(O.gemv(p, x)[0], O.gemv(c, x)[0])
    pr = O.pack_2bitcsr_rows(w[:4], O.prune_n4_magnitude(w[:4], 1), [1, 1, 1, 1], g, O.VAL_INT4_PAIRED)
    assert np.array_equal(O.dense_from_packed_rows(pr),
                          O.dense_from_packed(O.pack_2bitcsr(w[:4], O.prune_n4_magnitude(w[:4], 1), 1, g, O.VAL_INT4)))
