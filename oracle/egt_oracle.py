"""CPU oracle for the SparseGemv path: prune -> quantise -> 2bit-CSR -> y = W.x

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the HIP
library is checked against.  Nothing in the product path may import it; it
imports nothing from the product either (numpy only).  All floating-point work
is float64 unless a rounding to FP16 is part of the format.

What the paper fixes and what it leaves open
--------------------------------------------
The paper (Sec. 3.2 "Sparsification", Sec. 3.3 "Sparse Index Structure" and
"Computational Acceleration") gives, in prose only:
  * N:M semi-structured sparsity with M = 4 and N in {2, 1}, chosen per layer;
  * weights group-wise quantised FP16 -> INT4, activations stay FP16;
  * non-zeros are extracted, their column positions recorded in a compact index,
    the indices turned into binary, grouped and packed into uint16_t words,
    stored in "reverse order" so that bit operations recover them;
  * a CSR-like row structure;
  * index + weights take 30 % of the size of the original CSR.
It prints no bit layout, no quantiser formula and no worked example.  Every
layout decision below is therefore this build's reading of that prose (listed in
the design notes of the repository); those readings are *parity unpinned against
the paper*: they are pinned only by the closed forms, invariants, brute-force
checks and the hand-worked fixture in tests/.

The one number the paper does print for the format, the 30 % ratio, is
reproduced exactly by `size_model` (INT4 value + 2-bit index = 6 bits against
INT4 value + 16-bit column index = 20 bits).

The product y = W.x itself has a plain definition: it is the ordinary
matrix-vector product with the *decoded* matrix.  `gemv`/`gemm_smallm` are that
definition written out.

Canonical format (shared wording with the library's header, no shared code)
--------------------------------------------------------------------------
R rows, K columns, K % 32 == 0.  Columns are cut into 4-groups [4c, 4c+4).
n = n_keep in {1, 2, 3, 4}.  Every row has S = n*K/4 slots in ascending column
order; 4-group c owns slots [n*c, n*c + n) whose in-group offsets (0..3) are
strictly ascending.
  row_ptr : uint32[R+1], slot units, row_ptr[r] = r*S.
  idx     : uint16[total_slots/8]; global slot t sits in word t>>3 at bits
            [2*(t&7), 2*(t&7)+1] (first slot in the least-significant bits).
  values  : INT4 - byte t>>1, low nibble for even t;  FP16 - uint16[t] raw bits.
  qparams : INT4 only, uint16[R][K/g][2] = FP16 bits of {scale, zero}; the
            quantisation groups are ranges of g *dense* columns.

Rows of different lengths (Sec. 3.2: N of N:4 is chosen adaptively; Sec. 3.3: the format is
CSR-like, i.e. it has row pointers).  Row r keeps n_r in {1..4} entries per 4-group and has
S_r = n_r*K/4 slots; row_ptr is the running sum of the S_r.  Since every row starts on a
whole index word and a whole value byte (K % 32 == 0) and the quantiser works row by row,
such a matrix is, by definition here, the row-by-row concatenation of the uniform encodings
of its rows: that is how `pack_2bitcsr_rows` builds it, and `decode_row` / `gemv_rows` walk
row_ptr as any CSR product does.  The dict says n_keep = 0 and carries row_n_keep.
"""
from __future__ import annotations

import numpy as np

VAL_INT4 = 0
VAL_FP16 = 1
VAL_INT4_PAIRED = 2      # INT4 codes in the second nibble order, see PAIRED_ORDER

# Sec. 3.3 reorders what it stores so that bit operations recover it cheaply; the reading
# taken here for the codes: inside every word of eight slots (the 32 bits of values that one
# index word speaks for) the nibbles, from the least-significant one up, hold the slots
# 0, 2, 4, 6, 1, 3, 5, 7.  Then `word & 0x000F000F` is the slot pair (0, 1), `word & 0x00F000F0`
# the pair (2, 3), and the same masks on `word >> 8` give (4, 5) and (6, 7).
PAIRED_ORDER = (0, 2, 4, 6, 1, 3, 5, 7)


# --------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------
def _is_int4(val_kind: int) -> bool:
    return val_kind in (VAL_INT4, VAL_INT4_PAIRED)


def _code_position(t, val_kind: int):
    """Byte index and bit shift of the code of global slot t (array or scalar)."""
    t = np.asarray(t, dtype=np.int64)
    if val_kind == VAL_INT4_PAIRED:
        nibble_of_slot = np.argsort(np.array(PAIRED_ORDER))      # slot j of a word -> its nibble
        pos = nibble_of_slot[t & 7]
        return 4 * (t >> 3) + (pos >> 1), 4 * (pos & 1)
    return t >> 1, 4 * (t & 1)


def _as_f16(w) -> np.ndarray:
    w = np.asarray(w)
    if w.dtype == np.uint16:
        w = w.view(np.float16)
    if w.dtype != np.float16:
        raise TypeError("weights/activations must be float16 (or their uint16 bits)")
    return w


def check_shape(rows: int, cols: int, n_keep: int, group: int, val_kind: int) -> None:
    """Shape rules of the format (K % 32 == 0 keeps whole idx words per row)."""
    if rows < 0 or cols < 0:
        raise ValueError("negative shape")
    if cols % 32 != 0:
        raise ValueError("cols must be a multiple of 32")
    if n_keep not in (1, 2, 3, 4):
        raise ValueError("n_keep must be 1..4")
    if val_kind in (VAL_INT4, VAL_INT4_PAIRED):
        if group <= 0 or group % 4 != 0 or cols % group != 0:
            raise ValueError("group must be a positive multiple of 4 dividing cols")
    elif val_kind == VAL_FP16:
        if group != 0:
            raise ValueError("group must be 0 for FP16 values")
    else:
        raise ValueError("val_kind")


# --------------------------------------------------------------------------
# O1  pruning helper  (Sec. 3.2 "Sparsification": N:M, importance ranking;
#     Eq. (3) with constant activation norm and gradient = plain magnitude)
# --------------------------------------------------------------------------
def prune_n4_magnitude(w, n_keep: int) -> np.ndarray:
    """Mask (uint8, R x K) keeping, in every 4-group of consecutive columns, the
    n_keep entries of largest |w|; among equal magnitudes the lower column wins.
    -0.0 counts as magnitude 0."""
    w = _as_f16(w)
    R, K = w.shape
    if K % 4 != 0:
        raise ValueError("cols must be a multiple of 4")
    mag = np.abs(w.astype(np.float64)).reshape(R, K // 4, 4)
    # rank of entry j inside its group = number of entries that beat it:
    # strictly larger magnitude, or equal magnitude at a lower column.
    beats = np.zeros(mag.shape, dtype=np.int64)
    for j in range(4):
        for i in range(4):
            if i == j:
                continue
            if i < j:
                beats[:, :, j] += mag[:, :, i] >= mag[:, :, j]
            else:
                beats[:, :, j] += mag[:, :, i] > mag[:, :, j]
    return (beats < n_keep).astype(np.uint8).reshape(R, K)


def importance_eq3(w, act_norm, grad_abs) -> np.ndarray:
    """Eq. (3): |W_ij| * ||X_j||_2 + |W_ij| * |dE/dW_ij| (float64)."""
    a = np.abs(_as_f16(w).astype(np.float64))
    return a * np.asarray(act_norm, dtype=np.float64)[None, :] + a * np.asarray(grad_abs, dtype=np.float64)


def prune_n4_importance(w, act_norm, grad_abs, n_keep: int) -> np.ndarray:
    """Mask keeping, in every 4-group, the n_keep entries of largest Eq. (3) score;
    equal scores: the lower column wins (Sec. 3.2 "Sparsification")."""
    w16 = _as_f16(w)
    R, K = w16.shape
    if grad_abs is None:
        grad_abs = np.zeros((R, K))
    score = importance_eq3(w16, act_norm, grad_abs).reshape(R, K // 4, 4)
    mask = np.zeros((R, K // 4, 4), dtype=np.uint8)
    for j in range(4):
        beats = np.zeros((R, K // 4), dtype=np.int64)
        for i in range(4):
            if i == j:
                continue
            if i < j:
                beats += score[:, :, i] >= score[:, :, j]
            else:
                beats += score[:, :, i] > score[:, :, j]
        mask[:, :, j] = beats < n_keep
    return mask.reshape(R, K)


# --------------------------------------------------------------------------
# O2  slot selection
# --------------------------------------------------------------------------
def choose_slots(mask, n_keep: int) -> np.ndarray:
    """For every 4-group return the n_keep chosen in-group offsets, ascending.

    A group whose mask keeps fewer than n_keep entries is padded with the
    smallest offsets the mask did not keep (they carry an exact zero).  A group
    that keeps more than n_keep is an error.
    Returns `chosen`, bool (R, K/4, 4) with exactly n_keep True per group."""
    mask = np.asarray(mask)
    R, K = mask.shape
    kept = (mask.reshape(R, K // 4, 4) != 0)
    count = kept.sum(axis=2)
    if np.any(count > n_keep):
        raise ValueError("mask keeps more than n_keep entries in a 4-group")
    chosen = kept.copy()
    have = count.copy()
    for j in range(4):                       # smallest unused offsets first
        add = (~kept[:, :, j]) & (have < n_keep)
        chosen[:, :, j] |= add
        have = have + add
    assert np.all(chosen.sum(axis=2) == n_keep)
    return chosen


# --------------------------------------------------------------------------
# O3  group-wise asymmetric INT4 quantiser (Sec. 3.2 "Adaptive Group-Wise
#     Quantization": FP16 -> INT4 per group; formula = this build's reading)
# --------------------------------------------------------------------------
def quant_params(vmin: np.ndarray, vmax: np.ndarray):
    """Scale (float16) and integer zero point from the extrema of the kept values
    of each group.  The range is widened to contain 0 so that an exact zero is
    representable (code == zero point)."""
    xmin = np.minimum(0.0, np.asarray(vmin, dtype=np.float64))
    xmax = np.maximum(0.0, np.asarray(vmax, dtype=np.float64))
    s16 = ((xmax - xmin) / 15.0).astype(np.float16)     # one RNE rounding f64 -> f16
    s16 = np.where(s16 == 0, np.float16(1.0), s16).astype(np.float16)
    s = s16.astype(np.float64)
    z = np.clip(np.rint(-xmin / s), 0.0, 15.0)          # rint: ties to even
    z = z + 0.0                                          # an integer 0..15: never -0.0
    return s16, z


def quant_codes(v: np.ndarray, s: np.ndarray, z: np.ndarray) -> np.ndarray:
    """q = clamp(rint(v/s) + z, 0, 15) in float64 with the *rounded* scale."""
    return np.clip(np.rint(np.asarray(v, dtype=np.float64) / s) + z, 0.0, 15.0)


# --------------------------------------------------------------------------
# O4  pack
# --------------------------------------------------------------------------
def pack_2bitcsr(w, mask, n_keep: int, group: int, val_kind: int, row_group=None) -> dict:
    """Dense FP16 W (R x K) + 0/1 mask + n_keep + group size -> 2bit-CSR.

    Returns a dict of numpy arrays: row_ptr (uint32), values (uint8 bytes),
    idx (uint16), qparams (uint16 (R, K/g, 2) or None) plus the scalars.

    row_group (INT4 only): per-row group sizes (Sec. 3.2 "Adaptive Group-Wise
    Quantization": sensitive channels get more, smaller groups).  Row r is quantised in
    groups of row_group[r] columns, a multiple of `group` that divides K; the stored
    parameters keep the granularity `group`, every coarse group repeating its pair."""
    w = _as_f16(w)
    R, K = w.shape
    check_shape(R, K, n_keep, group, val_kind)
    mask = np.asarray(mask)
    if mask.shape != (R, K):
        raise ValueError("mask shape")
    kept = mask.reshape(R, K // 4, 4) != 0
    wf = w.astype(np.float64).reshape(R, K // 4, 4)
    if not np.all(np.isfinite(wf[kept])):
        raise FloatingPointError("non-finite kept weight")

    chosen = choose_slots(mask, n_keep)                   # (R, K/4, 4)
    S = n_keep * K // 4
    # np.nonzero walks C order: row, then 4-group, then offset -> ascending columns
    offs = np.nonzero(chosen)[2].reshape(R, S).astype(np.int64)
    grp4 = np.repeat(np.arange(K // 4, dtype=np.int64), n_keep)[None, :]
    col = 4 * grp4 + offs                                  # dense column of each slot
    rows = np.arange(R)[:, None]
    slot_kept = kept.reshape(R, K)[rows, col]              # False for padding slots

    row_ptr = (np.arange(R + 1, dtype=np.uint64) * S)
    if row_ptr[-1] >= 2 ** 32:
        raise ValueError("too many slots for uint32 row_ptr")
    row_ptr = row_ptr.astype(np.uint32)

    # ---- indices: 8 two-bit fields per uint16, first slot in the low bits
    o = offs.reshape(-1, 8).astype(np.uint32)
    words = np.zeros(o.shape[0], dtype=np.uint32)
    for k in range(8):
        words |= o[:, k] << (2 * k)
    idx = words.astype(np.uint16)

    out = dict(rows=R, cols=K, n_keep=n_keep, group=group, val_kind=val_kind,
               row_ptr=row_ptr, idx=idx, qparams=None)

    if val_kind == VAL_FP16:
        bits = w.view(np.uint16)[rows, col]
        bits = np.where(slot_kept, bits, np.uint16(0)).astype(np.uint16)   # padding = +0.0
        out["values"] = bits.reshape(-1).view(np.uint8).copy()
        return out

    # ---- INT4: per (row, dense-column group) parameters from the kept values only
    G = K // group
    wk = w.astype(np.float64).reshape(R, G, group)
    mk = kept.reshape(R, G, group)
    vmin = np.where(mk, wk, np.inf).min(axis=2)
    vmax = np.where(mk, wk, -np.inf).max(axis=2)
    if row_group is not None:
        rg = np.asarray(row_group, dtype=np.int64)
        if rg.shape != (R,) or np.any(rg <= 0) or np.any(rg % group != 0) or np.any(K % rg != 0):
            raise ValueError("row_group entries must be multiples of group that divide cols")
        for m in np.unique(rg // group):                   # rows whose groups span m stored groups
            sel = np.nonzero(rg // group == m)[0]
            lo = vmin[sel].reshape(len(sel), G // m, m).min(axis=2)
            hi = vmax[sel].reshape(len(sel), G // m, m).max(axis=2)
            vmin[sel] = np.repeat(lo, m, axis=1)
            vmax[sel] = np.repeat(hi, m, axis=1)
    vmin = np.where(np.isfinite(vmin), vmin, 0.0)          # group with nothing kept
    vmax = np.where(np.isfinite(vmax), vmax, 0.0)
    s16, z = quant_params(vmin, vmax)                      # (R, G)
    sg = s16.astype(np.float64)
    gcol = col // group                                    # quantisation group of each slot
    s_slot = sg[rows, gcol]
    z_slot = z[rows, gcol]
    v_slot = w.astype(np.float64)[rows, col]
    q = np.where(slot_kept, quant_codes(v_slot, s_slot, z_slot), z_slot).astype(np.uint8)

    if val_kind == VAL_INT4_PAIRED:                        # nibble k of a word of eight slots holds slot PAIRED_ORDER[k]
        q = q.reshape(-1, 8)[:, list(PAIRED_ORDER)]
    qf = q.reshape(-1, 2)
    out["values"] = (qf[:, 0] | (qf[:, 1] << 4)).astype(np.uint8)   # first of a pair = low nibble
    qp = np.empty((R, G, 2), dtype=np.uint16)
    qp[:, :, 0] = s16.view(np.uint16)
    qp[:, :, 1] = z.astype(np.float16).view(np.uint16)
    out["qparams"] = qp
    return out


# --------------------------------------------------------------------------
# O5  decode
# --------------------------------------------------------------------------
def decode_2bitcsr(p: dict):
    """2bit-CSR -> per-slot dense column (int64 (R,S)) and decoded weight (float64
    (R,S)).  For INT4 also returns the raw codes; for FP16 the raw bits."""
    R, K, n, g = p["rows"], p["cols"], p["n_keep"], p["group"]
    S = n * K // 4
    row_ptr = p["row_ptr"].astype(np.int64)
    if not np.array_equal(row_ptr, np.arange(R + 1, dtype=np.int64) * S):
        raise ValueError("row_ptr is not the uniform n*K/4 progression")
    t = row_ptr[:-1, None] + np.arange(S, dtype=np.int64)[None, :]         # global slot ids
    words = p["idx"].astype(np.int64)
    offs = (words[t >> 3] >> (2 * (t & 7))) & 3
    col = 4 * (np.arange(S, dtype=np.int64) // n)[None, :] + offs
    rows = np.arange(R)[:, None]
    if p["val_kind"] == VAL_FP16:
        bits = p["values"].view(np.uint16)[t]
        return col, bits.view(np.float16).astype(np.float64), bits
    where, shift = _code_position(t, p["val_kind"])
    q = (p["values"].astype(np.int64)[where] >> shift) & 15
    qp = p["qparams"]
    s = qp[:, :, 0].view(np.float16).astype(np.float64)
    z = qp[:, :, 1].view(np.float16).astype(np.float64)
    gcol = col // g
    w_hat = s[rows, gcol] * (q.astype(np.float64) - z[rows, gcol])
    return col, w_hat, q


def dense_from_packed(p: dict) -> np.ndarray:
    """Decoded matrix W_hat as dense float64 (R x K); empty positions are 0."""
    col, w_hat, _ = decode_2bitcsr(p)
    W = np.zeros((p["rows"], p["cols"]), dtype=np.float64)
    W[np.arange(p["rows"])[:, None], col] = w_hat
    return W


def mask_from_packed(p: dict) -> np.ndarray:
    """Positions that own a slot (kept entries plus padding), uint8 R x K."""
    col, _, _ = decode_2bitcsr(p)
    m = np.zeros((p["rows"], p["cols"]), dtype=np.uint8)
    m[np.arange(p["rows"])[:, None], col] = 1
    return m


# --------------------------------------------------------------------------
# O6  the product (Sec. 3.3: y = W.x over the stored non-zeros)
# --------------------------------------------------------------------------
def gemv(p: dict, x):
    """y_ref[r] = sum over the slots of row r of w_hat * x[col]  (float64, no final
    rounding) and A[r] = sum |w_hat * x[col]| for the tolerance."""
    x = _as_f16(x).astype(np.float64)
    if x.shape != (p["cols"],):
        raise ValueError("x length")
    col, w_hat, _ = decode_2bitcsr(p)
    return gemv_decoded(col, w_hat, x)


def gemv_decoded(col, w_hat, x):
    """The product step of `gemv` alone, on an already decoded matrix (per-slot dense
    column and weight, as `decode_2bitcsr` returns them); x is float64."""
    prod = w_hat * x[col]
    return prod.sum(axis=1), np.abs(prod).sum(axis=1)


def gemm_smallm(p: dict, X):
    """Y_ref[m][r] = sum_k W_hat[r][k] * X[m][k]; also A[m][r] = sum |.|."""
    X = _as_f16(X).astype(np.float64)
    if X.ndim != 2 or X.shape[1] != p["cols"]:
        raise ValueError("X shape")
    col, w_hat, _ = decode_2bitcsr(p)
    Y = np.empty((X.shape[0], p["rows"]), dtype=np.float64)
    A = np.empty_like(Y)
    for m in range(X.shape[0]):
        prod = w_hat * X[m][col]
        Y[m] = prod.sum(axis=1)
        A[m] = np.abs(prod).sum(axis=1)
    return Y, A


# --------------------------------------------------------------------------
# O6b  rows of different lengths (Sec. 3.2 adaptive N:4, Sec. 3.3 CSR-like row pointers)
# --------------------------------------------------------------------------
def pack_2bitcsr_rows(w, mask, row_n_keep, group: int, val_kind: int) -> dict:
    """Row r keeps row_n_keep[r] (1..4) entries per 4-group.  The result is the uniform
    encoding of every row by itself, laid end to end; row_ptr is the running sum of the row
    lengths."""
    w = _as_f16(w)
    R, K = w.shape
    mask = np.asarray(mask)
    if mask.shape != (R, K):
        raise ValueError("mask shape")
    nk = np.asarray(row_n_keep, dtype=np.int64)
    if nk.shape != (R,) or np.any(nk < 1) or np.any(nk > 4):
        raise ValueError("row_n_keep: one entry in 1..4 per row")
    check_shape(R, K, 1, group, val_kind)
    row_ptr = np.concatenate([[0], np.cumsum(nk * (K // 4))])
    if row_ptr[-1] >= 2 ** 32:
        raise ValueError("too many slots for uint32 row_ptr")
    values, idx, qparams = [], [], []
    for r in range(R):
        one = pack_2bitcsr(w[r:r + 1], mask[r:r + 1], int(nk[r]), group, val_kind)
        values.append(one["values"])
        idx.append(one["idx"])
        if _is_int4(val_kind):
            qparams.append(one["qparams"])
    cat = lambda parts, dt: np.concatenate(parts) if parts else np.zeros(0, dtype=dt)
    return dict(rows=R, cols=K, n_keep=0, row_n_keep=nk.astype(np.int32), group=group, val_kind=val_kind,
                row_ptr=row_ptr.astype(np.uint32), values=cat(values, np.uint8), idx=cat(idx, np.uint16),
                qparams=(cat(qparams, np.uint16).reshape(R, K // group, 2) if _is_int4(val_kind) else None),
                total_slots=int(row_ptr[-1]))


def decode_row(p: dict, r: int):
    """Dense columns and decoded weights (float64) of the slots of row r, read through
    row_ptr: slots row_ptr[r] .. row_ptr[r+1]-1, n_r = (their number) / (K/4) per 4-group."""
    K, g = p["cols"], p["group"]
    t0, t1 = int(p["row_ptr"][r]), int(p["row_ptr"][r + 1])
    S = t1 - t0
    if S <= 0 or S % (K // 4) or S // (K // 4) > 4 or t0 % 8:
        raise ValueError("row_ptr does not describe a whole row of 1..4 entries per 4-group")
    n = S // (K // 4)
    t = t0 + np.arange(S, dtype=np.int64)
    offs = (p["idx"].astype(np.int64)[t >> 3] >> (2 * (t & 7))) & 3
    col = 4 * (np.arange(S, dtype=np.int64) // n) + offs
    if p["val_kind"] == VAL_FP16:
        return col, p["values"].view(np.uint16)[t].view(np.float16).astype(np.float64)
    where, shift = _code_position(t, p["val_kind"])
    q = (p["values"].astype(np.int64)[where] >> shift) & 15
    s = p["qparams"][r, :, 0].view(np.float16).astype(np.float64)
    z = p["qparams"][r, :, 1].view(np.float16).astype(np.float64)
    return col, s[col // g] * (q.astype(np.float64) - z[col // g])


def dense_from_packed_rows(p: dict) -> np.ndarray:
    """Decoded matrix of a ragged encoding, dense float64; positions without a slot are 0."""
    W = np.zeros((p["rows"], p["cols"]), dtype=np.float64)
    for r in range(p["rows"]):
        col, w_hat = decode_row(p, r)
        W[r, col] = w_hat
    return W


def mask_from_packed_rows(p: dict) -> np.ndarray:
    m = np.zeros((p["rows"], p["cols"]), dtype=np.uint8)
    for r in range(p["rows"]):
        m[r, decode_row(p, r)[0]] = 1
    return m


def gemm_rows(p: dict, X):
    """Y_ref[m][r] = sum over the slots of row r of w_hat * X[m][col] and A = sum |.|,
    the CSR product written out row by row (float64)."""
    X = _as_f16(X).astype(np.float64)
    if X.ndim != 2 or X.shape[1] != p["cols"]:
        raise ValueError("X shape")
    Y = np.zeros((X.shape[0], p["rows"]), dtype=np.float64)
    A = np.zeros_like(Y)
    for r in range(p["rows"]):
        col, w_hat = decode_row(p, r)
        prod = w_hat[None, :] * X[:, col]
        Y[:, r] = prod.sum(axis=1)
        A[:, r] = np.abs(prod).sum(axis=1)
    return Y, A


def gemv_rows(p: dict, x):
    Y, A = gemm_rows(p, _as_f16(x)[None, :])
    return Y[0], A[0]


def buffer_sizes_rows(cols: int, row_n_keep, group: int, val_kind: int):
    """Bytes of (row_ptr, values, idx, qparams) of a ragged encoding."""
    nk = np.asarray(row_n_keep, dtype=np.int64)
    T = int(nk.sum()) * (cols // 4)
    R = len(nk)
    return (4 * (R + 1), T // 2 if _is_int4(val_kind) else 2 * T, T // 4,
            4 * R * (cols // group) if _is_int4(val_kind) else 0)


# --------------------------------------------------------------------------
# O7  dense INT4 (the "previous generation of Gemv", Sec. 3.3)
# --------------------------------------------------------------------------
def quant_int4_dense(w, group: int):
    """All columns kept.  Returns q bytes (R, K/2) - column c in byte c>>1, low
    nibble for even c - and qparams uint16 (R, K/g, 2)."""
    w = _as_f16(w)
    R, K = w.shape
    if K % 2 or group <= 0 or K % group or group % 2:
        raise ValueError("shape")
    wf = w.astype(np.float64)
    if not np.all(np.isfinite(wf)):
        raise FloatingPointError("non-finite weight")
    G = K // group
    wg = wf.reshape(R, G, group)
    s16, z = quant_params(wg.min(axis=2), wg.max(axis=2))
    q = quant_codes(wg, s16.astype(np.float64)[:, :, None], z[:, :, None]).astype(np.uint8).reshape(R, K)
    qbytes = (q[:, 0::2] | (q[:, 1::2] << 4)).astype(np.uint8)
    qp = np.empty((R, G, 2), dtype=np.uint16)
    qp[:, :, 0] = s16.view(np.uint16)
    qp[:, :, 1] = z.astype(np.float16).view(np.uint16)
    return qbytes, qp


def dequant_int4_dense(qbytes, qparams, group: int) -> np.ndarray:
    qbytes = np.asarray(qbytes, dtype=np.uint8)
    R, K2 = qbytes.shape
    K = 2 * K2
    q = np.empty((R, K), dtype=np.float64)
    q[:, 0::2] = qbytes & 15
    q[:, 1::2] = qbytes >> 4
    s = qparams[:, :, 0].view(np.float16).astype(np.float64)
    z = qparams[:, :, 1].view(np.float16).astype(np.float64)
    return (np.repeat(s, group, axis=1) * (q - np.repeat(z, group, axis=1)))


def int4_gemv(qbytes, qparams, group: int, x):
    """y_ref = W_hat . x for the dense group-quantised matrix (float64) and A."""
    x = _as_f16(x).astype(np.float64)
    W = dequant_int4_dense(qbytes, qparams, group)
    prod = W * x[None, :]
    return prod.sum(axis=1), np.abs(prod).sum(axis=1)


# --------------------------------------------------------------------------
# O8  byte-size model (Sec. 1 contribution list: "30% of the original CSR size")
# --------------------------------------------------------------------------
def buffer_sizes(rows: int, cols: int, n_keep: int, group: int, val_kind: int):
    """Bytes of (row_ptr, values, idx, qparams)."""
    check_shape(rows, cols, n_keep, group, val_kind)
    slots = rows * n_keep * cols // 4
    b_row = 4 * (rows + 1)
    b_val = slots // 2 if _is_int4(val_kind) else 2 * slots
    b_idx = 2 * (slots // 8)
    b_qp = 4 * rows * (cols // group) if _is_int4(val_kind) else 0
    return b_row, b_val, b_idx, b_qp


def size_model(rows: int, cols: int, n_keep: int, value_bits: int, csr_index_bits: int,
               group: int = 0, csr_value_bits: int | None = None) -> dict:
    """Bytes of 2bit-CSR (values + 2-bit indices, optionally + group parameters)
    against a standard CSR with `csr_index_bits` column indices.  The row
    pointers are the same on both sides and are reported separately."""
    if csr_value_bits is None:
        csr_value_bits = value_bits
    nnz = rows * n_keep * cols // 4
    ours = nnz * (value_bits + 2) / 8.0
    if group:
        ours += 4.0 * rows * (cols // group)
    csr = nnz * (csr_value_bits + csr_index_bits) / 8.0
    return dict(nnz=nnz, bytes_2bitcsr=ours, bytes_csr=csr, ratio=ours / csr,
                bytes_row_ptr=4 * (rows + 1))


# --------------------------------------------------------------------------
# O9  trigger cost model (Sec. 3.4 "Parallel Verification Trigger": verification cost
#     linear in the number of candidates, autoregressive step constant; trigger where
#     "time to generate the remaining tokens minus time to verify them" is largest)
# --------------------------------------------------------------------------
def fit_verify_cost(m, t):
    """Least-squares line t ~ a + b*m (normal equations via numpy.linalg.lstsq)."""
    m = np.asarray(m, dtype=np.float64)
    t = np.asarray(t, dtype=np.float64)
    A = np.stack([np.ones_like(m), m], axis=1)
    (a, b), *_ = np.linalg.lstsq(A, t, rcond=None)
    return float(a), float(b)


def trigger_depth(t_ar, a, b, cand, remaining):
    """Depth with the largest positive benefit remaining*t_ar - (a + b*cand), else -1."""
    best, top = -1, 0.0
    for d, (c, r) in enumerate(zip(cand, remaining)):
        gain = r * t_ar - (a + b * c)
        if gain > top:
            best, top = d, gain
    return best, top
