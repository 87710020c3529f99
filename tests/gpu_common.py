"""Helpers of the GPU parity tests: upload, call through the C ABI, compare with
the oracle under the stated tolerance."""
import functools

import numpy as np

from oracle import egt_oracle as O
from paper_2605_11582_amd import binding as B, synth

RTOL_ABS_SUM = 1e-2      # |y - y_ref| <= 1e-2 * sum|w_hat * x| + 1e-3, per element
ATOL = 1e-3
CANARY = 0x7BFF          # a finite FP16 pattern no result of these tests equals (65504)


def torch_mod():
    import torch
    return torch


def to_dev(a):
    torch = torch_mod()
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def assert_close(y, y_ref, a_ref, what=""):
    y = np.asarray(y, dtype=np.float64)
    assert np.all(np.isfinite(y)), f"{what}: non-finite output"
    err = np.abs(y - y_ref)
    bound = RTOL_ABS_SUM * a_ref + ATOL
    bad = np.argwhere(err > bound)
    assert bad.size == 0, f"{what}: {bad.shape[0]} outputs out of tolerance, first at {bad[0]}: " \
                          f"got {y[tuple(bad[0])]}, want {y_ref[tuple(bad[0])]}, bound {bound[tuple(bad[0])]}"
    return float((err / bound).max()) if err.size else 0.0


def run_sparse_gemv(p_host: B.Packed, x: np.ndarray, guard: int = 64) -> np.ndarray:
    """y through egt_sparse_gemv; the output buffer carries canaries on both sides."""
    torch = torch_mod()
    pd = p_host.to("cuda")
    xd = to_dev(x.view(np.uint16)).view(torch.float16)
    buf = torch.full((p_host.rows + 2 * guard,), CANARY, dtype=torch.int16, device="cuda")
    y = buf[guard:guard + p_host.rows].view(torch.float16)
    B.sparse_gemv(pd, xd, y)
    torch.cuda.synchronize()
    host = buf.cpu().numpy().view(np.uint16)
    assert np.all(host[:guard] == CANARY) and np.all(host[guard + p_host.rows:] == CANARY), "write outside y"
    return host[guard:guard + p_host.rows].view(np.float16)


def run_sparse_gemm(p_host: B.Packed, X: np.ndarray, ldx_pad: int = 0, ldy_pad: int = 0) -> np.ndarray:
    torch = torch_mod()
    M, K = X.shape
    pd = p_host.to("cuda")
    Xbuf = torch.zeros((M, K + ldx_pad), dtype=torch.float16, device="cuda")
    Xbuf[:, :K] = to_dev(X.view(np.uint16)).view(torch.float16)
    Ybuf = torch.full((M + 2, p_host.rows + ldy_pad), CANARY, dtype=torch.int16, device="cuda")
    Y = Ybuf[1:M + 1, :p_host.rows].view(torch.float16)
    B.sparse_gemm_smallm(pd, Xbuf[:, :K], Y)
    torch.cuda.synchronize()
    host = Ybuf.cpu().numpy().view(np.uint16)
    assert np.all(host[0] == CANARY) and np.all(host[M + 1] == CANARY), "write outside Y rows"
    if ldy_pad:
        assert np.all(host[:, p_host.rows:] == CANARY), "write into the Y row padding"
    return host[1:M + 1, :p_host.rows].view(np.float16)


def run_int4_gemv(q: np.ndarray, qp: np.ndarray, group: int, x: np.ndarray, guard: int = 64) -> np.ndarray:
    torch = torch_mod()
    rows, cols = q.shape[0], q.shape[1] * 2
    qd, qpd = to_dev(q), to_dev(qp)
    xd = to_dev(x.view(np.uint16)).view(torch.float16)
    buf = torch.full((rows + 2 * guard,), CANARY, dtype=torch.int16, device="cuda")
    y = buf[guard:guard + rows].view(torch.float16)
    B.int4_gemv(qd, qpd, rows, cols, group, xd, y)
    torch.cuda.synchronize()
    host = buf.cpu().numpy().view(np.uint16)
    assert np.all(host[:guard] == CANARY) and np.all(host[guard + rows:] == CANARY), "write outside y"
    return host[guard:guard + rows].view(np.float16)


def oracle_view(p: B.Packed) -> dict:
    """The library's packed bytes handed to the oracle's own decoder."""
    return dict(rows=p.rows, cols=p.cols, n_keep=p.n_keep, group=p.group, val_kind=p.val_kind,
                row_ptr=np.asarray(p.row_ptr), values=np.asarray(p.values), idx=np.asarray(p.idx),
                qparams=None if p.qparams is None else np.asarray(p.qparams), total_slots=p.total_slots)


def row_subset(p: B.Packed, rows: np.ndarray) -> dict:
    """Oracle-side view of a few rows of a library-packed matrix (slices of the
    row-major buffers with a rebased row_ptr)."""
    S = p.n_keep * p.cols // 4
    vb = 2 * S if p.val_kind == B.VAL_FP16 else S // 2
    values = np.concatenate([p.values[r * vb:(r + 1) * vb] for r in rows])
    idx = np.concatenate([p.idx[r * (S // 8):(r + 1) * (S // 8)] for r in rows])
    qp = None if p.qparams is None else p.qparams[rows]
    return dict(rows=len(rows), cols=p.cols, n_keep=p.n_keep, group=p.group, val_kind=p.val_kind,
                row_ptr=(np.arange(len(rows) + 1, dtype=np.uint64) * S).astype(np.uint32),
                values=values, idx=idx, qparams=qp)


@functools.lru_cache(maxsize=4)
def packed_full(rows: int, cols: int, n_keep: int, group: int, kind: int, seed: int):
    """A full-size matrix packed by the library (host) + its dense weights and mask."""
    w = synth.weights(rows, cols, seed)
    mask = B.prune_n4(w, n_keep)
    return w, mask, B.pack_2bitcsr(w, mask, n_keep, group, kind)


def sample_rows(rows: int, count: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    pick = set(rng.choice(rows, size=min(count, rows), replace=False).tolist())
    pick.update([0, 1, rows - 1, rows // 2])
    return np.array(sorted(pick))
