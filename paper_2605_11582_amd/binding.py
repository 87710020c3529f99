"""Thin ctypes binding of libegt.so: argument marshalling only.

Host functions take and return numpy arrays; device functions take torch tensors
(used for device memory and the current stream, nothing else).  There is no CPU
fallback: if the built library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# EGT_LIBRARY names another build of the same library (a tuning or ablation build made with
# EGT_EXTRA_HIPCC_FLAGS, see build.py); the default is the in-tree one
LIB_PATH = os.environ.get("EGT_LIBRARY") or os.path.join(_PKG, "libegt.so")

VAL_INT4 = 0
VAL_FP16 = 1
VAL_INT4_PAIRED = 2       # INT4 codes in the paired nibble order (egt.h)

SYMBOLS = (
    "egt_status_str", "egt_last_hip_error", "egt_2bitcsr_sizes", "egt_prune_n4", "egt_pack_2bitcsr",
    "egt_unpack_2bitcsr", "egt_quant_int4", "egt_int4_gemv", "egt_sparse_gemv",
    "egt_sparse_gemm_smallm", "egt_stream_read", "egt_sparse_gemv_batch", "egt_int4_gemv_batch",
    "egt_fit_verify_cost", "egt_trigger_depth", "egt_prune_n4_importance", "egt_pack_2bitcsr_rowgroups",
    "egt_pack_2bitcsr_rows", "egt_2bitcsr_sizes_rows",
    "egt_gemv_stack_plan", "egt_gemv_stack_run", "egt_sparse_gemm_smallm_ws_bytes", "egt_sparse_gemm_smallm_ws",
    "egt_sparse_gemm_smallm_static", "egt_sparse_gemm_smallm_batch",
    "egt_gemm_stack_plan", "egt_gemm_stack_run",
)


class EgtError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"egt status {status}: {text}")
        self.status = status


class View(C.Structure):
    """Mirror of `egt_2bitcsr`."""
    _fields_ = [("rows", C.c_int32), ("cols", C.c_int32), ("n_keep", C.c_int32),
                ("group_size", C.c_int32), ("val_kind", C.c_int32),
                ("row_ptr", C.c_void_p), ("values", C.c_void_p), ("idx", C.c_void_p),
                ("qparams", C.c_void_p), ("total_slots", C.c_uint32)]


class GemvItem(C.Structure):
    """Mirror of `egt_gemv_item`."""
    _fields_ = [("sparse", C.POINTER(View)), ("q", C.c_void_p), ("qparams", C.c_void_p),
                ("rows", C.c_int32), ("cols", C.c_int32), ("group", C.c_int32),
                ("x", C.c_void_p), ("y", C.c_void_p)]


class StackPart(C.Structure):
    """Mirror of `egt_stack_part`: one launch of a planned table."""
    _fields_ = [("count", C.c_int32), ("mode", C.c_int32), ("grid_x", C.c_int32), ("block_threads", C.c_int32),
                ("lds_bytes", C.c_int32), ("x_pieces", C.c_int32), ("forms", C.c_int32), ("nitems", C.c_int32),
                ("part_offset", C.c_int32), ("reserved", C.c_int32), ("table_bytes", C.c_uint64)]


class GemmItem(C.Structure):
    """Mirror of `egt_gemm_item`."""
    _fields_ = [("sparse", C.POINTER(View)), ("X", C.c_void_p), ("Y", C.c_void_p)]


class GemmPlan(C.Structure):
    """Mirror of `egt_gemm_plan`."""
    _fields_ = [("count", C.c_int32), ("M", C.c_int32), ("grid_x", C.c_int32), ("block_threads", C.c_int32),
                ("lds_bytes", C.c_int32), ("n_keep", C.c_int32), ("table_bytes", C.c_uint64)]


STACK_MAX_PARTS = 2


class StackPlan(C.Structure):
    """Mirror of `egt_stack_plan`.  The launch shape of the first part is also reachable as
    attributes of the plan itself (`plan.mode`, `plan.grid_x`, ...)."""
    _fields_ = [("count", C.c_int32), ("nparts", C.c_int32), ("part", StackPart * STACK_MAX_PARTS), ("table_bytes", C.c_uint64)]

    _FIRST = ("mode", "grid_x", "block_threads", "lds_bytes", "x_pieces", "forms", "nitems", "part_offset")

    def __getattr__(self, name):
        if name in StackPlan._FIRST:
            return getattr(self.part[0], name)
        raise AttributeError(name)

    def __setattr__(self, name, value):
        if name in StackPlan._FIRST:
            setattr(self.part[0], name, value)
        elif name in ("count", "nparts", "part", "table_bytes"):
            super().__setattr__(name, value)
        else:
            raise AttributeError(f"egt_stack_plan has no field {name}")


STACK_ENTRY_BYTES = 160

_lib = None


def _declare(L: C.CDLL, names=None) -> C.CDLL:
    """Argument and result types of the entry points `names` (default: all) of a loaded library."""
    names = SYMBOLS if names is None else names
    sig = {
        "egt_status_str": ([C.c_int], C.c_char_p),
        "egt_last_hip_error": ([], C.c_char_p),
        "egt_2bitcsr_sizes": ([C.c_int] * 5 + [C.POINTER(C.c_size_t)], C.c_int),
        "egt_prune_n4": ([C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int64], C.c_int),
        "egt_prune_n4_importance": ([C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int,
                                     C.c_void_p, C.c_int64], C.c_int),
        "egt_pack_2bitcsr": ([C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                              C.POINTER(View)], C.c_int),
        "egt_pack_2bitcsr_rowgroups": ([C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int,
                                        C.c_int, C.c_void_p, C.POINTER(View)], C.c_int),
        "egt_2bitcsr_sizes_rows": ([C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_size_t)], C.c_int),
        "egt_pack_2bitcsr_rows": ([C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                   C.POINTER(View)], C.c_int),
        "egt_unpack_2bitcsr": ([C.POINTER(View), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64], C.c_int),
        "egt_quant_int4": ([C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p], C.c_int),
        "egt_int4_gemv": ([C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
        "egt_sparse_gemv": ([C.POINTER(View), C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
        "egt_sparse_gemm_smallm": ([C.POINTER(View), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int, C.c_void_p], C.c_int),
        "egt_stream_read": ([C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p], C.c_int),
        "egt_sparse_gemv_batch": ([C.POINTER(View), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int, C.c_void_p], C.c_int),
        "egt_sparse_gemm_smallm_batch": ([C.POINTER(View), C.POINTER(C.c_void_p), C.c_int64, C.POINTER(C.c_void_p), C.c_int64,
                                          C.c_int, C.c_int, C.c_void_p], C.c_int),
        "egt_int4_gemv_batch": ([C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int, C.c_int, C.c_int,
                                 C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int, C.c_void_p], C.c_int),
        "egt_fit_verify_cost": ([C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)], C.c_int),
        "egt_trigger_depth": ([C.c_double, C.c_double, C.c_double, C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_int),
                               C.POINTER(C.c_double)], C.c_int),
        "egt_gemv_stack_plan": ([C.POINTER(GemvItem), C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.POINTER(StackPlan)], C.c_int),
        "egt_gemv_stack_run": ([C.c_void_p, C.POINTER(StackPlan), C.c_void_p], C.c_int),
        "egt_gemm_stack_plan": ([C.POINTER(GemmItem), C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.POINTER(GemmPlan)], C.c_int),
        "egt_gemm_stack_run": ([C.c_void_p, C.POINTER(GemmPlan), C.c_void_p], C.c_int),
        "egt_sparse_gemm_smallm_ws_bytes": ([C.POINTER(View), C.c_int64, C.c_int, C.POINTER(C.c_size_t)], C.c_int),
        "egt_sparse_gemm_smallm_ws": ([C.POINTER(View), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int, C.c_void_p,
                                       C.c_size_t, C.c_void_p], C.c_int),
        "egt_sparse_gemm_smallm_static": ([C.POINTER(View), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int, C.c_void_p],
                                          C.c_int),
    }
    for name in names:
        fn = getattr(L, name)                           # AttributeError if the library lacks an entry point
        fn.argtypes, fn.restype = sig[name]
    return L


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2605_11582_amd.build` "
                               "(there is no fallback path)")
        # One HIP runtime per process: PyTorch ships its own libamdhip64 (same soname
        # as the system one).  Importing torch first makes the loader bind libegt.so
        # to that copy, so streams and device pointers mean the same thing on both
        # sides; loading libegt.so first would pull in a second runtime.
        import torch  # noqa: F401
        _lib = _declare(C.CDLL(LIB_PATH))
    return _lib


def status_str(status: int) -> str:
    return lib().egt_status_str(int(status)).decode()


def _check(status: int) -> None:
    if status != 0:
        text = status_str(status)
        if status == 7:
            text += ": " + lib().egt_last_hip_error().decode()
        raise EgtError(status, text)


def _np_ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _f16_bits(a: np.ndarray) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("expected float16 or its uint16 bits")
    return a


def _row_major(a: np.ndarray) -> np.ndarray:
    if a.ndim != 2 or a.strides[1] != a.itemsize or a.strides[0] % a.itemsize:
        a = np.ascontiguousarray(a)
    return a


def _ld(a: np.ndarray) -> int:
    """Leading dimension in elements (numpy reports stride 0 for empty arrays)."""
    return max(a.strides[0] // a.itemsize, a.shape[1])


# ------------------------------------------------------------------ host calls
def sizes(rows: int, cols: int, n_keep: int, group: int, val_kind: int):
    out = (C.c_size_t * 4)()
    _check(lib().egt_2bitcsr_sizes(rows, cols, n_keep, group, val_kind, out))
    return tuple(int(v) for v in out)


def prune_n4(w: np.ndarray, n_keep: int) -> np.ndarray:
    w = _row_major(_f16_bits(w))
    rows, cols = w.shape
    mask = np.empty((rows, cols), dtype=np.uint8)
    _check(lib().egt_prune_n4(_np_ptr(w), _ld(w), rows, cols, n_keep, _np_ptr(mask), cols))
    return mask


def prune_n4_importance(w: np.ndarray, act_norm: np.ndarray, grad_abs, n_keep: int) -> np.ndarray:
    w = _row_major(_f16_bits(w))
    rows, cols = w.shape
    norm = np.ascontiguousarray(act_norm, dtype=np.float32)
    if norm.shape != (cols,):
        raise ValueError("act_norm must have one entry per column")
    grad = None if grad_abs is None else np.ascontiguousarray(grad_abs, dtype=np.float32)
    if grad is not None and grad.shape != (rows, cols):
        raise ValueError("grad_abs must have the shape of w")
    mask = np.empty((rows, cols), dtype=np.uint8)
    _check(lib().egt_prune_n4_importance(_np_ptr(w), _ld(w), _np_ptr(norm), None if grad is None else _np_ptr(grad),
                                         cols, rows, cols, n_keep, _np_ptr(mask), cols))
    return mask


@dataclass
class Packed:
    """One matrix in 2bit-CSR; the four buffers are numpy (host) or torch (device)."""
    rows: int
    cols: int
    n_keep: int
    group: int
    val_kind: int
    row_ptr: object
    values: object
    idx: object
    qparams: object
    total_slots: int = 0          # rows of different lengths (n_keep == 0): row_ptr[rows]
    row_n_keep: object = None     # ... and the entries kept per 4-group in each row (host copy)

    def _ptr(self, b):
        if b is None:
            return None
        return b.ctypes.data if isinstance(b, np.ndarray) else b.data_ptr()

    def view(self) -> View:
        return View(self.rows, self.cols, self.n_keep, self.group, self.val_kind,
                    self._ptr(self.row_ptr), self._ptr(self.values), self._ptr(self.idx),
                    self._ptr(self.qparams), self.total_slots)

    def sizes(self):
        """Bytes of (row_ptr, values, idx, qparams) the view speaks for."""
        if self.n_keep == 0:                             # total_slots is what the kernels trust
            T, int4 = self.total_slots, self.val_kind != VAL_FP16
            return (4 * (self.rows + 1), T // 2 if int4 else 2 * T, T // 4,
                    4 * self.rows * (self.cols // self.group) if int4 else 0)
        return sizes(self.rows, self.cols, self.n_keep, self.group, self.val_kind)

    def nbytes(self) -> int:
        return sum(self.sizes())

    def to(self, device) -> "Packed":
        import torch
        def up(b):
            if b is None:
                return None
            return torch.from_numpy(np.ascontiguousarray(b).view(np.uint8).reshape(-1)).to(device)
        return Packed(self.rows, self.cols, self.n_keep, self.group, self.val_kind,
                      up(self.row_ptr), up(self.values), up(self.idx), up(self.qparams),
                      self.total_slots, self.row_n_keep)


def concat_rows(packs) -> Packed:
    """The host matrices `packs` (same columns, kept count, group size and value kind, uniform rows)
    as one matrix with their rows one after the other: q/k/v or gate/up as a single product.  A row
    of 2bit-CSR depends on nothing outside it, so this is a concatenation of the buffers (with the
    row pointers continued) and equals packing the stacked dense matrix."""
    p0 = packs[0]
    for p in packs:
        if not isinstance(p.values, np.ndarray):
            raise ValueError("concat_rows takes host matrices")
        if (p.cols, p.n_keep, p.group, p.val_kind) != (p0.cols, p0.n_keep, p0.group, p0.val_kind) or p.n_keep == 0:
            raise ValueError("concat_rows takes uniformly shaped matrices of one format")
    rows = sum(p.rows for p in packs)
    slots_per_row = p0.n_keep * (p0.cols // 4)
    if rows * slots_per_row >= 1 << 32:
        raise ValueError("row pointers are 32-bit")
    row_ptr = (np.arange(rows + 1, dtype=np.uint64) * slots_per_row).astype(np.uint32)
    qparams = None if p0.qparams is None else np.concatenate([p.qparams for p in packs], axis=0)
    return Packed(rows, p0.cols, p0.n_keep, p0.group, p0.val_kind, row_ptr,
                  np.concatenate([p.values for p in packs]), np.concatenate([p.idx for p in packs]), qparams)


def pack_2bitcsr(w: np.ndarray, mask: np.ndarray, n_keep: int, group: int, val_kind: int,
                 row_group=None) -> Packed:
    w = _row_major(_f16_bits(w))
    mask = _row_major(np.asarray(mask, dtype=np.uint8))
    rows, cols = w.shape
    if mask.shape != w.shape:
        raise ValueError("mask shape")
    b = sizes(rows, cols, n_keep, group, val_kind)
    row_ptr = np.empty(b[0] // 4, dtype=np.uint32)
    values = np.empty(b[1], dtype=np.uint8)
    idx = np.empty(b[2] // 2, dtype=np.uint16)
    qparams = np.empty((rows, cols // group, 2), dtype=np.uint16) if val_kind != VAL_FP16 else None
    p = Packed(rows, cols, n_keep, group, val_kind, row_ptr, values, idx, qparams)
    v = p.view()
    if row_group is None:
        _check(lib().egt_pack_2bitcsr(_np_ptr(w), _ld(w), _np_ptr(mask), _ld(mask),
                                      rows, cols, n_keep, group, val_kind, C.byref(v)))
    else:
        rg = np.ascontiguousarray(row_group, dtype=np.int32)
        if rg.shape != (rows,):
            raise ValueError("row_group must have one entry per row")
        _check(lib().egt_pack_2bitcsr_rowgroups(_np_ptr(w), _ld(w), _np_ptr(mask), _ld(mask), rows, cols, n_keep,
                                                group, val_kind, _np_ptr(rg), C.byref(v)))
    return p


def sizes_rows(rows: int, cols: int, row_n_keep, group: int, val_kind: int):
    nk = np.ascontiguousarray(row_n_keep, dtype=np.int32)
    if nk.shape != (rows,):
        raise ValueError("row_n_keep must have one entry per row")
    out = (C.c_size_t * 4)()
    _check(lib().egt_2bitcsr_sizes_rows(rows, cols, _np_ptr(nk), group, val_kind, out))
    return tuple(int(v) for v in out)


def pack_2bitcsr_rows(w: np.ndarray, mask: np.ndarray, row_n_keep, group: int, val_kind: int) -> Packed:
    """Rows of different lengths: row r keeps row_n_keep[r] entries per 4-group."""
    w = _row_major(_f16_bits(w))
    mask = _row_major(np.asarray(mask, dtype=np.uint8))
    rows, cols = w.shape
    if mask.shape != w.shape:
        raise ValueError("mask shape")
    nk = np.ascontiguousarray(row_n_keep, dtype=np.int32)
    b = sizes_rows(rows, cols, nk, group, val_kind)
    row_ptr = np.empty(b[0] // 4, dtype=np.uint32)
    values = np.empty(b[1], dtype=np.uint8)
    idx = np.empty(b[2] // 2, dtype=np.uint16)
    qparams = np.empty((rows, cols // group, 2), dtype=np.uint16) if val_kind != VAL_FP16 else None
    p = Packed(rows, cols, 0, group, val_kind, row_ptr, values, idx, qparams, 0, nk)
    v = p.view()
    _check(lib().egt_pack_2bitcsr_rows(_np_ptr(w), _ld(w), _np_ptr(mask), _ld(mask), rows, cols, _np_ptr(nk),
                                       group, val_kind, C.byref(v)))
    p.total_slots = int(v.total_slots)
    return p


def unpack_2bitcsr(p: Packed):
    w = np.empty((p.rows, p.cols), dtype=np.uint16)
    mask = np.empty((p.rows, p.cols), dtype=np.uint8)
    v = p.view()
    _check(lib().egt_unpack_2bitcsr(C.byref(v), _np_ptr(w), p.cols, _np_ptr(mask), p.cols))
    return w.view(np.float16), mask


def quant_int4(w: np.ndarray, group: int):
    w = _row_major(_f16_bits(w))
    rows, cols = w.shape
    if cols % 2 or group <= 0 or cols % group:
        _check(2)                                        # EGT_ERR_SHAPE, before the buffers are sized
    q = np.empty((rows, cols // 2), dtype=np.uint8)
    qparams = np.empty((rows, cols // group, 2), dtype=np.uint16)
    _check(lib().egt_quant_int4(_np_ptr(w), _ld(w), rows, cols, group, _np_ptr(q), _np_ptr(qparams)))
    return q, qparams


def fit_verify_cost(m, t):
    m = np.ascontiguousarray(m, dtype=np.int32)
    t = np.ascontiguousarray(t, dtype=np.float64)
    a, b = C.c_double(), C.c_double()
    _check(lib().egt_fit_verify_cost(_np_ptr(m), _np_ptr(t), len(m), C.byref(a), C.byref(b)))
    return a.value, b.value


def trigger_depth(t_ar: float, a: float, b: float, cand, remaining):
    cand = np.ascontiguousarray(cand, dtype=np.int32)
    remaining = np.ascontiguousarray(remaining, dtype=np.int32)
    best, gain = C.c_int(), C.c_double()
    _check(lib().egt_trigger_depth(t_ar, a, b, _np_ptr(cand), _np_ptr(remaining), len(cand), C.byref(best), C.byref(gain)))
    return best.value, gain.value


# ------------------------------------------------------------------ device calls
def _stream_ptr(stream=None) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _dev(t):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return t.data_ptr()


# The C ABI sees pointers only: a tensor of the wrong type or too short would become an
# out-of-bounds access on the device, so sizes and types are checked here, on the host.
def _need(t, nbytes: int, what: str, f16: bool = False):
    import torch
    if f16 and t.dtype != torch.float16:
        raise ValueError(f"{what}: expected a float16 tensor, got {t.dtype}")
    if t.numel() * t.element_size() < nbytes:
        raise ValueError(f"{what}: {t.numel() * t.element_size()} bytes, needs {nbytes}")
    return _dev(t)


def _check_packed_dev(p: "Packed") -> None:
    b = p.sizes()
    for name, nb in zip(("row_ptr", "values", "idx", "qparams"), b):
        t = getattr(p, name)
        if t is None:
            if nb and name != "qparams":
                raise ValueError(f"packed matrix: {name} is missing")
            continue
        _need(t, nb, "packed matrix " + name)


def _check_int4_dev(q, qparams, rows: int, cols: int, group: int) -> None:
    if rows < 0 or cols < 0 or group <= 0 or cols % group:
        return                                           # the library reports the shape error
    _need(q, rows * (cols // 2), "q")
    _need(qparams, 4 * rows * (cols // group), "qparams")


def int4_gemv(q, qparams, rows: int, cols: int, group: int, x, y, stream=None) -> None:
    """q, qparams, x, y: device tensors (uint8 / int16-viewable / float16 / float16)."""
    _check_int4_dev(q, qparams, rows, cols, group)
    _check(lib().egt_int4_gemv(_dev(q), _dev(qparams), rows, cols, group, _need(x, 2 * cols, "x", True),
                               _need(y, 2 * rows, "y", True), _stream_ptr(stream)))


def sparse_gemv(p: Packed, x, y, stream=None) -> None:
    v = p.view()
    _check_packed_dev(p)
    _check(lib().egt_sparse_gemv(C.byref(v), _need(x, 2 * p.cols, "x", True), _need(y, 2 * p.rows, "y", True),
                                 _stream_ptr(stream)))


def _check_xy(p: "Packed", X, Y) -> None:
    import torch
    if X.dim() != 2 or Y.dim() != 2 or (X.shape[1] > 1 and X.stride(1) != 1) or (Y.shape[1] > 1 and Y.stride(1) != 1):
        raise ValueError("X and Y must be row-major 2-D tensors")
    if not (X.is_cuda and Y.is_cuda) or X.dtype != torch.float16 or Y.dtype != torch.float16:
        raise ValueError("X and Y must be float16 device tensors")
    if X.shape[1] != p.cols or tuple(Y.shape) != (X.shape[0], p.rows):
        raise ValueError(f"X must be (M, {p.cols}) and Y (M, {p.rows}); got {tuple(X.shape)} and {tuple(Y.shape)}")
    _check_packed_dev(p)


def sparse_gemm_smallm(p: Packed, X, Y, stream=None) -> None:
    """X: (M, K) float16 device tensor, Y: (M, R) float16 device tensor; rows may be strided."""
    _check_xy(p, X, Y)
    v = p.view()
    _check(lib().egt_sparse_gemm_smallm(C.byref(v), X.data_ptr(), X.stride(0), Y.data_ptr(),
                                        Y.stride(0), X.shape[0], _stream_ptr(stream)))


# Pre-marshalled calls: the arguments are converted once, the returned function only
# crosses the C ABI (for launch-rate-sensitive loops; same entry points, same checks).
# The stream defaults to the one current at preparation; pass `stream_ptr` (an int)
# to launch elsewhere, e.g. on a capturing stream.
def prepared_sparse_gemv(p: Packed, x, y, stream=None):
    fn, v = lib().egt_sparse_gemv, p.view()
    _check_packed_dev(p)
    ref, xp, yp, sp = C.byref(v), _need(x, 2 * p.cols, "x", True), _need(y, 2 * p.rows, "y", True), _stream_ptr(stream)

    def call(stream_ptr=sp, _keep=(v, p, x, y)):
        st = fn(ref, xp, yp, stream_ptr)
        if st:
            _check(st)
    return call


def prepared_sparse_gemm_smallm(p: Packed, X, Y, stream=None):
    fn, v = lib().egt_sparse_gemm_smallm, p.view()
    _check_xy(p, X, Y)
    args = (C.byref(v), X.data_ptr(), X.stride(0), Y.data_ptr(), Y.stride(0), X.shape[0])
    sp = _stream_ptr(stream)

    def call(stream_ptr=sp, _keep=(v, p, X, Y)):
        st = fn(*args, stream_ptr)
        if st:
            _check(st)
    return call


def smallm_ws_bytes(p: Packed, M: int, ldx=None) -> int:
    """Bytes of device workspace `sparse_gemm_smallm_ws` needs (0: none)."""
    out = C.c_size_t()
    v = p.view()
    _check(lib().egt_sparse_gemm_smallm_ws_bytes(C.byref(v), p.cols if ldx is None else ldx, M, C.byref(out)))
    return int(out.value)


def prepared_sparse_gemm_smallm_ws(p: Packed, X, Y, workspace, stream=None):
    """The K-split form; `workspace`: a device tensor of at least smallm_ws_bytes bytes (or None
    when that is 0)."""
    fn, v = lib().egt_sparse_gemm_smallm_ws, p.view()
    _check_xy(p, X, Y)
    need = smallm_ws_bytes(p, X.shape[0], X.stride(0))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        raise ValueError(f"workspace of {need} bytes required")
    wp = 0 if workspace is None else _dev(workspace)
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    args = (C.byref(v), X.data_ptr(), X.stride(0), Y.data_ptr(), Y.stride(0), X.shape[0], wp, wb)
    sp = _stream_ptr(stream)

    def call(stream_ptr=sp, _keep=(v, p, X, Y, workspace)):
        st = fn(*args, stream_ptr)
        if st:
            _check(st)
    return call


def sparse_gemm_smallm_static(p: Packed, X, Y, stream=None) -> None:
    """The K-split form on the library's built-in scratch buffer (allocates nothing)."""
    _check_xy(p, X, Y)
    v = p.view()
    _check(lib().egt_sparse_gemm_smallm_static(C.byref(v), X.data_ptr(), X.stride(0), Y.data_ptr(), Y.stride(0),
                                               X.shape[0], _stream_ptr(stream)))


def sparse_gemm_smallm_ws(p: Packed, X, Y, workspace, stream=None) -> None:
    prepared_sparse_gemm_smallm_ws(p, X, Y, workspace, stream)()


def prepared_int4_gemv(q, qparams, rows: int, cols: int, group: int, x, y, stream=None):
    fn = lib().egt_int4_gemv
    _check_int4_dev(q, qparams, rows, cols, group)
    args = (_dev(q), _dev(qparams), rows, cols, group, _need(x, 2 * cols, "x", True), _need(y, 2 * rows, "y", True))
    sp = _stream_ptr(stream)

    def call(stream_ptr=sp, _keep=(q, qparams, x, y)):
        st = fn(*args, stream_ptr)
        if st:
            _check(st)
    return call


def _ptr_array(tensors):
    return (C.c_void_p * len(tensors))(*[_dev(t) for t in tensors])


def prepared_sparse_gemv_batch(ps, xs, ys, stream=None):
    """One launch for len(ps) identically shaped matrices: ys[k] = W[k].xs[k]."""
    fn = lib().egt_sparse_gemv_batch
    for p, x, y in zip(ps, xs, ys):
        _check_packed_dev(p)
        _need(x, 2 * p.cols, "x", True)
        _need(y, 2 * p.rows, "y", True)
    views = (View * len(ps))(*[p.view() for p in ps])
    xa, ya, n, sp = _ptr_array(xs), _ptr_array(ys), len(ps), _stream_ptr(stream)

    def call(stream_ptr=sp, _keep=(views, ps, xs, ys, xa, ya)):
        st = fn(views, xa, ya, n, stream_ptr)
        if st:
            _check(st)
    return call


def prepared_sparse_gemm_smallm_batch(ps, Xs, Ys, stream=None):
    """One launch for len(ps) identically shaped matrices and M tokens each: Ys[k] = Xs[k] . W[k]^T.
    Xs[k]: (M, K), Ys[k]: (M, R) float16 device tensors, all Xs with one row stride, all Ys with one
    (the members may share one X)."""
    fn = lib().egt_sparse_gemm_smallm_batch
    for p, X, Y in zip(ps, Xs, Ys):
        _check_xy(p, X, Y)
        if X.shape[0] != Xs[0].shape[0] or X.stride(0) != Xs[0].stride(0) or Y.stride(0) != Ys[0].stride(0):
            raise ValueError("the members of a batch share M, ldx and ldy")
    views = (View * len(ps))(*[p.view() for p in ps])
    xa = (C.c_void_p * len(ps))(*[X.data_ptr() for X in Xs])
    ya = (C.c_void_p * len(ps))(*[Y.data_ptr() for Y in Ys])
    args = (views, xa, Xs[0].stride(0), ya, Ys[0].stride(0), Xs[0].shape[0], len(ps))
    sp = _stream_ptr(stream)

    def call(stream_ptr=sp, _keep=(views, ps, Xs, Ys, xa, ya)):
        st = fn(*args, stream_ptr)
        if st:
            _check(st)
    return call


def sparse_gemm_smallm_batch(ps, Xs, Ys, stream=None) -> None:
    prepared_sparse_gemm_smallm_batch(ps, Xs, Ys, stream)()


def prepared_int4_gemv_batch(qs, qparams, rows: int, cols: int, group: int, xs, ys, stream=None):
    fn = lib().egt_int4_gemv_batch
    for q, qp, x, y in zip(qs, qparams, xs, ys):
        _check_int4_dev(q, qp, rows, cols, group)
        _need(x, 2 * cols, "x", True)
        _need(y, 2 * rows, "y", True)
    qa, pa, xa, ya = _ptr_array(qs), _ptr_array(qparams), _ptr_array(xs), _ptr_array(ys)
    n, sp = len(qs), _stream_ptr(stream)

    def call(stream_ptr=sp, _keep=(qs, qparams, xs, ys, qa, pa, xa, ya)):
        st = fn(qa, pa, rows, cols, group, xa, ya, n, stream_ptr)
        if st:
            _check(st)
    return call


def sparse_gemv_batch(ps, xs, ys, stream=None) -> None:
    prepared_sparse_gemv_batch(ps, xs, ys, stream)()


def int4_gemv_batch(qs, qparams, rows: int, cols: int, group: int, xs, ys, stream=None) -> None:
    prepared_int4_gemv_batch(qs, qparams, rows, cols, group, xs, ys, stream)()


STACK_AUTO, STACK_GRID, STACK_RESIDENT = 0, 1, 2


def prepared_gemv_stack(items, stream=None, form=STACK_AUTO):
    """One launch for a list of products of different shapes and storage forms.

    items: tuples ("sparse", Packed, x, y) or ("dense", q, qparams, rows, cols, group, x, y)
    with device tensors.  The descriptor table is planned by the library on the host and
    uploaded here into a device tensor that the returned call keeps alive."""
    import torch
    n = len(items)
    arr = (GemvItem * n)()
    views, keep = [], []
    for k, it in enumerate(items):
        if it[0] == "sparse":
            _, p, x, y = it
            _check_packed_dev(p)
            v = p.view()
            views.append(v)
            arr[k].sparse = C.pointer(v)
            arr[k].x, arr[k].y = _need(x, 2 * p.cols, "x", True), _need(y, 2 * p.rows, "y", True)
            keep.append((p, x, y))
        else:
            _, q, qp, rows, cols, group, x, y = it
            _check_int4_dev(q, qp, rows, cols, group)
            arr[k].q, arr[k].qparams = _dev(q), _dev(qp)
            arr[k].rows, arr[k].cols, arr[k].group = rows, cols, group
            arr[k].x, arr[k].y = _need(x, 2 * cols, "x", True), _need(y, 2 * rows, "y", True)
            keep.append((q, qp, x, y))
    plan = StackPlan()
    _check(lib().egt_gemv_stack_plan(arr, n, form, None, 0, C.byref(plan)))    # size query
    table = np.zeros(int(plan.table_bytes), dtype=np.uint8)
    _check(lib().egt_gemv_stack_plan(arr, n, form, _np_ptr(table), table.nbytes, C.byref(plan)))
    dev = keep[0][-1].device
    table_dev = torch.from_numpy(table).to(dev)
    fn, tp, ref, sp = lib().egt_gemv_stack_run, table_dev.data_ptr(), C.byref(plan), _stream_ptr(stream)

    def call(stream_ptr=sp, _keep=(table_dev, plan, keep, views, arr)):
        st = fn(tp, ref, stream_ptr)
        if st:
            _check(st)
    call.plan = plan
    return call


def _prepared_gemm_table(items, M, stream):
    import torch
    n = len(items)
    arr = (GemmItem * n)()
    views = []
    for k, (p, X, Y) in enumerate(items):
        v = p.view()
        views.append(v)
        arr[k].sparse = C.pointer(v)
        arr[k].X, arr[k].Y = _dev(X), _dev(Y)
    plan = GemmPlan()
    _check(lib().egt_gemm_stack_plan(arr, n, M, None, 0, C.byref(plan)))    # size query
    table = np.zeros(int(plan.table_bytes), dtype=np.uint8)
    _check(lib().egt_gemm_stack_plan(arr, n, M, _np_ptr(table), table.nbytes, C.byref(plan)))
    table_dev = torch.from_numpy(table).to(items[0][2].device)
    return lib().egt_gemm_stack_run, table_dev.data_ptr(), C.byref(plan), plan, (table_dev, views, arr, items)


def prepared_gemm_stack(items, stream=None):
    """One launch per storage form for a list of small-M products Y = X . W^T under the same
    number of tokens.

    items: tuples (Packed, X, Y) with contiguous device tensors X (M, cols) and Y (M, rows).
    A list that holds 2:4 and 1:4 matrices becomes two tables (the library takes one form
    per table), run one after the other.  The descriptor tables are planned by the library
    on the host and uploaded here into device tensors that the returned call keeps alive."""
    if not items:
        raise ValueError("no items")
    M = int(items[0][1].shape[0])
    by_form = {}
    for (p, X, Y) in items:
        _check_xy(p, X, Y)
        if X.shape[0] != M or not X.is_contiguous() or not Y.is_contiguous():
            raise ValueError("every X and Y of the table must be contiguous and hold the same number of tokens")
        by_form.setdefault(p.n_keep, []).append((p, X, Y))
    tables = [_prepared_gemm_table(group, M, stream) for group in by_form.values()]
    sp = _stream_ptr(stream)

    def call(stream_ptr=sp, _tables=tables):
        for fn, tp, ref, _, _ in _tables:
            st = fn(tp, ref, stream_ptr)
            if st:
                _check(st)
    call.plans = [t[3] for t in tables]
    call.plan = call.plans[0]
    return call


def prepared_stream_read(src, nbytes: int, sink, stream=None):
    fn = lib().egt_stream_read
    if src.numel() * src.element_size() < nbytes or sink.numel() * sink.element_size() < 4 * 4096:
        raise ValueError("stream_read: src shorter than nbytes, or sink shorter than 4096 words")
    args = (_dev(src), nbytes, _dev(sink))
    sp = _stream_ptr(stream)

    def call(stream_ptr=sp, _keep=(src, sink)):
        st = fn(*args, stream_ptr)
        if st:
            _check(st)
    return call


def stream_read(src, nbytes: int, sink, stream=None) -> None:
    prepared_stream_read(src, nbytes, sink, stream)()
