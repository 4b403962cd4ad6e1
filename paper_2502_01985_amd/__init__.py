"""Python binding of libilargi (MI355X / gfx950): factorized linear algebra over
``T = sum_k I_k D_k M_k^T`` (paper, Sec. 2.1-2.2).

The binding only marshals arguments: torch tensors become raw device pointers plus the current
HIP stream, and every step of every operator runs in the library's kernels.  There is no CPU or
PyTorch fallback: importing this package fails if the compiled library is missing.

Functions carry the names of the C entry points declared in ``include/ilargi.h``.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libilargi.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
        "or python paper_2502_01985_amd/build.py). There is no fallback path.")

# PyTorch ships its own copy of the HIP runtime.  It has to be in the process before libilargi.so is
# loaded so that the library binds to that same runtime (same soname) and shares torch's device context.
import torch  # noqa: E402,F401

lib = ctypes.CDLL(LIB_PATH)

OK, ERR_NULL, ERR_SHAPE, ERR_COLMAP, ERR_INDEX_RANGE, ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_DEVICE = range(8)
F32, BF16_IN_F32_ACC = 0, 1
LINEAR, LOGISTIC = 0, 1
STATUS_NAMES = ["OK", "ERR_NULL", "ERR_SHAPE", "ERR_COLMAP", "ERR_INDEX_RANGE", "ERR_WORKSPACE",
                "ERR_UNSUPPORTED", "ERR_DEVICE"]

EXPORTED = [
    "ilargi_plan_workspace_bytes", "ilargi_plan_create", "ilargi_plan_create_static", "ilargi_plan_destroy",
    "ilargi_plan_cluster_bytes", "ilargi_plan_cluster", "ilargi_lmm", "ilargi_tmm",
    "ilargi_rmm", "ilargi_crossprod", "ilargi_materialize", "ilargi_gd_step", "ilargi_kmeans_step", "ilargi_gnmf_step",
    "ilargi_elementwise", "ilargi_row_sum",
    "ilargi_col_sum", "ilargi_choose", "ilargi_segment_sum",
    "ilargi_plan_inverse_index", "ilargi_plan_trace_begin", "ilargi_plan_trace_label", "ilargi_plan_trace_end",
    "ilargi_plan_trace_name", "ilargi_stream_probe",
    "ilargi_static_scratch_bytes",
    "ilargi_last_error",
    "ilargi_version",
]


class SourceStruct(ctypes.Structure):
    _fields_ = [("D", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("row_idx", ctypes.c_void_p), ("col_map", ctypes.c_void_p),
                ("csr_rowptr", ctypes.c_void_p), ("csr_col", ctypes.c_void_p), ("csr_val", ctypes.c_void_p),
                ("nnz", ctypes.c_int64)]


_vp, _i64, _int = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
lib.ilargi_plan_workspace_bytes.argtypes = [_int, ctypes.POINTER(SourceStruct), _i64, _i64, _i64,
                                            ctypes.POINTER(ctypes.c_size_t)]
lib.ilargi_plan_create.argtypes = [_int, ctypes.POINTER(SourceStruct), _i64, _i64, _i64, _vp, ctypes.c_size_t, _vp,
                                   ctypes.POINTER(_vp)]
lib.ilargi_plan_create_static.argtypes = [_int, ctypes.POINTER(SourceStruct), _i64, _i64, _i64, _vp, ctypes.POINTER(_vp)]
lib.ilargi_static_scratch_bytes.argtypes = []
lib.ilargi_plan_destroy.argtypes = [_vp]
lib.ilargi_plan_cluster_bytes.argtypes = [_vp, ctypes.POINTER(ctypes.c_size_t)]
lib.ilargi_plan_cluster.argtypes = [_vp, _vp, ctypes.c_size_t, _vp, _vp]
lib.ilargi_lmm.argtypes = [_vp, _vp, _i64, _vp, _int, _vp]
lib.ilargi_tmm.argtypes = [_vp, _vp, _i64, _vp, _int, _vp]
lib.ilargi_rmm.argtypes = [_vp, _vp, _i64, _vp, _int, _vp]
lib.ilargi_crossprod.argtypes = [_vp, _vp, _vp]
lib.ilargi_materialize.argtypes = [_vp, _vp, _vp]
lib.ilargi_gd_step.argtypes = [_vp, _int, _vp, _i64, _vp, _vp, _vp, _int, _vp]
lib.ilargi_kmeans_step.argtypes = [_vp, _vp, _i64, _vp, _vp, _vp]
lib.ilargi_gnmf_step.argtypes = [_vp, _vp, _vp, _i64, _vp]
lib.ilargi_segment_sum.argtypes = [_vp, _int, _vp, _i64, _vp, _vp]
lib.ilargi_elementwise.argtypes = [_vp, _int, ctypes.c_float, _vp, _vp]
lib.ilargi_row_sum.argtypes = [_vp, _vp, _vp]
lib.ilargi_col_sum.argtypes = [_vp, _vp, _vp]
lib.ilargi_plan_inverse_index.argtypes = [_vp, _int, ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.POINTER(_i64)]
lib.ilargi_plan_trace_begin.argtypes = [_vp, ctypes.c_char_p, _int]
lib.ilargi_plan_trace_end.argtypes = [_vp, ctypes.POINTER(ctypes.c_float), _int, ctypes.POINTER(_int)]
lib.ilargi_plan_trace_label.argtypes = [_vp, ctypes.c_char_p]
lib.ilargi_plan_trace_name.argtypes = [_vp, _int, ctypes.c_char_p, _int]
lib.ilargi_stream_probe.argtypes = [_int, _vp, _vp, _i64, _int, _vp]
for _name in EXPORTED[:-3]:
    getattr(lib, _name).restype = _int
lib.ilargi_static_scratch_bytes.restype = ctypes.c_size_t
lib.ilargi_last_error.restype = ctypes.c_char_p
lib.ilargi_version.restype = ctypes.c_char_p


class IlargiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.ilargi_last_error().decode()
        super().__init__(f"{where}: {STATUS_NAMES[status] if 0 <= status < 8 else status}: {msg}")


def _check(status: int, where: str) -> None:
    if status != OK:
        raise IlargiError(status, where)


def ilargi_last_error() -> str:
    return lib.ilargi_last_error().decode()


def ilargi_version() -> str:
    return lib.ilargi_version().decode()


def _torch():
    import torch
    return torch


def _stream_ptr(stream=None) -> int:
    torch = _torch()
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _dev_f32(t, name: str):
    torch = _torch()
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous float32 CUDA tensor")
    return t


class CSR:
    """A source table in compressed sparse rows: int32 CUDA tensors ``rowptr`` (rows + 1) and ``col`` (nnz), a
    float32 CUDA tensor ``val`` (nnz), and the dense shape."""

    def __init__(self, rowptr, col, val, shape):
        self.rowptr, self.col, self.val = rowptr, col, val
        self.shape = (int(shape[0]), int(shape[1]))

    @property
    def nnz(self) -> int:
        return int(self.val.numel())

    @property
    def device(self):
        return self.rowptr.device

    @classmethod
    def from_dense(cls, D: np.ndarray, device="cuda:0"):
        """Keeps the non-zero cells of a host array (row-major order, so columns ascend within a row)."""
        torch = _torch()
        D = np.asarray(D, dtype=np.float32)
        r, c = np.nonzero(D)
        rowptr = np.zeros(D.shape[0] + 1, dtype=np.int32)
        np.cumsum(np.bincount(r, minlength=D.shape[0]), out=rowptr[1:])
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
        return cls(t(rowptr), t(c.astype(np.int32)), t(D[r, c]), D.shape)


def make_source_array(sources: Sequence[tuple]):
    """ctypes array from ``(D_ptr, rows, cols, row_idx_ptr_or_0, col_map int32 ndarray)`` tuples, optionally
    extended by ``(csr_rowptr_ptr, csr_col_ptr, csr_val_ptr, nnz)``.
    Returns the array and the objects that must stay alive while it is used."""
    arr = (SourceStruct * len(sources))()
    keep = []
    for k, src in enumerate(sources):
        dptr, rows, cols, iptr, cmap = src[:5]
        cm = np.ascontiguousarray(cmap, dtype=np.int32)
        keep.append(cm)
        arr[k].D = dptr or None
        arr[k].rows = rows
        arr[k].cols = cols
        arr[k].row_idx = iptr or None
        arr[k].col_map = cm.ctypes.data if cm.size else None
        if len(src) > 5:
            arr[k].csr_rowptr, arr[k].csr_col, arr[k].csr_val = src[5] or None, src[6] or None, src[7] or None
            arr[k].nnz = src[8]
    return arr, keep


def ilargi_plan_workspace_bytes(sources, r_T: int, c_T: int, max_cx: int) -> int:
    arr, _keep = make_source_array(sources)
    out = ctypes.c_size_t(0)
    _check(lib.ilargi_plan_workspace_bytes(len(sources), arr, r_T, c_T, max_cx, ctypes.byref(out)),
           "ilargi_plan_workspace_bytes")
    return int(out.value)


class Plan:
    """Owns the plan handle, its device workspace and references to the borrowed tensors."""

    def __init__(self, handle: int, workspace, borrowed, r_T: int, c_T: int, max_cx: int, src_shapes, device=None):
        self.handle = handle
        self.workspace = workspace          # None: the plan lives in the library's static scratch array
        self.device = device if device is not None else workspace.device
        self._borrowed = borrowed
        self.r_T, self.c_T, self.max_cx = r_T, c_T, max_cx
        self.src_shapes = src_shapes
        self._cluster = None                # (buffer, labels) handed to ilargi_plan_cluster: kept alive with the plan

    def destroy(self) -> None:
        if self.handle:
            lib.ilargi_plan_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _marshal_sources(sources, r_T: int):
    torch = _torch()
    tuples, borrowed, shapes = [], [], []
    for D, row_idx, col_map in sources:
        if row_idx is not None:
            if not (row_idx.is_cuda and row_idx.dtype == torch.int32 and row_idx.is_contiguous()
                    and row_idx.numel() == r_T):
                raise TypeError("row_idx must be a contiguous int32 CUDA tensor of length r_T")
        iptr = row_idx.data_ptr() if row_idx is not None else 0
        if isinstance(D, CSR):
            for t_, dt in ((D.rowptr, torch.int32), (D.col, torch.int32), (D.val, torch.float32)):
                if not (t_.is_cuda and t_.dtype == dt and t_.is_contiguous()):
                    raise TypeError("CSR parts must be contiguous CUDA tensors: int32 rowptr, int32 col, float32 val")
            if D.rowptr.numel() != D.shape[0] + 1 or D.col.numel() != D.val.numel():
                raise TypeError("CSR parts have inconsistent lengths")
            borrowed.append((D, row_idx))
            shapes.append(D.shape)
            tuples.append((0, D.shape[0], D.shape[1], iptr, np.asarray(col_map, dtype=np.int32),
                           D.rowptr.data_ptr(), D.col.data_ptr() if D.nnz else 0, D.val.data_ptr() if D.nnz else 0, D.nnz))
            continue
        _dev_f32(D, "D")
        if D.dim() != 2:
            raise TypeError("D must be 2-D")
        borrowed.append((D, row_idx))
        shapes.append((int(D.shape[0]), int(D.shape[1])))
        tuples.append((D.data_ptr(), int(D.shape[0]), int(D.shape[1]), iptr, np.asarray(col_map, dtype=np.int32)))
    return tuples, borrowed, shapes


def _source_device(sources):
    D = sources[0][0]
    return D.device


def ilargi_plan_create(sources, r_T: int, c_T: int, max_cx: int = 1, stream=None) -> Plan:
    """``sources``: list of ``(D, row_idx, col_map)`` with ``D`` a float32 CUDA tensor ``r_k x c_k``,
    ``row_idx`` an int32 CUDA tensor of length ``r_T`` or ``None`` (identity) and ``col_map`` an int32
    host array of length ``c_k``."""
    torch = _torch()
    tuples, borrowed, shapes = _marshal_sources(sources, r_T)
    arr, keep = make_source_array(tuples)
    nbytes = ctypes.c_size_t(0)
    _check(lib.ilargi_plan_workspace_bytes(len(tuples), arr, r_T, c_T, max_cx, ctypes.byref(nbytes)),
           "ilargi_plan_workspace_bytes")
    workspace = torch.empty(int(nbytes.value) + 256, dtype=torch.uint8, device=_source_device(sources))
    base = workspace.data_ptr()
    aligned = (base + 255) // 256 * 256
    handle = _vp(0)
    _check(lib.ilargi_plan_create(len(tuples), arr, r_T, c_T, max_cx, aligned, int(nbytes.value),
                                  _stream_ptr(stream), ctypes.byref(handle)), "ilargi_plan_create")
    del keep
    return Plan(handle.value, workspace, borrowed, r_T, c_T, max_cx, shapes)


def ilargi_plan_cluster_bytes(plan: Plan) -> int:
    nbytes = ctypes.c_size_t(0)
    _check(lib.ilargi_plan_cluster_bytes(plan.handle, ctypes.byref(nbytes)), "ilargi_plan_cluster_bytes")
    return int(nbytes.value)


def ilargi_plan_cluster(plan: Plan, buffer="new", y=None, stream=None) -> None:
    """Keeps a join-ordered copy of the entity table of a two-table star join with the plan.  ``buffer``: a uint8
    CUDA tensor of at least ``ilargi_plan_cluster_bytes(plan)`` bytes (256-byte aligned), ``"new"`` to allocate one
    here, or ``None`` to make the plan forget the copy.  ``y``: the labels (float32 CUDA tensor of length r_T) to keep
    in join order as well; ``ilargi_gd_step`` called with this same tensor then reads them from the copy."""
    torch = _torch()
    if buffer is None:
        _check(lib.ilargi_plan_cluster(plan.handle, None, 0, None, _stream_ptr(stream)), "ilargi_plan_cluster")
        plan._cluster = None
        return
    if isinstance(buffer, str):
        buffer = torch.empty(ilargi_plan_cluster_bytes(plan), dtype=torch.uint8, device=plan.device)
    if not (buffer.is_cuda and buffer.dtype == torch.uint8 and buffer.is_contiguous()):
        raise TypeError("buffer must be a contiguous uint8 CUDA tensor")
    if y is not None:
        _dev_f32(y, "y")
        if y.numel() != plan.r_T:
            raise TypeError("y must have r_T entries")
    _check(lib.ilargi_plan_cluster(plan.handle, buffer.data_ptr(), buffer.numel(), y.data_ptr() if y is not None else None,
                                   _stream_ptr(stream)), "ilargi_plan_cluster")
    plan._cluster = (buffer, y)


def ilargi_static_scratch_bytes() -> int:
    return int(lib.ilargi_static_scratch_bytes())


def ilargi_plan_create_static(sources, r_T: int, c_T: int, max_cx: int = 1, stream=None) -> Plan:
    """Like ``ilargi_plan_create``, but the plan lives in the library's static scratch array: no device memory
    is allocated, here or in the library.  One such plan per device at a time (``plan.destroy()`` frees the array)."""
    torch = _torch()
    tuples, borrowed, shapes = _marshal_sources(sources, r_T)
    arr, keep = make_source_array(tuples)
    device = _source_device(sources)
    handle = _vp(0)
    with torch.cuda.device(device):
        _check(lib.ilargi_plan_create_static(len(tuples), arr, r_T, c_T, max_cx, _stream_ptr(stream),
                                             ctypes.byref(handle)), "ilargi_plan_create_static")
    del keep
    return Plan(handle.value, None, borrowed, r_T, c_T, max_cx, shapes, device=device)


def ilargi_lmm(plan: Plan, X, out=None, precision: int = F32, stream=None):
    torch = _torch()
    _dev_f32(X, "X")
    cx = X.shape[1] if X.dim() == 2 else 1
    if X.numel() != plan.c_T * cx:
        raise ValueError("X must be c_T x cx")
    if out is None:
        out = torch.empty((plan.r_T, cx), dtype=torch.float32, device=X.device)
    _dev_f32(out, "out")
    _check(lib.ilargi_lmm(plan.handle, X.data_ptr(), cx, out.data_ptr(), precision, _stream_ptr(stream)), "ilargi_lmm")
    return out


def ilargi_tmm(plan: Plan, Y, out=None, precision: int = F32, stream=None):
    torch = _torch()
    _dev_f32(Y, "Y")
    cx = Y.shape[1] if Y.dim() == 2 else 1
    if Y.numel() != plan.r_T * cx:
        raise ValueError("Y must be r_T x cx")
    if out is None:
        out = torch.empty((plan.c_T, cx), dtype=torch.float32, device=Y.device)
    _dev_f32(out, "out")
    _check(lib.ilargi_tmm(plan.handle, Y.data_ptr(), cx, out.data_ptr(), precision, _stream_ptr(stream)), "ilargi_tmm")
    return out


def ilargi_rmm(plan: Plan, X, out=None, precision: int = F32, stream=None):
    """``X`` is ``cx x r_T``; returns ``X T`` (``cx x c_T``)."""
    torch = _torch()
    _dev_f32(X, "X")
    cx = X.shape[0] if X.dim() == 2 else 1
    if X.numel() != plan.r_T * cx:
        raise TypeError("X must be cx x r_T")
    if out is None:
        out = torch.empty((cx, plan.c_T), dtype=torch.float32, device=plan.device)
    _dev_f32(out, "out")
    _check(lib.ilargi_rmm(plan.handle, X.data_ptr() if X.numel() else None, cx, out.data_ptr(), precision,
                          _stream_ptr(stream)), "ilargi_rmm")
    return out


def _dev_i32(t, name):
    torch = _torch()
    if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous int32 device tensor")


def ilargi_kmeans_step(plan: Plan, C, assign=None, counts=None, stream=None):
    """One Lloyd iteration; ``C`` (``c_T x k``, column j = centroid j) is updated in place.
    ``assign`` (int32[r_T]) and ``counts`` (int32[k]) are optional outputs."""
    _dev_f32(C, "C")
    k = C.shape[1] if C.dim() == 2 else 1
    if C.numel() != plan.c_T * k:
        raise TypeError("C must be c_T x k")
    if assign is not None:
        _dev_i32(assign, "assign")
        if assign.numel() != plan.r_T:
            raise TypeError("assign must hold r_T values")
    if counts is not None:
        _dev_i32(counts, "counts")
        if counts.numel() != k:
            raise TypeError("counts must hold k values")
    _check(lib.ilargi_kmeans_step(plan.handle, C.data_ptr(), k,
                                  assign.data_ptr() if assign is not None and assign.numel() else None,
                                  counts.data_ptr() if counts is not None else None, _stream_ptr(stream)),
           "ilargi_kmeans_step")
    return C


def ilargi_gnmf_step(plan: Plan, W, Ht, stream=None):
    """One round of multiplicative updates; ``W`` (``r_T x r``) and ``Ht`` (``c_T x r``, the transpose of H)
    are updated in place."""
    _dev_f32(W, "W"); _dev_f32(Ht, "Ht")
    r = Ht.shape[1] if Ht.dim() == 2 else 1
    if Ht.numel() != plan.c_T * r or W.numel() != plan.r_T * r:
        raise TypeError("W must be r_T x r and Ht c_T x r")
    _check(lib.ilargi_gnmf_step(plan.handle, W.data_ptr() if W.numel() else None, Ht.data_ptr(), r,
                                _stream_ptr(stream)), "ilargi_gnmf_step")
    return W, Ht


def ilargi_crossprod(plan: Plan, out=None, stream=None):
    torch = _torch()
    if out is None:
        out = torch.empty((plan.c_T, plan.c_T), dtype=torch.float32, device=plan.device)
    _dev_f32(out, "out")
    _check(lib.ilargi_crossprod(plan.handle, out.data_ptr(), _stream_ptr(stream)), "ilargi_crossprod")
    return out


def ilargi_materialize(plan: Plan, out=None, stream=None):
    torch = _torch()
    if out is None:
        out = torch.empty((plan.r_T, plan.c_T), dtype=torch.float32, device=plan.device)
    _dev_f32(out, "T")
    _check(lib.ilargi_materialize(plan.handle, out.data_ptr(), _stream_ptr(stream)), "ilargi_materialize")
    return out


def ilargi_gd_step(plan: Plan, model: int, W, y, lr, loss=None, precision: int = F32, stream=None):
    """In-place update of ``W`` (``c_T x m``); ``loss`` (optional, float32[m]) receives the pre-update loss."""
    _dev_f32(W, "W"); _dev_f32(y, "y"); _dev_f32(lr, "lr")
    m = W.shape[1] if W.dim() == 2 else 1
    if W.numel() != plan.c_T * m or y.numel() != plan.r_T or lr.numel() != m:
        raise ValueError("W must be c_T x m, y of length r_T, lr of length m")
    lptr = 0
    if loss is not None:
        _dev_f32(loss, "loss")
        if loss.numel() != m:
            raise ValueError("loss must have m entries")
        lptr = loss.data_ptr()
    _check(lib.ilargi_gd_step(plan.handle, model, W.data_ptr(), m, y.data_ptr(), lr.data_ptr(), lptr or None,
                              precision, _stream_ptr(stream)), "ilargi_gd_step")
    return W


class WorkloadStruct(ctypes.Structure):
    _fields_ = [("iterations", ctypes.c_int64), ("models", ctypes.c_int64), ("bytes_per_second", ctypes.c_double),
                ("launch_seconds", ctypes.c_double)]


class ChoiceStruct(ctypes.Structure):
    _fields_ = [("factorize", ctypes.c_int), ("complexity_ratio", ctypes.c_double), ("tuple_ratio", ctypes.c_double),
                ("feature_ratio", ctypes.c_double), ("morpheus_rule", ctypes.c_int), ("bytes_factorized", ctypes.c_double),
                ("bytes_materialized", ctypes.c_double), ("bytes_join", ctypes.c_double),
                ("seconds_factorized", ctypes.c_double), ("seconds_materialized", ctypes.c_double)]


lib.ilargi_choose.argtypes = [_int, ctypes.POINTER(SourceStruct), _i64, _i64, ctypes.POINTER(WorkloadStruct),
                              ctypes.POINTER(ChoiceStruct)]


def ilargi_choose(shapes, r_T: int, c_T: int, iterations: int = 200, models: int = 1,
                  bytes_per_second: float = 0.0, launch_seconds: float = 0.0) -> dict:
    """``shapes``: one ``(rows, cols, has_row_idx)`` or ``(rows, cols, has_row_idx, nnz)`` (a sparse table)
    per source.  Host-only; returns the fields of ``ilargi_choice_t`` as a dict."""
    arr = (SourceStruct * len(shapes))()
    for k, shp in enumerate(shapes):
        rows, cols, has = shp[:3]
        arr[k].D = None
        arr[k].rows, arr[k].cols = int(rows), int(cols)
        arr[k].row_idx = 1 if has else None      # only tested against NULL
        arr[k].col_map = None
        if len(shp) > 3:
            arr[k].csr_rowptr = 1                # only tested against NULL
            arr[k].nnz = int(shp[3])
    w = WorkloadStruct(int(iterations), int(models), float(bytes_per_second), float(launch_seconds))
    c = ChoiceStruct()
    _check(lib.ilargi_choose(len(shapes), arr, r_T, c_T, ctypes.byref(w), ctypes.byref(c)), "ilargi_choose")
    return {name: getattr(c, name) for name, _ in ChoiceStruct._fields_}


OPS = {"mul": 0, "div": 1, "add": 2, "sub": 3, "pow": 4, "exp": 5, "log": 6, "sqrt": 7, "abs": 8, "square": 9}


def ilargi_elementwise(plan: Plan, op, x: float = 0.0, outs=None, stream=None):
    """``op``: a name from ``OPS`` or its code.  ``outs``: one float32 CUDA tensor per source, shaped like
    the source tables (``None``: new tensors; the source tensors themselves: in place).  Returns ``outs``."""
    torch = _torch()
    code = OPS[op] if isinstance(op, str) else int(op)
    if outs is None:
        outs = [torch.empty_like(D.val if isinstance(D, CSR) else D) for D, _ in plan._borrowed]
    if len(outs) != len(plan._borrowed):
        raise TypeError("one output tensor per source")
    ptrs = (ctypes.c_void_p * len(outs))()
    for k, (o, (D, _)) in enumerate(zip(outs, plan._borrowed)):
        _dev_f32(o, "outs[k]")
        like = D.val if isinstance(D, CSR) else D
        if tuple(o.shape) != tuple(like.shape):
            raise TypeError("outs[k] must have the shape of source k (of its values for a sparse source)")
        ptrs[k] = o.data_ptr() if o.numel() > 0 else None
    _check(lib.ilargi_elementwise(plan.handle, code, float(x), ptrs, _stream_ptr(stream)), "ilargi_elementwise")
    return outs


def ilargi_row_sum(plan: Plan, out=None, stream=None):
    torch = _torch()
    if out is None:
        out = torch.empty(plan.r_T, dtype=torch.float32, device=plan.device)
    _dev_f32(out, "out")
    _check(lib.ilargi_row_sum(plan.handle, out.data_ptr() if out.numel() else None, _stream_ptr(stream)), "ilargi_row_sum")
    return out


def ilargi_col_sum(plan: Plan, out=None, stream=None):
    torch = _torch()
    if out is None:
        out = torch.empty(plan.c_T, dtype=torch.float32, device=plan.device)
    _dev_f32(out, "out")
    _check(lib.ilargi_col_sum(plan.handle, out.data_ptr(), _stream_ptr(stream)), "ilargi_col_sum")
    return out


def ilargi_segment_sum(plan: Plan, k: int, Y, out=None, stream=None):
    torch = _torch()
    _dev_f32(Y, "Y")
    cx = Y.shape[1] if Y.dim() == 2 else 1
    if Y.numel() != plan.r_T * cx:
        raise ValueError("Y must be r_T x cx")
    if out is None:
        out = torch.empty((plan.src_shapes[k][0], cx), dtype=torch.float32, device=Y.device)
    _check(lib.ilargi_segment_sum(plan.handle, k, Y.data_ptr(), cx, out.data_ptr(), _stream_ptr(stream)),
           "ilargi_segment_sum")
    return out


def ilargi_plan_inverse_index(plan: Plan, k: int):
    """``(rowptr, perm)`` of source ``k`` copied to host int32 arrays, or ``(None, None)`` for an identity source."""
    torch = _torch()
    rp, pm, nnz = _vp(0), _vp(0), _i64(0)
    _check(lib.ilargi_plan_inverse_index(plan.handle, k, ctypes.byref(rp), ctypes.byref(pm), ctypes.byref(nnz)),
           "ilargi_plan_inverse_index")
    if not rp.value:
        return None, None
    torch.cuda.synchronize()
    r_k = plan.src_shapes[k][0]

    def fetch(ptr, count):
        # a plain device-to-host copy of `count` int32 values through the HIP runtime the library is bound to
        host = np.empty(count, dtype=np.int32)
        if count:
            rc = lib.hipMemcpy(_vp(host.ctypes.data), _vp(ptr), ctypes.c_size_t(4 * count), 2)   # 2 = device to host
            if rc != 0:
                raise RuntimeError(f"hipMemcpy failed with {rc}")
        return host

    return fetch(rp.value, r_k + 1), fetch(pm.value, int(nnz.value))


def ilargi_plan_trace_begin(plan: Plan, tag: str, max_launches: int) -> None:
    _check(lib.ilargi_plan_trace_begin(plan.handle, tag.encode(), max_launches), "ilargi_plan_trace_begin")


def ilargi_plan_trace_label(plan: Plan, label: str) -> None:
    _check(lib.ilargi_plan_trace_label(plan.handle, label.encode()), "ilargi_plan_trace_label")


def ilargi_plan_trace_end(plan: Plan, capacity: int, names: bool = False):
    """Elapsed milliseconds of the traced launches (numpy float32 array); with ``names`` also their names."""
    buf = (ctypes.c_float * max(capacity, 1))()
    cnt = _int(0)
    got = []
    if names:
        # names have to be read before trace_end releases the events' bookkeeping of this run
        i = 0
        nb = ctypes.create_string_buffer(128)
        while lib.ilargi_plan_trace_name(plan.handle, i, nb, 128) == OK:
            got.append(nb.value.decode())
            i += 1
    _check(lib.ilargi_plan_trace_end(plan.handle, buf, capacity, ctypes.byref(cnt)), "ilargi_plan_trace_end")
    ms = np.array(buf[:min(cnt.value, capacity)], dtype=np.float32)
    return (ms, got[:len(ms)]) if names else ms


def ilargi_stream_probe(kind: int, dst, src, n_floats: int, blocks: int = 4096, stream=None) -> None:
    _check(lib.ilargi_stream_probe(kind, dst.data_ptr(), src.data_ptr() if src is not None else None, n_floats,
                                   blocks, _stream_ptr(stream)), "ilargi_stream_probe")


def schema_to_device(schema, device="cuda:0", sparse=False):
    """Uploads a ``datagen.Schema`` and returns the ``(D, row_idx, col_map)`` list for ilargi_plan_create.
    ``sparse``: ``True`` (every table) or a collection of source numbers to upload in compressed sparse rows."""
    torch = _torch()
    out = []
    for k, s in enumerate(schema.sources):
        as_csr = sparse is True or (sparse not in (False, None) and k in sparse)
        D = CSR.from_dense(s.D, device) if as_csr else torch.from_numpy(np.ascontiguousarray(s.D)).to(device)
        idx = None if s.row_idx is None else torch.from_numpy(np.ascontiguousarray(s.row_idx)).to(device)
        out.append((D, idx, s.col_map))
    return out
