"""Thin ctypes binding of the C ABI in include/comet.h.

Argument marshalling only: every function checks dtypes / devices / contiguity of the torch
tensors it is given, passes their device pointers and the current HIP stream to the library,
and wraps what comes back.  PyTorch is used for device memory and streams; all arithmetic runs
in the HIP kernels of libcomet_hip.so.  There is no fallback: if the shared library is missing
the import of this module's functions fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcomet_hip.so")

COMET_D, COMET_CU, COMET_CN, COMET_S = 0, 1, 2, 3
COMET_BORROW, COMET_COPY, COMET_VALIDATE, COMET_LEAN = 0, 1, 2, 4
COMET_OK = 0
COMET_MAX_ORDER = 4

_STATUS_NAMES = {0: "COMET_OK", 1: "COMET_ERR_INVALID_ARG", 2: "COMET_ERR_BAD_FORMAT", 3: "COMET_ERR_SHAPE",
                 4: "COMET_ERR_UNSUPPORTED", 5: "COMET_ERR_ALLOC", 6: "COMET_ERR_DEVICE"}

EXPORTS = ["comet_tensor_create", "comet_tensor_destroy", "comet_tensor_info", "comet_spmv", "comet_spmm",
           "comet_ttv", "comet_ttm", "comet_mttkrp", "comet_status_string", "comet_tensor_set_variant",
           "comet_tensor_reorder", "comet_tensor_convert", "comet_tensor_reserve", "comet_spmv_static",
           "comet_calibrate_read", "comet_calibrate_gather", "comet_spmv_axpby", "comet_spmm_axpby",
           "comet_mttkrp_axpby"]


class CometError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().comet_status_string(status).decode() if _LIB is not None else ""
        super().__init__("%s: %s (%s)" % (where, _STATUS_NAMES.get(status, status), msg))


class _Info(ctypes.Structure):
    _fields_ = [("order", ctypes.c_int32),
                ("dims", ctypes.c_int64 * COMET_MAX_ORDER),
                ("levels", ctypes.c_int32 * COMET_MAX_ORDER),
                ("pos", ctypes.c_void_p * COMET_MAX_ORDER),
                ("pos_len", ctypes.c_int64 * COMET_MAX_ORDER),
                ("crd", ctypes.c_void_p * COMET_MAX_ORDER),
                ("crd_len", ctypes.c_int64 * COMET_MAX_ORDER),
                ("vals", ctypes.c_void_p),
                ("nvals", ctypes.c_int64),
                ("mode_of_level", ctypes.c_int32 * COMET_MAX_ORDER),
                ("heavy_rows", ctypes.c_int64),
                ("heavy_nnz", ctypes.c_int64),
                ("heavy_stream_bytes", ctypes.c_int64)]


_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
                              "or paper_2102_05187_amd.build.build())" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        lib.comet_tensor_create.argtypes = [ctypes.POINTER(vp), ci, vp, vp, vp, vp, vp, vp, vp, i64, ctypes.c_uint, vp]
        lib.comet_tensor_destroy.argtypes = [vp]
        lib.comet_tensor_info.argtypes = [vp, ctypes.POINTER(_Info)]
        lib.comet_spmv.argtypes = [vp, vp, vp, vp]
        lib.comet_spmv_static.argtypes = [vp, vp, vp, vp]
        lib.comet_tensor_reserve.argtypes = [vp, i64, vp]
        lib.comet_calibrate_read.argtypes = [vp, i64, vp, vp]
        lib.comet_calibrate_gather.argtypes = [vp, i64, i64, i64, vp, vp]
        lib.comet_spmm.argtypes = [vp, vp, i64, vp, vp]
        lib.comet_ttv.argtypes = [vp, ci, vp, ctypes.POINTER(vp), vp]
        lib.comet_ttm.argtypes = [vp, ci, vp, i64, ctypes.POINTER(vp), vp]
        lib.comet_mttkrp.argtypes = [vp, ci, vp, i64, vp, vp]
        f64 = ctypes.c_double
        lib.comet_spmv_axpby.argtypes = [vp, f64, vp, f64, vp, vp]
        lib.comet_spmm_axpby.argtypes = [vp, f64, vp, i64, f64, vp, vp]
        lib.comet_mttkrp_axpby.argtypes = [vp, ci, f64, vp, i64, f64, vp, vp]
        lib.comet_tensor_set_variant.argtypes = [vp, ci]
        lib.comet_tensor_reorder.argtypes = [vp, vp, ctypes.POINTER(vp), vp]
        lib.comet_tensor_convert.argtypes = [vp, vp, vp, ctypes.POINTER(vp), vp]
        lib.comet_status_string.argtypes = [ci]
        lib.comet_status_string.restype = ctypes.c_char_p
        for n in EXPORTS:
            if n != "comet_status_string":
                getattr(lib, n).restype = ci
        _LIB = lib
    return _LIB


def _check(status: int, where: str):
    if status != COMET_OK:
        raise CometError(status, where)


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev(t: Optional[torch.Tensor], dtype, what: str) -> Optional[torch.Tensor]:
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a torch tensor in device memory" % what)
    if t.dtype != dtype:
        raise TypeError("%s must have dtype %s, got %s" % (what, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % what)
    return t


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None or t.numel() == 0 else t.data_ptr()


class _DeviceView:
    """Exposes a raw device pointer through __cuda_array_interface__ so torch can wrap it."""

    def __init__(self, ptr: int, n: int, typestr: str, owner):
        self.__cuda_array_interface__ = {"shape": (n,), "typestr": typestr, "data": (ptr, False), "version": 2}
        self._owner = owner


class Tensor:
    """A library tensor handle plus the torch tensors it borrows (kept alive with it)."""

    def __init__(self, handle: int, keep: Sequence = (), parent: "Tensor" = None):
        self._h = ctypes.c_void_p(handle)
        self._keep = list(keep)
        self._parent = parent      # a result shares level arrays with its input
        self._dims = None

    @property
    def handle(self) -> ctypes.c_void_p:
        if not self._h:
            raise ValueError("tensor handle was destroyed")
        return self._h

    def info(self) -> _Info:
        inf = _Info()
        _check(_lib().comet_tensor_info(self.handle, ctypes.byref(inf)), "comet_tensor_info")
        return inf

    def _wrap(self, ptr, n, typestr, dtype, copy=True):
        if not ptr or n == 0:
            return torch.empty(0, dtype=dtype, device="cuda")
        view = torch.as_tensor(_DeviceView(ptr, n, typestr, self), device="cuda")
        return view.clone() if copy else view

    def levels(self) -> List[int]:
        inf = self.info()
        return [int(inf.levels[l]) for l in range(inf.order)]

    def dims(self) -> List[int]:
        # sizes per level never change for a handle: looked up once (the products are launch-bound on small inputs)
        if self._dims is None:
            inf = self.info()
            self._dims = [int(inf.dims[l]) for l in range(inf.order)]
        return list(self._dims)

    def mode_of_level(self) -> List[int]:
        inf = self.info()
        return [int(inf.mode_of_level[l]) for l in range(inf.order)]

    def heavy_plan(self):
        """(rows, nonzeros) that comet_spmm hands to its heavy-row sweep; (0, 0) when none is planned."""
        inf = self.info()
        return int(inf.heavy_rows), int(inf.heavy_nnz)

    def heavy_stream_bytes(self) -> int:
        """Device memory held by the re-ordered copy of the heavy rows that the sweep reads (0: no sweep planned)."""
        return int(self.info().heavy_stream_bytes)

    def mode_dims(self) -> List[int]:
        """Sizes indexed by tensor mode (dims() is indexed by level)."""
        inf = self.info()
        out = [0] * inf.order
        for l in range(inf.order):
            out[int(inf.mode_of_level[l])] = int(inf.dims[l])
        return out

    def pos(self, l: int) -> Optional[torch.Tensor]:
        inf = self.info()
        return None if inf.pos_len[l] == 0 else self._wrap(inf.pos[l], inf.pos_len[l], "<i4", torch.int32)

    def crd(self, l: int) -> Optional[torch.Tensor]:
        inf = self.info()
        if int(inf.levels[l]) == COMET_D:
            return None
        return self._wrap(inf.crd[l], inf.crd_len[l], "<i4", torch.int32)

    def vals(self, copy: bool = True) -> torch.Tensor:
        """The value array; copy=False returns a view of the library's memory (valid while the handle lives)."""
        inf = self.info()
        return self._wrap(inf.vals, inf.nvals, "<f8", torch.float64, copy)

    def reserve(self, R: int, stream=None) -> "Tensor":
        _check(_lib().comet_tensor_reserve(self.handle, int(R), _stream(stream)), "comet_tensor_reserve")
        return self

    def set_variant(self, variant: int) -> "Tensor":
        _check(_lib().comet_tensor_set_variant(self.handle, variant), "comet_tensor_set_variant")
        return self

    def destroy(self):
        if self._h:
            _check(_lib().comet_tensor_destroy(self._h), "comet_tensor_destroy")
            self._h = ctypes.c_void_p(None)
            self._keep = []

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def comet_tensor_create(dims: Sequence[int], levels: Sequence[int], pos: Sequence[Optional[torch.Tensor]],
                        crd: Sequence[Optional[torch.Tensor]], vals: torch.Tensor,
                        flags: int = COMET_VALIDATE, stream=None) -> Tensor:
    order = len(dims)
    if not (len(levels) == len(pos) == len(crd) == order):
        raise ValueError("dims, levels, pos and crd must have one entry per level")
    pos = [_dev(p, torch.int32, "pos[%d]" % l) for l, p in enumerate(pos)]
    crd = [_dev(c, torch.int32, "crd[%d]" % l) for l, c in enumerate(crd)]
    vals = _dev(vals, torch.float64, "vals")
    c_dims = (ctypes.c_int64 * order)(*[int(d) for d in dims])
    c_lv = (ctypes.c_int * order)(*[int(t) for t in levels])
    c_pos = (ctypes.c_void_p * order)(*[_ptr(p) for p in pos])
    c_crd = (ctypes.c_void_p * order)(*[_ptr(c) for c in crd])
    c_pl = (ctypes.c_int64 * order)(*[0 if p is None else p.numel() for p in pos])
    c_cl = (ctypes.c_int64 * order)(*[0 if c is None else c.numel() for c in crd])
    out = ctypes.c_void_p(None)
    st = _lib().comet_tensor_create(ctypes.byref(out), order, c_dims, c_lv, c_pos, c_pl, c_crd, c_cl,
                                    _ptr(vals), vals.numel(), flags, _stream(stream))
    _check(st, "comet_tensor_create")
    keep = [] if (flags & COMET_COPY) else [*pos, *crd, vals]
    return Tensor(out.value, keep)


def comet_tensor_destroy(t: Tensor):
    t.destroy()


def comet_tensor_reorder(X: Tensor, mode_order: Sequence[int], stream=None) -> Tensor:
    order = len(X.dims())
    if len(mode_order) != order:
        raise CometError(1, "comet_tensor_reorder")
    c_order = (ctypes.c_int32 * order)(*[int(m) for m in mode_order])
    out = ctypes.c_void_p(None)
    _check(_lib().comet_tensor_reorder(X.handle, c_order, ctypes.byref(out), _stream(stream)), "comet_tensor_reorder")
    return Tensor(out.value)


def comet_tensor_convert(X: Tensor, mode_order: Sequence[int], levels: Sequence[int], stream=None) -> Tensor:
    order = len(X.dims())
    if len(mode_order) != order or len(levels) != order:
        raise CometError(1, "comet_tensor_convert")
    c_order = (ctypes.c_int32 * order)(*[int(m) for m in mode_order])
    c_lv = (ctypes.c_int * order)(*[int(t) for t in levels])
    out = ctypes.c_void_p(None)
    _check(_lib().comet_tensor_convert(X.handle, c_order, c_lv, ctypes.byref(out), _stream(stream)), "comet_tensor_convert")
    return Tensor(out.value)


def comet_spmv(A: Tensor, x: torch.Tensor, y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    x = _dev(x, torch.float64, "x")
    if len(A.dims()) != 2:
        raise CometError(4, "comet_spmv")
    I, J = A.dims()
    if x.numel() != J:
        raise CometError(3, "comet_spmv")
    if y is None:
        y = torch.empty(I, dtype=torch.float64, device=x.device)
    y = _dev(y, torch.float64, "y")
    if y.numel() != I:
        raise CometError(3, "comet_spmv")
    _check(_lib().comet_spmv(A.handle, x.data_ptr(), y.data_ptr(), _stream(stream)), "comet_spmv")
    return y


def comet_spmv_axpby(A: Tensor, alpha: float, x: torch.Tensor, beta: float, y: torch.Tensor, stream=None) -> torch.Tensor:
    """y = alpha * A x + beta * y, in place."""
    x, y = _dev(x, torch.float64, "x"), _dev(y, torch.float64, "y")
    if len(A.dims()) != 2:
        raise CometError(4, "comet_spmv_axpby")
    I, J = A.dims()
    if x.numel() != J or y.numel() != I:
        raise CometError(3, "comet_spmv_axpby")
    _check(_lib().comet_spmv_axpby(A.handle, float(alpha), x.data_ptr(), float(beta), y.data_ptr(), _stream(stream)),
           "comet_spmv_axpby")
    return y


def comet_spmm_axpby(A: Tensor, alpha: float, B: torch.Tensor, beta: float, C: torch.Tensor, stream=None) -> torch.Tensor:
    """C = alpha * A B + beta * C, in place."""
    B, C = _dev(B, torch.float64, "B"), _dev(C, torch.float64, "C")
    if len(A.dims()) != 2:
        raise CometError(4, "comet_spmm_axpby")
    I, J = A.dims()
    if B.dim() != 2 or B.shape[0] != J or tuple(C.shape) != (I, B.shape[1]):
        raise CometError(3, "comet_spmm_axpby")
    _check(_lib().comet_spmm_axpby(A.handle, float(alpha), B.data_ptr(), B.shape[1], float(beta), C.data_ptr(),
                                   _stream(stream)), "comet_spmm_axpby")
    return C


def comet_spmv_static(A: Tensor, x: torch.Tensor, y: torch.Tensor, stream=None) -> torch.Tensor:
    """comet_spmv for callers that cannot allocate: the caller passes y, the library's scratch is static."""
    x, y = _dev(x, torch.float64, "x"), _dev(y, torch.float64, "y")
    if len(A.dims()) != 2:
        raise CometError(4, "comet_spmv_static")
    I, J = A.dims()
    if x.numel() != J or y.numel() != I:
        raise CometError(3, "comet_spmv_static")
    _check(_lib().comet_spmv_static(A.handle, x.data_ptr(), y.data_ptr(), _stream(stream)), "comet_spmv_static")
    return y


def comet_calibrate_read(data: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    data, sink = _dev(data, torch.float64, "data"), _dev(sink, torch.float64, "sink")
    _check(_lib().comet_calibrate_read(data.data_ptr(), data.numel(), sink.data_ptr(), _stream(stream)), "comet_calibrate_read")


def comet_calibrate_gather(table: torch.Tensor, gathers: int, sink: torch.Tensor, stream=None) -> None:
    table, sink = _dev(table, torch.float64, "table"), _dev(sink, torch.float64, "sink")
    if table.dim() != 2:
        raise CometError(3, "comet_calibrate_gather")
    _check(_lib().comet_calibrate_gather(table.data_ptr(), table.shape[0], table.shape[1], int(gathers), sink.data_ptr(),
                                         _stream(stream)), "comet_calibrate_gather")


def comet_spmm(A: Tensor, B: torch.Tensor, C: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    B = _dev(B, torch.float64, "B")
    if len(A.dims()) != 2:
        raise CometError(4, "comet_spmm")
    I, J = A.dims()
    if B.dim() != 2 or B.shape[0] != J:
        raise CometError(3, "comet_spmm")
    R = B.shape[1]
    if C is None:
        C = torch.empty((I, R), dtype=torch.float64, device=B.device)
    C = _dev(C, torch.float64, "C")
    if tuple(C.shape) != (I, R):
        raise CometError(3, "comet_spmm")
    _check(_lib().comet_spmm(A.handle, B.data_ptr(), R, C.data_ptr(), _stream(stream)), "comet_spmm")
    return C


def comet_ttv(X: Tensor, mode: int, v: torch.Tensor, Y: Optional[Tensor] = None, stream=None) -> Tensor:
    v = _dev(v, torch.float64, "v")
    dims = X.mode_dims()
    if len(dims) != 3:
        raise CometError(4, "comet_ttv")
    if 0 <= mode < 3 and v.numel() != dims[mode]:
        raise CometError(3, "comet_ttv")
    h = ctypes.c_void_p(Y.handle.value if Y is not None else None)
    _check(_lib().comet_ttv(X.handle, mode, v.data_ptr(), ctypes.byref(h), _stream(stream)), "comet_ttv")
    return Y if Y is not None else Tensor(h.value, parent=X)


def comet_ttm(X: Tensor, mode: int, U: torch.Tensor, Y: Optional[Tensor] = None, stream=None) -> Tensor:
    U = _dev(U, torch.float64, "U")
    dims = X.mode_dims()
    if len(dims) != 3:
        raise CometError(4, "comet_ttm")
    if U.dim() != 2 or (0 <= mode < 3 and U.shape[0] != dims[mode]):
        raise CometError(3, "comet_ttm")
    h = ctypes.c_void_p(Y.handle.value if Y is not None else None)
    _check(_lib().comet_ttm(X.handle, mode, U.data_ptr(), U.shape[1], ctypes.byref(h), _stream(stream)), "comet_ttm")
    return Y if Y is not None else Tensor(h.value, parent=X)


def comet_mttkrp(X: Tensor, mode: int, factors: Sequence[Optional[torch.Tensor]],
                 M: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    dims = X.mode_dims()
    if len(dims) != 3 or len(factors) != 3:
        raise CometError(4, "comet_mttkrp")
    fs = [None if (f is None or l == mode) else _dev(f, torch.float64, "factors[%d]" % l) for l, f in enumerate(factors)]
    R = None
    for l, f in enumerate(fs):
        if f is None:
            continue
        if f.dim() != 2 or f.shape[0] != dims[l] or (R is not None and f.shape[1] != R):
            raise CometError(3, "comet_mttkrp")
        R = f.shape[1]
    if R is None or not (0 <= mode < 3):
        raise CometError(1, "comet_mttkrp")
    dev = next(f for f in fs if f is not None).device
    if M is None:
        M = torch.empty((dims[mode], R), dtype=torch.float64, device=dev)
    M = _dev(M, torch.float64, "M")
    if tuple(M.shape) != (dims[mode], R):
        raise CometError(3, "comet_mttkrp")
    c_f = (ctypes.c_void_p * 3)(*[_ptr(f) for f in fs])
    _check(_lib().comet_mttkrp(X.handle, mode, c_f, R, M.data_ptr(), _stream(stream)), "comet_mttkrp")
    return M


def comet_mttkrp_axpby(X: Tensor, mode: int, alpha: float, factors: Sequence[Optional[torch.Tensor]], beta: float,
                       M: torch.Tensor, stream=None) -> torch.Tensor:
    """M = alpha * MTTKRP(X, factors) + beta * M, in place."""
    dims = X.mode_dims()
    if len(dims) != 3 or len(factors) != 3:
        raise CometError(4, "comet_mttkrp_axpby")
    fs = [None if (f is None or l == mode) else _dev(f, torch.float64, "factors[%d]" % l) for l, f in enumerate(factors)]
    R = None
    for l, f in enumerate(fs):
        if f is None:
            continue
        if f.dim() != 2 or f.shape[0] != dims[l] or (R is not None and f.shape[1] != R):
            raise CometError(3, "comet_mttkrp_axpby")
        R = f.shape[1]
    if R is None or not (0 <= mode < 3):
        raise CometError(1, "comet_mttkrp_axpby")
    M = _dev(M, torch.float64, "M")
    if tuple(M.shape) != (dims[mode], R):
        raise CometError(3, "comet_mttkrp_axpby")
    c_f = (ctypes.c_void_p * 3)(*[_ptr(f) for f in fs])
    _check(_lib().comet_mttkrp_axpby(X.handle, mode, float(alpha), c_f, R, float(beta), M.data_ptr(), _stream(stream)),
           "comet_mttkrp_axpby")
    return M


def from_levels(T, flags: int = COMET_VALIDATE, stream=None) -> Tensor:
    """Create a handle from a synth.LevelTensor-like object (dims, tags, pos, crd, vals on the GPU)."""
    return comet_tensor_create(T.dims, T.tags, T.pos, T.crd, T.vals, flags, stream)
