"""Thin ctypes binding of libf3m.so (include/f3m.h): argument marshalling only.

Tensors are torch CUDA(HIP) tensors used purely as device memory; every step of
the path runs inside the library's kernels.  There is no fallback: if the
library is missing, importing a symbol from it raises.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libf3m.so")

MAX_DIM = 7
MAX_LEVELS = 20

STATUS = {0: "F3M_OK", 1: "F3M_ERR_INVALID_ARG", 2: "F3M_ERR_NONFINITE", 3: "F3M_ERR_UNSUPPORTED",
          4: "F3M_ERR_OOM", 5: "F3M_ERR_HIP", 6: "F3M_ERR_BREAKDOWN"}


class F3MError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("%s: %s" % (STATUS.get(status, status), msg))
        self.status = status


class Options(ctypes.Structure):
    _fields_ = [("leaf_max", ctypes.c_int32), ("max_depth", ctypes.c_int32),
                ("force_all_near", ctypes.c_int32), ("overlap", ctypes.c_int32),
                ("eta_smooth", ctypes.c_float), ("adaptive_far", ctypes.c_int32), ("small_field", ctypes.c_int32),
                ("route_min_points", ctypes.c_int32)]


class Info(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("D", ctypes.c_int32), ("interp_nodes", ctypes.c_int32),
                ("nodes_per_box", ctypes.c_int32), ("depth", ctypes.c_int32), ("quant_depth", ctypes.c_int32),
                ("far_threshold", ctypes.c_int32), ("edge", ctypes.c_float), ("scale", ctypes.c_float),
                ("alpha", ctypes.c_float * MAX_DIM),
                ("nboxes", ctypes.c_int64 * (MAX_LEVELS + 1)), ("max_box", ctypes.c_int64 * (MAX_LEVELS + 1)),
                ("near_pairs", ctypes.c_int64 * (MAX_LEVELS + 1)), ("far_pairs", ctypes.c_int64 * (MAX_LEVELS + 1)),
                ("far_point_pairs", ctypes.c_int64 * (MAX_LEVELS + 1)),
                ("near_point_pairs", ctypes.c_int64), ("device_bytes", ctypes.c_int64),
                ("smooth_depth", ctypes.c_int32), ("level_nodes", ctypes.c_int32 * (MAX_LEVELS + 1)),
                ("small_pairs", ctypes.c_int64 * (MAX_LEVELS + 1)),
                ("small_point_pairs", ctypes.c_int64 * (MAX_LEVELS + 1))]


class SourceInfo(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("two_sets", ctypes.c_int32), ("alpha", ctypes.c_float * MAX_DIM),
                ("nboxes", ctypes.c_int64 * (MAX_LEVELS + 1)), ("max_box", ctypes.c_int64 * (MAX_LEVELS + 1))]


class Times(ctypes.Structure):
    _fields_ = [(k, ctypes.c_float) for k in
                ("bbox_keys", "sort", "gather", "boxes", "lists", "tables", "plan_total",
                 "permute_in", "p2p", "p2m", "m2l", "l2p", "permute_out", "kmvm_total")]

    def as_dict(self):
        return {k: float(getattr(self, k)) for k, _ in self._fields_}


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libf3m.so is missing (%s): build it with "
                               "`python -m paper_2202_01085_amd.build`; there is no fallback path" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, ci, cf = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
        L.f3m_plan.argtypes = [vp, i64, ci, cf, ci, cf, vp, ctypes.POINTER(vp)]
        L.f3m_plan_ex.argtypes = [vp, i64, ci, cf, ci, cf, ctypes.POINTER(Options), vp, ctypes.POINTER(vp)]
        L.f3m_plan_xy.argtypes = [vp, i64, vp, i64, ci, cf, ci, cf, ctypes.POINTER(Options), vp, ctypes.POINTER(vp)]
        L.f3m_kmvm.argtypes = [vp, vp, vp, vp]
        L.f3m_kmvm_multi.argtypes = [vp, vp, i64, vp, i64, ci, vp]
        L.f3m_kmvm_multi.restype = ci
        L.f3m_cg_solve.argtypes = [vp, cf, vp, vp, ci, cf, ctypes.POINTER(ci), vp, vp]
        L.f3m_cg_solve.restype = ci
        L.direct_kmvm_xy.argtypes = [vp, i64, vp, i64, ci, cf, vp, vp, vp]
        L.direct_kmvm_xy_rows_f64.argtypes = [vp, i64, vp, i64, ci, cf, vp, vp, i64, vp, vp]
        L.f3m_plan_source_info.argtypes = [vp, ctypes.POINTER(SourceInfo)]
        L.f3m_plan_get_source_perm.argtypes = [vp, vp]
        L.f3m_plan_get_source_boxes.argtypes = [vp, ci, vp, vp]
        L.direct_kmvm.argtypes = [vp, i64, ci, cf, vp, vp, vp]
        L.direct_kmvm_rows_f64.argtypes = [vp, i64, ci, cf, vp, vp, i64, vp, vp]
        L.direct_kmvm_rows_f64_static.argtypes = [vp, i64, ci, cf, vp, vp, i64, vp, vp]
        L.f3m_destroy.argtypes = [vp]
        L.f3m_destroy.restype = None
        L.f3m_trim_memory.argtypes = []
        L.f3m_trim_memory.restype = ctypes.c_int64
        L.f3m_last_error.restype = ctypes.c_char_p
        L.f3m_plan_info.argtypes = [vp, ctypes.POINTER(Info)]
        L.f3m_plan_get_perm.argtypes = [vp, vp]
        L.f3m_plan_get_point_keys.argtypes = [vp, vp]
        L.f3m_plan_get_boxes.argtypes = [vp, ci, vp, vp]
        L.f3m_plan_get_list.argtypes = [vp, ci, ci, vp, vp]
        L.f3m_stage_times.argtypes = [vp, ctypes.POINTER(Times)]
        L.f3m_level_times.argtypes = [vp, ci, vp]
        for name in ("f3m_plan", "f3m_plan_ex", "f3m_kmvm", "direct_kmvm", "direct_kmvm_rows_f64", "f3m_plan_info",
                     "f3m_plan_get_perm", "f3m_plan_get_point_keys", "f3m_plan_get_boxes", "f3m_plan_get_list",
                     "f3m_stage_times", "f3m_level_times", "f3m_plan_xy", "direct_kmvm_xy", "direct_kmvm_xy_rows_f64",
                     "f3m_plan_source_info", "f3m_plan_get_source_perm", "f3m_plan_get_source_boxes",
                     "direct_kmvm_rows_f64_static"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise F3MError(status, lib().f3m_last_error().decode())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_f32(t, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous float32 device tensor" % name)
    return ctypes.c_void_p(t.data_ptr())


def _np_ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


class Plan:
    """f3m_plan / f3m_plan_ex: the partition and interaction lists of one point set;
    with Y given, f3m_plan_xy: targets X and sources Y, for v = K(X, Y) b."""

    def __init__(self, X, lengthscale, interp_nodes, eta=2.0, leaf_max=0, max_depth=0, force_all_near=False,
                 overlap=False, stream=None, eta_smooth=0.0, adaptive_far=False, small_field=0, Y=None,
                 route_min_points=0):
        n, D = X.shape
        self.n, self.D = int(n), int(D)
        self.ns = self.n
        self._h = ctypes.c_void_p()
        opt = Options(int(leaf_max), int(max_depth), int(bool(force_all_near)), int(bool(overlap)),
                      float(eta_smooth), int(bool(adaptive_far)), int(small_field), int(route_min_points))
        xp = _dev_f32(X, "X") if n > 0 else ctypes.c_void_p()
        if Y is None:
            _check(lib().f3m_plan_ex(xp, self.n, self.D, float(lengthscale), int(interp_nodes), float(eta),
                                     ctypes.byref(opt), _stream(stream), ctypes.byref(self._h)))
        else:
            if Y.shape[1] != D:
                raise ValueError("X and Y must have the same number of columns")
            self.ns = int(Y.shape[0])
            yp = _dev_f32(Y, "Y") if self.ns > 0 else ctypes.c_void_p()
            _check(lib().f3m_plan_xy(xp, self.n, yp, self.ns, self.D, float(lengthscale), int(interp_nodes),
                                     float(eta), ctypes.byref(opt), _stream(stream), ctypes.byref(self._h)))

    def close(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:      # _lib is already gone when the interpreter shuts down
            _lib.f3m_destroy(h)

    __del__ = close

    def kmvm(self, b, y=None, stream=None):
        """f3m_kmvm: y ~= K(X,X) b, or K(X,Y) b for a two-set plan (asynchronous on the stream)."""
        if y is None:
            y = torch.empty(self.n, dtype=torch.float32, device=b.device)
        if self.n == 0:
            return y
        if b.numel() != self.ns or y.numel() != self.n:
            raise ValueError("b must have one entry per source and y one per target")
        _check(lib().f3m_kmvm(self._h, _dev_f32(b, "b") if self.ns else None, _dev_f32(y, "y"), _stream(stream)))
        return y

    def kmvm_multi(self, B, Y=None, stream=None):
        """f3m_kmvm_multi: B is an (m, sources) tensor, one right-hand side per ROW (each row contiguous);
        returns Y of shape (m, n) with Y[j] = product of B[j]."""
        m = int(B.shape[0])
        if B.dim() != 2 or B.shape[1] != self.ns:
            raise ValueError("B must have shape (m, sources)")
        if Y is None:
            Y = torch.empty((m, self.n), dtype=torch.float32, device=B.device)
        if Y.shape != (m, self.n):
            raise ValueError("Y must have shape (m, n)")
        if m and self.n:
            _check(lib().f3m_kmvm_multi(self._h, _dev_f32(B, "B") if self.ns else None, self.ns, _dev_f32(Y, "Y"), self.n,
                                        m, _stream(stream)))
        return Y

    def cg_solve(self, b, lam, tol=1e-6, max_iter=100, x=None, stream=None):
        """f3m_cg_solve: x = (K + lam I)^{-1} b by conjugate gradients; returns (x, iterations, history)."""
        if x is None:
            x = torch.empty_like(b)
        iters = ctypes.c_int(0)
        hist = np.zeros(max_iter + 1, dtype=np.float32)
        _check(lib().f3m_cg_solve(self._h, float(lam), _dev_f32(b, "b") if self.n else None,
                                  _dev_f32(x, "x") if self.n else None, int(max_iter), float(tol), ctypes.byref(iters),
                                  _np_ptr(hist), _stream(stream)))
        return x, int(iters.value), hist[:iters.value + 1]

    def source_info(self):
        out = SourceInfo()
        _check(lib().f3m_plan_source_info(self._h, ctypes.byref(out)))
        return out

    def source_perm(self):
        out = np.empty(self.ns, dtype=np.uint32)
        _check(lib().f3m_plan_get_source_perm(self._h, _np_ptr(out)))
        return out

    def source_boxes(self, level):
        nb = int(self.source_info().nboxes[level])
        keys = np.empty(nb, dtype=np.uint32)
        starts = np.empty(nb + 1, dtype=np.uint32)
        _check(lib().f3m_plan_get_source_boxes(self._h, int(level), _np_ptr(keys), _np_ptr(starts)))
        return keys, starts

    def info(self):
        out = Info()
        _check(lib().f3m_plan_info(self._h, ctypes.byref(out)))
        return out

    def perm(self):
        out = np.empty(self.n, dtype=np.uint32)
        _check(lib().f3m_plan_get_perm(self._h, _np_ptr(out)))
        return out

    def point_keys(self):
        out = np.empty(self.n, dtype=np.uint32)
        _check(lib().f3m_plan_get_point_keys(self._h, _np_ptr(out)))
        return out

    def boxes(self, level):
        nb = int(self.info().nboxes[level])
        keys = np.empty(nb, dtype=np.uint32)
        starts = np.empty(nb + 1, dtype=np.uint32)
        _check(lib().f3m_plan_get_boxes(self._h, int(level), _np_ptr(keys), _np_ptr(starts)))
        return keys, starts

    def interactions(self, level, kind):
        inf = self.info()
        nb = int(inf.nboxes[level])
        sz = int((inf.near_pairs, inf.far_pairs, inf.small_pairs)[kind][level])
        ptr = np.empty(nb + 1, dtype=np.uint64)
        cols = np.empty(max(sz, 1), dtype=np.uint32)
        _check(lib().f3m_plan_get_list(self._h, int(level), int(kind), _np_ptr(ptr), _np_ptr(cols)))
        return ptr, cols[:sz]

    def level_times(self, level):
        """(P2M, M2L, L2P) milliseconds of one depth in the last kmvm"""
        out = (ctypes.c_float * 3)()
        _check(lib().f3m_level_times(self._h, int(level), out))
        return tuple(float(v) for v in out)

    def stage_times(self):
        out = Times()
        _check(lib().f3m_stage_times(self._h, ctypes.byref(out)))
        return out.as_dict()


def trim_memory():
    """f3m_trim_memory: give the library's cached device blocks back to the device; returns the bytes freed."""
    return int(lib().f3m_trim_memory())


def f3m_plan(X, lengthscale, interp_nodes, eta=2.0, **kw):
    return Plan(X, lengthscale, interp_nodes, eta, **kw)


def f3m_kmvm(plan, b, y=None, stream=None):
    return plan.kmvm(b, y, stream)


def direct_kmvm(X, b, lengthscale, y=None, stream=None):
    """direct_kmvm: exact y = K(X,X) b in fp32, O(n^2)."""
    n, D = X.shape
    if y is None:
        y = torch.empty_like(b)
    _check(lib().direct_kmvm(_dev_f32(X, "X") if n else None, int(n), int(D), float(lengthscale),
                             _dev_f32(b, "b") if n else None, _dev_f32(y, "y") if n else None, _stream(stream)))
    return y


def direct_kmvm_rows_f64(X, b, lengthscale, rows, stream=None):
    """direct_kmvm_rows_f64: exact fp64 sums for the selected rows (device int64 tensor)."""
    n, D = X.shape
    rows = rows.to(device=X.device, dtype=torch.int64).contiguous()
    y64 = torch.empty(rows.numel(), dtype=torch.float64, device=X.device)
    _check(lib().direct_kmvm_rows_f64(_dev_f32(X, "X"), int(n), int(D), float(lengthscale), _dev_f32(b, "b"),
                                      ctypes.c_void_p(rows.data_ptr()), int(rows.numel()),
                                      ctypes.c_void_p(y64.data_ptr()), _stream(stream)))
    return y64


def direct_kmvm_rows_f64_static(X, b, lengthscale, rows, y64, stream=None):
    """direct_kmvm_rows_f64_static: the same sums into the caller's y64 (device float64, one entry per row);
    the library call allocates nothing (at most 16384 rows).  rows: device int64 tensor."""
    n, D = X.shape
    if not (rows.is_cuda and rows.dtype == torch.int64 and rows.is_contiguous()):
        raise TypeError("rows must be a contiguous int64 device tensor")
    if not (y64.is_cuda and y64.dtype == torch.float64 and y64.is_contiguous() and y64.numel() >= rows.numel()):
        raise TypeError("y64 must be a contiguous float64 device tensor with one entry per row")
    _check(lib().direct_kmvm_rows_f64_static(_dev_f32(X, "X"), int(n), int(D), float(lengthscale), _dev_f32(b, "b"),
                                             ctypes.c_void_p(rows.data_ptr()), int(rows.numel()),
                                             ctypes.c_void_p(y64.data_ptr()), _stream(stream)))
    return y64


def direct_kmvm_xy(X, Y, b, lengthscale, y=None, stream=None):
    """direct_kmvm_xy: exact y = K(X,Y) b in fp32."""
    nx, D = X.shape
    ny = Y.shape[0]
    if y is None:
        y = torch.empty(nx, dtype=torch.float32, device=X.device)
    _check(lib().direct_kmvm_xy(_dev_f32(X, "X") if nx else None, int(nx), _dev_f32(Y, "Y") if ny else None, int(ny),
                                int(D), float(lengthscale), _dev_f32(b, "b") if ny else None,
                                _dev_f32(y, "y") if nx else None, _stream(stream)))
    return y


def direct_kmvm_xy_rows_f64(X, Y, b, lengthscale, rows, stream=None):
    """direct_kmvm_xy_rows_f64: exact fp64 sums of K(X,Y) b for the selected rows of X."""
    nx, D = X.shape
    ny = Y.shape[0]
    rows = rows.to(device=X.device, dtype=torch.int64).contiguous()
    y64 = torch.empty(rows.numel(), dtype=torch.float64, device=X.device)
    _check(lib().direct_kmvm_xy_rows_f64(_dev_f32(X, "X"), int(nx), _dev_f32(Y, "Y") if ny else None, int(ny), int(D),
                                         float(lengthscale), _dev_f32(b, "b") if ny else None,
                                         ctypes.c_void_p(rows.data_ptr()), int(rows.numel()),
                                         ctypes.c_void_p(y64.data_ptr()), _stream(stream)))
    return y64
