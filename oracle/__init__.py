"""ctypes front end of the CPU oracle (oracle/f3m_oracle.c).

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and the cpu_baseline
leg of bench.py may import this package.  It never touches the HIP library.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "f3m_oracle.c")
_LIB = os.path.join(_HERE, "libf3m_oracle.so")


def build(force=False):
    """Compile the oracle with gcc (fp contraction off so that the fp32 cell
    expression is evaluated as two separately rounded operations)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-D_GNU_SOURCE", "-fopenmp", "-ffp-contract=off", "-fPIC",
             "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        c_i64, c_int, c_dbl, c_vp = ctypes.c_int64, ctypes.c_int, ctypes.c_double, ctypes.c_void_p
        L.oracle_num_threads.restype = c_int
        L.oracle_set_verbose.argtypes = [c_int]
        L.oracle_rows_k.argtypes = [c_vp, c_i64, c_int, c_dbl, c_int, c_int, c_vp, c_vp, c_i64, c_vp]
        L.oracle_cheb2_nodes.argtypes = [c_int, c_vp]
        L.oracle_lagrange_product.argtypes = [c_int, c_vp, c_dbl, c_vp]
        L.oracle_lagrange_barycentric.argtypes = [c_int, c_vp, c_dbl, c_vp]
        L.oracle_quant_depth.argtypes = [c_int]
        L.oracle_quant_depth.restype = c_int
        L.oracle_tree_build.argtypes = [c_vp, c_i64, c_int, c_dbl, c_i64, c_int, c_int]
        L.oracle_tree_build.restype = c_vp
        L.oracle_tree_build_ex.argtypes = [c_vp, c_i64, c_int, c_dbl, c_i64, c_int, c_int, c_dbl, c_dbl]
        L.oracle_tree_build_ex.restype = c_vp
        L.oracle_tree_build_ex2.argtypes = [c_vp, c_i64, c_int, c_dbl, c_i64, c_int, c_int, c_dbl, c_dbl, c_i64]
        L.oracle_tree_build_ex2.restype = c_vp
        L.oracle_tree_build_rows.argtypes = [c_vp, c_i64, c_int, c_dbl, c_i64, c_int, c_int, c_dbl, c_dbl, c_vp, c_i64]
        L.oracle_tree_build_rows.restype = c_vp
        L.oracle_f3m_apply_rows.argtypes = [c_vp, c_vp, c_dbl, c_int, c_int, c_int, c_vp, c_vp, c_i64, c_vp, c_int]
        L.oracle_f3m_apply_rows.restype = c_int
        L.oracle_is_smooth_depth.argtypes = [c_dbl, c_int, c_int, c_dbl, c_dbl]
        L.oracle_is_smooth_depth.restype = c_int
        L.oracle_adaptive_nodes.argtypes = [c_dbl, c_int, c_dbl, c_int]
        L.oracle_adaptive_nodes.restype = c_int
        L.oracle_tree_free.argtypes = [c_vp]
        for name in ("oracle_tree_depth", "oracle_tree_quant_depth", "oracle_tree_smooth_depth"):
            getattr(L, name).argtypes = [c_vp]
            getattr(L, name).restype = c_int
        L.oracle_tree_edge.argtypes = [c_vp]
        L.oracle_tree_edge.restype = c_dbl
        L.oracle_tree_alpha.argtypes = [c_vp, c_vp]
        L.oracle_tree_nboxes.argtypes = [c_vp, c_int]
        L.oracle_tree_nboxes.restype = c_i64
        L.oracle_tree_perm.argtypes = [c_vp, c_vp]
        L.oracle_tree_point_keys.argtypes = [c_vp, c_vp]
        L.oracle_tree_boxes.argtypes = [c_vp, c_int, c_vp, c_vp]
        L.oracle_tree_list_size.argtypes = [c_vp, c_int, c_int]
        L.oracle_tree_list_size.restype = c_i64
        L.oracle_tree_list.argtypes = [c_vp, c_int, c_int, c_vp, c_vp]
        L.oracle_beta.argtypes = [c_vp, c_int, c_vp]
        L.oracle_p2m_level.argtypes = [c_vp, c_vp, c_vp, c_int, c_int, c_vp]
        L.oracle_f3m_apply.argtypes = [c_vp, c_vp, c_dbl, c_int, c_int, c_int, c_vp, c_vp, c_int]
        L.oracle_f3m_apply.restype = c_int
        L.oracle_f3m_apply_ex.argtypes = [c_vp, c_vp, c_dbl, c_int, c_int, c_int, c_vp, c_vp, c_int, c_int]
        L.oracle_f3m_apply_ex.restype = c_int
        L.oracle_rows_xy.argtypes = [c_vp, c_i64, c_vp, c_i64, c_int, c_dbl, c_int, c_int, c_vp, c_vp, c_i64, c_vp]
        L.oracle_tree2_build.argtypes = [c_vp, c_i64, c_vp, c_i64, c_int, c_dbl, c_i64, c_int, c_int, c_dbl, c_dbl,
                                         c_i64]
        L.oracle_tree2_build.restype = c_vp
        L.oracle_tree2_free.argtypes = [c_vp]
        for name in ("oracle_tree2_depth", "oracle_tree2_smooth_depth"):
            getattr(L, name).argtypes = [c_vp]
            getattr(L, name).restype = c_int
        L.oracle_tree2_edge.argtypes = [c_vp]
        L.oracle_tree2_edge.restype = c_dbl
        L.oracle_tree2_side.argtypes = [c_vp, c_int]
        L.oracle_tree2_side.restype = c_vp
        L.oracle_tree2_list_size.argtypes = [c_vp, c_int, c_int]
        L.oracle_tree2_list_size.restype = c_i64
        L.oracle_tree2_list.argtypes = [c_vp, c_int, c_int, c_vp, c_vp]
        L.oracle_f3m2_apply.argtypes = [c_vp, c_vp, c_vp, c_dbl, c_int, c_int, c_int, c_vp, c_vp, c_int]
        L.oracle_f3m2_apply.restype = c_int
        _lib = L
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def set_verbose(on):
    """Progress lines on stderr, one per finished step of a tree build or a product."""
    lib().oracle_set_verbose(int(bool(on)))


def num_threads():
    return int(lib().oracle_num_threads())


def rows(X, b, gamma, rows=None, kernel_id=0, kparam=0):
    """Exact y_i = sum_j k(x_i, x_j) b_j (fp64) for the given rows (all rows if None)."""
    X = _f32(X)
    b = _f32(b)
    n, D = X.shape
    if rows is None:
        idx, m, rp = None, n, None
    else:
        idx = np.ascontiguousarray(rows, dtype=np.int64)
        m, rp = idx.size, _ptr(idx)
    y = np.empty(m, dtype=np.float64)
    lib().oracle_rows_k(_ptr(X), n, D, float(gamma), kernel_id, kparam, _ptr(b), rp, m, _ptr(y))
    return y


def direct(X, b, gamma, kernel_id=0, kparam=0):
    return rows(X, b, gamma, None, kernel_id, kparam)


def cheb2_nodes(p):
    s = np.empty(p, dtype=np.float64)
    lib().oracle_cheb2_nodes(p, _ptr(s))
    return s


def lagrange_product(p, t):
    s = cheb2_nodes(p)
    out = np.empty(p, dtype=np.float64)
    lib().oracle_lagrange_product(p, _ptr(s), float(t), _ptr(out))
    return out


def lagrange_barycentric(p, t):
    s = cheb2_nodes(p)
    out = np.empty(p, dtype=np.float64)
    lib().oracle_lagrange_barycentric(p, _ptr(s), float(t), _ptr(out))
    return out


def quant_depth(D):
    return int(lib().oracle_quant_depth(D))


class Tree:
    """Partition + interaction lists of Algorithm 1 for one point set."""

    def __init__(self, X, theta=2.0, zeta=128, max_depth=0, force_all_near=False, gamma=0.0, eta_smooth=0.0,
                 small_field=0, rows=None):
        """eta_smooth > 0 switches the smooth field of Sec. 4.3 on (needs the lengthscale gamma);
        small_field = rho > 0 the small field of Sec. 4.2.  rows: build the interaction rows only for
        the boxes that hold these points (for apply_rows on large inputs; not with the small field)."""
        self.X = _f32(X)
        self.n, self.D = self.X.shape
        if rows is None:
            self._h = lib().oracle_tree_build_ex2(_ptr(self.X), self.n, self.D, float(theta), int(zeta),
                                                  int(max_depth), int(bool(force_all_near)), float(gamma),
                                                  float(eta_smooth), int(small_field))
        else:
            if small_field:
                raise ValueError("a row-subset tree is not offered with the small field")
            idx = np.ascontiguousarray(rows, dtype=np.int64)
            self._h = lib().oracle_tree_build_rows(_ptr(self.X), self.n, self.D, float(theta), int(zeta),
                                                   int(max_depth), int(bool(force_all_near)), float(gamma),
                                                   float(eta_smooth), _ptr(idx), idx.size)
        if not self._h:
            raise ValueError("oracle_tree_build rejected its arguments")
        self.L = int(lib().oracle_tree_depth(self._h))
        self.smooth_depth = int(lib().oracle_tree_smooth_depth(self._h))
        self.Lq = int(lib().oracle_tree_quant_depth(self._h))
        self.E = float(lib().oracle_tree_edge(self._h))
        a = np.empty(self.D, dtype=np.float64)
        lib().oracle_tree_alpha(self._h, _ptr(a))
        self.alpha = a

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and lib is not None:   # module globals may be gone at interpreter shutdown
            lib().oracle_tree_free(h)

    def nboxes(self, level):
        return int(lib().oracle_tree_nboxes(self._h, level))

    def perm(self):
        out = np.empty(self.n, dtype=np.int64)
        lib().oracle_tree_perm(self._h, _ptr(out))
        return out

    def point_keys(self):
        out = np.empty(self.n, dtype=np.uint64)
        lib().oracle_tree_point_keys(self._h, _ptr(out))
        return out

    def boxes(self, level):
        nb = self.nboxes(level)
        keys = np.empty(nb, dtype=np.uint64)
        starts = np.empty(nb + 1, dtype=np.int64)
        lib().oracle_tree_boxes(self._h, level, _ptr(keys), _ptr(starts))
        return keys, starts

    def interactions(self, level, kind):
        """CSR (row_ptr, cols) by target rank; kind 0 = near, 1 = far, 2 = small field."""
        nb = self.nboxes(level)
        sz = int(lib().oracle_tree_list_size(self._h, level, kind))
        ptr = np.empty(nb + 1, dtype=np.int64)
        cols = np.empty(max(sz, 1), dtype=np.int64)
        lib().oracle_tree_list(self._h, level, kind, _ptr(ptr), _ptr(cols))
        return ptr, cols[:sz]

    def beta(self, level):
        out = np.empty(self.n, dtype=np.uint64)
        lib().oracle_beta(self._h, level, _ptr(out))
        return out

    def p2m(self, b, p, level):
        b = _f32(b)
        r = p ** self.D
        W = np.empty((self.nboxes(level), r), dtype=np.float64)
        lib().oracle_p2m_level(self._h, _ptr(self.X), _ptr(b), p, level, _ptr(W))
        return W

    def apply(self, b, gamma, p, kernel_id=0, kparam=0, literal=False, adaptive=False):
        b = _f32(b)
        y = np.empty(self.n, dtype=np.float64)
        rc = lib().oracle_f3m_apply_ex(self._h, _ptr(self.X), float(gamma), int(p), kernel_id, kparam,
                                       _ptr(b), _ptr(y), int(bool(literal)), int(bool(adaptive)))
        if rc:
            raise ValueError("oracle_f3m_apply rejected its arguments")
        return y

    def apply_rows(self, b, gamma, p, rows, kernel_id=0, kparam=0, adaptive=False):
        """The rows `rows` of apply(): the same steps over the boxes that hold them (same bits)."""
        b = _f32(b)
        idx = np.ascontiguousarray(rows, dtype=np.int64)
        y = np.empty(idx.size, dtype=np.float64)
        rc = lib().oracle_f3m_apply_rows(self._h, _ptr(self.X), float(gamma), int(p), kernel_id, kparam, _ptr(b),
                                         _ptr(idx), idx.size, _ptr(y), int(bool(adaptive)))
        if rc:
            raise ValueError("oracle_f3m_apply_rows rejected its arguments (%d)" % rc)
        return y


def adaptive_nodes(E, depth, gamma, p):
    """Nodes per dimension of a depth under the adaptive far-field rule of Sec. 4.3 (0 = dropped)."""
    return int(lib().oracle_adaptive_nodes(float(E), int(depth), float(gamma), int(p)))


def f3m(X, b, gamma, p, theta=2.0, zeta=128, max_depth=0, force_all_near=False, eta_smooth=0.0, adaptive=False,
        small_field=0):
    """CPU F3M product (fp64), original point order."""
    return Tree(X, theta, zeta, max_depth, force_all_near, gamma, eta_smooth, small_field).apply(b, gamma, p,
                                                                                               adaptive=adaptive)


def rows_xy(X, Y, b, gamma, rows=None, kernel_id=0, kparam=0):
    """Exact v_i = sum_j k(x_i, y_j) b_j (fp64) for the given rows of X (all rows if None)."""
    X, Y, b = _f32(X), _f32(Y), _f32(b)
    nx, D = X.shape
    ny = Y.shape[0]
    assert Y.shape[1] == D and b.shape == (ny,)
    if rows is None:
        idx, m, rp = None, nx, None
    else:
        idx = np.ascontiguousarray(rows, dtype=np.int64)
        m, rp = idx.size, _ptr(idx)
    y = np.empty(m, dtype=np.float64)
    lib().oracle_rows_xy(_ptr(X), nx, _ptr(Y), ny, D, float(gamma), kernel_id, kparam, _ptr(b), rp, m, _ptr(y))
    return y


class _Side:
    """One set's partition inside a Tree2 (borrowed handle): perm, point keys, boxes, beta."""

    def __init__(self, owner, side, n, D):
        self._owner, self.n, self.D = owner, n, D   # the owner keeps the handle alive
        self._h = lib().oracle_tree2_side(owner._h, side)
        a = np.empty(D, dtype=np.float64)
        lib().oracle_tree_alpha(self._h, _ptr(a))
        self.alpha = a
        self.Lq = int(lib().oracle_tree_quant_depth(self._h))

    nboxes = Tree.nboxes
    perm = Tree.perm
    point_keys = Tree.point_keys
    boxes = Tree.boxes
    beta = Tree.beta


class Tree2:
    """Partitions of X (targets) and Y (sources) and the interaction lists of Algorithm 1 for K(X, Y)."""

    def __init__(self, X, Y, theta=2.0, zeta=128, max_depth=0, force_all_near=False, gamma=0.0, eta_smooth=0.0,
                 small_field=0):
        self.X, self.Y = _f32(X), _f32(Y)
        self.nx, self.D = self.X.shape
        self.ny = self.Y.shape[0]
        assert self.Y.shape[1] == self.D
        self._h = lib().oracle_tree2_build(_ptr(self.X), self.nx, _ptr(self.Y), self.ny, self.D, float(theta),
                                           int(zeta), int(max_depth), int(bool(force_all_near)), float(gamma),
                                           float(eta_smooth), int(small_field))
        if not self._h:
            raise ValueError("oracle_tree2_build rejected its arguments")
        self.L = int(lib().oracle_tree2_depth(self._h))
        self.smooth_depth = int(lib().oracle_tree2_smooth_depth(self._h))
        self.E = float(lib().oracle_tree2_edge(self._h))
        self.tx = _Side(self, 0, self.nx, self.D)
        self.ty = _Side(self, 1, self.ny, self.D)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and lib is not None:
            lib().oracle_tree2_free(h)

    def interactions(self, level, kind):
        """CSR (row_ptr, cols): rows are boxes of X, columns ranks of boxes of Y; kind 0 near, 1 far, 2 small."""
        nb = self.tx.nboxes(level)
        sz = int(lib().oracle_tree2_list_size(self._h, level, kind))
        ptr = np.empty(nb + 1, dtype=np.int64)
        cols = np.empty(max(sz, 1), dtype=np.int64)
        lib().oracle_tree2_list(self._h, level, kind, _ptr(ptr), _ptr(cols))
        return ptr, cols[:sz]

    def apply(self, b, gamma, p, kernel_id=0, kparam=0, adaptive=False):
        b = _f32(b)
        assert b.shape == (self.ny,)
        y = np.empty(self.nx, dtype=np.float64)
        rc = lib().oracle_f3m2_apply(self._h, _ptr(self.X), _ptr(self.Y), float(gamma), int(p), kernel_id, kparam,
                                     _ptr(b), _ptr(y), int(bool(adaptive)))
        if rc:
            raise ValueError("oracle_f3m2_apply rejected its arguments")
        return y


def f3m_xy(X, Y, b, gamma, p, theta=2.0, zeta=128, max_depth=0, force_all_near=False, eta_smooth=0.0, adaptive=False,
           small_field=0):
    """CPU F3M product K(X, Y) b (fp64), original order of X."""
    return Tree2(X, Y, theta, zeta, max_depth, force_all_near, gamma, eta_smooth, small_field).apply(
        b, gamma, p, adaptive=adaptive)


# ----------------------------------------------------------------------------
# kernel ridge regression by conjugate gradients (Sec. 5 "Kernel Ridge Regression experiment":
# alpha = (k(X,X) + lambda I)^{-1} b, with F3M as the matrix-vector product of the solver)
# ----------------------------------------------------------------------------
def apply64(T, v, gamma, p, **kw):
    """T.apply for an fp64 vector: the C routine takes fp32 weights, and the product is linear, so
    v = hi + lo with hi = fl32(v), lo = fl32(v - hi) gives it to about 2^-48."""
    v = np.asarray(v, dtype=np.float64)
    hi = v.astype(np.float32)
    lo = (v - hi.astype(np.float64)).astype(np.float32)
    return T.apply(hi, gamma, p, **kw) + T.apply(lo, gamma, p, **kw)


def cg_solve(T, b, lam, gamma, p, tol=1e-6, max_iter=100, **kw):
    """Textbook conjugate gradients (Hestenes-Stiefel) for (K + lam I) x = b, K the F3M operator of the
    tree T, from x_0 = 0, in fp64.  Stops after the first iteration with |r_k| <= tol |b|, or after
    max_iter iterations.  Returns (x, history) with history[k] = |r_k| / |b|, k = 0..iterations."""
    b = np.asarray(b, dtype=np.float64)
    x = np.zeros_like(b)
    r = b.copy()
    d = r.copy()
    rs = float(r @ r)
    nb = np.sqrt(rs)
    hist = [1.0 if nb > 0 else 0.0]
    if nb == 0:
        return x, np.array(hist)
    for _ in range(max_iter):
        Ad = apply64(T, d, gamma, p, **kw) + lam * d
        alpha = rs / float(d @ Ad)
        x = x + alpha * d
        r = r - alpha * Ad
        rs_new = float(r @ r)
        hist.append(np.sqrt(rs_new) / nb)
        if np.sqrt(rs_new) <= tol * nb:
            break
        d = r + (rs_new / rs) * d
        rs = rs_new
    return x, np.array(hist)
