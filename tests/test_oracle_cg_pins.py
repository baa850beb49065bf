"""Pins of the oracle's conjugate-gradient solve of (K + lambda I) x = b (Sec. 5 "Kernel Ridge
Regression experiment": alpha = (k(X,X) + lambda I)^{-1} b with F3M as the solver's product).
No GPU.  The solve is pinned to dense linear algebra, not to itself."""
import numpy as np

import oracle
from paper_2202_01085_amd import inputs


def _dense_operator(T, gamma, p, **kw):
    n = T.n
    A = np.empty((n, n))
    for j in range(n):
        e = np.zeros(n, dtype=np.float32)
        e[j] = 1.0
        A[:, j] = T.apply(e, gamma, p, **kw)
    return A


def test_apply64_is_the_product_of_an_fp64_vector():
    X = inputs.points_uniform(400, 2, 11).numpy()
    T = oracle.Tree(X, zeta=16, force_all_near=True)          # exact K
    v = np.random.default_rng(0).standard_normal(400) * np.pi
    d2 = ((X.astype(np.float64)[:, None] - X.astype(np.float64)[None]) ** 2).sum(-1)
    want = np.exp(-d2 / (2 * 0.3 ** 2)) @ v
    got = oracle.apply64(T, v, 0.3, 3)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)
    assert not np.allclose(T.apply(v.astype(np.float32), 0.3, 3), want, rtol=1e-10, atol=1e-10)   # fp32 rounding of v shows


def test_cg_on_the_exact_kernel_matrix_equals_the_dense_solve():
    X = inputs.points_normal(250, 3, 12).numpy()
    b = inputs.rhs_normal(250, 13).numpy().astype(np.float64)
    T = oracle.Tree(X, zeta=8, force_all_near=True)
    d2 = ((X.astype(np.float64)[:, None] - X.astype(np.float64)[None]) ** 2).sum(-1)
    K = np.exp(-d2 / (2 * 0.5 ** 2))
    for lam in (1.0, 0.05):
        want = np.linalg.solve(K + lam * np.eye(250), b)
        x, hist = oracle.cg_solve(T, b, lam, 0.5, 3, tol=1e-13, max_iter=400)
        assert hist[-1] <= 1e-13 and np.allclose(x, want, rtol=1e-9, atol=1e-9 * np.abs(want).max())


def test_cg_on_the_f3m_operator_equals_the_dense_solve_with_its_matrix():
    X = inputs.points_uniform(300, 2, 14).numpy()
    b = inputs.rhs_normal(300, 15).numpy().astype(np.float64)
    T = oracle.Tree(X, zeta=6)
    assert T.L >= 2 and sum(len(T.interactions(l, 1)[1]) for l in range(1, T.L + 1)) > 0
    A = _dense_operator(T, 0.3, 4)
    assert np.allclose(A, A.T, rtol=1e-12, atol=1e-12)
    want = np.linalg.solve(A + 0.5 * np.eye(300), b)
    x, hist = oracle.cg_solve(T, b, 0.5, 0.3, 4, tol=1e-12, max_iter=300)
    assert np.allclose(x, want, rtol=1e-8, atol=1e-8 * np.abs(want).max())
    # the recorded residual norms are the true ones
    assert abs(hist[-1] - np.linalg.norm(b - (A + 0.5 * np.eye(300)) @ x) / np.linalg.norm(b)) <= 1e-10


def test_cg_ends_in_at_most_n_steps_and_its_residuals_are_orthogonal():
    # textbook properties: n distinct eigenvalues -> exact after n steps; r_i . r_j = 0 for i != j
    X = np.array([[0.0], [0.9], [2.1], [3.7], [4.2], [6.0]], dtype=np.float32)
    b = np.array([1.0, -2.0, 0.5, 3.0, -1.0, 2.0])
    T = oracle.Tree(X, zeta=64)                                # one box: exact
    d2 = (X.astype(np.float64) - X.astype(np.float64).T) ** 2
    A = np.exp(-d2 / 2.0) + 0.3 * np.eye(6)
    x, hist = oracle.cg_solve(T, b, 0.3, 1.0, 2, tol=0.0, max_iter=6)
    assert len(hist) == 7 and hist[-1] < 1e-12
    assert np.allclose(x, np.linalg.solve(A, b), rtol=1e-11, atol=1e-11)
    res = []
    for k in range(1, 5):
        xk, _ = oracle.cg_solve(T, b, 0.3, 1.0, 2, tol=0.0, max_iter=k)
        res.append(b - A @ xk)
    for i in range(len(res)):
        for j in range(i):
            assert abs(res[i] @ res[j]) <= 1e-10 * np.linalg.norm(res[i]) * np.linalg.norm(res[j]) + 1e-14
    # and every iterate minimises the A-norm of the error over the Krylov space: it decreases
    xs = np.linalg.solve(A, b)
    errs = [float((xs - oracle.cg_solve(T, b, 0.3, 1.0, 2, tol=0.0, max_iter=k)[0]) @ A @
                  (xs - oracle.cg_solve(T, b, 0.3, 1.0, 2, tol=0.0, max_iter=k)[0])) for k in range(0, 6)]
    assert all(errs[k + 1] < errs[k] for k in range(5))


def test_cg_stops_on_the_tolerance_and_handles_a_zero_right_hand_side():
    X = inputs.points_uniform(500, 3, 16).numpy()
    b = inputs.rhs_normal(500, 17).numpy().astype(np.float64)
    T = oracle.Tree(X, zeta=16)
    x, hist = oracle.cg_solve(T, b, 1.0, 0.4, 4, tol=1e-4, max_iter=200)
    assert hist[-1] <= 1e-4 < hist[-2] and len(hist) < 200
    x0, h0 = oracle.cg_solve(T, np.zeros(500), 1.0, 0.4, 4)
    assert np.all(x0 == 0) and len(h0) == 1
