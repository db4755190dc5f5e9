"""Pins for the oracle's dual coordinate-ascent solver (Section 2 equation (2), Section 3 "Shrinking").

The optimum of the problem is unique in w, so independent solvers (LIBLINEAR through scikit-learn, a
bound-constrained quasi-Newton method through scipy) pin it; closed forms pin the single step; KKT
conditions and weak duality, evaluated here in numpy, pin the stopping rule.
"""
import numpy as np
import pytest
import scipy.optimize


def _problem(seed, n, r, margin=0.0):
    rng = np.random.default_rng(seed)
    G = (rng.standard_normal((n, r)) / np.sqrt(r)).astype(np.float32)
    v = rng.standard_normal(r)
    s = G.astype(np.float64) @ v
    y = np.where(s + margin * rng.standard_normal(n) >= 0, 1.0, -1.0).astype(np.float32)
    return G, y


def _dual(G, y, alpha):
    w = (alpha * y) @ G.astype(np.float64)
    return alpha.sum() - 0.5 * w @ w, w


def _primal(G, y, w, C):
    return 0.5 * w @ w + C * np.maximum(0.0, 1.0 - y * (G.astype(np.float64) @ w)).sum()


def _kkt(G, y, alpha, w, C):
    grad = 1.0 - y * (G.astype(np.float64) @ w)
    v = np.where(alpha <= 0, np.maximum(grad, 0), np.where(alpha >= C, np.maximum(-grad, 0), np.abs(grad)))
    return v.max()


def test_single_variable_closed_form(oracle):
    g = np.array([[0.6, 0.8, 0.0]], dtype=np.float32)        # ||g||^2 = 1
    for C, expect in [(10.0, 1.0), (0.25, 0.25)]:
        a, w, st = oracle.cd_solve(g, [0], [1.0], C, eps=1e-12)
        assert abs(a[0] - expect) < 1e-7
        assert np.allclose(w, expect * g[0], atol=1e-7)
        assert st["converged"]
    a, w, st = oracle.cd_solve(g, [0], [-1.0], 10.0, eps=1e-12)
    assert abs(a[0] - 1.0) < 1e-7 and np.allclose(w, -g[0], atol=1e-7)


def test_first_step_is_the_truncated_newton_step(oracle):
    # from alpha = 0, w = 0: the first step on variable i gives clip(1 / ||g_i||^2, 0, C)
    G, y = _problem(1, 6, 4)
    q = (G.astype(np.float64) ** 2).sum(axis=1)
    a, w, st = oracle.cd_solve(G[:1], [0], y[:1], 100.0, eps=1e-12)
    assert abs(a[0] - min(1.0 / q[0], 100.0)) < 1e-9


def test_zero_row_goes_to_upper_bound(oracle):
    G = np.zeros((2, 3), dtype=np.float32)
    G[1] = [1, 0, 0]
    a, w, st = oracle.cd_solve(G, [0, 1], [1.0, 1.0], 0.5, eps=1e-9)
    assert a[0] == 0.5 and abs(a[1] - 0.5) < 1e-12 and st["converged"]


@pytest.mark.parametrize("C", [0.1, 1.0, 10.0])
@pytest.mark.parametrize("shrink_k", [0, 5])
def test_optimum_against_bounded_quasi_newton(oracle, C, shrink_k):
    G, y = _problem(2, 60, 8, margin=0.3)
    rows = np.arange(60)
    a, w, st = oracle.cd_solve(G, rows, y, C, eps=1e-9, max_epochs=200000, shrink_k=shrink_k)
    assert st["converged"]
    Q = (y[:, None] * G.astype(np.float64)) @ (y[:, None] * G.astype(np.float64)).T
    res = scipy.optimize.minimize(lambda x: 0.5 * x @ Q @ x - x.sum(), np.zeros(60), jac=lambda x: Q @ x - 1.0,
                                  bounds=[(0.0, C)] * 60, method="L-BFGS-B",
                                  options={"maxiter": 100000, "ftol": 1e-15, "gtol": 1e-10})
    d_ref = -(res.fun)
    d, w_chk = _dual(G, y, a)
    assert abs(d - st["dual"]) < 1e-9 * max(1.0, abs(d))
    assert abs(d - d_ref) <= 1e-6 * max(1.0, abs(d_ref))
    assert d >= d_ref - 1e-9                       # the oracle is at least as good as the reference optimum
    assert np.allclose(w, w_chk, atol=1e-9)        # w is kept consistent with alpha
    assert _kkt(G, y, a, w, C) <= 1e-7         # violations are measured before each step of the last epoch
    assert np.all(a >= 0) and np.all(a <= C)


def test_optimum_against_liblinear(oracle):
    sklearn_svm = pytest.importorskip("sklearn.svm")
    G, y = _problem(3, 300, 12, margin=0.5)
    C = 2.0
    a, w, st = oracle.cd_solve(G, np.arange(300), y, C, eps=1e-8, max_epochs=100000)
    clf = sklearn_svm.LinearSVC(loss="hinge", dual=True, fit_intercept=False, C=C, tol=1e-10, max_iter=2000000)
    clf.fit(G.astype(np.float64), y)
    w_ref = clf.coef_[0]
    assert np.linalg.norm(w - w_ref) <= 1e-4 * np.linalg.norm(w_ref)
    # weak duality closes: P(w) - D(alpha) ~ 0
    assert abs(_primal(G, y, w, C) - st["dual"]) <= 1e-5 * abs(st["dual"])


def test_dual_objective_never_decreases_over_epochs(oracle):
    G, y = _problem(4, 200, 10, margin=0.4)
    prev = -1.0
    for e in range(1, 12):
        a, w, st = oracle.cd_solve(G, np.arange(200), y, 1.0, eps=0.0, max_epochs=e)
        assert st["epochs"] == e
        assert st["dual"] >= prev - 1e-12
        prev = st["dual"]


def test_shrinking_saves_steps_and_reaches_the_same_optimum(oracle):
    # overlapping classes in 10 dimensions: at the optimum all but ~10 variables sit at 0 or C; they are
    # removed after k unchanged steps and the late epochs run over a handful of variables
    rng = np.random.default_rng(5)
    n, r = 3000, 10
    G = (rng.standard_normal((n, r)) / np.sqrt(r)).astype(np.float32)
    v = rng.standard_normal(r)
    y = np.where(G.astype(np.float64) @ v + 0.15 * rng.standard_normal(n) >= 0, 1.0, -1.0).astype(np.float32)
    a0, w0, s0 = oracle.cd_solve(G, np.arange(n), y, 1.0, eps=1e-5, max_epochs=100000, shrink_k=0)
    a1, w1, s1 = oracle.cd_solve(G, np.arange(n), y, 1.0, eps=1e-5, max_epochs=100000, shrink_k=5)
    assert s0["converged"] and s1["converged"]
    assert abs(s0["dual"] - s1["dual"]) <= 1e-8 * abs(s0["dual"])
    assert np.linalg.norm(w0 - w1) <= 1e-4 * np.linalg.norm(w0)
    assert s1["steps"] < 0.1 * s0["steps"]         # the paper reports two orders of magnitude on its data
    assert s1["active"] < 100                      # the final active set is small
    assert _kkt(G, y, a1, w1, 1.0) <= 1e-4         # removed variables were verified before stopping
    # without the eta share nothing is re-checked until the final sweep; the optimum is the same
    a2, w2, s2 = oracle.cd_solve(G, np.arange(n), y, 1.0, eps=1e-5, max_epochs=100000, shrink_k=5, eta=0.0)
    assert s2["converged"] and abs(s2["dual"] - s0["dual"]) <= 1e-8 * abs(s0["dual"])


def test_visiting_order_and_row_subset(oracle):
    G, y = _problem(6, 80, 7, margin=0.2)
    rows = np.random.default_rng(0).permutation(80)[:50]
    a, w, st = oracle.cd_solve(G, rows, y[rows], 1.0, eps=1e-9, max_epochs=100000)
    a2, w2, st2 = oracle.cd_solve(G[rows], np.arange(50), y[rows], 1.0, eps=1e-9, max_epochs=100000)
    assert np.array_equal(a, a2) and np.array_equal(w, w2)     # a row list is just indirection
    a3, w3, st3 = oracle.cd_solve(G, rows[::-1].copy(), y[rows[::-1]], 1.0, eps=1e-9, max_epochs=100000)
    assert np.linalg.norm(w3 - w) <= 1e-6 * np.linalg.norm(w)  # other order, same optimum


def test_warm_start_at_the_solution_stops_at_once(oracle):
    G, y = _problem(7, 100, 9, margin=0.3)
    a, w, st = oracle.cd_solve(G, np.arange(100), y, 1.0, eps=1e-7, max_epochs=100000)
    a2, w2, st2 = oracle.cd_solve(G, np.arange(100), y, 1.0, eps=1e-6, max_epochs=100000, alpha0=a)
    assert st2["epochs"] == 1 and st2["converged"]
    assert np.linalg.norm(w2 - w) <= 1e-6 * np.linalg.norm(w)
