"""Pins for the oracle's dual coordinate-ascent solver (Section 2 equation (2), Section 4 "Shrinking").

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


# ---------------------------------------------------------------- the discrete rules, traced by hand
#
# Section 4, "Shrinking", gives k = 5 and eta = 5 % and no more; the oracle's header lists the reading.  The
# cases below are small enough to follow step by step on paper, use numbers that are exact in binary, and
# assert the counters the trace predicts.  Two kinds of variables:
#   inert    g = unit vector of a coordinate of its own: the first step takes alpha to 1 (C = 10), every later
#            step leaves it unchanged;
#   busy     a: g = (2, 0, ..), b: g = (1, 1, ..), labels +1.  Their steps are alpha_a <- (1 - 2 alpha_b) / 4 and
#            alpha_b <- (1 - 2 alpha_a) / 2: after epoch e, alpha_a = 2^-(e+1), alpha_b = 1/2 - 2^-(e+1), both
#            change in every epoch, and the largest violation seen in epoch e + 1 is 2^-e (a's gradient before
#            its step), so with a tiny eps the stopping rule stays out of the way;
#   sleeper  s: g = (beta, 0, .., 1 in a coordinate of its own), beta = 2 - 2^-j, label +1.  At alpha_s = 0 its
#            gradient is 1 - beta w_1 with w_1 = 2 alpha_a + alpha_b: w_1 = 1/2 + 2^-(e+1) after b's step of epoch
#            e (gradient < 0 for e <= j: the step leaves alpha_s = 0) and w_1 = 1/2 exactly between a's and b's
#            steps of any later epoch (gradient 2^-(j+1) > 0: the step moves alpha_s to 2^-(j+1) / (beta^2 + 1)).

def _trace_problem(names, j=6):
    r = 2 + len(names)
    G = np.zeros((len(names), r), dtype=np.float32)
    for i, nm in enumerate(names):
        if nm == "a":
            G[i, 0] = 2.0
        elif nm == "b":
            G[i, 0] = G[i, 1] = 1.0
        elif nm == "u":
            G[i, 2 + i] = 1.0
        else:
            G[i, 0] = 2.0 - 2.0 ** -j
            G[i, 2 + i] = 1.0
    return G, np.arange(len(names)), np.ones(len(names), dtype=np.float32)


def test_removal_after_exactly_k_unchanged_steps(oracle):
    # a, b, then 40 inert variables.  Epoch 1 changes all 42; epochs 2..6 leave the inert ones unchanged for the
    # 1st..5th time in a row, so with k = 5 they are all still listed after epoch 5 and all gone after epoch 6.
    G, rows, y = _trace_problem(["a", "b"] + ["u"] * 40)
    for k, last_full in ((4, 4), (5, 5), (6, 6)):
        for E in range(1, 9):
            _, _, st = oracle.cd_solve(G, rows, y, 10.0, eps=2.0 ** -40, max_epochs=E, shrink_k=k)
            assert st["epochs"] == E and not st["converged"]
            assert st["active"] == (42 if E <= last_full else 2), (k, E)


def test_one_recheck_after_every_19_active_steps(oracle):
    # eta = 5 %: S = round(0.95 / 0.05) = 19.  Same problem; epochs 1..5 cost 42 steps each and nothing is
    # removed yet, so the counter of active steps since the last re-check stands far above S when epoch 6 begins.
    # Epoch 6, position by position: a, b, the first inert variable (removed: the queue is no longer empty), then
    # a re-check before position 3, and one more before every 19th position after it: positions 3, 22, 41 of the
    # 42.  Each re-check finds its variable unchanged.  Steps after 6 epochs: 5 * 42 + 42 + 3 = 255.
    # With 39 inert variables the positions are 3 and 22 (41 positions in all): 5 * 41 + 41 + 2 = 248.
    # S = 18 would give 3 re-checks in the second case (3, 21, 39), S = 20 two in the first (3, 23): 249 / 254.
    for m, steps6 in ((40, 255), (39, 248)):
        G, rows, y = _trace_problem(["a", "b"] + ["u"] * m)
        _, _, st = oracle.cd_solve(G, rows, y, 10.0, eps=2.0 ** -40, max_epochs=6, shrink_k=5, eta=0.05)
        assert st["steps"] == steps6 and st["active"] == 2
    G, rows, y = _trace_problem(["a", "b"] + ["u"] * 39)
    assert oracle.cd_solve(G, rows, y, 10.0, eps=2.0 ** -40, max_epochs=6, eta=1.0 / 19.0)[2]["steps"] == 249   # S = 18
    G, rows, y = _trace_problem(["a", "b"] + ["u"] * 40)
    assert oracle.cd_solve(G, rows, y, 10.0, eps=2.0 ** -40, max_epochs=6, eta=1.0 / 21.0)[2]["steps"] == 254   # S = 20
    # later epochs have two active steps each; after the re-check at position 41 of epoch 6 one active step
    # followed, so the counter reads 1 + 2 (e - 6) after epoch e and reaches 19 after epoch 15: the next re-check
    # opens epoch 16.  Steps: 255 + 2 * 9 = 273 after epoch 15, 273 + 1 + 2 = 276 after epoch 16.
    for E, steps in ((15, 273), (16, 276)):
        assert oracle.cd_solve(G, rows, y, 10.0, eps=2.0 ** -40, max_epochs=E, eta=0.05)[2]["steps"] == steps


_FIFO_ORDER = ["a", "b", "u", "s", "u"]


def _fifo_trace_expectation(j=6):
    beta = 2.0 - 2.0 ** -j
    alpha_s = 2.0 ** -(j + 1) / (beta * beta + 1.0)
    return {"steps": 19, "active": 3, "alpha_a": 1.0 / 32.0, "alpha_s": alpha_s,
            "alpha_b": 15.0 / 32.0 - beta * alpha_s / 2.0}


def test_recheck_takes_the_oldest_removed_variable(oracle):
    # Order a, b, u1, s, u2; k = 2; eta = 1/4, so S = 3.  c = active steps since the last re-check, Q = queue.
    #   epoch 1  a, b, u1 change; s sees w_1 = 3/4: unchanged (1st time); u2 changes.  c = 5, 5 steps.
    #   epoch 2  a, b change; u1 unchanged (1st); s sees 5/8: unchanged (2nd) -> removed, Q = [s].  Before u2:
    #            c = 9 >= 3 and Q is not empty -> re-check of s, still 5/8: unchanged, back to the tail, c = 0.
    #            u2 unchanged (1st), c = 1.  Steps 5 + 4 + 1 + 1 = 11, list for epoch 3: a, b, u1, u2.
    #   epoch 3  a (c = 2), b (c = 3); before u1: re-check of s, w_1 = 9/16: unchanged, c = 0.  u1 unchanged (2nd)
    #            -> removed, u2 likewise: Q = [s, u1, u2], c = 2.  Steps 11 + 4 + 1 = 16, list: a, b.
    #   epoch 4  a (c = 3); before b: re-check of the OLDEST entry, s, between a's and b's step: w_1 = 1/2, the
    #            step moves alpha_s to 2^-7 / (beta^2 + 1) and s rejoins.  Then b, whose gradient now contains s:
    #            alpha_b = 7/16 + (1/16 - beta alpha_s) / 2.  Steps 16 + 2 + 1 = 19, list for epoch 5: a, s, b.
    # Taking the newest entry instead (u2) finds it unchanged: alpha_s stays 0 and two variables stay listed.
    G, rows, y = _trace_problem(_FIFO_ORDER)
    for E, steps, active in ((1, 5, 5), (2, 11, 4), (3, 16, 2)):
        a, _, st = oracle.cd_solve(G, rows, y, 10.0, eps=2.0 ** -40, max_epochs=E, shrink_k=2, eta=0.25)
        assert (st["steps"], st["active"]) == (steps, active) and a[3] == 0.0
    a, w, st = oracle.cd_solve(G, rows, y, 10.0, eps=2.0 ** -40, max_epochs=4, shrink_k=2, eta=0.25)
    exp = _fifo_trace_expectation()
    assert (st["steps"], st["active"]) == (exp["steps"], exp["active"])
    assert a[0] == exp["alpha_a"] and a[2] == 1.0 and a[4] == 1.0
    assert abs(a[3] - exp["alpha_s"]) <= 1e-16 and abs(a[1] - exp["alpha_b"]) <= 1e-15
    # S = 4 (eta = 1/5) moves the re-checks: the one of epoch 4 does not happen, s stays asleep
    a, _, st = oracle.cd_solve(G, rows, y, 10.0, eps=2.0 ** -40, max_epochs=4, shrink_k=2, eta=0.2)
    assert a[3] == 0.0 and st["active"] == 2


def test_stop_is_confirmed_by_an_epoch_that_started_from_w_of_alpha(oracle):
    # Four orthonormal rows, C = 1/2: epoch 1 takes every alpha from 0 to C (violation 1 before each step);
    # from then on nothing changes and no violation is seen (at alpha = C a positive gradient is none).
    # Epoch 2 meets the criterion, w is set to sum alpha y g (4 rows read), nothing is removed or violating, but
    # the epoch had started from the increments of epoch 1 -> not yet; epoch 3 started from that w -> stop.
    # Steps: 3 epochs * 4 + 2 * 4 rows read = 20.
    G = np.eye(4, dtype=np.float32)
    a, w, st = oracle.cd_solve(G, np.arange(4), np.ones(4, dtype=np.float32), 0.5, eps=1e-3)
    assert st["converged"] and st["epochs"] == 3 and st["steps"] == 20 and np.all(a == 0.5)
    # a start at the solution is confirmed by its first epoch (the start w is computed from the start alpha)
    a, w, st = oracle.cd_solve(G, np.arange(4), np.ones(4, dtype=np.float32), 0.5, eps=1e-3, alpha0=a)
    assert st["converged"] and st["epochs"] == 1 and st["steps"] == 4 + 4


def test_sweep_at_the_stopping_check_brings_violators_back(oracle):
    # a, b, sleeper with j = 3, no interleaved re-checks (eta = 0), k = 2: s is removed in epoch 2 and nobody looks
    # at it again until the criterion is met.  The largest violation of epoch e + 1 is 2^-e, so eps = 1.5 * 2^-10 is
    # met in epoch 11.  The sweep then shows s the state after b's step of epoch 11, w_1 = 1/2 + 2^-12: its
    # gradient 1 - (2 - 1/8) w_1 = 1/16 - 2^-11 + 2^-15 is far above eps -> s rejoins and the solver goes on.
    G, rows, y = _trace_problem(["a", "b", "s"], j=3)
    eps = 1.5 * 2.0 ** -10
    for E in (3, 10):
        a, _, st = oracle.cd_solve(G, rows, y, 10.0, eps=eps, max_epochs=E, shrink_k=2, eta=0.0)
        assert st["active"] == 2 and a[2] == 0.0 and not st["converged"]
        assert a[0] == 2.0 ** -(E + 1) and a[1] == 0.5 - 2.0 ** -(E + 1)
    a, _, st = oracle.cd_solve(G, rows, y, 10.0, eps=eps, max_epochs=11, shrink_k=2, eta=0.0)
    assert st["active"] == 3 and not st["converged"] and st["max_violation"] == 2.0 ** -10
    # steps: 3 (epoch 1) + 3 (epoch 2) + 2 * 9 (epochs 3..11) + 2 rows read for w (alpha_s = 0 is skipped) + 1 sweep
    assert st["steps"] == 3 + 3 + 18 + 2 + 1
    a, w, st = oracle.cd_solve(G, rows, y, 10.0, eps=eps, max_epochs=100000, shrink_k=2, eta=0.0)
    assert st["converged"] and a[2] > 0.0 and _kkt(G, y, a, w, 10.0) <= eps


# The same traces must FAIL for an oracle with the rule changed: copies of the C source with one planted mistake
# each are built on the CPU and run through the hand-traced cases.

def _mutant(tmp_path, name, old, new):
    import ctypes
    import subprocess
    from oracle import lpd_oracle
    src = open(lpd_oracle._SRC).read()
    assert src.count(old) == 1, "the planted mistake no longer matches the oracle's source"
    c_file, so = tmp_path / f"{name}.c", tmp_path / f"{name}.so"
    c_file.write_text(src.replace(old, new))
    subprocess.run(["gcc", "-O2", "-fPIC", "-shared", "-std=c11", "-o", str(so), str(c_file), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    f32p, f64p, i64 = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double), ctypes.c_int64
    lib.orc_cd_solve.argtypes = [f32p, i64, i64, ctypes.POINTER(i64), f32p, i64, ctypes.c_double, ctypes.c_double,
                                 i64, i64, ctypes.c_double, f64p, f64p, f64p]
    lib.orc_cd_solve.restype = None

    def solve(G, rows, y, C, eps, max_epochs, shrink_k, eta):
        G = np.ascontiguousarray(G, dtype=np.float32)
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        y = np.ascontiguousarray(y, dtype=np.float32)
        alpha, w, st = np.zeros(len(rows)), np.zeros(G.shape[1]), np.zeros(6)
        lib.orc_cd_solve(G.ctypes.data_as(f32p), G.shape[1], G.shape[1], rows.ctypes.data_as(ctypes.POINTER(i64)),
                         y.ctypes.data_as(f32p), len(rows), C, eps, max_epochs, shrink_k, eta,
                         alpha.ctypes.data_as(f64p), w.ctypes.data_as(f64p), st.ctypes.data_as(f64p))
        return alpha, w, {"epochs": int(st[0]), "steps": int(st[1]), "converged": bool(st[2]), "active": int(st[3])}
    return solve


def test_planted_mistakes_in_the_discrete_rules_fail_the_traces(oracle, tmp_path):
    exp = _fifo_trace_expectation()
    G, rows, y = _trace_problem(_FIFO_ORDER)
    # (1) the re-check takes the newest removed variable instead of the oldest
    lifo = _mutant(tmp_path, "lifo",
                   "                const int64_t t = rem[head];\n"
                   "                head = (head + 1) % (np + 1);\n"
                   "                --n_rem;\n"
                   "                const float *g = G + rows[t] * ldg;\n"
                   "                double q = 0.0;",
                   "                const int64_t t = rem[(head + n_rem - 1) % (np + 1)];\n"
                   "                --n_rem;\n"
                   "                const float *g = G + rows[t] * ldg;\n"
                   "                double q = 0.0;")
    a, _, st = lifo(G, rows, y, 10.0, 2.0 ** -40, 4, 2, 0.25)
    assert a[3] == 0.0 and st["active"] == 2 and st["active"] != exp["active"]
    # (2) removal one unchanged step late
    late = _mutant(tmp_path, "late", "++cnt[t] >= shrink_k", "++cnt[t] > shrink_k")
    Gk, rk, yk = _trace_problem(["a", "b"] + ["u"] * 40)
    assert late(Gk, rk, yk, 10.0, 2.0 ** -40, 6, 5, 0.05)[2]["active"] == 42      # the trace says 2
    # (3) a re-check after every S + 1 active steps
    slow = _mutant(tmp_path, "slow", "since >= S && n_rem > 0", "since > S && n_rem > 0")
    assert slow(Gk, rk, yk, 10.0, 2.0 ** -40, 6, 5, 0.05)[2]["steps"] == 254      # the trace says 255
    # (4) no confirming epoch
    hasty = _mutant(tmp_path, "hasty", "if (back == 0 && fresh) converged = 1;", "if (back == 0) converged = 1;")
    _, _, st = hasty(np.eye(4), np.arange(4), np.ones(4), 0.5, 1e-3, 1000, 5, 0.05)
    assert st["converged"] and st["epochs"] == 2 and st["steps"] == 12            # the trace says 3 and 20
