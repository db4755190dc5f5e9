"""Pins for the CPU oracle: things the paper and the mathematics fix, none of them the oracle itself.

Each test names the mistake it would catch.  All CPU, double precision, tiny seeded inputs.
"""
import math
import os

import numpy as np
import pytest
import scipy.spatial.distance as ssd

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "two_landmark_closed_form.txt")


def _rng(seed):
    return np.random.default_rng(seed)


def _relfro(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def _points(seed, n, d):
    return _rng(seed).standard_normal((n, d)).astype(np.float32)


# ---------------------------------------------------------------- Section 5 kernel

def test_kernel_two_point_hand_values(oracle):
    # d=1, x=0, x'=1, gamma=ln2 -> 1/2 ; d=3 with squared distance 9, gamma=0.1 -> exp(-0.9)
    z = oracle.kernel_block(np.array([[0.0]]), np.array([[1.0]]), math.log(2.0))
    assert abs(z[0, 0] - 0.5) < 1e-15
    z = oracle.kernel_block(np.array([[1.0, 2.0, 3.0]]), np.array([[0.0, 0.0, 1.0]]), 0.1)
    assert abs(z[0, 0] - math.exp(-0.9)) < 1e-15
    # a wrong sign of gamma or a missing square would give > 1 or exp(-0.5)
    assert 0.0 < z[0, 0] < 1.0


def test_kernel_diagonal_symmetry_range(oracle):
    L = _points(1, 40, 7)
    K = oracle.kernel_block(L, L, 0.3)
    assert np.all(np.diag(K) == 1.0)           # exact: direct differences give exp(0)
    assert np.array_equal(K, K.T)
    assert np.all(K > 0.0) and np.all(K <= 1.0)


def test_kernel_block_rows_of_landmarks_are_one(oracle):
    X = _points(2, 50, 5)
    idx = np.array([3, 17, 42])
    Z = oracle.kernel_block(X, X[idx], 0.7)
    for b, i in enumerate(idx):
        assert Z[i, b] == 1.0


def test_kernel_block_against_scipy_sqeuclidean(oracle):
    # independent library routine for the squared distance; catches a transposed or mis-strided operand
    X = _points(3, 33, 11)
    L = _points(4, 9, 11)
    gamma = 0.05
    Z = oracle.kernel_block(X, L, gamma)
    ref = np.exp(-gamma * ssd.cdist(X.astype(np.float64), L.astype(np.float64), "sqeuclidean"))
    assert Z.shape == (33, 9)
    assert np.max(np.abs(Z - ref)) < 1e-14


# ---------------------------------------------------------------- Figure 1 step 1b

def test_jacobi_against_lapack_and_residual(oracle):
    L = _points(5, 48, 6)
    K = oracle.kernel_block(L, L, 0.2)
    ev, V = oracle.jacobi_eigh(K)
    ref = np.linalg.eigvalsh(K)
    assert np.max(np.abs(np.sort(ev) - ref)) < 1e-12
    assert _relfro(V @ np.diag(ev) @ V.T, K) < 1e-13
    assert np.linalg.norm(V.T @ V - np.eye(48)) < 1e-12
    assert abs(ev.sum() - 48.0) < 1e-11      # trace of a Gaussian kernel matrix is B


def test_jacobi_known_2x2(oracle):
    ev, V = oracle.jacobi_eigh(np.array([[1.0, 0.5], [0.5, 1.0]]))
    assert np.allclose(np.sort(ev), [0.5, 1.5], atol=1e-15)


def test_library_eigendecomposition_path_above_the_jacobi_limit(oracle):
    # 600 landmarks in 4 dimensions, above the size where the oracle hands step 1b to LAPACK.  The spectrum
    # decays fast, so the dropping rule of Section 4 is active too.  What must hold whatever routine did 1b:
    # the kept part reproduces the kernel matrix up to the dropped eigenvalues, W K W^T = I_r, trace = B.
    from oracle import lpd_oracle
    assert 600 > lpd_oracle.JACOBI_MAX_B
    Lm = _points(21, 600, 4)
    gamma, tau = 0.25, 1e-10
    W, eig, rank, K = oracle.whiten(Lm, gamma, tau=tau)                  # "auto" -> LAPACK + self-check
    assert 0 < rank < 600 and np.all(np.diff(eig) <= 0)
    assert eig[rank - 1] >= tau * eig[0] > eig[rank]
    assert abs(eig.sum() - 600.0) < 1e-9
    Wr = W[:rank]
    GL = oracle.apply_whitening(K, W, rank)                              # landmark rows of the factor: Z = K_LL
    dropped = np.sqrt(np.sum(eig[rank:] ** 2))
    assert np.linalg.norm(GL @ GL.T - K) <= dropped + 1e-9 * np.linalg.norm(K)
    # W K W^T = I_r: the error of row j carries a factor 1 / eig_j of the eigenvector's own rounding
    I_r = Wr @ K @ Wr.T
    assert np.max(np.abs(I_r - np.eye(rank)) * np.sqrt(np.outer(eig[:rank], eig[:rank]))) < 1e-9
    assert np.all(W[rank:] == 0.0)


def test_library_and_jacobi_paths_agree(oracle):
    # 300 landmarks, well-conditioned kernel matrix: both routes of step 1b must give the same eigenvalues, the
    # same rank, and the same basis-independent quantities K~ = G_L G_L^T and W^T W (= K^-1 when nothing is dropped).
    Lm = _points(22, 300, 16)
    gamma = 1.0 / 16
    Wj, ej, rj, K = oracle.whiten(Lm, gamma, method="jacobi")
    Wl, el, rl, _ = oracle.whiten(Lm, gamma, method="lapack")
    assert rj == rl == 300
    assert np.max(np.abs(ej - el)) <= 1e-11 * ej[0]
    Gj, Gl = oracle.apply_whitening(K, Wj), oracle.apply_whitening(K, Wl)
    assert _relfro(Gj @ Gj.T, Gl @ Gl.T) < 1e-10 and _relfro(Gl @ Gl.T, K) < 1e-10
    assert _relfro(Wj.T @ Wj, Wl.T @ Wl) < 1e-7
    assert _relfro(Wl.T @ Wl, np.linalg.inv(K)) < 1e-7
    # simple spectrum: the rows themselves agree, sign convention included
    gaps = np.min(np.abs(np.diff(ej))) / ej[0]
    if gaps > 1e-6:
        assert np.max(np.abs(Wj - Wl) * np.sqrt(ej)[:, None]) < 1e-6


def test_library_eigendecomposition_is_checked_before_use(oracle):
    # a decomposition that does not reproduce K, or whose vectors are not orthonormal, must be refused
    Lm = _points(23, 40, 5)
    K = oracle.kernel_block(Lm, Lm, 0.3)
    ev, V = np.linalg.eigh(K)
    oracle.check_eigendecomposition(K, ev, V)
    with pytest.raises(RuntimeError):
        oracle.check_eigendecomposition(K, ev[::-1].copy(), V)           # values paired with the wrong vectors
    V_bad = V.copy()
    V_bad[:, 0] *= 1.0 + 1e-9                                            # not normalised
    with pytest.raises(RuntimeError):
        oracle.check_eigendecomposition(K, ev, V_bad)
    V_rot = V.copy()
    V_rot[:, 1] += 1e-8 * V[:, 0]                                        # not orthogonal
    with pytest.raises(RuntimeError):
        oracle.check_eigendecomposition(K, ev, V_rot)


# ---------------------------------------------------------------- steps 1a-1d, closed form

def _read_golden():
    rows, W, D = [], None, None
    for line in open(GOLDEN):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "W":
            W = np.array(t[1:], dtype=np.float64).reshape(2, 2)
        elif t[0] == "D":
            D = np.array(t[1:], dtype=np.float64)
        else:
            rows.append([float(v) for v in t])
    return np.array(rows), W, D


@pytest.mark.parametrize("method", ["jacobi", "lapack"])
def test_two_landmark_closed_form(oracle, method):
    rows, Wg, Dg = _read_golden()
    Lm = np.array([[0.0], [1.0]], dtype=np.float32)
    gamma = math.log(2.0)
    W, eig, rank, K = oracle.whiten(Lm, gamma, method=method)
    assert rank == 2
    assert np.allclose(eig, Dg, atol=1e-14)
    assert np.allclose(W, Wg, atol=1e-14)       # includes order and sign convention
    X = rows[:, :1].astype(np.float32)
    Z = oracle.kernel_block(X, Lm, gamma)
    assert np.allclose(Z, rows[:, 1:3], atol=1e-15)
    G = oracle.apply_whitening(Z, W)
    assert np.allclose(G, rows[:, 3:5], atol=1e-14)
    # fp32-input entry point agrees (W here is exactly representable only approximately: 1e-7)
    G32 = oracle.nystrom_factor(X, Lm, gamma, W.astype(np.float32))
    assert np.allclose(G32, rows[:, 3:5], atol=1e-7)
    m = oracle.margins_f64(G, np.array([2.0, -3.0]))
    assert np.allclose(m, rows[:, 5], atol=1e-14)


# ---------------------------------------------------------------- invariants of the factor

@pytest.mark.parametrize("method", ["jacobi", "lapack"])
def test_landmark_rows_reproduce_landmark_kernel(oracle, method):
    # G_L G_L^T = K_LL ; G_L^T G_L = D ; sum D = B.   Fails by O(1) if W is applied untransposed
    # (G = Z W instead of Z W^T), if D^-1 replaces D^-1/2, or if eigenvectors are taken as rows.
    X = _points(6, 120, 8)
    idx = np.arange(0, 120, 5)                     # 24 landmarks
    Lm = X[idx]
    gamma = 1.0 / 8
    W, eig, rank, K = oracle.whiten(Lm, gamma, method=method)
    assert rank == 24
    Z = oracle.kernel_block(X, Lm, gamma)
    G = oracle.apply_whitening(Z, W)
    GL = G[idx]
    assert _relfro(GL @ GL.T, K) < 1e-10
    assert np.max(np.abs(GL.T @ GL - np.diag(eig))) < 1e-10
    assert abs(eig.sum() - 24.0) < 1e-10
    assert np.all(np.diff(eig) <= 0)
    # planted mistakes (CPU only): the other orientation, and D^-1 scaling, must break the identity
    G_wrong = Z @ W                                # = Z D^-1/2 U^T
    assert _relfro(G_wrong[idx] @ G_wrong[idx].T, K) > 1e-2
    W_inv = W * (1.0 / np.sqrt(eig))[:, None]      # rows scaled by D^-1 instead of D^-1/2
    G_inv = Z @ W_inv.T
    assert _relfro(G_inv[idx] @ G_inv[idx].T, K) > 1e-2


def test_all_points_landmarks_gives_full_kernel_bruteforce(oracle):
    # B = n: G G^T must equal K(X, X), computed here by an independent double loop
    n, d, gamma = 24, 3, 0.4
    X = _points(7, n, d)
    W, eig, rank, _ = oracle.whiten(X, gamma)
    assert rank == n
    G = oracle.nystrom_factor(X, X, gamma, W.astype(np.float32))   # fp32 W: 1e-7-level agreement
    Gd = oracle.apply_whitening(oracle.kernel_block(X, X, gamma), W)
    Kb = np.empty((n, n))
    for i in range(n):
        for j in range(n):
            s = 0.0
            for k in range(d):
                s += (float(X[i, k]) - float(X[j, k])) ** 2
            Kb[i, j] = math.exp(-gamma * s)
    assert _relfro(Gd @ Gd.T, Kb) < 1e-10
    assert _relfro(G @ G.T, Kb) < 1e-5


def test_projection_bound_on_every_row(oracle):
    # ||g_i||^2 = k~(x_i, x_i) <= k(x_i, x_i) = 1, with equality on landmark rows
    X = _points(8, 300, 10)
    idx = np.arange(0, 300, 10)
    W, eig, rank, _ = oracle.whiten(X[idx], 0.1)
    G = oracle.nystrom_factor(X, X[idx], 0.1, W.astype(np.float32))
    sq = (G * G).sum(axis=1)
    assert np.all(sq <= 1.0 + 1e-5)
    assert np.allclose(sq[idx], 1.0, atol=1e-5)
    assert sq.min() < 0.9                          # not trivially all ones


def test_gamma_zero_rank_one(oracle):
    # K_LL = 1 1^T: eigenvalues (B, 0, ...): rank 1, W[0] = 1^T / B, G[:,0] = 1
    X = _points(9, 20, 4)
    Lm = X[:6]
    W, eig, rank, K = oracle.whiten(Lm, 0.0)
    assert rank == 1
    assert abs(eig[0] - 6.0) < 1e-12 and np.max(np.abs(eig[1:])) < 1e-12
    assert np.allclose(W[0], 1.0 / 6.0, atol=1e-14)
    assert np.all(W[1:] == 0.0)
    G = oracle.apply_whitening(oracle.kernel_block(X, Lm, 0.0), W)
    assert np.allclose(G[:, 0], 1.0, atol=1e-13) and np.all(G[:, 1:] == 0.0)


@pytest.mark.parametrize("method", ["jacobi", "lapack"])
def test_duplicate_landmark_is_dropped(oracle, method):
    X = _points(10, 60, 5)
    Lm = np.concatenate([X[:12], X[3:4]])          # landmark 3 twice -> one zero eigenvalue
    gamma = 0.15
    W, eig, rank, K = oracle.whiten(Lm, gamma, method=method)
    assert rank == 12
    assert abs(eig[-1]) < 1e-12
    G = oracle.apply_whitening(oracle.kernel_block(Lm, Lm, gamma), W)
    assert _relfro(G @ G.T, K) < 1e-9             # still reproduces K_LL without the dropped direction
    assert np.all(W[12:] == 0.0)


def test_single_landmark(oracle):
    X = _points(11, 15, 3)
    Lm = X[4:5]
    W, eig, rank, _ = oracle.whiten(Lm, 0.5)
    assert rank == 1 and W.shape == (1, 1) and abs(W[0, 0] - 1.0) < 1e-15
    G = oracle.nystrom_factor(X, Lm, 0.5, W.astype(np.float32))
    assert np.allclose(G[:, 0], oracle.kernel_block(X, Lm, 0.5)[:, 0], atol=1e-15)


def test_sign_and_order_convention(oracle):
    X = _points(12, 30, 6)
    W, eig, rank, _ = oracle.whiten(X, 0.2)
    for j in range(rank):
        k = np.argmax(np.abs(W[j]))
        assert W[j, k] > 0.0
        assert abs(np.dot(W[j], W[j]) - 1.0 / eig[j]) < 1e-9 / eig[j]
    assert np.all(np.diff(eig) <= 0)


# ---------------------------------------------------------------- Figure 1 step 2a

def test_margins_unit_vectors_and_numpy(oracle):
    rng = _rng(13)
    G = rng.standard_normal((37, 10)).astype(np.float32)
    for j in (0, 4, 9):
        e = np.zeros(10, dtype=np.float32)
        e[j] = 1.0
        assert np.array_equal(oracle.margins(G, e), G[:, j].astype(np.float64))
    w = rng.standard_normal(10).astype(np.float32)
    assert np.allclose(oracle.margins(G, w), G.astype(np.float64) @ w.astype(np.float64), atol=1e-13)
    # leading dimension larger than r: trailing columns are ignored
    assert np.allclose(oracle.margins(G, w[:6], r=6), G[:, :6].astype(np.float64) @ w[:6].astype(np.float64),
                       atol=1e-13)


def test_margins_with_landmark_row_returns_kernel_column(oracle):
    # w = G_a^T for landmark a:  G G_a^T = Z K_LL^-1 K_LL[:,a] = Z[:,a]  -- ties the sweep to the kernel block
    X = _points(14, 80, 6)
    idx = np.arange(0, 80, 4)
    gamma = 0.2
    W, eig, rank, _ = oracle.whiten(X[idx], gamma)
    Z = oracle.kernel_block(X, X[idx], gamma)
    G = oracle.apply_whitening(Z, W)
    for a in (0, 7, 19):
        m = oracle.margins_f64(G, G[idx[a]])
        assert np.max(np.abs(m - Z[:, a])) < 1e-10


def test_workload_recipes_keep_landmark_kernel_well_conditioned(oracle):
    # on scaled-down versions of the five recipes no eigenvalue is near the drop threshold
    import torch
    from paper_2207_01016_amd import workloads as wl

    for name, w in wl.WORKLOADS.items():
        small = w.with_shape(n=600, B=64)
        X = wl.make_X(small).numpy()
        idx = wl.landmark_indices(small).numpy()
        W, eig, rank, _ = oracle.whiten(X[idx], small.gamma)
        assert rank == 64, name
        assert eig[-1] > 1e-3, (name, eig[-1])


# ---------------------------------------------------------------- prediction (Section 4, prediction step)

def test_predict_closed_form_two_landmarks(oracle):
    rows, Wg, Dg = _read_golden()
    Lm = np.array([[0.0], [1.0]], dtype=np.float32)
    X = rows[:, :1].astype(np.float32)
    F = oracle.predict(X, Lm, math.log(2.0), Wg.astype(np.float32), np.array([[2.0, -3.0]], dtype=np.float32))
    assert np.allclose(F[:, 0], rows[:, 5], atol=1e-6)          # fp32 W: 1/sqrt(3) is rounded


def test_predict_on_training_rows_equals_margins_of_the_factor(oracle):
    X = _points(20, 90, 6)
    idx = np.arange(0, 90, 3)
    gamma = 0.2
    W, eig, rank, _ = oracle.whiten(X[idx], gamma)
    W32 = W.astype(np.float32)
    G = oracle.nystrom_factor(X, X[idx], gamma, W32)
    Ws = _rng(21).standard_normal((3, rank)).astype(np.float32)
    F = oracle.predict(X, X[idx], gamma, W32, Ws)
    for j in range(3):
        assert np.allclose(F[:, j], oracle.margins_f64(G, Ws[j].astype(np.float64)), atol=1e-12)


def test_predict_is_the_kernel_expansion_when_all_points_are_landmarks(oracle):
    # B = n: the low-rank kernel is exact, so with w = sum_i a_i y_i g_i the score of a NEW point x is the
    # representer form f(x) = sum_i a_i y_i k(x, x_i) of Section 2, computed here by an independent loop
    n, d, gamma = 20, 3, 0.3
    X = _points(22, n, d)
    Xt = _points(23, 7, d)
    W, eig, rank, _ = oracle.whiten(X, gamma)
    assert rank == n
    G = oracle.apply_whitening(oracle.kernel_block(X, X, gamma), W)
    coef = _rng(24).standard_normal(n)                      # a_i y_i
    w = coef @ G
    F = oracle.predict(Xt, X, gamma, W.astype(np.float32), w.astype(np.float32)[None, :])
    for t in range(7):
        ref = 0.0
        for i in range(n):
            dist = sum((float(Xt[t, k]) - float(X[i, k])) ** 2 for k in range(d))
            ref += coef[i] * math.exp(-gamma * dist)
        assert abs(F[t, 0] - ref) <= 1e-4 * max(1.0, abs(ref))   # W and w were rounded to fp32


# ---------------------------------------------------------------- Section 4, kernel block of sparse rows

def _random_csr(seed, n, d, density, sort=True):
    """Rows as dicts {column: value}, and the same rows in compressed-row form."""
    g = _rng(seed)
    rows, row_ptr, cols, vals = [], [0], [], []
    for i in range(n):
        k = int(g.binomial(d, density)) if i % 5 else 0          # every fifth row is empty
        c = g.choice(d, size=k, replace=False)
        if sort:
            c = np.sort(c)
        v = g.standard_normal(k).astype(np.float32)
        rows.append({int(a): float(b) for a, b in zip(c, v)})
        cols.extend(int(a) for a in c)
        vals.extend(float(b) for b in v)
        row_ptr.append(len(cols))
    return rows, np.array(row_ptr, dtype=np.int64), np.array(cols, dtype=np.int32), np.array(vals, dtype=np.float32)


def test_csr_kernel_block_against_sparse_inner_products(oracle):
    """Independent formula: ||x - l||^2 = sum_nz x_k^2 + ||l||^2 - 2 sum_nz x_k l_k, from the dict rows.
    A dropped entry, an index shifted by one, or a value attached to the wrong row would show here."""
    d, B, gamma = 23, 9, 0.07
    rows, rp, ci, va = _random_csr(3, 31, d, 0.3)
    L = _points(4, B, d)
    Z = oracle.kernel_block_csr(rp, ci, va, d, L, gamma)
    for i, row in enumerate(rows):
        for b in range(B):
            l = L[b].astype(np.float64)
            sq = sum(v * v for v in row.values()) + float(l @ l) - 2.0 * sum(v * l[k] for k, v in row.items())
            assert abs(Z[i, b] - math.exp(-gamma * sq)) <= 1e-12


def test_csr_kernel_block_equals_dense_on_the_written_out_matrix(oracle):
    d, B, gamma = 40, 17, 0.02
    for sort in (True, False):                         # column order within a row does not matter
        rows, rp, ci, va = _random_csr(5, 50, d, 0.15, sort=sort)
        X = np.zeros((50, d), dtype=np.float32)
        for i, row in enumerate(rows):
            for k, v in row.items():
                X[i, k] = v
        L = _points(6, B, d)
        assert np.array_equal(oracle.kernel_block_csr(rp, ci, va, d, L, gamma), oracle.kernel_block(X, L, gamma))
    # an all-empty matrix gives exp(-gamma ||l||^2) in every row
    Z = oracle.kernel_block_csr(np.zeros(4, dtype=np.int64), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.float32),
                                d, L, gamma)
    assert np.allclose(Z, np.exp(-gamma * (L.astype(np.float64) ** 2).sum(axis=1))[None, :], rtol=1e-14)
    # stored zeros are harmless
    rp2 = np.array([0, 2], dtype=np.int64)
    Z0 = oracle.kernel_block_csr(rp2, np.array([3, 7], dtype=np.int32), np.array([0.0, 1.5], dtype=np.float32), d, L, gamma)
    Z1 = oracle.kernel_block_csr(np.array([0, 1], dtype=np.int64), np.array([7], dtype=np.int32),
                                 np.array([1.5], dtype=np.float32), d, L, gamma)
    assert np.array_equal(Z0, Z1)
