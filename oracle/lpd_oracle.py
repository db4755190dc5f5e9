"""Python face of the double-precision CPU oracle (TEST INFRASTRUCTURE, NOT THE PRODUCT).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module.  It marshals numpy arrays into ``lpd_oracle.c`` (plain C, built
with gcc) and adds the one step that is allowed to be a library primitive: for
landmark counts where the plain Jacobi sweep would take minutes, the symmetric
eigendecomposition of step 1b (Figure 1) is LAPACK's, through
``numpy.linalg.eigh``; ordering, dropping and sign convention stay in the C
code either way.

Notation follows Figure 1 of the paper: K_LL (1a), K_LL = U D U^T (1b),
W = (U sqrt(D^-1))^T with small components dropped (1c and Section 4),
Z and G = Z W^T (1d), m = G w (2a).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lpd_oracle.c")
_LIB = os.path.join(_HERE, "liblpd_oracle.so")

JACOBI_MAX_B = 256  # above this the eigendecomposition step is numpy.linalg.eigh

_i64 = ctypes.c_int64
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile lpd_oracle.c with gcc -O2 -fopenmp into oracle/liblpd_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.orc_kernel_block.argtypes = [_f32p, _i64, _i64, _i64, _f32p, _i64, _i64, ctypes.c_double, _f64p]
        lib.orc_kernel_block.restype = None
        lib.orc_kernel_block_csr.argtypes = [ctypes.c_void_p, ctypes.c_void_p, _f32p, _i64, _i64, _f32p, _i64, _i64,
                                             ctypes.c_double, _f64p]
        lib.orc_kernel_block_csr.restype = None
        lib.orc_jacobi_eigh.argtypes = [_f64p, _i64, _f64p, _f64p]
        lib.orc_jacobi_eigh.restype = ctypes.c_int
        lib.orc_whiten_from_eig.argtypes = [_f64p, _f64p, _i64, ctypes.c_double, _f64p, _f64p]
        lib.orc_whiten_from_eig.restype = _i64
        lib.orc_nystrom_factor.argtypes = [_f32p, _i64, _i64, _i64, _f32p, _i64, _i64, ctypes.c_double,
                                           _f32p, _i64, _i64, _f64p]
        lib.orc_nystrom_factor.restype = None
        lib.orc_apply_whitening.argtypes = [_f64p, _i64, _i64, _f64p, _i64, _f64p]
        lib.orc_apply_whitening.restype = None
        lib.orc_margins.argtypes = [_f32p, _i64, _i64, _i64, _f32p, _f64p]
        lib.orc_margins.restype = None
        lib.orc_margins_f64.argtypes = [_f64p, _i64, _i64, _i64, _f64p, _f64p]
        lib.orc_margins_f64.restype = None
        lib.orc_cd_solve.argtypes = [_f32p, _i64, _i64, ctypes.POINTER(_i64), _f32p, _i64, ctypes.c_double,
                                     ctypes.c_double, _i64, _i64, ctypes.c_double, _f64p, _f64p, _f64p]
        lib.orc_cd_solve.restype = None
        lib.orc_predict.argtypes = [_f32p, _i64, _i64, _i64, _f32p, _i64, _i64, ctypes.c_double, _f32p, _i64, _i64,
                                    _f32p, _i64, _i64, _f64p]
        lib.orc_predict.restype = None
        lib.orc_num_threads.restype = ctypes.c_int
        lib.orc_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p32(a):
    return a.ctypes.data_as(_f32p)


def _p64(a):
    return a.ctypes.data_as(_f64p)


def num_threads() -> int:
    return int(_load().orc_num_threads())


def set_num_threads(t: int) -> None:
    _load().orc_set_num_threads(int(t))


def kernel_block(X, L, gamma: float) -> np.ndarray:
    """Z[i,b] = exp(-gamma ||x_i - l_b||^2) (Section 5 kernel; Figure 1 steps 1a/1d)."""
    X, L = _f32(X), _f32(L)
    n, d = X.shape
    B, d2 = L.shape
    assert d == d2
    Z = np.empty((n, B), dtype=np.float64)
    _load().orc_kernel_block(_p32(X), n, d, d, _p32(L), B, d, float(gamma), _p64(Z))
    return Z


def kernel_block_csr(row_ptr, col_idx, values, d: int, L, gamma: float) -> np.ndarray:
    """Z[i,b] = exp(-gamma ||x_i - l_b||^2) with the rows x_i given in compressed-row form (Section 4, sparse
    kernel operations): distinct column indices per row, any order, absent coordinates zero."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    values = _f32(values)
    L = _f32(L)
    n = row_ptr.shape[0] - 1
    B, d2 = L.shape
    assert d == d2 and row_ptr[0] == 0 and row_ptr[-1] == col_idx.shape[0] == values.shape[0]
    assert np.all(np.diff(row_ptr) >= 0)
    if col_idx.size:
        assert col_idx.min() >= 0 and col_idx.max() < d
    Z = np.empty((n, B), dtype=np.float64)
    _load().orc_kernel_block_csr(row_ptr.ctypes.data_as(ctypes.c_void_p), col_idx.ctypes.data_as(ctypes.c_void_p),
                                 _p32(values), n, d, _p32(L), B, d, float(gamma), _p64(Z))
    return Z


def jacobi_eigh(K):
    """Cyclic Jacobi eigendecomposition (Figure 1 step 1b); returns (ev unsorted, V columns)."""
    A = _f64(K).copy()
    B = A.shape[0]
    V = np.empty((B, B), dtype=np.float64)
    ev = np.empty(B, dtype=np.float64)
    sweeps = _load().orc_jacobi_eigh(_p64(A), B, _p64(V), _p64(ev))
    if sweeps < 0:
        raise RuntimeError("oracle Jacobi did not converge")
    return ev, V


def check_eigendecomposition(K, ev, V, tol: float = 1e-12) -> None:
    """Accept a library eigendecomposition K = V diag(ev) V^T (Figure 1 step 1b) only if it reproduces K and V is
    orthogonal: ||K - V diag(ev) V^T||_F <= tol ||K||_F and ||V^T V - I||_F <= tol B.  Raises otherwise."""
    K, ev, V = _f64(K), _f64(ev), _f64(V)
    B = K.shape[0]
    if B == 0:
        return
    res = np.linalg.norm(K - (V * ev) @ V.T) / max(np.linalg.norm(K), np.finfo(np.float64).tiny)
    orth = np.linalg.norm(V.T @ V - np.eye(B))
    if not (res <= tol) or not (orth <= tol * B):
        raise RuntimeError(f"library eigendecomposition rejected: residual {res:.3e} (bound {tol:.1e}), "
                           f"orthogonality {orth:.3e} (bound {tol * B:.1e})")


def whiten(L, gamma: float, tau: float = 1e-10, method: str = "auto"):
    """Steps 1a-1c: returns (W float64 BxB with rows >= rank zero, eig descending, rank, K_LL)."""
    L = _f32(L)
    B = L.shape[0]
    K = kernel_block(L, L, gamma)
    if method == "auto":
        method = "jacobi" if B <= JACOBI_MAX_B else "lapack"
    if method == "jacobi":
        ev, V = jacobi_eigh(K)
    elif method == "lapack":
        ev, V = np.linalg.eigh(K)
        check_eigendecomposition(K, ev, V)
    else:
        raise ValueError(method)
    V = _f64(V)
    ev = _f64(ev)
    W = np.empty((B, B), dtype=np.float64)
    eig = np.empty(B, dtype=np.float64)
    rank = int(_load().orc_whiten_from_eig(_p64(V), _p64(ev), B, float(tau), _p64(W), _p64(eig)))
    return W, eig, rank, K


def nystrom_factor(X, L, gamma: float, W, r: int | None = None) -> np.ndarray:
    """Step 1d with fp32 inputs promoted to double: G (n x r) = Z W[:r]^T."""
    X, L, W = _f32(X), _f32(L), _f32(W)
    n, d = X.shape
    B = L.shape[0]
    if r is None:
        r = W.shape[0]
    assert W.shape[1] == B and r <= W.shape[0] and L.shape[1] == d
    G = np.empty((n, r), dtype=np.float64)
    _load().orc_nystrom_factor(_p32(X), n, d, d, _p32(L), B, d, float(gamma), _p32(W), r, W.shape[1], _p64(G))
    return G


def apply_whitening(Z, W, r: int | None = None) -> np.ndarray:
    """G = Z W[:r]^T entirely in double (for the pins)."""
    Z, W = _f64(Z), _f64(W)
    n, B = Z.shape
    if r is None:
        r = W.shape[0]
    assert W.shape[1] == B
    G = np.empty((n, r), dtype=np.float64)
    _load().orc_apply_whitening(_p64(Z), n, B, _p64(W), r, _p64(G))
    return G


def margins(G, w, r: int | None = None) -> np.ndarray:
    """Step 2a: m = G[:, :r] w, G and w fp32 (the buffers the sweep reads), sum in double."""
    G, w = _f32(G), _f32(w)
    n, ldg = G.shape
    if r is None:
        r = w.shape[0]
    assert r <= ldg and r <= w.shape[0]
    m = np.empty(n, dtype=np.float64)
    _load().orc_margins(_p32(G), n, r, ldg, _p32(w), _p64(m))
    return m


def margins_f64(G, w) -> np.ndarray:
    G, w = _f64(G), _f64(w)
    n, r = G.shape
    m = np.empty(n, dtype=np.float64)
    _load().orc_margins_f64(_p64(G), n, r, r, _p64(w), _p64(m))
    return m


def cd_solve(G, rows, y, C: float, eps: float = 1e-3, max_epochs: int = 1000, shrink_k: int = 5, eta: float = 0.05,
             alpha0=None, r: int | None = None):
    """Dual coordinate ascent with shrinking on the rows of G (Figure 1 steps 2a-2b; Section 4 "Shrinking").

    G: fp32 factor; rows: the problem's row indices in visiting order; y: +-1 per listed row.
    Returns (alpha float64 per listed row, w float64 (r), stats dict)."""
    G = _f32(G)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    y = _f32(y)
    n_p = rows.shape[0]
    assert y.shape[0] == n_p and G.ndim == 2
    r = G.shape[1] if r is None else int(r)
    alpha = np.zeros(n_p, dtype=np.float64) if alpha0 is None else _f64(alpha0).copy()
    w = np.zeros(r, dtype=np.float64)
    stats = np.zeros(6, dtype=np.float64)
    _load().orc_cd_solve(_p32(G), r, G.shape[1], rows.ctypes.data_as(ctypes.POINTER(_i64)), _p32(y), n_p, float(C),
                         float(eps), int(max_epochs), int(shrink_k), float(eta), _p64(alpha), _p64(w), _p64(stats))
    return alpha, w, {"epochs": int(stats[0]), "steps": int(stats[1]), "converged": bool(stats[2]),
                      "active": int(stats[3]), "max_violation": float(stats[4]), "dual": float(stats[5])}


def predict(X, L, gamma: float, W, Ws, r: int | None = None) -> np.ndarray:
    """Scores f_j(x_i) = ws_j . (W z(x_i)) of c classifiers (Section 4 prediction step). Ws: c x r. Returns n x c."""
    X, L, W = _f32(X), _f32(L), _f32(W)
    Ws = np.atleast_2d(_f32(Ws))
    n, d = X.shape
    B = L.shape[0]
    r = W.shape[0] if r is None else int(r)
    c = Ws.shape[0]
    assert W.shape[1] == B and Ws.shape[1] >= r and L.shape[1] == d
    F = np.empty((n, c), dtype=np.float64)
    _load().orc_predict(_p32(X), n, d, d, _p32(L), B, d, float(gamma), _p32(W), r, W.shape[1],
                        _p32(Ws), c, Ws.shape[1], _p64(F))
    return F
