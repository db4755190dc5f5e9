"""Thin ctypes binding over the C-ABI library ``liblpd.so`` (see ``include/lpd.h``).

Argument marshalling only: every function takes torch tensors (device memory and
the current stream come from PyTorch), checks dtype / device / contiguity, and
passes raw pointers, sizes and leading dimensions to the entry point of the same
name.  All arithmetic happens in the library's HIP kernels (or, for
``lpd_whiten_host``, in its host routine).  There is no fallback: if the shared
library is missing, loading fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblpd.so")

_i64 = ctypes.c_int64
_vp = ctypes.c_void_p
_sz = ctypes.c_size_t

LPD_OK = 0


class LpdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().lpd_strerror(status).decode()} (status {status})")


class FactorProfile(ctypes.Structure):
    _fields_ = [
        ("launches_norms", ctypes.c_int32),
        ("launches_kernel_block", ctypes.c_int32),
        ("launches_whiten", ctypes.c_int32),
        ("panel_rows", ctypes.c_int32),
        ("ms_norms", ctypes.c_float),
        ("ms_kernel_block", ctypes.c_float),
        ("ms_whiten", ctypes.c_float),
    ]


_FACTOR_ARGS = [_vp, _i64, _i64, _i64, _vp, _i64, _i64, ctypes.c_float, _vp, _i64, _i64, _vp, _i64, _vp, _sz, _vp]

SIGNATURES = {
    "lpd_version": (ctypes.c_int, []),
    "lpd_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "lpd_set_option": (ctypes.c_int, [ctypes.c_int, _i64]),
    "lpd_whiten_host": (ctypes.c_int, [_vp, _i64, _i64, _i64, ctypes.c_double, ctypes.c_double, _vp, _i64, _vp,
                                       ctypes.POINTER(_i64)]),
    "lpd_whiten_workspace": (ctypes.c_int, [_i64, ctypes.POINTER(_sz)]),
    "lpd_whiten": (ctypes.c_int, [_vp, _i64, _i64, _i64, ctypes.c_double, ctypes.c_double, _vp, _i64, _vp,
                                  ctypes.POINTER(_i64), _vp, _sz, _vp, ctypes.POINTER(ctypes.c_double)]),
    "lpd_nystrom_factor_workspace": (ctypes.c_int, [_i64, _i64, _i64, ctypes.POINTER(_sz), ctypes.POINTER(_sz)]),
    "lpd_nystrom_factor": (ctypes.c_int, _FACTOR_ARGS),
    "lpd_nystrom_factor_profiled": (ctypes.c_int, _FACTOR_ARGS + [ctypes.POINTER(FactorProfile)]),
    "lpd_nystrom_factor_to_host_workspace": (ctypes.c_int, [_i64, _i64, _i64, ctypes.POINTER(_i64),
                                                            ctypes.POINTER(_sz)]),
    "lpd_nystrom_factor_to_host": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _i64, ctypes.c_float, _vp, _i64,
                                                  _i64, _vp, _i64, _i64, _vp, _sz, _vp]),
    "lpd_nystrom_factor_csr_workspace": (ctypes.c_int, [_i64, _i64, _i64, _i64, ctypes.POINTER(_i64),
                                                        ctypes.POINTER(_sz)]),
    "lpd_nystrom_factor_csr": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _i64, _i64, ctypes.c_float, _vp,
                                              _i64, _i64, _vp, _i64, _i64, _vp, _sz, _vp]),
    "lpd_kernel_block_csr": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _i64, _i64, ctypes.c_float, _vp,
                                            _i64, _i64, _vp, _sz, _vp]),
    "lpd_predict_csr": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _i64, _i64, ctypes.c_float, _vp, _i64,
                                       _i64, _vp, _i64, _i64, _vp, _sz, _vp]),
    "lpd_kernel_block": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _i64, ctypes.c_float, _vp, _i64, _vp, _sz,
                                        _vp]),
    "lpd_margins": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _vp, _vp]),
    "lpd_margins_rows": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _vp]),
    "lpd_margins_multi": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _i64, _vp, _i64, _vp]),
    "lpd_fold_weights": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _i64, _vp, _i64, _vp]),
    "lpd_predict": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _i64, ctypes.c_float, _vp, _i64, _i64, _vp, _i64,
                                   _vp, _sz, _vp]),
    "lpd_predict_noalloc": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _i64, ctypes.c_float, _vp, _i64, _i64, _vp,
                                           _i64, _vp]),
    "lpd_row_sqnorms": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _vp]),
    "lpd_cd_solve_workspace": (ctypes.c_int, [_i64, _i64, ctypes.POINTER(_sz)]),
    "lpd_cd_solve": (ctypes.c_int, [_vp, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _vp, _vp, _vp, _i64, _vp,
                                    ctypes.c_float, ctypes.c_int32, ctypes.c_int32, ctypes.c_float, _vp, _sz, _vp]),
}

_lib = None


def lib() -> ctypes.CDLL:
    """Load liblpd.so (built by ``__graft_entry__.build()``); raise loudly if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} not found: the HIP library is not built. Run `python -c 'import __graft_entry__ as g; "
                "g.build()'` at the repository root (needs hipcc); there is no CPU fallback.")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _check(status: int, where: str) -> None:
    if status != LPD_OK:
        raise LpdError(status, where)


def _dev_f32(t: torch.Tensor, name: str, ndim: int) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or t.dtype != torch.float32 or t.dim() != ndim:
        raise TypeError(f"{name}: expected a {ndim}-D float32 tensor")
    if not t.is_cuda:
        raise ValueError(f"{name}: expected a tensor in device memory")
    if ndim == 2 and t.numel() > 0 and t.stride(1) != 1:
        raise ValueError(f"{name}: rows must be contiguous (stride(1) == 1)")
    if ndim == 1 and t.numel() > 1 and t.stride(0) != 1:
        raise ValueError(f"{name}: must be contiguous")
    return t


def _ld(t: torch.Tensor) -> int:
    return int(t.stride(0)) if t.shape[0] > 1 else max(int(t.shape[1]), 1)


def _stream(dev: torch.device) -> int:
    return int(torch.cuda.current_stream(dev).cuda_stream)


def lpd_version() -> int:
    return int(lib().lpd_version())


LPD_OPT_GEMM_TILE = 1
LPD_OPT_GEMM_PIPELINE = 2
LPD_OPT_CSR_ROUTE = 3
LPD_OPT_SMALL_PATH = 4
LPD_OPT_WHITEN_DC = 5
LPD_OPT_WHITEN_UPPER = 6
LPD_OPT_SWEEP_GRID = 7
LPD_OPT_FUSED_SCORES = 8
CSR_ROUTES = {"auto": 0, "dense": 1, "gather": 2}
GEMM_PIPELINE_DEFAULT = 2
GEMM_TILES = {"auto": 0, "128x128": 1, "256x128": 2, "256x256": 3, "64x128": 4}


def lpd_set_option(option: int, value: int) -> None:
    """Process-wide tuning knob (see include/lpd.h)."""
    _check(lib().lpd_set_option(int(option), int(value)), "lpd_set_option")


def lpd_whiten_host(L: torch.Tensor, gamma: float, clip_ratio: float = 1e-10):
    """Steps 1a-1c on the host. L: B x d float32 CPU tensor. Returns (W B x B float32 CPU, eig float64, rank)."""
    if L.dtype != torch.float32 or L.dim() != 2 or L.is_cuda:
        raise TypeError("L: expected a 2-D float32 CPU tensor")
    L = L.contiguous()
    B, d = L.shape
    W = torch.empty((B, B), dtype=torch.float32)
    eig = torch.empty(B, dtype=torch.float64)
    rank = _i64(0)
    st = lib().lpd_whiten_host(L.data_ptr(), B, d, max(d, 1), float(gamma), float(clip_ratio), W.data_ptr(),
                               max(B, 1), eig.data_ptr(), ctypes.byref(rank))
    _check(st, "lpd_whiten_host")
    return W, eig, int(rank.value)


def lpd_whiten_workspace(B: int) -> int:
    """Bytes of device scratch lpd_whiten needs for B landmarks."""
    nb = _sz(0)
    _check(lib().lpd_whiten_workspace(B, ctypes.byref(nb)), "lpd_whiten_workspace")
    return int(nb.value)


WHITEN_PHASES = ("kernel_matrix", "tridiagonalisation", "accumulation", "ql_rotations", "scaling")


def lpd_whiten(L: torch.Tensor, gamma: float, clip_ratio: float = 1e-10, workspace=None, phases: dict | None = None):
    """Steps 1a-1c with the cubic work on the device. L: B x d float32 device tensor.
    Returns (W B x B float32 on L's device, eig float64 CPU tensor, rank). Blocks until W is complete.
    `phases`, if given, receives the wall seconds of each phase (this drains the stream between phases)."""
    L = _dev_f32(L, "L", 2)
    B, d = L.shape
    W = torch.empty((B, B), dtype=torch.float32, device=L.device)
    eig = torch.empty(B, dtype=torch.float64)
    rank = _i64(0)
    nbytes = lpd_whiten_workspace(B)
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=L.device)
    if workspace.dtype != torch.uint8 or not workspace.is_cuda:
        raise TypeError("workspace: expected a uint8 device tensor")
    ph = (ctypes.c_double * 5)() if phases is not None else None
    st = lib().lpd_whiten(L.data_ptr(), B, d, _ld(L), float(gamma), float(clip_ratio), W.data_ptr(), max(B, 1),
                          eig.data_ptr(), ctypes.byref(rank), workspace.data_ptr(), workspace.numel(),
                          _stream(L.device), ph)
    _check(st, "lpd_whiten")
    if phases is not None:
        phases.update(zip(WHITEN_PHASES, ph))
    return W, eig, int(rank.value)


def lpd_nystrom_factor_workspace(n: int, d: int, B: int):
    """(recommended bytes, minimum bytes) of device scratch for a factor call of this shape."""
    rec, mn = _sz(0), _sz(0)
    _check(lib().lpd_nystrom_factor_workspace(n, d, B, ctypes.byref(rec), ctypes.byref(mn)),
           "lpd_nystrom_factor_workspace")
    return int(rec.value), int(mn.value)


def alloc_workspace(n: int, d: int, B: int, device, nbytes: int | None = None) -> torch.Tensor:
    """Device scratch as a uint8 tensor (torch's allocator returns 256-byte aligned blocks)."""
    rec, mn = lpd_nystrom_factor_workspace(n, d, B)
    nbytes = rec if nbytes is None else max(int(nbytes), mn)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def _factor_args(X, L, gamma, W, r, G, workspace):
    X = _dev_f32(X, "X", 2)
    L = _dev_f32(L, "L", 2)
    W = _dev_f32(W, "W", 2)
    G = _dev_f32(G, "G", 2)
    n, d = X.shape
    B = L.shape[0]
    if L.shape[1] != d or W.shape[1] != B or G.shape != (n, B):
        raise ValueError("shape mismatch: X n x d, L B x d, W r x B, G n x B")
    r = W.shape[0] if r is None else int(r)
    if r > W.shape[0]:
        raise ValueError("r exceeds the rows of W")
    if workspace.dtype != torch.uint8 or not workspace.is_cuda:
        raise TypeError("workspace: expected a uint8 device tensor")
    return (X.data_ptr(), n, d, _ld(X), L.data_ptr(), B, _ld(L), float(gamma), W.data_ptr(), r, _ld(W),
            G.data_ptr(), _ld(G), workspace.data_ptr(), workspace.numel(), _stream(X.device))


def lpd_nystrom_factor(X, L, gamma: float, W, G, workspace, r: int | None = None) -> torch.Tensor:
    """Step 1d: G[:, :r] = K(X, L) W[:r]^T, G[:, r:] = 0. Enqueued on torch's current stream."""
    args = _factor_args(X, L, gamma, W, r, G, workspace)
    _check(lib().lpd_nystrom_factor(*args), "lpd_nystrom_factor")
    return G


def lpd_nystrom_factor_profiled(X, L, gamma: float, W, G, workspace, r: int | None = None) -> FactorProfile:
    """Same work, blocking, returning the per-kernel HIP-event timings."""
    args = _factor_args(X, L, gamma, W, r, G, workspace)
    prof = FactorProfile()
    _check(lib().lpd_nystrom_factor_profiled(*args, ctypes.byref(prof)), "lpd_nystrom_factor_profiled")
    return prof


def lpd_nystrom_factor_to_host_workspace(n: int, d: int, B: int, chunk_rows: int = 0):
    """(chunk_rows, bytes): the chunk size in use (the suggested one for chunk_rows <= 0) and its scratch size."""
    cr, nb = _i64(int(chunk_rows)), _sz(0)
    _check(lib().lpd_nystrom_factor_to_host_workspace(n, d, B, ctypes.byref(cr), ctypes.byref(nb)),
           "lpd_nystrom_factor_to_host_workspace")
    return int(cr.value), int(nb.value)


def lpd_nystrom_factor_to_host(X, L, gamma: float, W, G_host=None, chunk_rows: int = 0, workspace=None,
                               r: int | None = None) -> torch.Tensor:
    """Step 1d streamed to host memory: G_host (pinned float32 CPU tensor, n x B) is filled chunk by chunk
    while the device computes the next chunk. Blocks until G_host is complete."""
    X = _dev_f32(X, "X", 2)
    L = _dev_f32(L, "L", 2)
    W = _dev_f32(W, "W", 2)
    n, d = X.shape
    B = L.shape[0]
    if L.shape[1] != d or W.shape[1] != B:
        raise ValueError("shape mismatch: X n x d, L B x d, W r x B")
    r = W.shape[0] if r is None else int(r)
    if r > W.shape[0]:
        raise ValueError("r exceeds the rows of W")
    if G_host is None:
        G_host = torch.empty((n, B), dtype=torch.float32, pin_memory=True)
    if G_host.is_cuda or G_host.dtype != torch.float32 or G_host.dim() != 2 or G_host.shape != (n, B) \
            or (G_host.numel() and G_host.stride(1) != 1):
        raise TypeError("G_host: expected a float32 CPU tensor n x B with unit column stride")
    chunk_rows, nbytes = lpd_nystrom_factor_to_host_workspace(n, d, B, chunk_rows)
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=X.device)
    if workspace.dtype != torch.uint8 or not workspace.is_cuda:
        raise TypeError("workspace: expected a uint8 device tensor")
    _check(lib().lpd_nystrom_factor_to_host(X.data_ptr(), n, d, _ld(X), L.data_ptr(), B, _ld(L), float(gamma),
                                            W.data_ptr(), r, _ld(W), G_host.data_ptr(), _ld(G_host), chunk_rows,
                                            workspace.data_ptr(), workspace.numel(), _stream(X.device)),
           "lpd_nystrom_factor_to_host")
    return G_host


def _csr_args(row_ptr, col_idx, values, d, validate=True):
    if not (row_ptr.is_cuda and row_ptr.dtype == torch.int64 and row_ptr.dim() == 1 and row_ptr.numel() >= 1):
        raise TypeError("row_ptr: expected a 1-D int64 device tensor with n + 1 entries")
    if not (col_idx.is_cuda and col_idx.dtype == torch.int32 and col_idx.dim() == 1):
        raise TypeError("col_idx: expected a 1-D int32 device tensor")
    if not (values.is_cuda and values.dtype == torch.float32 and values.shape == col_idx.shape):
        raise TypeError("values: expected a float32 device tensor shaped like col_idx")
    row_ptr, col_idx, values = row_ptr.contiguous(), col_idx.contiguous(), values.contiguous()
    n = row_ptr.numel() - 1
    # the row offsets are trusted by the kernels: check them here unless the caller vouches for them
    # (validate=False: no device-to-host synchronisation, the call only enqueues)
    if validate:
        if int(row_ptr[0]) != 0 or int(row_ptr[-1]) != col_idx.numel() or \
                (n and bool((row_ptr[1:] < row_ptr[:-1]).any())):
            raise ValueError("row_ptr: expected non-decreasing offsets from 0 to the number of entries")
        if col_idx.numel() and (int(col_idx.min()) < 0 or int(col_idx.max()) >= d):
            raise ValueError("col_idx: column index outside [0, d)")
    return row_ptr, col_idx, values, n


def lpd_nystrom_factor_csr_workspace(n: int, d: int, B: int, chunk_rows: int = 0, nnz: int = -1):
    """(chunk_rows, bytes) of the compressed-row entry points (the suggested chunk for chunk_rows <= 0); nnz
    selects the route, and with it the workspace, as in the calls themselves."""
    cr, nb = _i64(int(chunk_rows)), _sz(0)
    _check(lib().lpd_nystrom_factor_csr_workspace(n, d, B, int(nnz), ctypes.byref(cr), ctypes.byref(nb)),
           "lpd_nystrom_factor_csr_workspace")
    return int(cr.value), int(nb.value)


def lpd_nystrom_factor_csr(row_ptr, col_idx, values, d: int, L, gamma: float, W, G=None, chunk_rows: int = 0,
                           workspace=None, r: int | None = None, validate: bool = True) -> torch.Tensor:
    """Step 1d for X in compressed-row form (device tensors). Enqueued on torch's current stream.
    validate=True reads the row offsets and the column range back first (a blocking check); pass False in a
    hot loop or under graph capture once the structure is known to be sound."""
    row_ptr, col_idx, values, n = _csr_args(row_ptr, col_idx, values, d, validate)
    L = _dev_f32(L, "L", 2)
    W = _dev_f32(W, "W", 2)
    B = L.shape[0]
    if L.shape[1] != d or W.shape[1] != B:
        raise ValueError("shape mismatch: L B x d, W r x B")
    r = W.shape[0] if r is None else int(r)
    if r > W.shape[0]:
        raise ValueError("r exceeds the rows of W")
    if G is None:
        G = torch.empty((n, B), dtype=torch.float32, device=L.device)
    G = _dev_f32(G, "G", 2)
    if G.shape != (n, B):
        raise ValueError("G: expected n x B")
    chunk_rows, nbytes = lpd_nystrom_factor_csr_workspace(n, d, B, chunk_rows, col_idx.numel())
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=L.device)
    _check(lib().lpd_nystrom_factor_csr(row_ptr.data_ptr(), col_idx.data_ptr(), values.data_ptr(), n, d, col_idx.numel(), L.data_ptr(),
                                        B, _ld(L), float(gamma), W.data_ptr(), r, _ld(W), G.data_ptr(), _ld(G),
                                        chunk_rows, workspace.data_ptr(), workspace.numel(), _stream(L.device)),
           "lpd_nystrom_factor_csr")
    return G


def lpd_kernel_block_csr(row_ptr, col_idx, values, d: int, L, gamma: float, Z=None, chunk_rows: int = 0,
                         workspace=None, validate: bool = True) -> torch.Tensor:
    """Z = K(X, L) for X in compressed-row form (device tensors); validate as in lpd_nystrom_factor_csr."""
    row_ptr, col_idx, values, n = _csr_args(row_ptr, col_idx, values, d, validate)
    L = _dev_f32(L, "L", 2)
    B = L.shape[0]
    if L.shape[1] != d:
        raise ValueError("shape mismatch: L B x d")
    if Z is None:
        Z = torch.empty((n, B), dtype=torch.float32, device=L.device)
    Z = _dev_f32(Z, "Z", 2)
    if Z.shape != (n, B):
        raise ValueError("Z: expected n x B")
    chunk_rows, nbytes = lpd_nystrom_factor_csr_workspace(n, d, B, chunk_rows, col_idx.numel())
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=L.device)
    _check(lib().lpd_kernel_block_csr(row_ptr.data_ptr(), col_idx.data_ptr(), values.data_ptr(), n, d, col_idx.numel(), L.data_ptr(), B,
                                      _ld(L), float(gamma), Z.data_ptr(), _ld(Z), chunk_rows, workspace.data_ptr(),
                                      workspace.numel(), _stream(L.device)), "lpd_kernel_block_csr")
    return Z


def lpd_predict_csr(row_ptr, col_idx, values, d: int, L, gamma: float, V, F=None, chunk_rows: int = 0,
                    workspace=None, validate: bool = True) -> torch.Tensor:
    """Scores F[i, j] = V[j] . K(x_i, L) for new points in compressed-row form (n x c); validate as in
    lpd_nystrom_factor_csr."""
    row_ptr, col_idx, values, n = _csr_args(row_ptr, col_idx, values, d, validate)
    L = _dev_f32(L, "L", 2)
    V = _dev_f32(V, "V", 2)
    B, c = L.shape[0], V.shape[0]
    if L.shape[1] != d or V.shape[1] != B:
        raise ValueError("shape mismatch: L B x d, V c x B")
    if F is None:
        F = torch.empty((n, c), dtype=torch.float32, device=L.device)
    F = _dev_f32(F, "F", 2)
    if F.shape != (n, c):
        raise ValueError("F must be n x c")
    chunk_rows, nbytes = lpd_nystrom_factor_csr_workspace(n, d, B, chunk_rows, col_idx.numel())
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=L.device)
    _check(lib().lpd_predict_csr(row_ptr.data_ptr(), col_idx.data_ptr(), values.data_ptr(), n, d, col_idx.numel(), L.data_ptr(), B,
                                 _ld(L), float(gamma), V.data_ptr(), c, _ld(V), F.data_ptr(), _ld(F), chunk_rows,
                                 workspace.data_ptr(), workspace.numel(), _stream(L.device)), "lpd_predict_csr")
    return F


def lpd_kernel_block(X, L, gamma: float, Z, workspace) -> torch.Tensor:
    """Z = K(X, L) in full (steps 1a / 1d)."""
    X = _dev_f32(X, "X", 2)
    L = _dev_f32(L, "L", 2)
    Z = _dev_f32(Z, "Z", 2)
    n, d = X.shape
    B = L.shape[0]
    if L.shape[1] != d or Z.shape != (n, B):
        raise ValueError("shape mismatch: X n x d, L B x d, Z n x B")
    st = lib().lpd_kernel_block(X.data_ptr(), n, d, _ld(X), L.data_ptr(), B, _ld(L), float(gamma), Z.data_ptr(),
                                _ld(Z), workspace.data_ptr(), workspace.numel(), _stream(X.device))
    _check(st, "lpd_kernel_block")
    return Z


def lpd_margins(G, w, m=None, r: int | None = None) -> torch.Tensor:
    """Step 2a for all rows: m = G[:, :r] w."""
    G = _dev_f32(G, "G", 2)
    w = _dev_f32(w, "w", 1)
    n = G.shape[0]
    r = w.shape[0] if r is None else int(r)
    if r > w.shape[0] or r > G.shape[1]:
        raise ValueError("r exceeds w or the columns of G")
    if m is None:
        m = torch.empty(n, dtype=torch.float32, device=G.device)
    m = _dev_f32(m, "m", 1)
    if m.shape[0] != n:
        raise ValueError("m must have one entry per row of G")
    _check(lib().lpd_margins(G.data_ptr(), n, r, _ld(G), w.data_ptr(), m.data_ptr(), _stream(G.device)),
           "lpd_margins")
    return m


def lpd_margins_rows(G, rows, w, m=None, r: int | None = None) -> torch.Tensor:
    """Step 2a over a list of rows (int64 device tensor). Only enqueues: the kernel checks the indices itself
    (an index outside [0, n) gives NaN), so the call can be recorded into a HIP graph."""
    G = _dev_f32(G, "G", 2)
    w = _dev_f32(w, "w", 1)
    if rows.dtype != torch.int64 or rows.dim() != 1 or not rows.is_cuda or (rows.numel() > 1 and rows.stride(0) != 1):
        raise TypeError("rows: expected a contiguous 1-D int64 device tensor")
    n = G.shape[0]
    k = rows.shape[0]
    r = w.shape[0] if r is None else int(r)
    if r > w.shape[0] or r > G.shape[1]:
        raise ValueError("r exceeds w or the columns of G")
    if m is None:
        m = torch.empty(k, dtype=torch.float32, device=G.device)
    m = _dev_f32(m, "m", 1)
    if m.shape[0] != k:
        raise ValueError("m must have one entry per listed row")
    st = lib().lpd_margins_rows(G.data_ptr(), n, r, _ld(G), rows.data_ptr(), k, w.data_ptr(), m.data_ptr(),
                                _stream(G.device))
    _check(st, "lpd_margins_rows")
    return m


def lpd_row_sqnorms(G, gsq=None, r: int | None = None) -> torch.Tensor:
    """gsq[i] = ||G[i, :r]||^2, the diagonal of the dual problem."""
    G = _dev_f32(G, "G", 2)
    n = G.shape[0]
    r = G.shape[1] if r is None else int(r)
    if r > G.shape[1]:
        raise ValueError("r exceeds the columns of G")
    if gsq is None:
        gsq = torch.empty(n, dtype=torch.float32, device=G.device)
    gsq = _dev_f32(gsq, "gsq", 1)
    if gsq.shape[0] != n:
        raise ValueError("gsq must have one entry per row of G")
    _check(lib().lpd_row_sqnorms(G.data_ptr(), n, r, _ld(G), gsq.data_ptr(), _stream(G.device)), "lpd_row_sqnorms")
    return gsq


def lpd_cd_solve_workspace(n_problems: int, total_rows: int) -> int:
    b = _sz(0)
    _check(lib().lpd_cd_solve_workspace(n_problems, total_rows, ctypes.byref(b)), "lpd_cd_solve_workspace")
    return int(b.value)


CD_STATUS_DTYPE = [("steps", "<i8"), ("epochs", "<i4"), ("converged", "<i4"), ("active", "<i4"),
                   ("max_violation", "<f4"), ("dual", "<f4"), ("reserved", "<i4")]


def lpd_cd_solve(G, gsq, prob_off, rows, y, C, alpha, w=None, eps: float = 1e-3, max_epochs: int = 1000,
                 shrink_k: int = 5, eta: float = 0.05, r: int | None = None, workspace=None, validate: bool = True,
                 status=None):
    """Batch of dual coordinate-ascent problems on the rows of G (see include/lpd.h).

    prob_off: int64 device tensor of n_problems + 1 offsets; rows / y / alpha: concatenated per-problem lists
    (alpha is updated in place); C: float32 device tensor, one per problem.
    validate=True reads prob_off and the range of rows back and raises on inconsistent lists (blocking);
    validate=False leaves them to the kernel, which clamps them so that no access leaves the arrays.
    status: optional uint8 device tensor (n_problems x 32) for the result records; when given, the call only
    enqueues and returns it as a device tensor (view it with CD_STATUS_DTYPE after a synchronise).
    Returns (alpha, w [n_problems x r], status: numpy record array read back after a synchronise, or the
    device tensor passed in)."""
    G = _dev_f32(G, "G", 2)
    gsq = _dev_f32(gsq, "gsq", 1)
    y = _dev_f32(y, "y", 1)
    C = _dev_f32(C, "C", 1)
    alpha = _dev_f32(alpha, "alpha", 1)
    for name, t in (("prob_off", prob_off), ("rows", rows)):
        if t.dtype != torch.int64 or t.dim() != 1 or not t.is_cuda or (t.numel() > 1 and t.stride(0) != 1):
            raise TypeError(f"{name}: expected a contiguous 1-D int64 device tensor")
    n = G.shape[0]
    r = G.shape[1] if r is None else int(r)
    P = C.shape[0]
    total = rows.shape[0]
    if r > G.shape[1] or prob_off.shape[0] != P + 1 or y.shape[0] != total or alpha.shape[0] != total or \
            gsq.shape[0] != n:
        raise ValueError("shape mismatch between G, gsq, prob_off, rows, y, C, alpha")
    if validate:
        if P > 0:
            po = prob_off.cpu()
            if int(po[0]) != 0 or int(po[-1]) != total or bool((po[1:] < po[:-1]).any()):
                raise ValueError("prob_off must start at 0, be non-decreasing and end at len(rows)")
        if total > 0 and (int(rows.min()) < 0 or int(rows.max()) >= n):
            raise IndexError("rows: index outside [0, n)")
    if w is None:
        w = torch.empty((P, max(r, 1)), dtype=torch.float32, device=G.device)
    w = _dev_f32(w, "w", 2)
    if w.shape[0] != P or w.shape[1] < r:
        raise ValueError("w must be n_problems x r")
    need = lpd_cd_solve_workspace(P, total)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=G.device)
    enqueue_only = status is not None
    if status is None:
        status = torch.zeros((max(P, 1), 32), dtype=torch.uint8, device=G.device)
    elif status.dtype != torch.uint8 or not status.is_cuda or status.numel() < 32 * P or not status.is_contiguous():
        raise TypeError("status: expected a contiguous uint8 device tensor of n_problems x 32 bytes")
    st = lib().lpd_cd_solve(G.data_ptr(), n, r, _ld(G), gsq.data_ptr(), P, prob_off.data_ptr(), total,
                            rows.data_ptr(), y.data_ptr(), C.data_ptr(), alpha.data_ptr(), w.data_ptr(), _ld(w),
                            status.data_ptr(), float(eps), int(max_epochs), int(shrink_k), float(eta),
                            workspace.data_ptr(), workspace.numel(), _stream(G.device))
    _check(st, "lpd_cd_solve")
    if enqueue_only:
        return alpha, w, status
    import numpy as np
    rec = np.frombuffer(status.cpu().numpy().tobytes(), dtype=np.dtype(CD_STATUS_DTYPE))[:P]
    return alpha, w, rec


def lpd_fold_weights(W, Ws, V=None, r: int | None = None) -> torch.Tensor:
    """V = Ws[:, :r] W[:r]: classifier weights folded through the whitening map (c x B)."""
    W = _dev_f32(W, "W", 2)
    Ws = _dev_f32(Ws, "Ws", 2)
    r = W.shape[0] if r is None else int(r)
    B = W.shape[1]
    c = Ws.shape[0]
    if r > W.shape[0] or r > Ws.shape[1]:
        raise ValueError("r exceeds W or Ws")
    if V is None:
        V = torch.empty((c, B), dtype=torch.float32, device=W.device)
    V = _dev_f32(V, "V", 2)
    if V.shape != (c, B):
        raise ValueError("V must be c x B")
    _check(lib().lpd_fold_weights(W.data_ptr(), r, B, _ld(W), Ws.data_ptr(), c, _ld(Ws), V.data_ptr(), _ld(V),
                                  _stream(W.device)), "lpd_fold_weights")
    return V


def lpd_predict(X, L, gamma: float, V, F=None, workspace=None) -> torch.Tensor:
    """Scores F[i, j] = V[j] . K(x_i, L) of c folded classifiers (n x c)."""
    X = _dev_f32(X, "X", 2)
    L = _dev_f32(L, "L", 2)
    V = _dev_f32(V, "V", 2)
    n, d = X.shape
    B = L.shape[0]
    c = V.shape[0]
    if L.shape[1] != d or V.shape[1] != B:
        raise ValueError("shape mismatch: X n x d, L B x d, V c x B")
    if F is None:
        F = torch.empty((n, c), dtype=torch.float32, device=X.device)
    F = _dev_f32(F, "F", 2)
    if F.shape != (n, c):
        raise ValueError("F must be n x c")
    if workspace is None:
        workspace = alloc_workspace(n, d, B, X.device)
    st = lib().lpd_predict(X.data_ptr(), n, d, _ld(X), L.data_ptr(), B, _ld(L), float(gamma), V.data_ptr(), c, _ld(V),
                           F.data_ptr(), _ld(F), workspace.data_ptr(), workspace.numel(), _stream(X.device))
    _check(st, "lpd_predict")
    return F


def lpd_predict_noalloc(X, L, gamma: float, V, F) -> torch.Tensor:
    """lpd_predict without a workspace and without any allocation (F must be passed in): the scratch is a fixed
    array inside the library, shared by all calls on the GPU; see include/lpd.h for the size limit."""
    X = _dev_f32(X, "X", 2)
    L = _dev_f32(L, "L", 2)
    V = _dev_f32(V, "V", 2)
    F = _dev_f32(F, "F", 2)
    n, d = X.shape
    B = L.shape[0]
    c = V.shape[0]
    if L.shape[1] != d or V.shape[1] != B or F.shape != (n, c):
        raise ValueError("shape mismatch: X n x d, L B x d, V c x B, F n x c")
    st = lib().lpd_predict_noalloc(X.data_ptr(), n, d, _ld(X), L.data_ptr(), B, _ld(L), float(gamma), V.data_ptr(), c,
                                   _ld(V), F.data_ptr(), _ld(F), _stream(X.device))
    _check(st, "lpd_predict_noalloc")
    return F


def lpd_margins_multi(G, Ws, M=None, r: int | None = None) -> torch.Tensor:
    """Step 2a for k weight vectors at once: M = G[:, :r] Ws[:, :r]^T (n x k)."""
    G = _dev_f32(G, "G", 2)
    Ws = _dev_f32(Ws, "Ws", 2)
    n = G.shape[0]
    k = Ws.shape[0]
    r = Ws.shape[1] if r is None else int(r)
    if r > Ws.shape[1] or r > G.shape[1]:
        raise ValueError("r exceeds Ws or the columns of G")
    if M is None:
        M = torch.empty((n, k), dtype=torch.float32, device=G.device)
    M = _dev_f32(M, "M", 2)
    if M.shape != (n, k):
        raise ValueError("M must be n x k")
    _check(lib().lpd_margins_multi(G.data_ptr(), n, r, _ld(G), Ws.data_ptr(), k, _ld(Ws), M.data_ptr(), _ld(M),
                                   _stream(G.device)), "lpd_margins_multi")
    return M
