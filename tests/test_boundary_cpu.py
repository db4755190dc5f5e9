"""CPU-side checks of the C-ABI library: exported symbols, argument validation, host whitening.

No kernel is launched here; every device entry point is only driven down its error paths, which
return before any HIP call.
"""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2207_01016_amd import lpd
    return lpd.lib()


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "lpd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(lpd_[a-z_]+)\s*\(", header))
    assert {"lpd_nystrom_factor", "lpd_margins", "lpd_whiten_host", "lpd_kernel_block"} <= declared
    from paper_2207_01016_amd import lpd
    assert declared == set(lpd.SIGNATURES), declared ^ set(lpd.SIGNATURES)
    for name in declared:
        assert hasattr(L, name), name


def test_header_is_valid_c_and_links_from_c(tmp_path):
    """include/lpd.h is a plain C header: a C99 program that includes it compiles without warnings, links against
    the library and runs (version call only: no device is touched)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    from paper_2207_01016_amd import lpd
    lpd.lib()
    pkg = os.path.join(ROOT, "paper_2207_01016_amd")
    src = tmp_path / "abi.c"
    src.write_text('#include <stdio.h>\n#include "lpd.h"\n'
                   'int main(void) { size_t b = 0, m = 0;\n'
                   '  if (lpd_nystrom_factor_workspace(1000, 16, 128, &b, &m) != LPD_OK || b < m) return 2;\n'
                   '  printf("%d %s\\n", lpd_version(), lpd_strerror(LPD_ERR_WORKSPACE)); return 0; }\n')
    exe = tmp_path / "abi"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", pkg, "-llpd", f"-Wl,-rpath,{pkg}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(maxsplit=1)
    assert int(out[0]) >= 100 and "workspace" in out[1]


def test_version_and_strerror(L):
    assert L.lpd_version() >= 100
    for st in range(-7, 1):
        assert len(L.lpd_strerror(st)) > 0


def test_workspace_query(L):
    rec, mn = ctypes.c_size_t(0), ctypes.c_size_t(0)
    assert L.lpd_nystrom_factor_workspace(1000, 16, 128, ctypes.byref(rec), ctypes.byref(mn)) == 0
    assert rec.value >= mn.value > 4 * (1000 + 128)
    assert rec.value % 256 == 0
    assert L.lpd_nystrom_factor_workspace(-1, 16, 128, ctypes.byref(rec), None) == -2
    assert L.lpd_nystrom_factor_workspace(10, 16, 128, None, None) == -1
    # the recommended panel never exceeds about 32 Mi kernel values (half the Infinity Cache) plus the norms
    assert L.lpd_nystrom_factor_workspace(2_000_000, 256, 16384, ctypes.byref(rec), ctypes.byref(mn)) == 0
    assert rec.value < 4 * (2_000_000 + 16384 + 256 + (32 << 20) + 16384 * 300)


def test_factor_argument_errors(L):
    buf = (ctypes.c_float * 4096)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    f = L.lpd_nystrom_factor
    #        X  n   d  ldx L  B  ldl gamma W  r  ldw G  ldg ws  bytes stream
    assert f(p, 0, 4, 4, p, 8, 4, 0.5, p, 8, 8, p, 8, None, 0, None) == 0          # n = 0: nothing to do
    assert f(p, 4, 4, 4, p, 0, 4, 0.5, p, 0, 1, p, 1, None, 0, None) == 0          # B = 0
    assert f(p, -1, 4, 4, p, 8, 4, 0.5, p, 8, 8, p, 8, None, 0, None) == -2
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 9, 8, p, 8, None, 0, None) == -2         # r > B
    assert f(None, 4, 4, 4, p, 8, 4, 0.5, p, 8, 8, p, 8, None, 0, None) == -1
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, None, 8, 8, p, 8, None, 0, None) == -1
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 8, 8, None, 8, None, 0, None) == -1
    assert f(p, 4, 4, 3, p, 8, 4, 0.5, p, 8, 8, p, 8, None, 0, None) == -3         # ldx < d
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 8, 7, p, 8, None, 0, None) == -3         # ldw < B
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 8, 8, p, 7, None, 0, None) == -3         # ldg < B
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 8, 8, p, 8, None, 0, None) == -4         # no workspace
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 8, 8, p, 8, p, 16, None) == -4           # too small


def test_streaming_factor_query_and_argument_errors(L):
    cr, nb = ctypes.c_int64(0), ctypes.c_size_t(0)
    q = L.lpd_nystrom_factor_to_host_workspace
    assert q(1_000_000, 784, 4096, ctypes.byref(cr), ctypes.byref(nb)) == 0
    assert 0 < cr.value <= 1_000_000 and nb.value % 256 == 0
    assert nb.value >= 2 * cr.value * 4096 * 4                       # two chunk buffers plus scratch
    cr2, nb2 = ctypes.c_int64(1000), ctypes.c_size_t(0)
    assert q(1_000_000, 784, 4096, ctypes.byref(cr2), ctypes.byref(nb2)) == 0
    assert cr2.value == 1000 and nb2.value < nb.value                # a given chunk size is kept
    cr3 = ctypes.c_int64(0)
    assert q(10, 4, 8, ctypes.byref(cr3), ctypes.byref(nb2)) == 0 and cr3.value == 10   # never above n
    assert q(10, 4, 8, None, ctypes.byref(nb2)) == -1
    assert q(-1, 4, 8, ctypes.byref(cr3), ctypes.byref(nb2)) == -2

    buf = (ctypes.c_float * 4096)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    f = L.lpd_nystrom_factor_to_host
    #        X  n  d  ldx L  B  ldl gamma W  r  ldw G  ldg chunk ws bytes stream
    assert f(p, 0, 4, 4, p, 8, 4, 0.5, p, 8, 8, p, 8, 4, None, 0, None) == 0       # n = 0: nothing to do
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 8, 8, p, 8, 0, None, 0, None) == -2      # chunk_rows must be > 0
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 9, 8, p, 8, 4, None, 0, None) == -2      # r > B
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 8, 8, None, 8, 4, None, 0, None) == -1
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 8, 8, p, 7, 4, None, 0, None) == -3      # ldg < B
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 8, 8, p, 8, 4, None, 0, None) == -4      # no workspace
    assert f(p, 4, 4, 4, p, 8, 4, 0.5, p, 8, 8, p, 8, 4, p, 256, None) == -4       # too small


def test_margins_and_kernel_block_argument_errors(L):
    buf = (ctypes.c_float * 1024)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    assert L.lpd_margins(p, 0, 8, 8, p, p, None) == 0
    assert L.lpd_margins(p, 4, 8, 7, p, p, None) == -3
    assert L.lpd_margins(None, 4, 8, 8, p, p, None) == -1
    assert L.lpd_margins(p, 4, 8, 8, p, None, None) == -1
    assert L.lpd_margins(p, 4, -8, 8, p, p, None) == -2
    assert L.lpd_margins_rows(p, 4, 8, 8, p, 0, p, p, None) == 0
    assert L.lpd_margins_rows(p, 4, 8, 8, None, 2, p, p, None) == -1
    assert L.lpd_kernel_block(p, 4, 4, 4, p, 8, 4, 0.5, p, 7, p, 4096, None) == -3
    assert L.lpd_kernel_block(p, 4, 4, 4, p, 8, 4, 0.5, p, 8, None, 0, None) == -4
    assert L.lpd_kernel_block(p, 0, 4, 4, p, 8, 4, 0.5, p, 8, None, 0, None) == 0
    assert L.lpd_set_option(1, 3) == 0 and L.lpd_set_option(1, 4) == 0 and L.lpd_set_option(1, 0) == 0
    assert L.lpd_set_option(1, 5) == -2 and L.lpd_set_option(1, 9) == -2 and L.lpd_set_option(77, 0) == -2


def test_solver_and_predict_argument_errors(L):
    buf = (ctypes.c_float * 4096)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    nb = ctypes.c_size_t(0)
    assert L.lpd_cd_solve_workspace(3, 100, ctypes.byref(nb)) == 0 and nb.value >= 3 * 103 * 4 + 100
    assert L.lpd_cd_solve_workspace(-1, 100, ctypes.byref(nb)) == -2
    cd = L.lpd_cd_solve
    #       G  n   r  ldg gsq P  off tot rows y  C  alpha w  ldw st eps  ep  k  eta  ws    bytes stream
    assert cd(p, 10, 8, 8, p, 0, p, 0, p, p, p, p, p, 8, p, 1e-3, 10, 5, 0.05, None, 0, None) == 0     # no problems
    assert cd(p, 10, 8, 8, p, 1, p, 10, p, p, p, p, p, 8, p, 1e-3, 10, 5, 0.05, None, 0, None) == -4   # no workspace
    assert cd(p, 10, 8, 7, p, 1, p, 10, p, p, p, p, p, 8, p, 1e-3, 10, 5, 0.05, p, 4096, None) == -3   # ldg < r
    assert cd(p, 10, 8, 8, p, 1, p, 10, p, p, p, p, p, 7, p, 1e-3, 10, 5, 0.05, p, 4096, None) == -3   # ldw < r
    assert cd(p, 10, 8, 8, p, 1, None, 10, p, p, p, p, p, 8, p, 1e-3, 10, 5, 0.05, p, 4096, None) == -1
    assert cd(p, 10, 8, 8, p, 1, p, 10, p, p, p, p, p, 8, p, 1e-3, 10, 300, 0.05, p, 4096, None) == -2  # k > 255
    assert cd(p, 10, 8, 8, p, 1, p, 10, p, p, p, p, p, 8, p, 1e-3, 10, 5, 1.0, p, 4096, None) == -2     # eta >= 1
    assert cd(p, 10, 20000, 20000, p, 1, p, 10, p, p, p, p, p, 20000, p, 1e-3, 10, 5, 0.05, p, 4096, None) == -2
    # a factor without columns or without rows cannot be stepped over: refused on the host, no launch
    assert cd(None, 10, 0, 0, p, 1, p, 10, p, p, p, p, None, 0, p, 1e-3, 10, 5, 0.05, p, 4096, None) == -2   # r = 0
    assert cd(p, 10, 0, 8, p, 1, p, 10, p, p, p, p, p, 8, p, 1e-3, 10, 5, 0.05, p, 4096, None) == -2        # r = 0
    assert cd(p, 0, 8, 8, p, 1, p, 10, p, p, p, p, p, 8, p, 1e-3, 10, 5, 0.05, p, 4096, None) == -2         # n = 0
    assert cd(None, 10, 8, 8, p, 1, p, 10, p, p, p, p, p, 8, p, 1e-3, 10, 5, 0.05, p, 4096, None) == -1     # G NULL
    assert L.lpd_margins_rows(p, 0, 8, 8, p, 5, p, p, None) == -2                    # rows listed, G has none
    assert L.lpd_row_sqnorms(p, 0, 8, 8, p, None) == 0
    assert L.lpd_row_sqnorms(p, 4, 8, 7, p, None) == -3
    assert L.lpd_row_sqnorms(p, 4, 8, 8, None, None) == -1
    assert L.lpd_fold_weights(p, 4, 8, 8, p, 0, 4, p, 8, None) == 0
    assert L.lpd_fold_weights(p, 4, 8, 7, p, 2, 4, p, 8, None) == -3
    assert L.lpd_fold_weights(p, 4, 8, 8, p, 2, 4, None, 8, None) == -1
    assert L.lpd_margins_multi(p, 4, 8, 8, p, 0, 8, p, 1, None) == 0
    assert L.lpd_margins_multi(p, 4, 8, 8, p, 3, 8, p, 2, None) == -3                # ldm < k
    assert L.lpd_margins_multi(p, 4, 8, 8, None, 3, 8, p, 3, None) == -1
    pr = L.lpd_predict
    assert pr(p, 4, 4, 4, p, 8, 4, 0.5, p, 0, 8, p, 1, None, 0, None) == 0           # no classifiers
    assert pr(p, 4, 4, 4, p, 8, 4, 0.5, p, 9, 8, p, 9, None, 0, None) == -2          # c > B
    assert pr(p, 4, 4, 4, p, 8, 4, 0.5, p, 2, 8, p, 1, p, 4096, None) == -3          # ldf < c
    assert pr(p, 4, 4, 4, p, 8, 4, 0.5, p, 2, 8, p, 2, None, 0, None) == -4


def test_binding_rejects_host_tensors():
    from paper_2207_01016_amd import lpd
    with pytest.raises(ValueError):
        lpd.lpd_margins(torch.zeros(4, 8), torch.zeros(8))
    with pytest.raises(TypeError):
        lpd.lpd_margins(torch.zeros(4, 8, dtype=torch.float64), torch.zeros(8))


# ---------------------------------------------------------------- host whitening (steps 1a-1c)

@pytest.mark.parametrize("name,B", [("tiny", 128), ("small", 200), ("digit", 97), ("cnn", 64), ("highrank", 333)])
def test_whiten_host_against_oracle(oracle, name, B):
    """Rotation-invariant comparison: eigenvalues, rank, W K W^T = I, and the sign convention."""
    from paper_2207_01016_amd import lpd, workloads
    wl = workloads.WORKLOADS[name].with_shape(n=max(2 * B, 1000), B=B)
    X = workloads.make_X(wl)
    Lm = X[workloads.landmark_indices(wl)].contiguous()
    W, eig, rank = lpd.lpd_whiten_host(Lm, wl.gamma)
    Wo, eo, ro, K = oracle.whiten(Lm.numpy(), wl.gamma, method="lapack")
    assert rank == ro == B
    assert np.max(np.abs(eig.numpy() - eo)) <= 1e-10 * eo[0]
    Wd = W.double().numpy()
    assert np.linalg.norm(Wd @ K @ Wd.T - np.eye(B)) <= 2e-6 * B
    # eigenvalues here are simple, so rows agree with the oracle's up to fp32 rounding of W
    gap = np.min(np.abs(np.diff(eo)))
    if gap > 1e-6:
        assert np.max(np.abs(Wd - Wo)) <= 1e-5 * np.max(np.abs(Wo)) / min(1.0, gap * 1e3)
    for j in range(B):
        assert Wd[j, np.argmax(np.abs(Wd[j]))] > 0.0


def test_whiten_host_degenerate_cases(oracle):
    from paper_2207_01016_amd import lpd
    g = torch.Generator().manual_seed(5)
    X = torch.randn((40, 6), generator=g)
    # gamma = 0: rank one, W[0] = 1/B
    W, eig, rank = lpd.lpd_whiten_host(X[:9].contiguous(), 0.0)
    assert rank == 1
    assert abs(eig[0].item() - 9.0) < 1e-12
    assert torch.allclose(W[0], torch.full((9,), 1.0 / 9.0), atol=1e-7) and torch.all(W[1:] == 0)
    # duplicated landmark: one component dropped, remaining ones still whiten K
    Ld = torch.cat([X[:12], X[3:4]]).contiguous()
    W, eig, rank = lpd.lpd_whiten_host(Ld, 0.15)
    assert rank == 12 and abs(eig[-1].item()) < 1e-12
    K = oracle.kernel_block(Ld.numpy(), Ld.numpy(), 0.15)
    Wd = W.double().numpy()[:12]
    assert np.linalg.norm(Wd @ K @ Wd.T - np.eye(12)) < 1e-5
    assert torch.all(W[12:] == 0)
    # B = 1 and B = 2
    W, eig, rank = lpd.lpd_whiten_host(X[:1].contiguous(), 0.3)
    assert rank == 1 and W.item() == 1.0
    W, eig, rank = lpd.lpd_whiten_host(torch.tensor([[0.0], [1.0]]), float(np.log(2.0)))
    assert rank == 2
    assert torch.allclose(eig, torch.tensor([1.5, 0.5], dtype=torch.float64), atol=1e-14)
    assert torch.allclose(W, torch.tensor([[3 ** -0.5, 3 ** -0.5], [1.0, -1.0]]), atol=1e-7)
    # B = 0
    W, eig, rank = lpd.lpd_whiten_host(torch.zeros((0, 3)), 0.3)
    assert rank == 0 and W.shape == (0, 0)


def test_whiten_host_errors(L):
    r = ctypes.c_int64(0)
    buf = (ctypes.c_float * 64)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    assert L.lpd_whiten_host(p, 4, 2, 1, 0.5, 1e-10, p, 4, None, ctypes.byref(r)) == -3
    assert L.lpd_whiten_host(p, 4, 2, 2, 0.5, 1e-10, None, 4, None, ctypes.byref(r)) == -1
    assert L.lpd_whiten_host(p, 4, 2, 2, 0.5, 1e-10, p, 4, None, None) == -1
    assert L.lpd_whiten_host(p, -4, 2, 2, 0.5, 1e-10, p, 4, None, ctypes.byref(r)) == -2


def test_whiten_device_query_and_argument_errors(L):
    nb = ctypes.c_size_t(0)
    assert L.lpd_whiten_workspace(4096, ctypes.byref(nb)) == 0
    assert nb.value >= 2 * 4096 * 4096 * 8 and nb.value % 256 == 0
    assert L.lpd_whiten_workspace(4096, None) == -1
    assert L.lpd_whiten_workspace(-1, ctypes.byref(nb)) == -2
    assert L.lpd_whiten_workspace(50_000, ctypes.byref(nb)) == -2          # above the supported B
    r = ctypes.c_int64(7)
    buf = (ctypes.c_float * 64)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    f = L.lpd_whiten
    #        L  B  d  ldl gamma clip  W  ldw eig   rank             ws    bytes stream phases
    assert f(p, 0, 2, 2, 0.5, 1e-10, p, 1, None, ctypes.byref(r), None, 0, None, None) == 0 and r.value == 0
    assert f(p, 4, 2, 1, 0.5, 1e-10, p, 4, None, ctypes.byref(r), None, 0, None, None) == -3
    assert f(p, 4, 2, 2, 0.5, 1e-10, p, 3, None, ctypes.byref(r), None, 0, None, None) == -3
    assert f(p, 4, 2, 2, 0.5, 1e-10, None, 4, None, ctypes.byref(r), None, 0, None, None) == -1
    assert f(p, 4, 2, 2, 0.5, 1e-10, p, 4, None, None, None, 0, None, None) == -1
    assert f(p, -4, 2, 2, 0.5, 1e-10, p, 4, None, ctypes.byref(r), None, 0, None, None) == -2
    assert f(p, 4, 2, 2, 0.5, 1e-10, p, 4, None, ctypes.byref(r), None, 0, None, None) == -4   # no workspace
    assert f(p, 4, 2, 2, 0.5, 1e-10, p, 4, None, ctypes.byref(r), p, 256, None, None) == -4    # too small


def test_csr_query_and_argument_errors(L):
    cr, nb = ctypes.c_int64(0), ctypes.c_size_t(0)
    q = L.lpd_nystrom_factor_csr_workspace
    assert q(1_000_000, 784, 4096, -1, ctypes.byref(cr), ctypes.byref(nb)) == 0
    assert 0 < cr.value <= 1_000_000 and nb.value >= cr.value * 784 * 4 and nb.value % 256 == 0
    # a density under 8 % selects the gather route: transposed landmarks instead of a dense panel of X
    cr2, nb2 = ctypes.c_int64(cr.value), ctypes.c_size_t(0)
    assert q(1_000_000, 784, 4096, 784 * 10_000, ctypes.byref(cr2), ctypes.byref(nb2)) == 0
    assert nb2.value >= 784 * 4096 * 4 + cr2.value * 4096 * 4 and nb2.value != nb.value
    cr3, nb3 = ctypes.c_int64(cr.value), ctypes.c_size_t(0)
    assert q(1_000_000, 784, 4096, 784 * 200_000, ctypes.byref(cr3), ctypes.byref(nb3)) == 0 and nb3.value == nb.value
    assert q(10, 4, 8, -1, None, ctypes.byref(nb)) == -1
    assert q(10, -4, 8, -1, ctypes.byref(cr), ctypes.byref(nb)) == -2
    buf = (ctypes.c_float * 4096)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    f = L.lpd_nystrom_factor_csr
    #        rp ci va n  d  nnz L  B  ldl gamma W  r  ldw G  ldg chunk ws  bytes stream
    assert f(p, p, p, 0, 4, -1, p, 8, 4, 0.5, p, 8, 8, p, 8, 4, None, 0, None) == 0          # no rows
    assert f(None, p, p, 4, 4, -1, p, 8, 4, 0.5, p, 8, 8, p, 8, 4, None, 0, None) == -1
    assert f(p, p, p, 4, 4, -1, p, 8, 4, 0.5, p, 9, 8, p, 8, 4, None, 0, None) == -2         # r > B
    assert f(p, p, p, 4, 4, -1, p, 8, 4, 0.5, p, 8, 8, p, 8, 0, None, 0, None) == -2         # chunk_rows must be > 0
    assert f(p, p, p, 4, 4, -1, p, 8, 3, 0.5, p, 8, 8, p, 8, 4, None, 0, None) == -3         # ldl < d
    assert f(p, p, p, 4, 4, -1, p, 8, 4, 0.5, p, 8, 8, p, 7, 4, None, 0, None) == -3         # ldg < B
    assert f(p, p, p, 4, 4, -1, p, 8, 4, 0.5, p, 8, 8, p, 8, 4, None, 0, None) == -4         # no workspace
    assert f(p, p, p, 4, 4, -1, p, 8, 4, 0.5, p, 8, 8, p, 8, 4, p, 256, None) == -4          # too small
    assert f(p, p, p, 4, 4, 0, p, 8, 4, 0.5, p, 8, 8, p, 8, 4, p, 256, None) == -4           # gather route: too small
    k = L.lpd_kernel_block_csr
    #        rp ci va n  d  nnz L  B  ldl gamma Z  ldz chunk ws  bytes stream
    assert k(p, p, p, 4, 4, -1, p, 8, 4, 0.5, None, 8, 4, None, 0, None) == -1
    assert k(p, p, p, 4, 4, -1, p, 8, 4, 0.5, p, 7, 4, None, 0, None) == -3
    assert k(p, p, p, 4, 4, -1, p, 8, 4, 0.5, p, 8, 4, None, 0, None) == -4
    g = L.lpd_predict_csr
    #        rp ci va n  d  nnz L  B  ldl gamma V  c  ldv F  ldf chunk ws  bytes stream
    assert g(p, p, p, 4, 4, -1, p, 8, 4, 0.5, p, 9, 8, p, 9, 4, None, 0, None) == -2         # c > B
    assert g(p, p, p, 4, 4, -1, p, 8, 4, 0.5, p, 3, 8, p, 2, 4, None, 0, None) == -3         # ldf < c
    assert L.lpd_set_option(3, 2) == 0 and L.lpd_set_option(3, 3) == -2 and L.lpd_set_option(3, 0) == 0


def test_predict_noalloc_error_paths(L):
    """The allocation-free entry point checks shapes and its fixed 32 MiB limit on the host, before any HIP call."""
    p = ctypes.c_void_p(256)
    f = L.lpd_predict_noalloc
    assert f(p, 1000, 8, 8, p, 40000, 8, 0.5, p, 2, 40000, p, 2, None) == -7        # beyond the scratch
    assert f(p, 4_500_000, 8, 8, p, 16384, 8, 0.5, p, 2, 16384, p, 2, None) == -7   # the norms alone: 18 MB + panel 17 MB
    assert b"32 MiB" in L.lpd_strerror(-7)
    assert f(p, 10, 8, 8, p, 16, 8, 0.5, p, 17, 16, p, 17, None) == -2              # more classifiers than landmarks
    assert f(p, 10, 8, 7, p, 16, 8, 0.5, p, 2, 16, p, 2, None) == -3                # ldx < d
    assert f(p, 10, 8, 8, p, 16, 8, 0.5, p, 2, 16, p, 1, None) == -3                # ldf < c
    assert f(None, 10, 8, 8, p, 16, 8, 0.5, p, 2, 16, p, 2, None) == -1
    assert f(p, 0, 8, 8, p, 16, 8, 0.5, p, 2, 16, p, 2, None) == 0                  # nothing to do
    assert f(p, 10, 8, 8, p, 16, 8, 0.5, p, 0, 16, p, 1, None) == 0
