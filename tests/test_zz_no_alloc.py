"""The allocation-free prediction entry point against lpd_predict, through the C ABI.

lpd_predict_noalloc keeps its scratch (row norms, origin, kernel-block panel) in a fixed device array inside the
library instead of a caller workspace.  Two calls in a row, the second with a smaller input, must each give the
scores lpd_predict gives (the stale contents the first call leaves behind must not leak into the second), and
both must match the double-precision oracle to the factor's 1e-4.
"""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

TOL = 1e-4


def relfro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


@pytest.fixture(scope="module")
def lpd():
    from paper_2207_01016_amd import lpd as mod
    mod.lib()
    return mod


def _scores_both_ways(lpd, dev, X, L, gamma, V):
    """(lpd_predict, lpd_predict_noalloc) through raw ctypes calls on the library's C ABI."""
    lib = lpd.lib()
    n, d = X.shape
    B, c = L.shape[0], V.shape[0]
    stream = ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    ws = lpd.alloc_workspace(n, d, B, dev)
    F_ref = torch.full((n, c), float("nan"), dtype=torch.float32, device=dev)
    F_new = torch.full((n, c), float("nan"), dtype=torch.float32, device=dev)
    st = lib.lpd_predict(X.data_ptr(), n, d, d, L.data_ptr(), B, d, gamma, V.data_ptr(), c, B, F_ref.data_ptr(), c,
                         ws.data_ptr(), ws.numel(), stream)
    assert st == 0
    print(f"lpd_predict_noalloc n={n} d={d} B={B} c={c}", flush=True)
    st = lib.lpd_predict_noalloc(X.data_ptr(), n, d, d, L.data_ptr(), B, d, gamma, V.data_ptr(), c, B,
                                 F_new.data_ptr(), c, stream)
    assert st == 0
    torch.cuda.synchronize()
    return F_ref.cpu().numpy(), F_new.cpu().numpy()


@pytest.mark.parametrize("c", [3, 40])       # both consumers of the panel: sweeps and the MFMA product
def test_noalloc_predict_twice_second_call_smaller(lpd, oracle, dev, c):
    g = torch.Generator().manual_seed(4242 + c)
    d, B, gamma = 24, 300, 1.0 / 24
    L = torch.randn((B, d), generator=g)
    W, eig, rank, K = oracle.whiten(L.numpy(), gamma)
    W32 = W[:rank].astype(np.float32)
    Ws = (torch.randn((c, rank), generator=g) / rank ** 0.5)
    V = lpd.lpd_fold_weights(torch.from_numpy(W32).to(dev), Ws.to(dev))
    for n in (1500, 333):                      # second call smaller: rows and panel of the first stay behind
        X = torch.randn((n, d), generator=g)
        F_ref, F_new = _scores_both_ways(lpd, dev, X.to(dev), L.to(dev), gamma, V)
        assert np.all(np.isfinite(F_new))
        assert relfro(F_new, F_ref) <= 1e-6
        F_orc = oracle.predict(X.numpy(), L.numpy(), gamma, W32, Ws.numpy())
        assert relfro(F_new, F_orc) <= TOL
        assert relfro(F_ref, F_orc) <= TOL


def test_noalloc_predict_rejects_shapes_beyond_its_scratch(lpd, dev):
    lib = lpd.lib()
    p = ctypes.c_void_p(256)                   # never dereferenced: the limit is checked on the host first
    # 40,000 landmarks: 256 panel rows alone need 41 MB
    assert lib.lpd_predict_noalloc(p, 1000, 8, 8, p, 40000, 8, 0.5, p, 2, 40000, p, 2, None) == -7
    assert b"32 MiB" in lib.lpd_strerror(-7)
    assert lib.lpd_predict_noalloc(p, 0, 8, 8, p, 16, 8, 0.5, p, 2, 16, p, 2, None) == 0
    assert lib.lpd_predict_noalloc(p, 10, 8, 8, p, 16, 8, 0.5, p, 17, 16, p, 17, None) == -2     # c > B
