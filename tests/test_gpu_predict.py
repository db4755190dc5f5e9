"""GPU parity for prediction (lpd_fold_weights + lpd_predict) against the CPU oracle.

The oracle scores a point as ws . (W z(x)) -- features first, then the classifier, nothing folded;
the GPU folds v = W^T ws once and takes v . z(x).  Tolerance: relative Frobenius error <= 1e-4, as
for the factor (the scores are sums of the same products).
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def relfro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


@pytest.fixture(scope="module")
def lpd():
    from paper_2207_01016_amd import lpd as mod
    mod.lib()
    return mod


@pytest.mark.parametrize("r,B,c", [(50, 70, 1), (70, 70, 9), (128, 128, 16), (300, 333, 40)])
def test_fold_weights(lpd, dev, r, B, c):
    g = torch.Generator().manual_seed(r + B + c)
    W = torch.randn((B, B), generator=g).to(dev)
    Ws = torch.randn((c, r + 3), generator=g).to(dev)
    V = lpd.lpd_fold_weights(W, Ws[:, :r], r=r)
    torch.cuda.synchronize()
    ref = Ws[:, :r].double().cpu().numpy() @ W[:r].double().cpu().numpy()
    assert relfro(V.cpu().numpy(), ref) <= 1e-5


@pytest.mark.parametrize("name,n,B,n_test,c", [
    ("tiny", 1500, 128, 777, 1),
    ("small", 6000, 512, 2500, 3),       # sweep path, several panels
    ("digit", 3000, 300, 1111, 10),      # sweep path in two passes (8 + 2), nothing a multiple of a tile
    ("small", 3000, 256, 1500, 32),      # last class count served by sweeps
    ("small", 3000, 256, 1500, 33),      # first one served by the MFMA product
    ("cnn", 2500, 260, 900, 45),
    ("highrank", 4000, 640, 2000, 130),
])
def test_predict_matches_oracle(lpd, oracle, dev, name, n, B, n_test, c):
    from paper_2207_01016_amd import workloads
    wl = workloads.WORKLOADS[name].with_shape(n=n + n_test, B=B)
    X_all = workloads.make_X(wl, dev)
    X, Xt = X_all[:n], X_all[n:].contiguous()
    idx = workloads.landmark_indices(wl.with_rows(n))
    L = X[idx.to(dev)].contiguous()
    W, eig, rank = lpd.lpd_whiten_host(L.cpu(), wl.gamma)
    g = torch.Generator().manual_seed(c)
    Ws = torch.randn((c, rank), generator=g) / rank ** 0.5
    V = lpd.lpd_fold_weights(W.to(dev), Ws.to(dev), r=rank)
    _, mn = lpd.lpd_nystrom_factor_workspace(n_test, wl.d, B)
    ws = lpd.alloc_workspace(n_test, wl.d, B, dev, mn * 3)           # several panels, ragged last one
    F = torch.full((n_test, c), float("nan"), dtype=torch.float32, device=dev)
    lpd.lpd_predict(Xt, L, wl.gamma, V, F, ws)
    torch.cuda.synchronize()
    ref = oracle.predict(Xt.cpu().numpy(), L.cpu().numpy(), wl.gamma, W.numpy(), Ws.numpy(), r=rank)
    Fh = F.cpu().numpy()
    assert np.all(np.isfinite(Fh))
    assert relfro(Fh, ref) <= 1e-4


@pytest.mark.parametrize("tile", ["auto", "128x128", "256x256", "64x128", "256x128"])
@pytest.mark.parametrize("n,d,B,c,aligned", [
    (777, 20, 130, 1, True),        # one and a bit tile columns, ragged rows
    (1000, 64, 333, 5, True),       # B and n no multiple of anything
    (513, 19, 257, 7, False),       # d % 4 != 0: element-wise loader, plain schedule
    (300, 48, 64, 32, True),        # the most weight vectors that fit half the slots of the write-out
    (700, 36, 300, 33, True),       # one more: the full set of slots
    (1300, 64, 520, 64, True),      # the most weight vectors the write-out takes
    (2100, 16, 1040, 17, True),     # several tile rows and columns of every tile
    (260, 0, 96, 3, True),          # no features: z = 1, the scores are the row sums of V
    (50, 8, 3, 2, True),            # three landmarks
    (40, 8, 9, 9, True),            # as many weight vectors as landmarks (the most the entry point accepts)
])
def test_scores_contracted_in_the_kernel_block_launch_match_the_panel_route(lpd, oracle, dev, n, d, B, c, aligned, tile):
    """Prediction with few weight vectors multiplies the kernel block by them in the write-out of its own launch
    (Z never stored); the route that stores a panel of Z and sweeps it must give the same scores, and both the
    oracle's."""
    g = torch.Generator().manual_seed(n + 7 * B + c)
    ldx = d + (0 if aligned else 1)
    Xf = torch.randn((n, max(ldx, 1)), generator=g)
    Lf = torch.randn((B, max(ldx, 1)), generator=g)
    X, L = Xf.to(dev)[:, :d], Lf.to(dev)[:, :d]
    V = (torch.randn((c, B), generator=g) / B ** 0.5).to(dev)
    gamma = 0.5 / max(d, 1)
    _, mn = lpd.lpd_nystrom_factor_workspace(n, d, B)
    ws = lpd.alloc_workspace(n, d, B, dev, mn * 2)              # a few panels
    out = []
    lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, lpd.GEMM_TILES[tile])
    try:
        for fused in (1, 0):
            lpd.lpd_set_option(lpd.LPD_OPT_FUSED_SCORES, fused)
            F = torch.full((n, c), float("nan"), dtype=torch.float32, device=dev)
            lpd.lpd_predict(X, L, gamma, V, F, ws)
            torch.cuda.synchronize()
            out.append(F.cpu().numpy())
    finally:
        lpd.lpd_set_option(lpd.LPD_OPT_FUSED_SCORES, 1)
        lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, 0)
    Z = oracle.kernel_block(np.ascontiguousarray(Xf[:, :d].numpy()), np.ascontiguousarray(Lf[:, :d].numpy()), gamma)
    ref = Z @ V.cpu().numpy().astype(np.float64).T
    assert np.all(np.isfinite(out[0])) and np.all(np.isfinite(out[1]))
    assert relfro(out[0], ref) <= 1e-5 and relfro(out[1], ref) <= 1e-5
    assert relfro(out[0], out[1]) <= 2e-6


def test_predict_on_training_rows_equals_margins_of_the_factor(lpd, dev):
    from paper_2207_01016_amd import workloads
    wl = workloads.WORKLOADS["small"].with_shape(n=3000, B=256)
    X = workloads.make_X(wl, dev)
    L = X[workloads.landmark_indices(wl).to(dev)].contiguous()
    W, eig, rank = lpd.lpd_whiten_host(L.cpu(), wl.gamma)
    Wd = W.to(dev)
    G = torch.empty((wl.n, wl.B), dtype=torch.float32, device=dev)
    lpd.lpd_nystrom_factor(X, L, wl.gamma, Wd, G, lpd.alloc_workspace(wl.n, wl.d, wl.B, dev), r=rank)
    w = workloads.make_w(wl).to(dev)
    m = lpd.lpd_margins(G, w, r=rank)
    V = lpd.lpd_fold_weights(Wd, w[None, :].contiguous(), r=rank)
    F = lpd.lpd_predict(X, L, wl.gamma, V)
    torch.cuda.synchronize()
    assert float((F[:, 0].double() - m.double()).norm() / m.double().norm()) <= 1e-4


def test_predict_strided_output_and_zero_classifiers(lpd, dev):
    g = torch.Generator().manual_seed(3)
    X = torch.randn((500, 12), generator=g).to(dev)
    L = X[:40].contiguous()
    V = torch.randn((2, 40), generator=g).to(dev)
    Fbig = torch.zeros((500, 5), dtype=torch.float32, device=dev)
    lpd.lpd_predict(X, L, 0.1, V, Fbig[:, :2])
    torch.cuda.synchronize()
    assert torch.all(Fbig[:, 2:] == 0) and bool(Fbig[:, :2].abs().sum() > 0)
    ref = torch.exp(-0.1 * torch.cdist(X.double(), L.double()) ** 2) @ V.double().T
    assert float((Fbig[:, :2].double() - ref).norm() / ref.norm()) <= 1e-5


@pytest.mark.parametrize("n,d,B,c", [
    (40000, 24, 300, 5),       # stored panel of 40,000 rows: sweeps up to 4 classifiers, a narrow MFMA tile from 5 on
    (40000, 24, 300, 13),
    (40000, 24, 300, 64),
    (20000, 20, 200, 30),      # 20,000 rows: a 128-wide MFMA tile from 9 classifiers on
    (20000, 20, 200, 7),       #   sweeps below
    (9000, 16, 130, 50),       # 9,000 rows: sweeps up to 32 classifiers, 128-wide tiles above
    (9000, 16, 130, 20),
])
def test_routes_of_prediction_with_few_landmarks_match_the_oracle(lpd, oracle, dev, n, d, B, c):
    """With few landmarks a stored panel of the kernel block is long; with the contracted write-out switched off,
    which kernel consumes it depends on its rows and on the number of classifiers.  Every route gives the
    oracle's scores, and the contracted write-out (FMA up to 6 classifiers, MFMA above) the same."""
    g = torch.Generator().manual_seed(3 * n + B + c)
    Xf = torch.randn((n, d), generator=g)
    Lf = torch.randn((B, d), generator=g)
    V = (torch.randn((c, B), generator=g) / B ** 0.5).to(dev)
    X, L = Xf.to(dev), Lf.to(dev)
    gamma = 0.5 / d
    ws = lpd.alloc_workspace(n, d, B, dev)
    out = []
    try:
        for fused in (1, 0):
            lpd.lpd_set_option(lpd.LPD_OPT_FUSED_SCORES, fused)
            F = torch.full((n, c), float("nan"), dtype=torch.float32, device=dev)
            lpd.lpd_predict(X, L, gamma, V, F, ws)
            torch.cuda.synchronize()
            out.append(F.cpu().numpy())
    finally:
        lpd.lpd_set_option(lpd.LPD_OPT_FUSED_SCORES, 1)
    Z = oracle.kernel_block(Xf.numpy(), Lf.numpy(), gamma)
    ref = Z @ V.cpu().numpy().astype(np.float64).T
    assert np.all(np.isfinite(out[0])) and np.all(np.isfinite(out[1]))
    assert relfro(out[0], ref) <= 1e-5 and relfro(out[1], ref) <= 1e-5
    assert relfro(out[0], out[1]) <= 2e-6
