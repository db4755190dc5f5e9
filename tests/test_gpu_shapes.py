"""Seeded sweep over small, awkward shapes: every size odd or not, padded leading dimensions (aligned and not),
ranks below B, all tile choices.  Factor, sweep and prediction against the oracle on all rows."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def relfro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def _cases(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        n = int(rng.integers(1, 700))
        d = int(rng.integers(1, 300))
        B = int(rng.integers(1, 600))
        r = int(rng.integers(1, B + 1))
        pads = [int(rng.choice([0, 1, 3, 4, 8])) for _ in range(4)]
        tile = ["auto", "128x128", "256x128", "256x256", "64x128"][int(rng.integers(0, 5))]
        out.append(pytest.param(n, d, B, r, pads, tile, i, id=f"{i}-n{n}-d{d}-B{B}-r{r}-{tile}"))
    return out


@pytest.mark.parametrize("n,d,B,r,pads,tile,case", _cases(40, 20220701))
def test_factor_sweep_predict_on_awkward_shapes(oracle, n, d, B, r, pads, tile, case):
    from paper_2207_01016_amd import lpd
    lpd.lib()
    dev = torch.device("cuda:0")
    g = torch.Generator().manual_seed(1000 + case)
    px, pl, pw, pg = pads
    Xf = torch.randn((n, d + px), generator=g)
    Lf = torch.randn((B, d + pl), generator=g)
    Wf = torch.randn((B, B + pw), generator=g) / B ** 0.5
    X, L, W = Xf[:, :d].to(dev) if px == 0 else Xf.to(dev)[:, :d], Lf.to(dev)[:, :d], Wf.to(dev)[:, :B]
    gamma = 0.5 / d
    Gf = torch.full((n, B + pg), float("nan"), device=dev)
    G = Gf[:, :B]
    ws = lpd.alloc_workspace(n, d, B, dev)
    lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, lpd.GEMM_TILES[tile])
    try:
        lpd.lpd_nystrom_factor(X, L, gamma, W, G, ws, r=r)
        G_panels = None
        if B <= 256:
            # few landmarks take the one-launch kernel; the panel schedule must give the same factor
            G_panels = torch.full((n, B), float("nan"), device=dev)
            lpd.lpd_set_option(lpd.LPD_OPT_SMALL_PATH, 0)
            try:
                lpd.lpd_nystrom_factor(X, L, gamma, W, G_panels, ws, r=r)
            finally:
                lpd.lpd_set_option(lpd.LPD_OPT_SMALL_PATH, 1)
        w = torch.randn(r, generator=g).to(dev)
        m = lpd.lpd_margins(G, w, r=r)
        c = int(1 + case % 5) if case % 2 else min(B, 33 + case)
        V = (torch.randn((c, B), generator=g) / B ** 0.5).to(dev)
        F = lpd.lpd_predict(X, L, gamma, V)
        torch.cuda.synchronize()
    finally:
        lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, 0)
    Xh, Lh, Wh = Xf[:, :d].numpy(), Lf[:, :d].numpy(), Wf[:, :B].numpy()
    ref = oracle.nystrom_factor(np.ascontiguousarray(Xh), np.ascontiguousarray(Lh), gamma, np.ascontiguousarray(Wh), r=r)
    Gh = G.cpu().numpy()
    assert relfro(Gh[:, :r], ref) <= 1e-4
    assert not Gh[:, r:].any()                                       # zero fill past r
    if G_panels is not None:
        Gp = G_panels.cpu().numpy()
        assert relfro(Gp[:, :r], ref) <= 1e-4 and not Gp[:, r:].any()
        assert relfro(Gh, Gp) <= 2e-5
    if pg:
        assert torch.isnan(Gf[:, B:]).all()                          # padding untouched
    assert relfro(m.cpu().numpy(), oracle.margins(np.ascontiguousarray(Gh), w.cpu().numpy(), r=r)) <= 1e-5
    Z = oracle.kernel_block(np.ascontiguousarray(Xh), np.ascontiguousarray(Lh), gamma)
    assert relfro(F.cpu().numpy(), Z @ V.double().cpu().numpy().T) <= 1e-4
