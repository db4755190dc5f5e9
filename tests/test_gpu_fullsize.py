"""Full-size parity: the five workloads at their real n, d, B in the launch configuration bench.py times
(default workspace / panel size, automatic tile choice), compared with the CPU oracle on a seeded row
sample that contains landmark rows, plus properties that hold for every row.

W comes from the device-side preparation (`lpd_whiten`), as in bench.py; the host routine would need
minutes for the 16,384 landmarks of 'highrank'.  That case holds 131 GB of G.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

TOL_G = 1e-4
TOL_M = 1e-5


def relfro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


CASES = ["tiny", "small", "digit", "cnn", "highrank"]


@pytest.mark.parametrize("name", CASES)
def test_full_size_workload(oracle, name):
    from paper_2207_01016_amd import lpd, workloads
    lpd.lib()
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS[name]
    print(f"[{name}] generating X {wl.n} x {wl.d}", flush=True)
    X = workloads.make_X(wl, dev)
    idx = workloads.landmark_indices(wl)
    L = X[idx.to(dev)].contiguous()
    print(f"[{name}] device whitening, B = {wl.B}", flush=True)
    Wd, eig, rank = lpd.lpd_whiten(L, wl.gamma)
    assert rank == wl.B                       # the recipes are well conditioned: nothing is dropped
    assert abs(float(eig.sum()) - wl.B) <= 1e-8 * wl.B      # trace of K_LL
    W = Wd.cpu()
    torch.cuda.empty_cache()                  # the 2 B^2 doubles of eigensolver scratch go back before G is made
    G = torch.empty((wl.n, wl.B), dtype=torch.float32, device=dev)
    ws = lpd.alloc_workspace(wl.n, wl.d, wl.B, dev)          # recommended size, as in bench.py
    print(f"[{name}] factor", flush=True)
    lpd.lpd_nystrom_factor(X, L, wl.gamma, Wd, G, ws, r=rank)
    w = workloads.make_w(wl).to(dev)
    m = lpd.lpd_margins(G, w, r=rank)
    torch.cuda.synchronize()

    # ---- sampled rows against the oracle (first, last, random rows and landmark rows)
    rows = workloads.sample_rows(wl, 256, include=torch.cat([idx[:64], torch.tensor([0, wl.n - 1])]))
    rd = rows.to(dev)
    print(f"[{name}] oracle on {rows.numel()} rows", flush=True)
    ref = oracle.nystrom_factor(X[rd].cpu().numpy(), L.cpu().numpy(), wl.gamma, W.numpy(), r=rank)
    Gs = G[rd].cpu().numpy()
    err_g = relfro(Gs, ref)
    m_ref = oracle.margins(Gs, w.cpu().numpy(), r=rank)
    err_m = relfro(m[rd].cpu().numpy(), m_ref)
    chained = relfro(m[rd].cpu().numpy(), oracle.margins_f64(ref, w.cpu().numpy().astype(np.float64)))
    print(f"[{name}] relF(G) = {err_g:.3e}  relF(m) = {err_m:.3e}  chained = {chained:.3e}", flush=True)
    assert np.all(np.isfinite(Gs))
    assert err_g <= TOL_G
    assert err_m <= TOL_M

    # ---- properties over ALL rows: projection bound ||g_i||^2 <= 1, = 1 on landmark rows; margins finite
    sq_max = 0.0
    chunk = max(1, (1 << 28) // wl.B)
    for r0 in range(0, wl.n, chunk):
        g = G[r0:r0 + chunk]
        sq_max = max(sq_max, float((g * g).sum(dim=1).max()))
    assert sq_max <= 1.0 + 1e-3, sq_max
    lm = G[idx.to(dev)].double()
    assert torch.allclose((lm * lm).sum(dim=1), torch.ones(wl.B, dtype=torch.float64, device=dev), atol=1e-3)
    assert bool(torch.isfinite(m).all())
    # row-list sweep over the sample equals the full sweep on those rows, bit for bit
    assert torch.equal(lpd.lpd_margins_rows(G, rd, w, r=rank), m[rd])
