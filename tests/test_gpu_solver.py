"""GPU parity for the batched dual coordinate-ascent solver (lpd_cd_solve) against the CPU oracle.

The GPU works in fp32, the oracle in fp64, with the same visiting order and the same rules.  With
shrinking off and a fixed number of epochs the two trajectories are continuous functions of the
rounding, so alpha and w are compared directly.  With shrinking and the stopping rule the discrete
decisions (bit-for-bit "unchanged", violation <= eps) can fall differently in the two precisions, so
what is unique is compared -- the optimal w and the dual objective -- and the rest is checked for
validity: box constraints, w = sum alpha y g, KKT violation evaluated in double.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


@pytest.fixture(scope="module")
def lpd():
    from paper_2207_01016_amd import lpd as mod
    mod.lib()
    return mod


def _data(seed, n, r, ld=None, noise=0.15):
    rng = np.random.default_rng(seed)
    ld = r if ld is None else ld
    G = np.zeros((n, ld), dtype=np.float32)
    G[:, :r] = (rng.standard_normal((n, r)) / np.sqrt(r)).astype(np.float32)
    v = rng.standard_normal(r)
    y = np.where(G[:, :r].astype(np.float64) @ v + noise * rng.standard_normal(n) >= 0, 1.0, -1.0).astype(np.float32)
    return G, y


def _batch(lpd, dev, G, probs, r, **kw):
    """probs: list of (rows int64 array, y float32 array, C). Returns per-problem (alpha, w, status)."""
    Gd = torch.from_numpy(G).to(dev)
    gsq = lpd.lpd_row_sqnorms(Gd, r=r)
    off = np.zeros(len(probs) + 1, dtype=np.int64)
    for i, (rw, _, _) in enumerate(probs):
        off[i + 1] = off[i] + len(rw)
    rows = torch.from_numpy(np.concatenate([p[0] for p in probs]).astype(np.int64)).to(dev)
    y = torch.from_numpy(np.concatenate([p[1] for p in probs]).astype(np.float32)).to(dev)
    C = torch.tensor([p[2] for p in probs], dtype=torch.float32, device=dev)
    alpha0 = kw.pop("alpha0", None)
    alpha = torch.zeros(int(off[-1]), dtype=torch.float32, device=dev) if alpha0 is None else alpha0.clone()
    alpha, w, st = lpd.lpd_cd_solve(Gd, gsq, torch.from_numpy(off).to(dev), rows, y, C, alpha, r=r, **kw)
    torch.cuda.synchronize()
    a = alpha.cpu().numpy()
    wh = w.cpu().numpy()
    return [(a[off[i]:off[i + 1]], wh[i, :r], st[i]) for i in range(len(probs))], alpha


def _kkt(G, rows, y, alpha, w, C):
    grad = 1.0 - y * (G[rows].astype(np.float64) @ w.astype(np.float64))
    a = alpha.astype(np.float64)
    v = np.where(a <= 0, np.maximum(grad, 0), np.where(a >= C, np.maximum(-grad, 0), np.abs(grad)))
    return float(v.max())


def test_row_sqnorms(lpd, dev):
    G, _ = _data(0, 300, 70, ld=72)
    gsq = lpd.lpd_row_sqnorms(torch.from_numpy(G).to(dev), r=70)
    ref = (G[:, :70].astype(np.float64) ** 2).sum(axis=1)
    assert np.allclose(gsq.cpu().numpy(), ref, rtol=1e-5)


@pytest.mark.parametrize("r,ld", [(10, 12), (256, 256), (300, 300), (512, 512), (1000, 1024), (1024, 1024),
                                  (1024, 1026), (2048, 2048), (4096, 4096), (4100, 4100), (8192, 8192),
                                  (8200, 8200)])
def test_fixed_epochs_no_shrinking_matches_oracle(lpd, oracle, dev, r, ld):
    """Three plain epochs: alpha and w track the double-precision trajectory (every register layout)."""
    n = 400
    G, y = _data(r, n, r, ld=ld)
    rng = np.random.default_rng(1)
    rows = rng.permutation(n)[:333].astype(np.int64)
    res, _ = _batch(lpd, dev, G, [(rows, y[rows], 1.0)], r, eps=0.0, max_epochs=3, shrink_k=0, eta=0.0)
    a, w, st = res[0]
    a_ref, w_ref, s_ref = oracle.cd_solve(G, rows, y[rows], 1.0, eps=0.0, max_epochs=3, shrink_k=0, eta=0.0, r=r)
    assert st["epochs"] == 3 and st["steps"] == 3 * 333 and st["converged"] == 0
    assert np.linalg.norm(a - a_ref) <= 1e-4 * np.linalg.norm(a_ref)
    assert np.linalg.norm(w - w_ref) <= 1e-4 * np.linalg.norm(w_ref)
    assert abs(st["dual"] - s_ref["dual"]) <= 1e-4 * abs(s_ref["dual"])


def test_batch_to_convergence_matches_oracle_optimum(lpd, oracle, dev):
    """A batch with different row subsets, orders and C: unique quantities vs the oracle, validity of the rest."""
    n, r = 3000, 10
    G, y = _data(5, n, r)
    rng = np.random.default_rng(2)
    probs = []
    for C in (0.1, 1.0, 10.0):
        for frac in (1.0, 0.6):
            rows = rng.permutation(n)[: int(frac * n)].astype(np.int64)
            probs.append((rows, y[rows], C))
    probs.append((np.arange(5, dtype=np.int64), y[:5], 1.0))            # tiny problem
    probs.append((np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.float32), 1.0))   # empty problem
    eps = 1e-4
    res, _ = _batch(lpd, dev, G, probs, r, eps=eps, max_epochs=200000)
    for (rows, yy, C), (a, w, st) in zip(probs, res):
        if len(rows) == 0:
            assert st["converged"] == 1 and st["steps"] == 0 and st["epochs"] == 1 and np.all(w == 0)
            continue
        a_ref, w_ref, s_ref = oracle.cd_solve(G, rows, yy, C, eps=eps, max_epochs=200000, r=r)
        assert st["converged"] == 1 and s_ref["converged"]
        assert np.all(a >= 0) and np.all(a <= np.float32(C))
        w_from_alpha = (a.astype(np.float64) * yy) @ G[rows, :r].astype(np.float64)
        assert np.linalg.norm(w - w_from_alpha) <= 1e-4 * max(np.linalg.norm(w_from_alpha), 1e-9)
        assert np.linalg.norm(w - w_ref) <= 5e-3 * np.linalg.norm(w_ref)
        d_gpu = a.astype(np.float64).sum() - 0.5 * w_from_alpha @ w_from_alpha
        assert abs(d_gpu - s_ref["dual"]) <= 1e-5 * abs(s_ref["dual"])
        assert abs(st["dual"] - s_ref["dual"]) <= 1e-4 * abs(s_ref["dual"])
        assert _kkt(G[:, :r], rows, yy, a, w_from_alpha, C) <= 20 * eps
        # shrinking did its work on the larger problems: far fewer steps than epochs * variables
        if len(rows) >= 1000:
            assert st["steps"] < 0.2 * st["epochs"] * len(rows)
            assert st["active"] < 0.1 * len(rows)


def test_shrinking_off_and_eta_zero_reach_the_same_optimum(lpd, oracle, dev):
    n, r = 1500, 12
    G, y = _data(7, n, r)
    rows = np.arange(n, dtype=np.int64)
    base = oracle.cd_solve(G, rows, y, 1.0, eps=1e-4, max_epochs=200000, r=r)[2]["dual"]
    for kw in (dict(shrink_k=0), dict(shrink_k=5, eta=0.0), dict(shrink_k=2, eta=0.2)):
        res, _ = _batch(lpd, dev, G, [(rows, y, 1.0)], r, eps=1e-4, max_epochs=200000, **kw)
        a, w, st = res[0]
        assert st["converged"] == 1
        assert abs(st["dual"] - base) <= 1e-4 * abs(base), kw


def test_warm_start_at_the_solution(lpd, dev):
    n, r = 800, 20
    G, y = _data(8, n, r)
    rows = np.arange(n, dtype=np.int64)
    res, alpha = _batch(lpd, dev, G, [(rows, y, 1.0)], r, eps=1e-4, max_epochs=100000)
    a, w, st = res[0]
    res2, _ = _batch(lpd, dev, G, [(rows, y, 1.0)], r, eps=1e-3, max_epochs=100000, alpha0=alpha)
    a2, w2, st2 = res2[0]
    assert st2["converged"] == 1 and st2["epochs"] <= 2
    assert np.linalg.norm(w2 - w) <= 1e-3 * np.linalg.norm(w)


def test_solver_on_factor_of_small_workload(lpd, oracle, dev):
    """End to end on a scaled-down 'small' recipe: factor on the GPU, then one-vs-one problems on its rows."""
    from paper_2207_01016_amd import workloads
    wl = workloads.WORKLOADS["small"].with_shape(n=4000, B=256)
    X = workloads.make_X(wl, dev)
    idx = workloads.landmark_indices(wl)
    L = X[idx.to(dev)].contiguous()
    W, eig, rank = lpd.lpd_whiten_host(L.cpu(), wl.gamma)
    G = torch.empty((wl.n, wl.B), dtype=torch.float32, device=dev)
    lpd.lpd_nystrom_factor(X, L, wl.gamma, W.to(dev), G, lpd.alloc_workspace(wl.n, wl.d, wl.B, dev), r=rank)
    torch.cuda.synchronize()
    comp = workloads.mixture_components(wl).numpy()
    Gh = G.cpu().numpy()
    probs = []
    for (c0, c1) in [(0, 1), (2, 7), (3, 4)]:
        rows = np.nonzero((comp == c0) | (comp == c1))[0].astype(np.int64)
        yy = np.where(comp[rows] == c0, 1.0, -1.0).astype(np.float32)
        probs.append((rows, yy, 4.0))
    res, _ = _batch(lpd, dev, Gh, probs, rank, eps=1e-3, max_epochs=100000)
    for (rows, yy, C), (a, w, st) in zip(probs, res):
        a_ref, w_ref, s_ref = oracle.cd_solve(Gh, rows, yy, C, eps=1e-3, max_epochs=100000, r=rank)
        assert st["converged"] == 1
        assert abs(st["dual"] - s_ref["dual"]) <= 1e-3 * abs(s_ref["dual"])
        assert np.linalg.norm(w - w_ref) <= 2e-2 * np.linalg.norm(w_ref)
        # the classifier separates its two mixture components
        acc = np.mean(np.sign(Gh[rows, :rank] @ w) == yy)
        assert acc > 0.95
