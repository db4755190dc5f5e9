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
    torch.cuda.empty_cache()                  # blocks cached from earlier tests go back before the large allocations
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
    # the factor reproduces the kernel on the landmarks, off the diagonal too: G_L G_L^T = K_LL on a block
    # of 128 landmarks (this is where a wrong eigenvector basis from the device preparation would show)
    sub = idx[:: max(1, wl.B // 128)][:128]
    gl = G[sub.to(dev)].double()
    kll = oracle.kernel_block(L[:: max(1, wl.B // 128)][:128].cpu().numpy(), L[:: max(1, wl.B // 128)][:128].cpu().numpy(),
                              wl.gamma)
    assert relfro((gl @ gl.T).cpu().numpy(), kll) <= 1e-4
    # row-list sweep over the sample equals the full sweep on those rows, bit for bit
    assert torch.equal(lpd.lpd_margins_rows(G, rd, w, r=rank), m[rd])


def test_dropping_rule_at_size(oracle):
    """The dropping rule of Section 4 (second bullet) on 4,096 landmarks of which 37 are copies of others: the
    device preparation drops exactly those components, the factor keeps its columns from the rank on at zero, and
    both parity and the kernel identity on the landmarks hold on the kept ones."""
    from paper_2207_01016_amd import lpd, workloads
    lpd.lib()
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS["digit"].with_rows(262144)
    dup = 37
    torch.cuda.empty_cache()
    X = workloads.make_X(wl, dev)
    idx = workloads.landmark_indices(wl)
    idx[wl.B - dup:] = idx[:dup]                              # the last 37 landmarks repeat the first 37
    L = X[idx.to(dev)].contiguous()
    Wd, eig, rank = lpd.lpd_whiten(L, wl.gamma)
    assert rank == wl.B - dup
    assert abs(float(eig.sum()) - wl.B) <= 1e-8 * wl.B       # trace of K_LL
    assert float(eig[rank - 1]) > 1e-10 * float(eig[0]) >= abs(float(eig[rank]))
    assert not bool(Wd[rank:].any())
    torch.cuda.empty_cache()
    G = torch.full((wl.n, wl.B), float("nan"), dtype=torch.float32, device=dev)
    lpd.lpd_nystrom_factor(X, L, wl.gamma, Wd, G, lpd.alloc_workspace(wl.n, wl.d, wl.B, dev), r=rank)
    torch.cuda.synchronize()
    assert not bool(G[:, rank:].any())                        # exact zeros from the rank on
    rows = workloads.sample_rows(wl, 192, include=torch.cat([idx[:32], idx[wl.B - dup:][:8], torch.tensor([0, wl.n - 1])]))
    ref = oracle.nystrom_factor(X[rows.to(dev)].cpu().numpy(), L.cpu().numpy(), wl.gamma, Wd.cpu().numpy(), r=rank)
    Gs = G[rows.to(dev)].cpu().numpy()
    assert np.all(np.isfinite(Gs))
    assert relfro(Gs[:, :rank], ref[:, :rank]) <= TOL_G
    # landmark rows of G have norm 1; G_L G_L^T = K_LL on a block that holds copies
    lm = G[idx.to(dev)].double()
    assert torch.allclose((lm * lm).sum(dim=1), torch.ones(wl.B, dtype=torch.float64, device=dev), atol=1e-3)
    sub = torch.cat([torch.arange(0, 96), torch.arange(wl.B - 32, wl.B)])
    gl = lm[sub.to(dev)]
    kll = oracle.kernel_block(L[sub.to(dev)].cpu().numpy(), L[sub.to(dev)].cpu().numpy(), wl.gamma)
    assert relfro((gl @ gl.T).cpu().numpy(), kll) <= 1e-4


def test_full_size_predict_cnn(oracle):
    """bench.py --path predict at its size: 262,144 new points of the cnn recipe, 10 classifiers; oracle on sampled points."""
    from paper_2207_01016_amd import lpd, workloads
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS["cnn"].with_rows(262144)
    X = workloads.make_X(wl, dev)
    L = X[workloads.landmark_indices(wl).to(dev)].contiguous()
    W, eig, rank = lpd.lpd_whiten(L, wl.gamma)
    torch.cuda.empty_cache()
    c = 10
    Ws = torch.randn((c, rank), generator=torch.Generator().manual_seed(2)) / rank ** 0.5
    V = lpd.lpd_fold_weights(W, Ws.to(dev), r=rank)
    F = lpd.lpd_predict(X, L, wl.gamma, V)
    torch.cuda.synchronize()
    rows = workloads.sample_rows(wl, 128, include=torch.tensor([0, wl.n - 1]))
    ref = oracle.predict(X[rows.to(dev)].cpu().numpy(), L.cpu().numpy(), wl.gamma, W.cpu().numpy(), Ws.numpy(), r=rank)
    err = relfro(F[rows.to(dev)].cpu().numpy(), ref)
    print(f"[predict cnn] relF(scores) = {err:.3e}", flush=True)
    assert err <= TOL_G
    assert bool(torch.isfinite(F).all())


def test_full_size_sparse_digit(oracle):
    """bench.py --path sparse at its size: the digit recipe in compressed-row form, all 1,000,000 rows."""
    from paper_2207_01016_amd import lpd, workloads
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS["digit"]
    X = workloads.make_X(wl, dev)
    idx = workloads.landmark_indices(wl)
    L = X[idx.to(dev)].contiguous()
    W, eig, rank = lpd.lpd_whiten(L, wl.gamma)
    torch.cuda.empty_cache()
    rp, ci, va = workloads.to_csr(X)
    rows = workloads.sample_rows(wl, 256, include=torch.cat([idx[:32], torch.tensor([0, wl.n - 1])]))
    rd = rows.to(dev)
    Xs = X[rd].cpu().numpy()
    del X
    G = torch.empty((wl.n, wl.B), dtype=torch.float32, device=dev)
    lpd.lpd_nystrom_factor_csr(rp, ci, va, wl.d, L, wl.gamma, W, G, r=rank)      # suggested chunk size, as in bench.py
    torch.cuda.synchronize()
    ref = oracle.nystrom_factor(Xs, L.cpu().numpy(), wl.gamma, W.cpu().numpy(), r=rank)
    err = relfro(G[rd].cpu().numpy(), ref)
    print(f"[sparse digit] relF(G) = {err:.3e}", flush=True)
    assert err <= TOL_G
    sq = (G * G).sum(dim=1)
    assert float(sq.max()) <= 1.0 + 1e-3


def test_full_size_solver_batch(oracle):
    """bench.py --path solver at its size: the 1,125 one-vs-one problems on the 'small' factor solved in one launch;
    three of them (smallest, middle and largest C) against the oracle: dual optimum and weight vector."""
    import bench
    from paper_2207_01016_amd import lpd, workloads
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS["small"]
    X = workloads.make_X(wl, dev)
    L = X[workloads.landmark_indices(wl).to(dev)].contiguous()
    W, eig, rank = lpd.lpd_whiten(L, wl.gamma)
    G = torch.empty((wl.n, wl.B), dtype=torch.float32, device=dev)
    lpd.lpd_nystrom_factor(X, L, wl.gamma, W, G, lpd.alloc_workspace(wl.n, wl.d, wl.B, dev), r=rank)
    gsq = lpd.lpd_row_sqnorms(G, r=rank)
    probs = bench.solver_problems(wl, workloads.mixture_components(wl).numpy())
    P = len(probs)
    off = np.zeros(P + 1, dtype=np.int64)
    for i, pr in enumerate(probs):
        off[i + 1] = off[i] + len(pr[0])
    rows = torch.from_numpy(np.concatenate([pr[0] for pr in probs])).to(dev)
    y = torch.from_numpy(np.concatenate([pr[1] for pr in probs])).to(dev)
    C = torch.tensor([pr[2] for pr in probs], dtype=torch.float32, device=dev)
    alpha = torch.zeros(int(off[-1]), dtype=torch.float32, device=dev)
    alpha, w, st = lpd.lpd_cd_solve(G, gsq, torch.from_numpy(off).to(dev), rows, y, C, alpha, eps=1e-3,
                                    max_epochs=10000, r=rank)
    assert int(st["converged"].sum()) == P
    Gh = G.cpu().numpy()
    for p in (0, 2, 4):                     # the five C values of the first pair and fold come first
        pr = probs[p]
        a_ref, w_ref, s_ref = oracle.cd_solve(Gh, pr[0], pr[1], pr[2], eps=1e-5, max_epochs=100000, r=rank)
        assert s_ref["converged"]
        dual = float(st["dual"][p])
        wp = w[p].double().cpu().numpy()
        print(f"[solver C={pr[2]}] dual {dual:.4f} oracle {s_ref['dual']:.4f}  |w - w*|/|w*| = "
              f"{np.linalg.norm(wp - w_ref) / np.linalg.norm(w_ref):.2e}", flush=True)
        assert abs(dual - s_ref["dual"]) <= 1e-3 * abs(s_ref["dual"])
        assert np.linalg.norm(wp - w_ref) <= 2e-2 * np.linalg.norm(w_ref)
