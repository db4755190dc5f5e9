"""Device-side preparation (steps 1a-1c, `lpd_whiten`) against the oracle's whitening.

Eigenvectors are unique only up to sign (and rotation within a repeated eigenvalue), so the comparison
uses what is unique: the eigenvalues, the rank, W K W^T = I on the kept components, the sign rule, and,
where the spectrum is simple, the rows of W themselves.
"""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


@pytest.fixture(scope="module")
def lpd():
    from paper_2207_01016_amd import lpd as mod
    mod.lib()
    return mod


@pytest.mark.parametrize("name,B", [
    ("tiny", 128), ("small", 200), ("digit", 97), ("cnn", 64), ("highrank", 333),
    ("small", 35),        # a single, partial reflector panel
    ("highrank", 1030),   # several rotation passes, trailing matrix over many workgroups
])
def test_whiten_against_oracle(lpd, oracle, dev, name, B):
    from paper_2207_01016_amd import workloads
    wl = workloads.WORKLOADS[name].with_shape(n=max(2 * B, 1000), B=B)
    X = workloads.make_X(wl)
    Lm = X[workloads.landmark_indices(wl)].contiguous()
    W, eig, rank = lpd.lpd_whiten(Lm.to(dev), wl.gamma)
    Wo, eo, ro, K = oracle.whiten(Lm.numpy(), wl.gamma, method="lapack")
    assert rank == ro == B
    assert np.max(np.abs(eig.numpy() - eo)) <= 1e-10 * eo[0]
    Wd = W.double().cpu().numpy()
    assert np.linalg.norm(Wd @ K @ Wd.T - np.eye(B)) <= 2e-6 * B
    gap = np.min(np.abs(np.diff(eo)))
    if gap > 1e-6:
        assert np.max(np.abs(Wd - Wo)) <= 1e-5 * np.max(np.abs(Wo)) / min(1.0, gap * 1e3)
    for j in range(B):
        assert Wd[j, np.argmax(np.abs(Wd[j]))] > 0.0


def test_whiten_matches_host_routine(lpd, dev):
    """Same definition as the host routine: eigenvalues to rounding, W to fp32 rounding where the spectrum is simple."""
    from paper_2207_01016_amd import workloads
    wl = workloads.WORKLOADS["small"].with_shape(n=4000, B=640)
    X = workloads.make_X(wl)
    Lm = X[workloads.landmark_indices(wl)].contiguous()
    Wh, eh, rh = lpd.lpd_whiten_host(Lm, wl.gamma, 1e-6)
    Wd, ed, rd = lpd.lpd_whiten(Lm.to(dev), wl.gamma, 1e-6)
    assert rd == rh
    assert torch.max(torch.abs(ed - eh)).item() <= 1e-11 * eh[0].item()
    assert torch.all(Wd[rd:] == 0)
    # the factor built from either W spans the same space: W^T W (= K^+ on the kept range) agrees
    Ph = Wh.double().T @ Wh.double()
    Pd = Wd.double().cpu().T @ Wd.double().cpu()
    assert float((Ph - Pd).norm() / Ph.norm()) <= 1e-5


def test_whiten_degenerate_cases(lpd, oracle, dev):
    g = torch.Generator().manual_seed(5)
    X = torch.randn((40, 6), generator=g)
    # gamma = 0: rank one, W[0] = 1/B
    W, eig, rank = lpd.lpd_whiten(X[:9].to(dev), 0.0)
    assert rank == 1
    assert abs(eig[0].item() - 9.0) < 1e-12
    assert torch.allclose(W[0].cpu(), torch.full((9,), 1.0 / 9.0), atol=1e-7) and torch.all(W[1:] == 0)
    # duplicated landmark: one component dropped, remaining ones still whiten K
    Ld = torch.cat([X[:12], X[3:4]]).contiguous()
    W, eig, rank = lpd.lpd_whiten(Ld.to(dev), 0.15)
    assert rank == 12 and abs(eig[-1].item()) < 1e-12
    K = oracle.kernel_block(Ld.numpy(), Ld.numpy(), 0.15)
    Wd = W.double().cpu().numpy()[:12]
    assert np.linalg.norm(Wd @ K @ Wd.T - np.eye(12)) < 1e-5
    assert torch.all(W[12:] == 0)
    # B = 1, 2, 3 (no reflector, no reflector, one reflector)
    W, eig, rank = lpd.lpd_whiten(X[:1].to(dev), 0.3)
    assert rank == 1 and W.item() == 1.0
    W, eig, rank = lpd.lpd_whiten(torch.tensor([[0.0], [1.0]], device=dev), float(np.log(2.0)))
    assert rank == 2
    assert torch.allclose(eig, torch.tensor([1.5, 0.5], dtype=torch.float64), atol=1e-14)
    assert torch.allclose(W.cpu(), torch.tensor([[3 ** -0.5, 3 ** -0.5], [1.0, -1.0]]), atol=1e-7)
    W, eig, rank = lpd.lpd_whiten(X[:3].to(dev), 0.1)
    K = oracle.kernel_block(X[:3].numpy(), X[:3].numpy(), 0.1)
    Wd = W.double().cpu().numpy()
    assert rank == 3 and np.linalg.norm(Wd @ K @ Wd.T - np.eye(3)) < 1e-5
    # B = 0
    W, eig, rank = lpd.lpd_whiten(torch.zeros((0, 3), device=dev), 0.3)
    assert rank == 0 and W.shape == (0, 0)


@pytest.mark.parametrize("B,gamma,dup", [(600, 0.05, 50), (512, 1e-4, 0), (384, 3e-3, 7)])
def test_whiten_rank_deficient_matches_host_and_whitens(lpd, oracle, dev, B, gamma, dup):
    """Many eigenvalues at or below the clipping threshold (duplicated landmarks, or a kernel so wide that the
    spectrum decays under it): same rank and eigenvalues as the host routine, kept components whiten K_LL,
    dropped rows are exact zeros."""
    g = torch.Generator().manual_seed(B)
    X = torch.randn((B, 12), generator=g)
    if dup:
        X[B - dup:] = X[:dup]
    Wd, ed, rd = lpd.lpd_whiten(X.to(dev), gamma)
    Wh, eh, rh = lpd.lpd_whiten_host(X, gamma)
    assert rd == rh and rd < B
    assert torch.max(torch.abs(ed - eh)).item() <= 1e-11 * eh[0].item()
    assert torch.all(Wd[rd:] == 0)
    K = oracle.kernel_block(X.numpy(), X.numpy(), gamma)
    W64 = Wd[:rd].double().cpu().numpy()
    # fp32 rounding of W is amplified by 1/lambda on the smallest kept components: check the well-conditioned part
    keep = int((ed.numpy() >= 1e-4 * ed[0].item()).sum())
    assert keep >= 1
    P = W64[:keep] @ K @ W64[:keep].T
    assert np.linalg.norm(P - np.eye(keep)) <= 1e-3 * keep ** 0.5
    # both routines span the same space: W^T W (the pseudo-inverse of K_LL on the kept range) agrees
    # on its dominant part
    Ph = Wh[:keep].double().T @ Wh[:keep].double()
    Pd = Wd[:keep].double().cpu().T @ Wd[:keep].double().cpu()
    assert float((Ph - Pd).norm() / Ph.norm()) <= 1e-4


def test_whiten_feeds_the_factor(lpd, oracle, dev):
    """End to end on the device: W from lpd_whiten, G from lpd_nystrom_factor; landmark rows give G G^T = K_LL."""
    from paper_2207_01016_amd import workloads
    wl = workloads.WORKLOADS["small"].with_shape(n=3000, B=256)
    X = workloads.make_X(wl, dev)
    idx = workloads.landmark_indices(wl)
    Lm = X[idx.to(dev)].contiguous()
    W, eig, rank = lpd.lpd_whiten(Lm, wl.gamma)
    G = torch.empty((wl.n, wl.B), dtype=torch.float32, device=dev)
    ws = lpd.alloc_workspace(wl.n, wl.d, wl.B, dev)
    lpd.lpd_nystrom_factor(X, Lm, wl.gamma, W, G, ws, r=rank)
    torch.cuda.synchronize()
    GL = G[idx.to(dev)].double().cpu().numpy()
    K = oracle.kernel_block(Lm.cpu().numpy(), Lm.cpu().numpy(), wl.gamma)
    assert np.linalg.norm(GL @ GL.T - K) / np.linalg.norm(K) <= 1e-4


def test_whiten_workspace_too_small(lpd, dev):
    Lm = torch.randn((64, 8), device=dev)
    with pytest.raises(lpd.LpdError) as ei:
        lpd.lpd_whiten(Lm, 0.1, workspace=torch.empty(4096, dtype=torch.uint8, device=dev))
    assert ei.value.status == -4


def test_whiten_digit_workload_at_full_landmark_count(lpd, oracle, dev):
    """The 4,096 landmarks of the digit-shaped workload, as bench.py prepares them: eigenvalues against the
    oracle's LAPACK path to 1e-10 of the largest, the rank, and W K W^T = I."""
    from paper_2207_01016_amd import workloads
    wl = workloads.WORKLOADS["digit"].with_rows(65536)
    X = workloads.make_X(wl)
    Lm = X[workloads.landmark_indices(wl)].contiguous()
    W, eig, rank = lpd.lpd_whiten(Lm.to(dev), wl.gamma)
    Wo, eo, ro, K = oracle.whiten(Lm.numpy(), wl.gamma, method="lapack")
    assert rank == ro == wl.B
    assert np.max(np.abs(eig.numpy() - eo)) <= 1e-10 * eo[0]
    Wd = W.double()
    P = Wd @ torch.from_numpy(K).to(dev) @ Wd.T
    assert float((P - torch.eye(wl.B, dtype=torch.float64, device=dev)).norm()) <= 2e-6 * wl.B


@pytest.mark.parametrize("name,B", [("highrank", 1030), ("small", 2100), ("digit", 600)])
def test_torn_and_whole_problem_agree(lpd, oracle, dev, name, B):
    """From 512 landmarks on the tridiagonal problem is torn into 2 (4 from 2,048 on) leaves that are solved
    side by side and merged on the device.  Both ways must give the oracle's eigenvalues, the same rank, and
    the same basis-independent W^T W; the rows agree up to rotations within (near-)repeated eigenvalues."""
    from paper_2207_01016_amd import workloads
    wl = workloads.WORKLOADS[name].with_shape(n=max(2 * B, 1000), B=B)
    X = workloads.make_X(wl)
    Lm = X[workloads.landmark_indices(wl)].contiguous()
    out = {}
    for dc in (1, 0):
        lpd.lpd_set_option(lpd.LPD_OPT_WHITEN_DC, dc)
        try:
            out[dc] = lpd.lpd_whiten(Lm.to(dev), wl.gamma)
        finally:
            lpd.lpd_set_option(lpd.LPD_OPT_WHITEN_DC, 1)
    Wo, eo, ro, K = oracle.whiten(Lm.numpy(), wl.gamma, method="lapack")
    for dc in (1, 0):
        W, eig, rank = out[dc]
        assert rank == ro
        assert np.max(np.abs(eig.numpy() - eo)) <= 1e-10 * eo[0], dc
        Wd = W.double().cpu().numpy()[:rank]
        assert np.linalg.norm(Wd @ K @ Wd.T - np.eye(rank)) <= 2e-6 * B, dc
    A1, A0 = out[1][0].double()[:ro], out[0][0].double()[:ro]
    G1, G0 = A1.T @ A1, A0.T @ A0
    assert float((G1 - G0).norm() / G0.norm()) <= 1e-5


def test_whiten_8192_landmarks_three_levels_of_tearing(lpd, dev):
    """8,192 landmarks of the cnn-shaped workload: eight leaves, seven merges.  Checked against a library
    eigenvalue routine on the device (double precision) and by W K W^T = I."""
    from paper_2207_01016_amd import workloads
    wl = workloads.WORKLOADS["cnn"].with_rows(32768)
    X = workloads.make_X(wl, dev)
    Lm = X[workloads.landmark_indices(wl).to(dev)].contiguous()
    W, eig, rank = lpd.lpd_whiten(Lm, wl.gamma)
    assert rank == wl.B
    Ld = Lm.double()
    sq = (Ld * Ld).sum(1)
    K = torch.exp(-wl.gamma * (sq[:, None] + sq[None, :] - 2.0 * Ld @ Ld.T).clamp_(min=0.0))
    K.fill_diagonal_(1.0)
    ref = torch.linalg.eigvalsh(K).flip(0).cpu().numpy()
    assert np.max(np.abs(eig.numpy() - ref)) <= 1e-9 * ref[0]
    Wd = W.double()
    P = Wd @ K @ Wd.T
    assert float((P - torch.eye(wl.B, dtype=torch.float64, device=dev)).norm()) <= 2e-6 * wl.B


@pytest.mark.parametrize("B", [333, 1030, 2050])
def test_upper_triangle_reduction_matches_full_matrix_reduction(lpd, dev, B):
    """The reduction to tridiagonal form reads the upper triangle of the symmetric trailing matrix only (each
    element serves its row and its column).  The same decomposition must come out as from the pass over the
    whole matrix: eigenvalues to rounding, W^T W to fp32 rounding (odd and even sizes: both loaders)."""
    from paper_2207_01016_amd import workloads
    wl = workloads.WORKLOADS["highrank"].with_shape(n=max(2 * B, 1000), B=B)
    X = workloads.make_X(wl)
    Lm = X[workloads.landmark_indices(wl)].contiguous().to(dev)
    out = {}
    for upper in (1, 0):
        lpd.lpd_set_option(lpd.LPD_OPT_WHITEN_UPPER, upper)
        try:
            out[upper] = lpd.lpd_whiten(Lm, wl.gamma)
        finally:
            lpd.lpd_set_option(lpd.LPD_OPT_WHITEN_UPPER, 1)
    (W1, e1, r1), (W0, e0, r0) = out[1], out[0]
    assert r1 == r0 == B
    assert float((e1 - e0).abs().max()) <= 1e-11 * float(e0[0])
    G1, G0 = W1.double().T @ W1.double(), W0.double().T @ W0.double()
    assert float((G1 - G0).norm() / G0.norm()) <= 1e-5
    # and it is deterministic: no atomics, fixed order of the partial sums
    W2, e2, r2 = lpd.lpd_whiten(Lm, wl.gamma)
    assert torch.equal(W2, W1) and torch.equal(e2, e1)
