"""GPU parity on inputs that stress the fp32 evaluation of the Gaussian kernel's squared distance (Section 5).

The device expands ||x - l||^2 into norms and an inner product in fp32.  The cases here are the ones that
expansion can break on, each against the double-precision oracle (direct differences) with one shared W:
features with a large common offset, raw pixel-scale values with the paper's tiny kernel parameter, and data
where a share of the kernel arguments underflows fp32.  Tolerances as everywhere: factor 1e-4, margins 1e-5.
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


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch.device("cuda:0")


@pytest.fixture(scope="module")
def lpd():
    from paper_2207_01016_amd import lpd as mod
    mod.lib()
    return mod


def _offset_features(seed, n, d):
    g = torch.Generator().manual_seed(seed)
    return 30.0 + torch.randn((n, d), generator=g)


def _pixels(seed, n, d):
    g = torch.Generator().manual_seed(seed)
    mask = torch.rand((n, d), generator=g) < 0.2
    return torch.floor(torch.rand((n, d), generator=g) * 256.0).clamp_(0, 255) * mask


def _two_far_clusters(seed, n, d):
    g = torch.Generator().manual_seed(seed)
    X = torch.randn((n, d), generator=g)
    X[torch.rand(n, generator=g) < 0.5, 0] += 60.0
    return X


CASES = {
    # name: (generator, n, d, B, gamma)
    "offset_mean30_std1": (_offset_features, 3000, 128, 512, 1.0 / 128),
    "offset_unaligned_d": (_offset_features, 1500, 30, 200, 1.0 / 30),          # element-wise loader
    "raw_pixels_gamma_2^-22": (_pixels, 2500, 784, 600, 2.0 ** -22),            # Table 1, MNIST-8M setting
    "far_clusters_underflow": (_two_far_clusters, 3000, 32, 400, 1.0 / 32),     # gamma dist ~ 115 across clusters
}


def _run_case(lpd, oracle, dev, name):
    gen, n, d, B, gamma = CASES[name]
    Xh = gen(20220701 + len(name), n, d).to(torch.float32)
    idx = torch.randperm(n, generator=torch.Generator().manual_seed(5))[:B]
    Lh = Xh[idx].contiguous()
    Wd, eig, rank, K = oracle.whiten(Lh.numpy(), gamma)
    W32 = torch.from_numpy(Wd.astype(np.float32))
    X, L = Xh.to(dev), Lh.to(dev)
    Z = torch.empty((n, B), dtype=torch.float32, device=dev)
    ws = lpd.alloc_workspace(n, d, B, dev)
    lpd.lpd_kernel_block(X, L, gamma, Z, ws)
    G = torch.full((n, B), float("nan"), dtype=torch.float32, device=dev)
    lpd.lpd_nystrom_factor(X, L, gamma, W32.to(dev), G, ws, r=rank)
    w = (torch.randn(B, generator=torch.Generator().manual_seed(9)) / B ** 0.5).to(dev)
    m = lpd.lpd_margins(G, w, r=rank)
    torch.cuda.synchronize()
    Z_ref = oracle.kernel_block(Xh.numpy(), Lh.numpy(), gamma)
    G_ref = oracle.nystrom_factor(Xh.numpy(), Lh.numpy(), gamma, W32.numpy(), r=rank)
    Gh = G.cpu().numpy()
    m_ref = oracle.margins(Gh, w.cpu().numpy(), r=rank)
    return {"Z": relfro(Z.cpu().numpy(), Z_ref), "G": relfro(Gh[:, :rank], G_ref), "m": relfro(m.cpu().numpy(), m_ref),
            "rank": rank, "Zh": Z.cpu().numpy(), "Z_ref": Z_ref, "cond": float(eig[0] / eig[rank - 1]),
            "tail_zero": bool(np.all(Gh[:, rank:] == 0))}


@pytest.mark.parametrize("name", list(CASES))
def test_factor_and_margins_on_hard_input_domains(lpd, oracle, dev, name):
    out = _run_case(lpd, oracle, dev, name)
    print(f"{name}: relF(Z)={out['Z']:.2e} relF(G)={out['G']:.2e} relF(m)={out['m']:.2e} rank={out['rank']} "
          f"cond={out['cond']:.1e}")
    assert out["tail_zero"]
    assert out["Z"] <= 1e-5
    assert out["G"] <= TOL_G
    assert out["m"] <= TOL_M
    assert np.all(out["Zh"] >= 0.0) and np.all(out["Zh"] <= 1.0)


def test_underflowing_kernel_values_are_exact_zeros_or_tiny(lpd, oracle, dev):
    # across the two clusters gamma ||x - l||^2 is about 115: fp32 gives 0 where double gives < 1e-38
    out = _run_case(lpd, oracle, dev, "far_clusters_underflow")
    far = out["Z_ref"] < 1e-38
    assert far.mean() > 0.3                                  # a real share of the pairs
    assert np.all(out["Zh"][far] <= 1.2e-38)
    near = out["Z_ref"] > 1e-3
    assert np.max(np.abs(out["Zh"][near] / out["Z_ref"][near] - 1.0)) <= 1e-4


def test_kernel_block_does_not_depend_on_a_common_offset(lpd, oracle, dev):
    # a distance does not change when every point moves by the same vector: the block for features shifted
    # by 1000 must still match the oracle (whose direct differences are exact for such a shift)
    g = torch.Generator().manual_seed(77)
    n, d, B, gamma = 700, 64, 256, 1.0 / 64
    base = torch.randn((n, d), generator=g)
    for shift in (0.0, 100.0, 1000.0):
        Xh = (base + shift).to(torch.float32)
        Lh = Xh[:B].contiguous()
        Z = torch.empty((n, B), dtype=torch.float32, device=dev)
        lpd.lpd_kernel_block(Xh.to(dev), Lh.to(dev), gamma, Z, lpd.alloc_workspace(n, d, B, dev))
        torch.cuda.synchronize()
        ref = oracle.kernel_block(Xh.numpy(), Lh.numpy(), gamma)
        err = relfro(Z.cpu().numpy(), ref)
        print(f"shift {shift}: relF(Z) = {err:.2e}")
        assert err <= 1e-5
