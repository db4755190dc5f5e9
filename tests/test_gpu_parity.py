"""GPU parity: the HIP path, called through the C ABI, against the double-precision CPU oracle.

Tolerances (relative Frobenius error over the compared rows):
    factor G   <= 1e-4      margins  <= 1e-5
The factor is compared with ONE shared W (the fp32 W handed to the GPU is the W the oracle uses):
the eigenvector basis is a convention, the product G = Z W^T is not.  Margins are a function of G:
the oracle sweeps the same fp32 G buffer the GPU kernel read.
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
    mod.lib()   # fails loudly when the HIP library is not built
    return mod


@pytest.fixture(scope="module")
def wls():
    from paper_2207_01016_amd import workloads
    return workloads


def _prepare(lpd, wls, wl, dev):
    X = wls.make_X(wl, dev)
    idx = wls.landmark_indices(wl)
    L = X[idx.to(dev)].contiguous()
    W, eig, rank = lpd.lpd_whiten_host(L.cpu(), wl.gamma)
    return X, idx, L, W, eig, rank


def _factor(lpd, X, L, gamma, W, rank, ws_bytes=None):
    n, d = X.shape
    B = L.shape[0]
    G = torch.full((n, B), float("nan"), dtype=torch.float32, device=X.device)
    ws = lpd.alloc_workspace(n, d, B, X.device, ws_bytes)
    lpd.lpd_nystrom_factor(X, L, gamma, W.to(X.device), G, ws, r=rank)
    torch.cuda.synchronize()
    return G


# ---------------------------------------------------------------- kernel block (GEMM-1 + exp epilogue)

@pytest.mark.parametrize("n,d,B,gamma", [
    (300, 20, 70, 0.05),       # nothing a multiple of a tile, d % 4 == 0
    (257, 19, 33, 0.07),       # d % 4 != 0: element-wise loader
    (1, 5, 1, 0.3),
    (513, 128, 260, 1.0 / 128),
    (130, 1, 129, 0.5),
])
@pytest.mark.parametrize("tile", ["128x128", "256x128", "256x256", "64x128"])
def test_kernel_block_matches_oracle(lpd, oracle, dev, n, d, B, gamma, tile):
    g = torch.Generator().manual_seed(1000 + n + d + B)
    X = torch.randn((n, d), generator=g).to(dev)
    L = torch.cat([X[: min(B, n) // 2].cpu(), torch.randn((B - min(B, n) // 2, d), generator=g)]).to(dev)
    Z = torch.full((n, B), float("nan"), dtype=torch.float32, device=dev)
    ws = torch.empty(4 * (n + B + d) + 3 * 256, dtype=torch.uint8, device=dev)     # three parts, each rounded up to 256
    lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, lpd.GEMM_TILES[tile])
    try:
        lpd.lpd_kernel_block(X, L, gamma, Z, ws)
        torch.cuda.synchronize()
    finally:
        lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, 0)
    ref = oracle.kernel_block(X.cpu().numpy(), L.cpu().numpy(), gamma)
    Zh = Z.cpu().numpy()
    assert np.all(np.isfinite(Zh))
    assert np.all(Zh <= 1.0) and np.all(Zh >= 0.0)
    assert relfro(Zh, ref) <= 1e-5
    assert np.max(np.abs(Zh - ref)) <= 2e-5


def test_kernel_block_strided_operands(lpd, oracle, dev):
    """Leading dimensions larger than the rows, including ones that break 16-byte alignment."""
    g = torch.Generator().manual_seed(7)
    for ldx, ldl, ldz in [(24, 28, 80), (21, 23, 71)]:
        Xs = torch.randn((200, ldx), generator=g).to(dev)
        Ls = torch.randn((70, ldl), generator=g).to(dev)
        Zs = torch.zeros((200, ldz), dtype=torch.float32, device=dev)
        ws = torch.empty(4096, dtype=torch.uint8, device=dev)
        lpd.lpd_kernel_block(Xs[:, :20], Ls[:, :20], 0.04, Zs[:, :70], ws)
        torch.cuda.synchronize()
        ref = oracle.kernel_block(Xs[:, :20].cpu().numpy(), Ls[:, :20].cpu().numpy(), 0.04)
        assert relfro(Zs[:, :70].cpu().numpy(), ref) <= 1e-5
        assert torch.all(Zs[:, 70:] == 0)           # padding columns untouched


# ---------------------------------------------------------------- factor on the workload recipes

def test_factor_tiny_all_rows(lpd, wls, oracle, dev):
    wl = wls.WORKLOADS["tiny"]
    X, idx, L, W, eig, rank = _prepare(lpd, wls, wl, dev)
    assert rank == wl.B
    G = _factor(lpd, X, L, wl.gamma, W, rank)
    ref = oracle.nystrom_factor(X.cpu().numpy(), L.cpu().numpy(), wl.gamma, W.numpy())
    Gh = G.cpu().numpy()
    assert relfro(Gh, ref) <= TOL_G
    # projection bound: ||g_i||^2 <= 1 on every row, = 1 on landmark rows
    sq = (Gh.astype(np.float64) ** 2).sum(axis=1)
    assert np.all(sq <= 1.0 + 1e-4)
    assert np.allclose(sq[idx.numpy()], 1.0, atol=1e-4)
    # G_L G_L^T reproduces K_LL
    GL = Gh[idx.numpy()].astype(np.float64)
    K = oracle.kernel_block(L.cpu().numpy(), L.cpu().numpy(), wl.gamma)
    assert relfro(GL @ GL.T, K) <= 1e-4


@pytest.mark.parametrize("name,n,B", [
    ("small", 20_000, 1024),
    ("digit", 5_000, 700),
    ("cnn", 3_000, 520),
    ("highrank", 6_000, 1111),
])
@pytest.mark.parametrize("tile", ["128x128", "256x256"])
def test_factor_scaled_workloads_sampled_rows(lpd, wls, oracle, dev, name, n, B, tile):
    """Recipe-shaped inputs with fewer rows / landmarks; oracle on a row sample that includes landmarks."""
    wl = wls.WORKLOADS[name].with_shape(n=n, B=B)
    X, idx, L, W, eig, rank = _prepare(lpd, wls, wl, dev)
    lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, lpd.GEMM_TILES[tile])
    try:
        # a workspace of three 256-row panels' worth forces several panels and a ragged last one
        _, mn = lpd.lpd_nystrom_factor_workspace(n, wl.d, B)
        G = _factor(lpd, X, L, wl.gamma, W, rank, ws_bytes=mn * 3)
    finally:
        lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, 0)
    rows = wls.sample_rows(wl, 600, include=idx[:64])
    ref = oracle.nystrom_factor(X[rows.to(dev)].cpu().numpy(), L.cpu().numpy(), wl.gamma, W.numpy(), r=rank)
    Gs = G[rows.to(dev)].cpu().numpy()
    assert np.all(np.isfinite(Gs))
    assert relfro(Gs[:, :rank], ref) <= TOL_G
    sq = (G.double() ** 2).sum(dim=1)
    assert float(sq.max()) <= 1.0 + 1e-4
    assert torch.allclose(sq[idx.to(dev)], torch.ones(B, dtype=torch.float64, device=dev), atol=1e-4)


def test_factor_rank_deficient_zero_fills(lpd, wls, oracle, dev):
    """Duplicated landmarks: dropped components give r < B; columns r..B-1 of G are exact zeros."""
    wl = wls.WORKLOADS["tiny"].with_shape(n=900, B=150)
    X = wls.make_X(wl, dev)
    L = torch.cat([X[:140], X[5:15]]).contiguous()         # 10 duplicates
    W, eig, rank = lpd.lpd_whiten_host(L.cpu(), wl.gamma)
    assert rank == 140
    G = _factor(lpd, X, L, wl.gamma, W, rank)
    ref = oracle.nystrom_factor(X.cpu().numpy(), L.cpu().numpy(), wl.gamma, W.numpy(), r=rank)
    Gh = G.cpu().numpy()
    assert relfro(Gh[:, :rank], ref) <= TOL_G
    assert np.all(Gh[:, rank:] == 0.0)
    # r = 0 writes only zeros
    G0 = _factor(lpd, X, L, wl.gamma, W, 0)
    assert torch.all(G0 == 0)


def test_factor_gamma_zero(lpd, wls, dev):
    wl = wls.WORKLOADS["tiny"].with_shape(n=500, B=40)
    X = wls.make_X(wl, dev)
    L = X[:40].contiguous()
    W, eig, rank = lpd.lpd_whiten_host(L.cpu(), 0.0)
    assert rank == 1
    G = _factor(lpd, X, L, 0.0, W, rank)
    assert torch.allclose(G[:, 0], torch.ones(500, device=dev), atol=1e-6)
    assert torch.all(G[:, 1:] == 0)


def test_factor_is_deterministic_and_tile_independent(lpd, wls, dev):
    wl = wls.WORKLOADS["small"].with_shape(n=3000, B=384)
    X, idx, L, W, eig, rank = _prepare(lpd, wls, wl, dev)
    outs = {}
    for tile in ["128x128", "256x128", "256x256", "64x128"]:
        lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, lpd.GEMM_TILES[tile])
        try:
            a = _factor(lpd, X, L, wl.gamma, W, rank)
            b = _factor(lpd, X, L, wl.gamma, W, rank)
        finally:
            lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, 0)
        assert torch.equal(a, b), tile                 # bitwise: no atomics, fixed summation order
        outs[tile] = a
    ref = outs["128x128"].double()
    for tile, a in outs.items():
        assert float((a.double() - ref).norm() / ref.norm()) <= 1e-6, tile


def test_factor_profiled_matches_plain(lpd, wls, dev):
    for B in (320, 256):
        wl = wls.WORKLOADS["small"].with_shape(n=5000, B=B)
        X, idx, L, W, eig, rank = _prepare(lpd, wls, wl, dev)
        G1 = _factor(lpd, X, L, wl.gamma, W, rank)
        G2 = torch.empty_like(G1)
        ws = lpd.alloc_workspace(wl.n, wl.d, wl.B, dev)
        prof = lpd.lpd_nystrom_factor_profiled(X, L, wl.gamma, W.to(dev), G2, ws, r=rank)
        assert torch.equal(G1, G2)
        if B > 256:     # panel schedule: one kernel-block launch per whitening launch
            assert prof.launches_whiten == prof.launches_kernel_block >= 1 and prof.launches_norms == 3
            assert prof.ms_whiten > 0 and prof.ms_kernel_block > 0
        else:           # one launch does it all and is booked under the whitening product
            assert (prof.launches_whiten, prof.launches_kernel_block, prof.launches_norms) == (1, 0, 0)
            assert prof.ms_whiten > 0 and prof.panel_rows == wl.n


@pytest.mark.parametrize("chunk_rows,pinned,pad", [
    (3000, True, 0),       # 7 chunks, ragged last one, both buffers reused several times
    (512, True, 4),        # many small chunks into a padded host matrix
    (0, True, 0),          # the suggested chunk size (one chunk here)
    (7000, False, 0),      # pageable host memory: same result, copies just do not overlap
])
def test_streaming_factor_matches_device_factor_and_oracle(lpd, wls, oracle, dev, chunk_rows, pinned, pad):
    wl = wls.WORKLOADS["small"].with_shape(n=20000, B=512)
    X, idx, L, W, eig, rank = _prepare(lpd, wls, wl, dev)
    G_dev = _factor(lpd, X, L, wl.gamma, W, rank).cpu()
    host = torch.full((wl.n, wl.B + pad), float("nan"), dtype=torch.float32, pin_memory=pinned)
    G_host = lpd.lpd_nystrom_factor_to_host(X, L, wl.gamma, W.to(dev), host[:, :wl.B], chunk_rows=chunk_rows, r=rank)
    assert G_host.data_ptr() == host.data_ptr()
    # a row of G depends on its own row of X only, and the arithmetic per row is the same in
    # both schedules, so the streamed factor equals the resident one
    assert relfro(G_host.numpy(), G_dev.numpy()) <= 1e-6
    if pad:
        assert torch.isnan(host[:, wl.B:]).all()                     # padding columns untouched
    rows = wls.sample_rows(wl, 300, include=idx[:32])
    ref = oracle.nystrom_factor(X[rows.to(dev)].cpu().numpy(), L.cpu().numpy(), wl.gamma, W.numpy(), r=rank)
    assert relfro(G_host[rows].numpy()[:, :rank], ref) <= TOL_G
    assert not G_host[:, rank:].any()


def test_streaming_factor_zero_fills_dropped_components(lpd, wls, dev):
    """r < B: the host matrix gets exact zeros in columns r..B-1, as the resident factor does."""
    wl = wls.WORKLOADS["tiny"].with_shape(n=5000, B=160)
    X, idx, L, W, eig, rank = _prepare(lpd, wls, wl, dev)
    r = rank - 37
    G_dev = _factor(lpd, X, L, wl.gamma, W, r).cpu()
    host = torch.full((wl.n, wl.B), float("nan"), dtype=torch.float32, pin_memory=True)
    lpd.lpd_nystrom_factor_to_host(X, L, wl.gamma, W.to(dev), host, chunk_rows=1024, r=r)
    assert torch.equal(host[:, r:], torch.zeros((wl.n, wl.B - r)))
    assert relfro(host.numpy(), G_dev.numpy()) <= 1e-6


@pytest.mark.parametrize("tile", ["128x128", "256x128", "256x256", "64x128"])
@pytest.mark.parametrize("n,d,B", [
    (700, 16, 272),        # one k-tile in the kernel block, 17 in the whitening product (odd: the peeled last step)
    (300, 48, 288),        # 3 and 18 k-tiles (even)
    (513, 36, 340),        # a partial last k-tile in both products
    (260, 32, 260),        # 2 k-tiles and a partial one
    (1100, 64, 1040),      # 65 k-tiles, several tiles of every shape, ragged edges in both directions
    (256, 16, 16),         # a single k-tile in the whitening product
    (300, 16, 48),         # 3 k-tiles
])
def test_main_loop_schedules_agree_bit_for_bit(lpd, oracle, dev, n, d, B, tile):
    """The plain schedule, the pipelined one and the one with two staged tiles visit k in the same order."""
    g = torch.Generator().manual_seed(31 + n + B)
    X = torch.randn((n, d), generator=g).to(dev)
    L = torch.randn((B, d), generator=g).to(dev)
    W = (torch.randn((B, B), generator=g) / B ** 0.5).to(dev)
    gamma = 0.5 / d
    ws = lpd.alloc_workspace(n, d, B, dev)
    out = []
    lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, lpd.GEMM_TILES[tile])
    try:
        for schedule in (0, 1, 2):
            lpd.lpd_set_option(lpd.LPD_OPT_GEMM_PIPELINE, schedule)
            G = torch.full((n, B), float("nan"), device=dev)
            lpd.lpd_nystrom_factor(X, L, gamma, W, G, ws)
            torch.cuda.synchronize()
            out.append(G.cpu().numpy())
    finally:
        lpd.lpd_set_option(lpd.LPD_OPT_GEMM_PIPELINE, lpd.GEMM_PIPELINE_DEFAULT)
        lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, 0)
    ref = oracle.nystrom_factor(X.cpu().numpy(), L.cpu().numpy(), gamma, W.cpu().numpy())
    assert relfro(out[0], ref) <= 1e-4
    assert np.array_equal(out[0], out[1]) and np.array_equal(out[0], out[2])


@pytest.mark.parametrize("k", [5, 9, 32, 33, 64])
@pytest.mark.parametrize("n,r", [
    (300, 16), (300, 32), (257, 48), (300, 64),     # 1 to 4 k-tiles: fewer than the staged tiles of the schedule
    (513, 80), (300, 96), (300, 112), (300, 128),   # every remainder of the loop that is unrolled four times
    (700, 144), (1000, 1040),                       # several workgroups, a ragged last one
    (300, 100),                                     # a partial last k-tile
])
def test_narrow_tile_schedules_agree_bit_for_bit(lpd, oracle, dev, n, r, k):
    """5 to 64 weight vectors take the narrow tiles, whose default schedule keeps four k-tiles in flight and
    requests them in pairs; the plain and the one-tile schedules visit k in the same order."""
    g = torch.Generator().manual_seed(77 + n + r + k)
    G = torch.randn((n, r), generator=g).to(dev)
    Ws = torch.randn((k, r), generator=g).to(dev)
    out = []
    try:
        for schedule in (0, 1, 2):
            lpd.lpd_set_option(lpd.LPD_OPT_GEMM_PIPELINE, schedule)
            M = torch.full((n, k), float("nan"), device=dev)
            lpd.lpd_margins_multi(G, Ws, M)
            torch.cuda.synchronize()
            out.append(M.cpu().numpy())
    finally:
        lpd.lpd_set_option(lpd.LPD_OPT_GEMM_PIPELINE, lpd.GEMM_PIPELINE_DEFAULT)
    ref = np.stack([oracle.margins(G.cpu().numpy(), Ws[q].cpu().numpy(), r) for q in range(k)], axis=1)
    assert relfro(out[0], ref) <= 1e-5
    assert np.array_equal(out[0], out[1]) and np.array_equal(out[0], out[2])


@pytest.mark.parametrize("n,d,B,r,gamma", [
    (2000, 16, 128, 128, 1.0 / 16),     # the tiny workload's shape
    (1, 7, 1, 1, 0.3),
    (33, 19, 31, 31, 0.1),              # nothing a multiple of 4: element-wise loads
    (700, 1024, 256, 256, 1.0 / 1024),  # the largest shape the one-launch kernel takes
    (257, 64, 200, 137, 1.0 / 64),      # rank below B: zero-filled columns
    (100, 12, 64, 0, 0.2),              # no component kept
    (95, 0, 40, 40, 0.5),               # no features: all points coincide, Z = 1
    (300, 20, 96, 96, 0.0),             # gamma = 0: Z = 1
    (64, 33, 255, 255, 1.5),            # gamma dist ~ 100: kernel values underflow for most pairs
])
def test_one_launch_factor_for_few_landmarks(lpd, oracle, dev, n, d, B, r, gamma):
    """B <= 256: step 1d as one kernel with its rows of Z in LDS, against the oracle and against the panel
    schedule, on the shapes that bound it."""
    g = torch.Generator().manual_seed(n * 7 + d * 3 + B)
    X = 3.0 + torch.randn((n, d), generator=g)                       # an offset: the kernel shifts its origin
    L = torch.cat([X[: min(n, B) // 2], 3.0 + torch.randn((B - min(n, B) // 2, d), generator=g)])
    W = torch.randn((B, B), generator=g) / B ** 0.5
    Xd, Ld, Wd = X.to(dev), L.to(dev), W.to(dev)
    ws = lpd.alloc_workspace(n, d, B, dev)
    out = []
    for small in (1, 0):
        G = torch.full((n, B + 3), float("nan"), device=dev)         # padded rows: ldg > B, not a multiple of 4
        lpd.lpd_set_option(lpd.LPD_OPT_SMALL_PATH, small)
        try:
            lpd.lpd_nystrom_factor(Xd, Ld, gamma, Wd, G[:, :B], ws, r=r)
            torch.cuda.synchronize()
        finally:
            lpd.lpd_set_option(lpd.LPD_OPT_SMALL_PATH, 1)
        assert torch.isnan(G[:, B:]).all()
        out.append(G[:, :B].cpu().numpy())
    ref = oracle.nystrom_factor(X.numpy(), L.numpy(), gamma, W.numpy(), r=r)
    for Gh in out:
        assert np.all(np.isfinite(Gh)) and not Gh[:, r:].any()
        if r:
            assert relfro(Gh[:, :r], ref) <= TOL_G
    assert relfro(out[0], out[1]) <= 2e-5 or r == 0


def test_factor_zero_sizes(lpd, dev):
    ws = torch.empty(1 << 16, dtype=torch.uint8, device=dev)
    X = torch.zeros((0, 8), device=dev)
    L = torch.zeros((4, 8), device=dev)
    W = torch.zeros((4, 4), device=dev)
    G = torch.zeros((0, 4), device=dev)
    lpd.lpd_nystrom_factor(X, L, 0.5, W, G, ws)
    torch.cuda.synchronize()


# ---------------------------------------------------------------- margins (GEMV sweep)

@pytest.mark.parametrize("n,r,ld", [
    (2000, 128, 128),      # tiny's shape: 32 lanes per row
    (777, 1024, 1024),     # 64 lanes per row
    (1000, 64, 64),        # 16 lanes per row
    (513, 20, 20),         # 8 lanes per row
    (300, 1000, 1040),     # ld > r, r % 4 == 0
    (300, 1001, 1044),     # ragged tail columns
    (301, 517, 517),       # ld % 4 != 0: scalar loader
    (5, 3, 3),
    (64, 4100, 4100),
])
def test_margins_match_oracle(lpd, oracle, dev, n, r, ld):
    g = torch.Generator().manual_seed(n * 31 + r)
    Gfull = torch.randn((n, ld), generator=g).to(dev)
    w = (torch.randn(r, generator=g) / r ** 0.5).to(dev)
    m = lpd.lpd_margins(Gfull[:, :r] if ld > r else Gfull, w, r=r)
    torch.cuda.synchronize()
    ref = oracle.margins(Gfull.cpu().numpy(), w.cpu().numpy(), r=r)
    assert relfro(m.cpu().numpy(), ref) <= TOL_M


def test_margins_unit_vector_and_rows(lpd, oracle, dev):
    g = torch.Generator().manual_seed(99)
    G = torch.randn((1500, 300), generator=g).to(dev)
    e = torch.zeros(300, device=dev)
    e[123] = 1.0
    assert torch.equal(lpd.lpd_margins(G, e), G[:, 123])
    w = torch.randn(300, generator=g).to(dev)
    rows = torch.randperm(1500, generator=g)[:400].to(dev)
    mr = lpd.lpd_margins_rows(G, rows, w)
    mall = lpd.lpd_margins(G, w)
    torch.cuda.synchronize()
    assert torch.equal(mr, mall[rows])
    ref = oracle.margins(G[rows].cpu().numpy(), w.cpu().numpy())
    assert relfro(mr.cpu().numpy(), ref) <= TOL_M
    # indices outside [0, n) are caught on the device: NaN for that entry, nothing read out of bounds,
    # the valid entries around it unaffected
    bad = torch.tensor([0, 1500, 7, -1, 1499, 1 << 40], device=dev)
    mb = lpd.lpd_margins_rows(G, bad, w)
    torch.cuda.synchronize()
    assert torch.equal(torch.isnan(mb).cpu(), torch.tensor([False, True, False, True, False, True]))
    assert torch.equal(mb[[0, 2, 4]], mall[[0, 7, 1499]])


def test_row_list_sweep_and_solver_replay_from_a_hip_graph(lpd, oracle, dev):
    """The row-list sweep and the solver take their index arrays from device memory and check them there, so the
    binding only enqueues them: both can be recorded into a HIP graph and replayed."""
    g = torch.Generator().manual_seed(123)
    n, r = 4000, 520
    G = (torch.randn((n, r), generator=g) / r ** 0.5).to(dev)
    w = torch.randn(r, generator=g).to(dev)
    rows = torch.randperm(n, generator=g)[:900].to(dev)
    gsq = lpd.lpd_row_sqnorms(G)
    prob_off = torch.tensor([0, 500, 900], device=dev)
    y = torch.where(torch.randn(900, generator=g) > 0, 1.0, -1.0).to(dev)
    C = torch.tensor([1.0, 0.5], device=dev)
    ws = torch.empty(lpd.lpd_cd_solve_workspace(2, 900), dtype=torch.uint8, device=dev)

    def run(m, alpha, wout, status):
        lpd.lpd_margins_rows(G, rows, w, m)
        alpha.copy_(alpha0)
        lpd.lpd_cd_solve(G, gsq, prob_off, rows, y, C, alpha, wout, eps=1e-3, max_epochs=50, workspace=ws,
                         validate=False, status=status)

    alpha0 = torch.zeros(900, device=dev)
    bufs0 = (torch.empty(900, device=dev), torch.empty(900, device=dev), torch.empty((2, r), device=dev),
             torch.zeros((2, 32), dtype=torch.uint8, device=dev))
    run(*bufs0)
    torch.cuda.synchronize()
    ref = oracle.margins(G[rows].cpu().numpy(), w.cpu().numpy())
    assert relfro(bufs0[0].cpu().numpy(), ref) <= TOL_M
    bufs1 = tuple(torch.zeros_like(b) for b in bufs0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(*bufs1)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(*bufs1)
    for rep in range(3):
        for b in bufs1[:3]:
            b.fill_(float("nan"))
        junk = (G @ G.T[:, :64]).sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(bufs1, bufs0)), rep
        assert bool(torch.isfinite(junk))


def test_margins_on_factor_output_tiny(lpd, wls, oracle, dev):
    """Whole path on the tiny workload: factor, then sweep; plus the chained error as information."""
    wl = wls.WORKLOADS["tiny"]
    X, idx, L, W, eig, rank = _prepare(lpd, wls, wl, dev)
    G = _factor(lpd, X, L, wl.gamma, W, rank)
    w = wls.make_w(wl).to(dev)
    m = lpd.lpd_margins(G, w, r=rank)
    torch.cuda.synchronize()
    ref = oracle.margins(G.cpu().numpy(), w.cpu().numpy(), r=rank)
    assert relfro(m.cpu().numpy(), ref) <= TOL_M
    # w = G_a^T for a landmark row returns the kernel column Z[:, a]
    a = 17
    ma = lpd.lpd_margins(G, G[idx[a]].contiguous(), r=rank)
    Z = oracle.kernel_block(X.cpu().numpy(), L.cpu().numpy(), wl.gamma)
    assert np.max(np.abs(ma.cpu().numpy() - Z[:, a])) <= 2e-4
    chained = oracle.margins_f64(oracle.nystrom_factor(X.cpu().numpy(), L.cpu().numpy(), wl.gamma, W.numpy()),
                                 w.cpu().numpy().astype(np.float64))
    print("chained rel error (oracle G -> oracle m vs GPU G -> GPU m):", relfro(m.cpu().numpy(), chained))


@pytest.mark.parametrize("n,r,ld,k", [(700, 300, 300, 1), (1000, 1024, 1024, 3), (513, 1001, 1004, 8),
                                       (301, 517, 517, 5), (2000, 640, 640, 9), (900, 260, 264, 150),
                                       # five to eight vectors: MFMA tile when 16-byte loads apply, else the plain kernel
                                       (1000, 1024, 1024, 5), (700, 640, 644, 8), (900, 512, 512, 4), (640, 250, 252, 7),
                                       # the narrow MFMA tiles (up to 32 and up to 64 vectors), aligned and not,
                                       # rows not a multiple of the tile, and the first count past them
                                       (1500, 512, 512, 16), (777, 333, 333, 32), (1030, 400, 400, 33),
                                       (600, 1024, 1028, 64), (515, 256, 256, 65)])
def test_margins_multi_match_oracle(lpd, oracle, dev, n, r, ld, k):
    g = torch.Generator().manual_seed(n + r + k)
    Gfull = torch.randn((n, ld), generator=g).to(dev)
    Ws = (torch.randn((k, ld), generator=g) / r ** 0.5).to(dev)
    M = torch.full((n, k), float("nan"), dtype=torch.float32, device=dev)
    lpd.lpd_margins_multi(Gfull, Ws, M, r=r)
    torch.cuda.synchronize()
    Gh, Wh = Gfull.cpu().numpy(), Ws.cpu().numpy()
    for q in range(k):
        ref = oracle.margins(Gh, Wh[q], r=r)
        assert relfro(M[:, q].cpu().numpy(), ref) <= TOL_M, q
    if k <= 8:
        # the single-vector sweep of the same row gives the same bits only up to summation order: compare loosely
        m0 = lpd.lpd_margins(Gfull, Ws[0].contiguous(), r=r)
        assert float((m0.double() - M[:, 0].double()).norm() / m0.double().norm()) <= 1e-6


def test_factor_sweep_and_predict_replay_from_a_hip_graph(lpd, wls, dev):
    """The device entry points only enqueue kernels on the caller's stream (no allocation, no memset, no wait), so
    they can be recorded into a HIP graph.  Replays, with eager work and synchronisations between them, must give
    the eager result bit for bit every time."""
    wl = wls.WORKLOADS["small"].with_shape(n=9000, B=384)
    X, idx, L, W, eig, rank = _prepare(lpd, wls, wl, dev)
    Wd = W.to(dev)
    w = wls.make_w(wl).to(dev)
    _, mn = lpd.lpd_nystrom_factor_workspace(wl.n, wl.d, wl.B)
    ws = lpd.alloc_workspace(wl.n, wl.d, wl.B, dev, mn * 5)          # several panels per call
    V = lpd.lpd_fold_weights(Wd, torch.randn((3, rank), generator=torch.Generator().manual_seed(1)).to(dev), r=rank)

    def run(G, m, F):
        lpd.lpd_nystrom_factor(X, L, wl.gamma, Wd, G, ws, r=rank)
        lpd.lpd_margins(G, w, m, r=rank)
        lpd.lpd_predict(X, L, wl.gamma, V, F, ws)

    G0, m0, F0 = (torch.empty((wl.n, wl.B), device=dev), torch.empty(wl.n, device=dev), torch.empty((wl.n, 3), device=dev))
    run(G0, m0, F0)
    torch.cuda.synchronize()
    G1, m1, F1 = torch.zeros_like(G0), torch.zeros_like(m0), torch.zeros_like(F0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(G1, m1, F1)                                              # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(G1, m1, F1)
    for rep in range(3):
        G1.fill_(float("nan")); m1.fill_(float("nan")); F1.fill_(float("nan"))
        junk = (X @ X.T[:, :64]).sum()                               # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(G1, G0) and torch.equal(m1, m0) and torch.equal(F1, F0), rep
        assert bool(torch.isfinite(junk))
