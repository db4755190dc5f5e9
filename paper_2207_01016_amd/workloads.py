"""Seeded synthetic inputs shaped like the paper's workloads (Section 5, Table 1).

This module only draws numbers: it holds none of the method's arithmetic (no
kernel, no eigendecomposition, no products) and imports neither the HIP
binding nor the CPU oracle, so both sides of a parity test can be fed from it.

The paper's data sets (Adult, Epsilon, SUSY, MNIST-8M, ImageNet features) are
not available offline; the five recipes below stand in for them with the same
shapes, sparsity and value ranges:

  tiny      2,000 x 16     i.i.d. N(0,1); landmarks = first 128 rows
  small     100,000 x 128  10-component Gaussian mixture, means ~ N(0, 4I)
  digit     1,000,000 x 784   ~80 % exact zeros, non-zeros ~ U(0,1)  (MNIST-8M-like)
  cnn       1,280,000 x 2,048 max(0, N(0,1)), rows L2-normalised     (ReLU-feature-like)
  highrank  2,000,000 x 256   i.i.d. N(0,1), B = 16,384

All values are fp32.  X is filled on the requested torch device in row chunks
from one seeded generator; landmark indices, the sweep vector w and labels come
from CPU generators so they do not depend on the device.  Labels are produced
for completeness; nothing on the factor / sweep path reads them.
"""
from __future__ import annotations

import dataclasses
import math

import torch

BASE_SEED = 20220701


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int          # position in the config list (0-based)
    n: int
    d: int
    B: int
    gamma: float
    landmarks: str      # "first" or "random"
    features: str       # recipe key for X
    density: float = 0.2   # share of non-zeros of the "sparse_uniform" recipe (0.2 = the digit-shaped workload)

    def seed(self, what: int) -> int:
        # 0: X, 1: landmark indices, 2: w, 3: labels, 4: row sample
        return BASE_SEED + 10 * (self.index + 1) + what

    def with_rows(self, n: int) -> "Workload":
        """Same recipe with a different number of rows (for test-sized cases)."""
        return dataclasses.replace(self, n=int(n))

    def with_density(self, density: float) -> "Workload":
        """The "sparse_uniform" recipe with another share of non-zeros (for the sparse-route measurements)."""
        return dataclasses.replace(self, density=float(density))

    def with_shape(self, n: int | None = None, d: int | None = None, B: int | None = None) -> "Workload":
        return dataclasses.replace(self, n=int(n or self.n), d=int(d or self.d), B=int(B or self.B))


WORKLOADS = {
    "tiny": Workload("tiny", 0, 2_000, 16, 128, 1.0 / 16, "first", "normal"),
    "small": Workload("small", 1, 100_000, 128, 1_024, 1.0 / 128, "random", "mixture"),
    "digit": Workload("digit", 2, 1_000_000, 784, 4_096, 0.02, "random", "sparse_uniform"),
    "cnn": Workload("cnn", 3, 1_280_000, 2_048, 8_192, 1.0, "random", "relu_normalised"),
    "highrank": Workload("highrank", 4, 2_000_000, 256, 16_384, 1.0 / 256, "random", "normal"),
}

_CHUNK_ROWS = 1 << 16


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_X(wl: Workload, device="cpu") -> torch.Tensor:
    """n x d fp32 feature matrix of the workload's recipe, resident on `device`."""
    device = torch.device(device)
    g = _gen(device, wl.seed(0))
    X = torch.empty((wl.n, wl.d), dtype=torch.float32, device=device)
    if wl.features == "mixture":
        gc = _gen("cpu", wl.seed(0) + 1000)
        means = (2.0 * torch.randn((10, wl.d), generator=gc, dtype=torch.float32)).to(device)
        comp_all = mixture_components(wl).to(device)
    for r0 in range(0, wl.n, _CHUNK_ROWS):
        r1 = min(wl.n, r0 + _CHUNK_ROWS)
        out = X[r0:r1]
        if wl.features == "normal":
            out.normal_(0.0, 1.0, generator=g)
        elif wl.features == "mixture":
            out.normal_(0.0, 1.0, generator=g)
            out += means[comp_all[r0:r1]]
        elif wl.features == "sparse_uniform":
            out.uniform_(0.0, 1.0, generator=g)
            keep = torch.rand(out.shape, generator=g, device=device, dtype=torch.float32) < wl.density
            out *= keep
        elif wl.features == "relu_normalised":
            out.normal_(0.0, 1.0, generator=g)
            out.clamp_(min=0.0)
            nrm = out.norm(dim=1, keepdim=True).clamp_(min=1e-12)
            out /= nrm
        else:
            raise ValueError(wl.features)
    return X


def mixture_components(wl: Workload) -> torch.Tensor:
    """Mixture component (0..9) of every row of the "mixture" recipe."""
    g = _gen("cpu", wl.seed(0) + 2000)
    return torch.randint(0, 10, (wl.n,), generator=g)


def landmark_indices(wl: Workload) -> torch.Tensor:
    """B distinct row indices: the first B rows, or a uniform draw without replacement."""
    if wl.landmarks == "first":
        return torch.arange(wl.B, dtype=torch.int64)
    g = _gen("cpu", wl.seed(1))
    return torch.randperm(wl.n, generator=g)[: wl.B].contiguous()


def make_w(wl: Workload, r: int | None = None) -> torch.Tensor:
    """Sweep vector w ~ N(0, 1/B) (variance 1/B), fp32, on the CPU."""
    g = _gen("cpu", wl.seed(2))
    r = wl.B if r is None else r
    return torch.randn(r, generator=g, dtype=torch.float32) / math.sqrt(wl.B)


def sample_rows(wl: Workload, m: int, include: torch.Tensor | None = None) -> torch.Tensor:
    """Sorted row sample for parity checks: up to m random rows plus `include` (e.g. landmark rows)."""
    g = _gen("cpu", wl.seed(4))
    m = min(m, wl.n)
    idx = torch.randperm(wl.n, generator=g)[:m]
    if include is not None:
        idx = torch.cat([idx, include.to(torch.int64)])
    return torch.unique(idx)  # sorted, distinct


def make_labels(wl: Workload, X: torch.Tensor) -> torch.Tensor:
    """+-1 labels per the workload recipe (not read by the factor or the sweep)."""
    g = _gen("cpu", wl.seed(3))
    dev = X.device
    if wl.name == "tiny" or wl.name == "digit":
        v = torch.randn(wl.d, generator=g, dtype=torch.float32).to(dev)
        s = X @ v
        if wl.name == "digit":
            s = s - s.median()
        y = torch.where(s >= 0, 1.0, -1.0)
    elif wl.name == "small":
        y = torch.where(mixture_components(wl) % 2 == 0, 1.0, -1.0).to(dev)
    elif wl.name == "cnn":
        cls = torch.randint(0, 1000, (X.shape[0],), generator=g)
        y = torch.where(cls == 0, 1.0, -1.0).to(dev)
    else:
        A = torch.randn((wl.d, 16), generator=g, dtype=torch.float32).to(dev) / math.sqrt(wl.d)
        v = torch.randn(16, generator=g, dtype=torch.float32).to(dev)
        y = torch.where(torch.tanh(X @ A) @ v >= 0, 1.0, -1.0)
    return y.to(torch.float32)


def to_csr(X: torch.Tensor):
    """The nonzeros of a dense matrix in compressed-row form: (row_ptr int64 [n+1], col_idx int32, values float32),
    on X's device. A change of storage format only; the entries are X's."""
    nz = X != 0
    counts = nz.sum(dim=1, dtype=torch.int64)
    row_ptr = torch.zeros(X.shape[0] + 1, dtype=torch.int64, device=X.device)
    row_ptr[1:] = torch.cumsum(counts, dim=0)
    idx = nz.nonzero(as_tuple=False)            # row-major order: rows ascending, columns ascending within a row
    col_idx = idx[:, 1].to(torch.int32).contiguous()
    values = X[nz].contiguous()
    return row_ptr, col_idx, values
