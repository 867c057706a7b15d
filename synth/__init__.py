"""Seeded synthetic gradients shaped like the paper's workloads.

This module only draws inputs.  It holds none of the method's arithmetic and is the one piece
shared by the CPU oracle's tests and the HIP path's tests / benchmark: both sides are handed
the very same bits.

The paper trains linear models (Section 6.1) and CNNs (Sections 6.2-6.3) on data sets that
are not available here; these generators stand in for them with the same vector lengths and
plausible value distributions (per-layer variances spread over decades for CNN gradients,
heavy tails, outliers).  Every generator works on any torch device and is a pure function of
(config, iteration, worker).
"""
from __future__ import annotations

import dataclasses
import math

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    P: int            # workers
    N: int            # elements per worker
    bucket: int
    s: int            # non-zero quantisation levels
    alpha: float
    beta: float
    iters: int
    kind: str         # which generator
    data_seed: int = 0
    norm: str = "linf"   # scaling factor of the quantiser: "linf" or "l2"

    @property
    def nb(self) -> int:
        return (self.N + self.bucket - 1) // self.bucket


# The five configurations of the benchmark definition, in its order.
WORKLOADS = {
    "tiny": Workload("tiny", P=4, N=4096, bucket=512, s=1, alpha=1.0, beta=1.0, iters=10,
                     kind="normal"),
    "linear": Workload("linear", P=8, N=1_048_576, bucket=1024, s=3, alpha=1.0, beta=0.9,
                       iters=100, kind="lsq"),
    "resnet50": Workload("resnet50", P=8, N=25_557_032, bucket=512, s=1, alpha=1.0, beta=0.9,
                         iters=20, kind="layered"),
    "alexnet": Workload("alexnet", P=16, N=61_100_840, bucket=2048, s=7, alpha=1.0, beta=0.95,
                        iters=10, kind="student_t"),
    "vgg16": Workload("vgg16", P=32, N=138_357_544, bucket=8192, s=1, alpha=1.0, beta=1.0,
                      iters=5, kind="outliers"),
}

# The quantiser settings the paper itself reports, on the metric workload's gradient (same
# P, N and value distribution as "resnet50"):
#   paper_cnn     Section 6.2 (CNN experiments): bucket 4096, l_2 scaling, s = 4, alpha = 0.01,
#                 beta = 1.0;
#   paper_linear  Section 6.1 (linear models): l_2 scaling, s = 4, alpha = 0.2, beta = 0.9; the
#                 paper scales the whole d-vector there (d <= 1024 features), which a bucket of
#                 1024 elements reproduces on a long flat gradient.
PAPER_SETTINGS = {
    "paper_cnn": Workload("paper_cnn", P=8, N=25_557_032, bucket=4096, s=4, alpha=0.01, beta=1.0,
                          iters=3, kind="layered", norm="l2"),
    "paper_linear": Workload("paper_linear", P=8, N=25_557_032, bucket=1024, s=4, alpha=0.2, beta=0.9,
                             iters=3, kind="layered", norm="l2"),
}
WORKLOADS.update(PAPER_SETTINGS)


def _gen(device, *seed_parts: int) -> torch.Generator:
    g = torch.Generator(device=device)
    seed = 0x9E3779B97F4A7C15
    for part in seed_parts:
        seed = (seed * 6364136223846793005 + 1442695040888963407 + int(part)) % (1 << 63)
    g.manual_seed(seed)
    return g


def _normal(wl, t, p, device):
    return torch.randn(wl.N, generator=_gen(device, wl.data_seed, t, p), device=device,
                       dtype=torch.float32)


def layer_sigmas(wl: Workload, segments: int = 161) -> torch.Tensor:
    """Per-segment standard deviations, log-uniform in [1e-4, 1e-1], drawn once per workload
    (shared by all workers and iterations)."""
    u = torch.rand(segments, generator=_gen("cpu", wl.data_seed, 777), dtype=torch.float64)
    return torch.exp(math.log(1e-4) + u * (math.log(1e-1) - math.log(1e-4))).to(torch.float32)


def _layered(wl, t, p, device, segments: int = 161):
    # `segments` contiguous runs of equal length (remainder in the last), each N(0, sigma_k^2).
    x = _normal(wl, t, p, device)
    seg = wl.N // segments
    idx = torch.clamp(torch.arange(wl.N, device=device) // seg, max=segments - 1)
    return x * layer_sigmas(wl, segments).to(device)[idx]


def _student_t(wl, t, p, device, nu: int = 3):
    # 1e-3 * Student-t(nu): z / sqrt(chi2_nu / nu).
    gen = _gen(device, wl.data_seed, t, p)
    z = torch.randn(wl.N, generator=gen, device=device, dtype=torch.float32)
    chi2 = torch.zeros(wl.N, device=device, dtype=torch.float32)
    for _ in range(nu):
        chi2 += torch.randn(wl.N, generator=gen, device=device, dtype=torch.float32) ** 2
    return 1e-3 * z / torch.sqrt(chi2 / nu)


def _outliers(wl, t, p, device):
    # N(0, variance 1e-4) with 1 % of the entries multiplied by 100.
    gen = _gen(device, wl.data_seed, t, p)
    x = 0.01 * torch.randn(wl.N, generator=gen, device=device, dtype=torch.float32)
    mask = torch.rand(wl.N, generator=gen, device=device) < 0.01
    return torch.where(mask, x * 100.0, x)


def _lsq(wl, t, p, device, rows: int = 256, density: float = 0.05):
    # Gradient of a synthetic least-squares minibatch: X^T (X w - y) / rows with X
    # `density`-dense, N(0,1) non-zeros; w fixed per workload, X and y redrawn per (t, p).
    gen = _gen(device, wl.data_seed, t, p)
    w = torch.randn(wl.N, generator=_gen(device, wl.data_seed, 4242), device=device,
                    dtype=torch.float32)
    y = torch.randn(rows, generator=gen, device=device, dtype=torch.float32)
    x = torch.randn(rows, wl.N, generator=gen, device=device, dtype=torch.float32)
    x *= torch.rand(rows, wl.N, generator=gen, device=device) < density
    resid = x @ w - y
    return (resid @ x) / rows


_KINDS = {"normal": _normal, "layered": _layered, "student_t": _student_t,
          "outliers": _outliers, "lsq": _lsq}


def gradient(wl: Workload, t: int, p: int, device="cpu") -> torch.Tensor:
    """Worker p's flat fp32 gradient at iteration t: a 1-D tensor of wl.N elements."""
    return _KINDS[wl.kind](wl, t, p, torch.device(device)).contiguous()


def gradients(wl: Workload, t: int, device="cpu", out: torch.Tensor | None = None) -> torch.Tensor:
    """All workers' gradients at iteration t as one [P, N] tensor (rows are workers)."""
    if out is None:
        out = torch.empty(wl.P, wl.N, device=device, dtype=torch.float32)
    for p in range(wl.P):
        out[p, : wl.N] = gradient(wl, t, p, device)
    return out


def scaled(wl: Workload, **changes) -> Workload:
    """A copy of a workload with some fields replaced (e.g. a smaller N for a CPU test)."""
    return dataclasses.replace(wl, **changes)
