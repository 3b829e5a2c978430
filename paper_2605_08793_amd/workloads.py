"""Seeded synthetic workloads: cost matrix M and marginals a, b.

This module serves both the GPU library's tests/benchmark and the CPU oracle's
tests.  It holds none of the method's arithmetic (no plan entries, sums,
Sinkhorn steps or thresholds): it only draws points and marginals from a seeded
numpy generator and forms the pairwise cost with elementwise torch operations
(subtract, multiply/abs, add, one division by the maximum), so the same recipe
can run on the host or on the GPU.

Recipes follow the paper's synthetic experiments (Sec. 6.1: M is divided by its
maximum; Sec. 6.2: squared-Euclidean Gaussian point clouds, and the 1-D
exponential-to-Gaussian-mixture grid problem) at the shapes and regularisation
values of the benchmark configurations.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Config:
    name: str
    n: int
    m: int
    d: int
    seed: int
    eta: float
    sweeps: int          # Sinkhorn sweeps (alpha then beta) from zero that define the dual point
    frac: float          # fraction of entries of T the threshold keeps
    recipe: str          # which point/marginal recipe below
    noise_sigma: float = 0.0   # std of the iid normal noise added to the dual point


CONFIGS = {
    # n=m=1000, d=2 Gaussian clouds, eta=0.01, 20 sweeps + N(0, var 0.01) noise, top 1 %
    "c1": Config("c1", 1000, 1000, 2, 1001, 0.01, 20, 0.01, "gauss_shift1", 0.1),
    # n=m=10000, d=10 Gaussian clouds, eta=0.01, 50 sweeps, top 1 %
    "c2": Config("c2", 10000, 10000, 10, 1002, 0.01, 50, 0.01, "gauss_shift05"),
    # n=m=20000, d=2, two 3-component mixtures, Dirichlet marginals, eta=0.001, 200 sweeps, top 0.5 %
    "c3": Config("c3", 20000, 20000, 2, 1003, 0.001, 200, 0.005, "mixture"),
    # n=40000, m=10000, d=64 uniform points, L1 cost, eta=0.01, 100 sweeps, top 1 %
    "c4": Config("c4", 40000, 10000, 64, 1004, 0.01, 100, 0.01, "uniform_l1"),
    # n=m=50000, d=3 Gaussian clouds, eta=0.005, 100 sweeps, top 0.2 %
    "c5": Config("c5", 50000, 50000, 3, 1005, 0.005, 100, 0.002, "gauss_shift03"),
    # the paper's own synthetic problems (Sec. 6.2), eta=0.001 as in its main runs
    "syn1_diff": Config("syn1_diff", 1600, 1200, 2, 2001, 0.001, 20, 0.01, "syn1_diff"),
    "syn2": Config("syn2", 1600, 1200, 1, 2002, 0.001, 20, 0.01, "syn2"),
}


@dataclass
class Problem:
    config: Config
    M: torch.Tensor          # (n, m) fp64, row-major, on `device`
    a: torch.Tensor          # (n,) fp64
    b: torch.Tensor          # (m,) fp64
    noise_alpha: Optional[np.ndarray] = None   # host arrays; zero-length-free: None when sigma == 0
    noise_beta: Optional[np.ndarray] = None
    meta: dict = field(default_factory=dict)

    @property
    def n(self):
        return self.M.shape[0]

    @property
    def m(self):
        return self.M.shape[1]

    @property
    def eta(self):
        return self.config.eta

    def k_keep(self) -> int:
        """Number of entries the top-k rule keeps: round(frac * n * m), at least 1."""
        return max(1, int(round(self.config.frac * self.n * self.m)))

    def host(self):
        """(M, a, b) as numpy arrays (copies off the device if needed)."""
        return self.M.cpu().numpy(), self.a.cpu().numpy(), self.b.cpu().numpy()


def _pairwise_cost(x: np.ndarray, y: np.ndarray, kind: str, device, chunk_bytes: int = 1 << 28) -> torch.Tensor:
    """M_ij = sum_k (x_ik - y_jk)^2 ("sq") or sum_k |x_ik - y_jk| ("l1"), then M / max(M).

    Coordinates are accumulated in ascending k with separate elementwise
    operations (no fused multiply-add, no BLAS), so the result does not depend
    on library kernels.
    """
    n, d = x.shape
    m = y.shape[0]
    xt = torch.from_numpy(np.ascontiguousarray(x)).to(device)
    yt = torch.from_numpy(np.ascontiguousarray(y)).to(device)
    M = torch.empty((n, m), dtype=torch.float64, device=device)
    rows = max(1, min(n, chunk_bytes // max(8 * m, 1)))
    for r0 in range(0, n, rows):
        r1 = min(n, r0 + rows)
        acc = M[r0:r1]
        acc.zero_()
        for k in range(d):
            diff = xt[r0:r1, k].unsqueeze(1) - yt[:, k].unsqueeze(0)
            if kind == "sq":
                diff.mul_(diff)
            elif kind == "l1":
                diff.abs_()
            else:
                raise ValueError(kind)
            acc.add_(diff)
    mx = M.max()
    M.div_(mx)
    return M


def _uniform_marginal(rng, length):
    v = rng.uniform(0.5, 1.5, size=length)
    return v / v.sum()


def _dirichlet_marginal(rng, length):
    v = rng.dirichlet(np.ones(length))
    v = np.maximum(v, 1e-8 * v.mean())
    return v / v.sum()


def make_problem(name: str, device="cpu", n: Optional[int] = None, m: Optional[int] = None,
                 seed: Optional[int] = None) -> Problem:
    """Build the workload `name`; n, m, seed override the configuration's (for small test variants)."""
    cfg = CONFIGS[name]
    if n is not None or m is not None or seed is not None:
        cfg = Config(cfg.name, cfg.n if n is None else int(n), cfg.m if m is None else int(m), cfg.d,
                     cfg.seed if seed is None else int(seed), cfg.eta, cfg.sweeps, cfg.frac, cfg.recipe,
                     cfg.noise_sigma)
    rng = np.random.default_rng(cfg.seed)
    n_, m_, d = cfg.n, cfg.m, cfg.d
    kind = "sq"
    r = cfg.recipe
    if r in ("gauss_shift1", "gauss_shift05", "gauss_shift03"):
        shift = {"gauss_shift1": 1.0, "gauss_shift05": 0.5, "gauss_shift03": 0.3}[r]
        x = rng.standard_normal((n_, d))
        y = rng.standard_normal((m_, d)) + shift
        a = _uniform_marginal(rng, n_)
        b = _uniform_marginal(rng, m_)
    elif r == "mixture":
        mu_x = rng.uniform(0.0, 4.0, size=(3, d))
        mu_y = rng.uniform(0.0, 4.0, size=(3, d))
        x = mu_x[rng.integers(0, 3, size=n_)] + 0.3 * rng.standard_normal((n_, d))
        y = mu_y[rng.integers(0, 3, size=m_)] + 0.3 * rng.standard_normal((m_, d))
        a = _dirichlet_marginal(rng, n_)
        b = _dirichlet_marginal(rng, m_)
    elif r == "uniform_l1":
        kind = "l1"
        x = rng.uniform(0.0, 1.0, size=(n_, d))
        y = rng.uniform(0.0, 1.0, size=(m_, d))
        a = np.full(n_, 1.0 / n_)
        b = _uniform_marginal(rng, m_)
    elif r == "syn1_diff":
        # Synthetic I, "diff": N(0,1) entries against N(1, variance 0.25) entries; uniform marginals
        x = rng.standard_normal((n_, d))
        y = 1.0 + 0.5 * rng.standard_normal((m_, d))
        a = np.full(n_, 1.0 / n_)
        b = np.full(m_, 1.0 / m_)
    elif r == "syn2":
        # Synthetic II: uniform grids on [0,5]; a ~ exp(-x); b ~ 0.2 N(1, var 0.04) + 0.8 N(3, var 0.25)
        x = np.linspace(0.0, 5.0, n_).reshape(n_, 1)
        y = np.linspace(0.0, 5.0, m_).reshape(m_, 1)
        a = np.exp(-x[:, 0])
        yy = y[:, 0]
        b = (0.2 * np.exp(-0.5 * (yy - 1.0) ** 2 / 0.04) / np.sqrt(2 * np.pi * 0.04)
             + 0.8 * np.exp(-0.5 * (yy - 3.0) ** 2 / 0.25) / np.sqrt(2 * np.pi * 0.25))
        a = a / a.sum()
        b = b / b.sum()
    else:
        raise ValueError(r)
    noise_a = noise_b = None
    if cfg.noise_sigma > 0:
        noise_a = cfg.noise_sigma * rng.standard_normal(n_)
        noise_b = cfg.noise_sigma * rng.standard_normal(m_)
    dev = torch.device(device)
    M = _pairwise_cost(x, y, kind, dev)
    return Problem(cfg, M, torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev), noise_a, noise_b,
                   meta=dict(cost=kind))


def random_small(n: int, m: int, seed: int, eta: float = 0.5):
    """Unstructured small dense problem on the host: M in [0,1], positive normalised a, b, N(0,1)*eta duals.

    For brute-force-size checks where no geometry is wanted.  Returns numpy arrays.
    """
    rng = np.random.default_rng(seed)
    M = rng.uniform(0.0, 1.0, size=(n, m))
    a = rng.uniform(0.5, 1.5, size=n)
    b = rng.uniform(0.5, 1.5, size=m)
    a /= a.sum()
    b /= b.sum()
    alpha = eta * rng.standard_normal(n)
    beta = eta * rng.standard_normal(m)
    return M, a, b, alpha, beta
