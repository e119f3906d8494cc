"""Seeded synthetic gradient generators (inputs only).

This module holds NONE of the method's arithmetic: it only draws the local
gradients g_n^t that the sparsifier consumes.  It serves both the HIP path and
the CPU oracle (the same tensor is handed to both), and runs on whatever torch
device it is given.

The shapes follow the workloads the paper trains on (the section "Numerical
Investigation"): a linear-regression problem with N = 20 workers, a CNN of the
size of ResNet-18 with N = 8, and larger vision models with N = 20; real
gradients would need the paper's datasets and weights, so seeded random vectors
with per-layer scales, heavy tails and a component shared by all workers stand
in for them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch

BASE_SEED = 20250105


@dataclass(frozen=True)
class Config:
    name: str
    N: int
    d: int
    k: int
    mu: float
    T: int
    kind: str          # "gauss_mix" | "linreg" | "layered" | "transformer"
    segments: int = 0
    marginal: str = "gauss"   # "student3" | "laplace" | "gauss"
    index: int = 0


CONFIGS = {
    # N, d, k as in the list of benchmark configurations.
    "tiny":        Config("tiny", 4, 10_000, 100, 1.0, 10, "gauss_mix", index=0),
    "linreg":      Config("linreg", 20, 100_000, 1_000, 1.0, 50, "linreg", index=1),
    "cnn":         Config("cnn", 8, 11_200_000, 11_200, 1.0, 20, "layered", 62, "student3", 2),
    "large_cnn":   Config("large_cnn", 16, 25_600_000, 256_000, 1.0, 20, "layered", 160, "laplace", 3),
    "transformer": Config("transformer", 4, 124_000_000, 124_000, 1.0, 10, "transformer", 151, "gauss", 4),
}


def scaled(cfg: Config, d: int, N: int | None = None, k: int | None = None, **kw) -> Config:
    """Same recipe at another size (for parity cases the oracle finishes quickly)."""
    N = cfg.N if N is None else N
    if k is None:
        k = max(1, int(round(cfg.k / cfg.d * d)))
    vals = dict(cfg.__dict__)
    vals.update(dict(N=N, d=d, k=k))
    vals.update(kw)
    return Config(**vals)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _draw(marginal: str, n: int, gen, device) -> torch.Tensor:
    if marginal == "gauss":
        return torch.randn(n, generator=gen, device=device, dtype=torch.float32)
    if marginal == "laplace":
        u = torch.rand(n, generator=gen, device=device, dtype=torch.float32) - 0.5
        return -torch.sign(u) * torch.log1p(-2.0 * u.abs()).clamp_(min=-80.0)
    if marginal == "student3":
        z = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
        c = torch.zeros(n, device=device, dtype=torch.float32)
        for _ in range(3):
            c += torch.randn(n, generator=gen, device=device, dtype=torch.float32) ** 2
        return z / torch.sqrt(c / 3.0).clamp_(min=1e-12)
    raise ValueError(marginal)


class Workload:
    """grads(t) -> [N, d] float32 tensor on ``device`` for round t (open loop)."""

    def __init__(self, cfg: Config, device="cpu", seed: int | None = None):
        self.cfg = cfg
        self.device = torch.device(device)
        self.seed = (BASE_SEED + cfg.index) if seed is None else seed
        dev = self.device
        g0 = _gen(dev, self.seed * 7919 + 1)
        d = cfg.d
        if cfg.kind == "gauss_mix":
            self.shared = torch.randn(d, generator=g0, device=dev)
        elif cfg.kind == "layered":
            self.scale = self._layer_scales(cfg.segments, d, g0, dev)
            self.shared = _draw(cfg.marginal, d, g0, dev)
        elif cfg.kind == "transformer":
            rows = min(50_260, max(1, (d * 38_600) // 124_000 // 768))
            self.emb_rows, self.emb_cols = rows, 768
            self.emb = rows * 768
            if self.emb >= d:      # tiny scaled-down variants
                self.emb_rows = max(1, d // (4 * 768))
                self.emb = self.emb_rows * 768
            rest = d - self.emb
            self.scale = self._layer_scales(cfg.segments - 1, rest, g0, dev)
            self.sigma0 = 0.02
            self.shared = torch.randn(rest, generator=g0, device=dev)
        elif cfg.kind == "linreg":
            pass
        else:
            raise ValueError(cfg.kind)

    @staticmethod
    def _layer_scales(n_seg: int, d: int, gen, dev) -> torch.Tensor:
        """[d] vector: per-entry scale, constant on each of n_seg contiguous layers."""
        u = torch.rand(n_seg, generator=gen, device=dev, dtype=torch.float64)
        w = torch.pow(2.0, 8.0 + 14.0 * u)                       # sizes ~ 2^U(8,22)
        sizes = torch.floor(w / w.sum() * d).to(torch.int64)
        sizes[-1] += d - int(sizes.sum())
        v = torch.rand(n_seg, generator=gen, device=dev, dtype=torch.float64)
        sigma = torch.pow(10.0, -4.0 + 3.0 * v).to(torch.float32)  # 10^U(-4,-1)
        return torch.repeat_interleave(sigma, sizes)

    def grads(self, t: int) -> torch.Tensor:
        cfg, dev = self.cfg, self.device
        out = torch.empty(cfg.N, cfg.d, device=dev, dtype=torch.float32)
        for n in range(cfg.N):
            gen = _gen(dev, (self.seed * 1_000_003 + t) * 1009 + n)
            if cfg.kind == "gauss_mix":
                p = torch.randn(cfg.d, generator=gen, device=dev) * math.sqrt(0.5)
                out[n] = self.shared + p
            elif cfg.kind == "layered":
                p = _draw(cfg.marginal, cfg.d, gen, dev)
                out[n] = self.scale * (math.sqrt(0.3) * self.shared + math.sqrt(0.7) * p)
            elif cfg.kind == "transformer":
                r = torch.randn(self.emb_rows, self.emb_cols, generator=gen, device=dev)
                active = torch.rand(self.emb_rows, generator=gen, device=dev) < 0.05
                rs = torch.where(active, torch.tensor(1.0, device=dev), torch.tensor(1e-6, device=dev))
                out[n, :self.emb] = (r * (self.sigma0 * rs)[:, None]).reshape(-1)
                p = torch.randn(cfg.d - self.emb, generator=gen, device=dev)
                out[n, self.emb:] = self.scale * (math.sqrt(0.3) * self.shared + math.sqrt(0.7) * p)
            else:
                raise ValueError("use LinRegWorkload for the closed-loop linear regression")
        return out


class LinRegWorkload:
    """Closed-loop distributed least squares: g_n = X_n^T (X_n theta - y_n).

    Mirrors the generator of the paper's linear-regression experiment (Gaussian
    design, labels from a linear model) at the larger d of the benchmark list,
    with 64 rows per worker and a sparse ground truth.
    """

    def __init__(self, cfg: Config, device="cpu", seed: int | None = None, rows: int = 64):
        self.cfg = cfg
        self.device = torch.device(device)
        self.seed = (BASE_SEED + cfg.index) if seed is None else seed
        dev = self.device
        g0 = _gen(dev, self.seed * 7919 + 1)
        N, d = cfg.N, cfg.d
        self.X = torch.randn(N, rows, d, generator=g0, device=dev)
        nz = torch.rand(d, generator=g0, device=dev) < 0.05
        self.theta_star = torch.randn(d, generator=g0, device=dev) * nz
        self.y = torch.einsum("nrd,d->nr", self.X, self.theta_star)
        self.eta = 1e-4

    def grads(self, theta: torch.Tensor) -> torch.Tensor:
        r = torch.einsum("nrd,d->nr", self.X, theta) - self.y
        return torch.einsum("nrd,nr->nd", self.X, r).contiguous()


class PaperLinReg:
    """The paper's own linear-regression experiment (section "Linear Regression
    Problem"): N workers with D_n data points each in J dimensions, rows
    x ~ N(0, I_J), a ground truth t_n ~ N(u_n, h^2 I_J) per worker with
    u_n ~ N(U, sigma^2), labels y_n = X_n t_n + e_n, e_n ~ N(0, eps^2 I).
    Local loss F_n = |X_n theta - y_n|^2 / D_n, so the local gradient is
    (2/D_n) X_n^T (X_n theta - y_n); the global optimum has the closed form
    [sum_n X_n^T X_n]^{-1} sum_n X_n^T y_n.  Defaults: the heterogeneous setting
    of the optimality-gap figures (N=20, J=100, D_n=500, U=0, sigma^2=5, h^2=1,
    eps^2=0.5, learning rate 1e-2).  ``normalised=False`` drops the factor 2/D_n
    from the gradient: with it the unsparsified run of the low-dimensional study
    of the appendix (N=2, J=4, D_n=20, sigma^2=1) decays at the rate of the
    curves plotted there (about 0.8 per iteration at first)."""

    def __init__(self, device="cpu", N=20, J=100, D=500, U=0.0, sigma2=5.0, h2=1.0, eps2=0.5,
                 eta=1e-2, seed: int = BASE_SEED + 100, normalised: bool = True):
        self.device = torch.device(device)
        self.N, self.J, self.D, self.eta = N, J, D, eta
        self.scale = 2.0 / D if normalised else 1.0
        g0 = torch.Generator(device="cpu")
        g0.manual_seed(seed)
        X = torch.randn(N, D, J, generator=g0, dtype=torch.float64)
        u = U + math.sqrt(sigma2) * torch.randn(N, generator=g0, dtype=torch.float64)
        truth = u[:, None] + math.sqrt(h2) * torch.randn(N, J, generator=g0, dtype=torch.float64)
        y = torch.einsum("ndj,nj->nd", X, truth) + math.sqrt(eps2) * torch.randn(N, D, generator=g0, dtype=torch.float64)
        A = torch.einsum("ndj,ndk->jk", X, X)
        b = torch.einsum("ndj,nd->j", X, y)
        self.theta_star = torch.linalg.solve(A, b).to(self.device)           # float64
        self.X = X.to(torch.float32).to(self.device)
        self.y = y.to(torch.float32).to(self.device)

    def grads(self, theta: torch.Tensor) -> torch.Tensor:
        r = torch.einsum("ndj,j->nd", self.X, theta) - self.y
        return (self.scale * torch.einsum("ndj,nd->nj", self.X, r)).contiguous()

    def gap(self, theta: torch.Tensor) -> float:
        """Optimality gap |theta - theta*|."""
        return float(torch.linalg.norm(theta.to(torch.float64) - self.theta_star))
