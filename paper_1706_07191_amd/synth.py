"""Seeded synthetic inputs shared by the tests, the bench and the CPU oracle.

This module only draws random numbers and assembles input matrices; it holds none of
the method's arithmetic (no sketching, orthonormalisation, SVD or shrinkage).

The matrices follow the data recipe of the paper's experiment section (a low-rank
matrix formed as the product of two Gaussian factors, Sec. 4 "Experiment environment
and setup"), extended with a prescribed diagonal scaling and additive Gaussian noise.
The robust-PCA input (low-rank background + sparse corruptions) stands in for the
image/video matrices of Table 2, which are not available offline.

Everything is generated with torch so the same code runs on the CPU (small cases) and
on the GPU (large cases, generated block by block).  The oracle and the HIP path always
read the *same buffer* produced by one call, so cross-device reproducibility of the
random streams is not needed.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Callable, Optional

import torch

BASE_SEED = 170607191


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def gaussian(rows: int, cols: int, seed: int, device="cpu", dtype=torch.float32) -> torch.Tensor:
    """rows x cols matrix of i.i.d. N(0,1) entries (the test matrix Omega of Alg. 1, step 1)."""
    return torch.randn(rows, cols, generator=_gen(seed, device), device=device, dtype=dtype)


def lowrank_plus_noise(m: int, n: int, sigma: torch.Tensor, noise: float, seed: int,
                       device="cpu", out: Optional[torch.Tensor] = None,
                       row_chunk: int = 8192, gen_device=None) -> torch.Tensor:
    """A = G1 * diag(sigma) * G2 + noise * N(0,1), G1 (m x r), G2 (r x n) i.i.d. N(0,1), fp32.

    The factors are *not* orthonormalised, so `sigma` shapes the spectrum without being the
    exact singular values.  `out` may be a preallocated (m, n) fp32 tensor on any device
    (e.g. pinned host memory); rows are produced `row_chunk` at a time on `gen_device`
    (defaults to `device`) so the peak extra memory is one chunk.
    """
    gen_device = gen_device or device
    sigma = sigma.to(device=gen_device, dtype=torch.float32)
    r = sigma.numel()
    g1 = torch.randn(m, r, generator=_gen(seed + 1, gen_device), device=gen_device)
    g2 = torch.randn(r, n, generator=_gen(seed + 2, gen_device), device=gen_device)
    gn = _gen(seed + 3, gen_device)
    if out is None:
        out = torch.empty(m, n, dtype=torch.float32, device=device)
    assert out.shape == (m, n) and out.dtype == torch.float32
    for r0 in range(0, m, row_chunk):
        r1 = min(m, r0 + row_chunk)
        blk = (g1[r0:r1] * sigma) @ g2
        if noise != 0.0:
            blk.add_(torch.randn(r1 - r0, n, generator=gn, device=gen_device), alpha=noise)
        out[r0:r1].copy_(blk)
    return out


def exact_spectrum_matrix(m: int, n: int, s: torch.Tensor, seed: int, dtype=torch.float64) -> torch.Tensor:
    """A = Q1 diag(s) Q2^T with orthonormal Q1 (m x r), Q2 (n x r): singular values exactly `s`.

    Used by tests that need a known spectrum (exact-recovery and error-bound pins)."""
    r = s.numel()
    q1, _ = torch.linalg.qr(torch.randn(m, r, generator=_gen(seed + 1, "cpu"), dtype=torch.float64))
    q2, _ = torch.linalg.qr(torch.randn(n, r, generator=_gen(seed + 2, "cpu"), dtype=torch.float64))
    return ((q1 * s.to(torch.float64)) @ q2.T).to(dtype)


def rpca_matrix(m: int, n: int, rank: int, frac: float, amp: float, noise: float, seed: int,
                device="cpu"):
    """D = L0 + S0 + noise*N(0,1): L0 = G1 (m x rank) G2 (rank x n) Gaussian, S0 has a fraction
    `frac` of entries (seeded Bernoulli mask) uniform in [-amp, amp].  Returns (D, L0, S0) fp32."""
    g1 = torch.randn(m, rank, generator=_gen(seed + 1, device), device=device)
    g2 = torch.randn(rank, n, generator=_gen(seed + 2, device), device=device)
    l0 = g1 @ g2
    mask = torch.rand(m, n, generator=_gen(seed + 3, device), device=device) < frac
    vals = (torch.rand(m, n, generator=_gen(seed + 4, device), device=device) * 2.0 - 1.0) * amp
    s0 = torch.where(mask, vals, torch.zeros((), device=device))
    d = l0 + s0
    if noise != 0.0:
        d = d + noise * torch.randn(m, n, generator=_gen(seed + 5, device), device=device)
    return d.float(), l0.float(), s0.float()


@dataclass
class Config:
    name: str
    m: int
    n: int
    k: int
    p: int
    q: int
    row_block: int
    rank: int
    sigma: Callable[[torch.Tensor], torch.Tensor]   # i (1-based index) -> sigma_i
    noise: float
    seed: int
    host_resident: bool = False
    device_budget: int = 0
    rpca: dict = field(default_factory=dict)

    @property
    def l(self) -> int:
        return self.k + self.p

    def sigma_vec(self) -> torch.Tensor:
        i = torch.arange(1, self.rank + 1, dtype=torch.float64)
        return self.sigma(i).float()

    def make_A(self, device="cpu", out=None, gen_device=None) -> torch.Tensor:
        return lowrank_plus_noise(self.m, self.n, self.sigma_vec(), self.noise, self.seed,
                                  device=device, out=out, gen_device=gen_device)

    def make_Omega(self, device="cpu", it: int = 0) -> torch.Tensor:
        return gaussian(self.n, self.l, self.seed + 7 + 100 * it, device=device)

    def scaled(self, m: int, n: int, row_block: Optional[int] = None) -> "Config":
        """Same recipe at a smaller shape (for tests the oracle finishes quickly)."""
        c = Config(**{**self.__dict__})
        c.m, c.n = m, n
        c.row_block = row_block or self.row_block
        c.name = f"{self.name}@{m}x{n}"
        return c


CONFIGS = {
    # tiny in-core
    "C1": Config("C1", 2000, 1000, 20, 10, 2, 512, 50, lambda i: 0.9 ** (i - 1), 1e-3, BASE_SEED + 1000),
    # in-core square (the configuration the headline metric is quoted on)
    "C2": Config("C2", 20000, 20000, 100, 10, 2, 4096, 200, lambda i: 1.0 / i, 1e-4, BASE_SEED + 2000),
    # in-core tall
    "C3": Config("C3", 100000, 50000, 256, 16, 1, 8192, 512, lambda i: torch.exp(-i / 64.0), 1e-5,
                 BASE_SEED + 3000),
    # out-of-core: A in pinned host memory, 16 GB device budget
    "C4": Config("C4", 200000, 100000, 128, 16, 1, 16384, 300, lambda i: i ** -0.5, 1e-4,
                 BASE_SEED + 4000, host_resident=True, device_budget=16 * 2 ** 30),
    # robust PCA by inexact ALM; sigma/noise describe the corruption recipe instead
    "C5": Config("C5", 76800, 2000, 10, 10, 1, 8192, 5, lambda i: torch.ones_like(i), 1e-3,
                 BASE_SEED + 5000, rpca=dict(frac=0.05, amp=50.0, iters=30)),
}


def make_rpca(cfg: Config, device="cpu", m: Optional[int] = None, n: Optional[int] = None):
    m = m or cfg.m
    n = n or cfg.n
    return rpca_matrix(m, n, cfg.rank, cfg.rpca["frac"], cfg.rpca["amp"], cfg.noise, cfg.seed, device=device)


def rpca_omegas(cfg: Config, n: int, iters: int, device="cpu") -> torch.Tensor:
    """One fresh Gaussian test matrix per ALM iteration, stacked: iters x n x l."""
    return torch.stack([gaussian(n, cfg.l, cfg.seed + 7 + 100 * i, device=device) for i in range(iters)])
