"""Seeded synthetic inputs for exact kNN.

This module only draws random numbers and arranges them; it holds none of the
method's arithmetic (no distance evaluation, sorting or selection), so both the GPU
library's callers and the CPU oracle's tests can take their inputs from it.

The paper's own experiment (Sect. 7) uses "randomly generated" vectors with
d = 256 and states no distribution; its motivating data are customer-preference
vectors after dimensionality reduction (Sect. 1).  The five workloads below give
that description concrete, reproducible shapes: i.i.d. Gaussian, clustered,
low-rank "embedding-like", unit-norm high-dimensional, and a query block of a
larger reference set.  Everything is generated on the host with torch's CPU
generator so that the same seed gives the same bits on every machine.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch

BASE_SEED = 9060231


@dataclass
class Workload:
    name: str
    R: torch.Tensor            # [nr, d] fp32, host: the reference set
    nq: int                    # queries are rows self_offset .. self_offset+nq of R
    self_offset: int
    k: int
    metric: str                # "sqeuclidean" | "cosine" | "hellinger" | "l1" | "linf" | "kl"
    symmetric: bool            # queries == whole reference set (all-pairs self kNN)

    @property
    def Q(self) -> torch.Tensor:
        return self.R[self.self_offset:self.self_offset + self.nq]

    @property
    def n(self) -> int:
        return self.R.shape[0]

    @property
    def d(self) -> int:
        return self.R.shape[1]


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def gaussian(n: int, d: int, seed: int, std: float = 1.0) -> torch.Tensor:
    """i.i.d. N(0, std^2) entries."""
    x = torch.randn(n, d, generator=_gen(seed), dtype=torch.float32)
    if std != 1.0:
        x.mul_(std)
    return x


def mixture(n: int, d: int, centers: int, seed: int, center_std: float = 2.0,
            noise_std: float = 1.0, chunk: int = 1 << 20) -> torch.Tensor:
    """Each row = one of `centers` Gaussian centres (entries N(0, center_std^2),
    picked uniformly) plus N(0, noise_std^2) noise."""
    g = _gen(seed)
    c = torch.randn(centers, d, generator=g, dtype=torch.float32) * center_std
    assign = torch.randint(0, centers, (n,), generator=g)
    x = torch.empty(n, d, dtype=torch.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        blk = torch.randn(e - s, d, generator=g, dtype=torch.float32)
        if noise_std != 1.0:
            blk.mul_(noise_std)
        blk.add_(c[assign[s:e]])
        x[s:e] = blk
    return x


def low_rank(n: int, d: int, rank: int, seed: int, noise_std: float = 0.1,
             chunk: int = 1 << 18) -> torch.Tensor:
    """X = U V + E with U[n, rank] ~ N(0,1), V[rank, d] ~ N(0, 1/rank),
    E ~ N(0, noise_std^2): what a truncated factorisation of a preference matrix
    looks like (Sect. 1 of the paper names SVD / LDA reduction)."""
    g = _gen(seed)
    v = torch.randn(rank, d, generator=g, dtype=torch.float32) * (rank ** -0.5)
    x = torch.empty(n, d, dtype=torch.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        u = torch.randn(e - s, rank, generator=g, dtype=torch.float32)
        blk = torch.randn(e - s, d, generator=g, dtype=torch.float32).mul_(noise_std)
        blk.addmm_(u, v)
        x[s:e] = blk
    return x


def unit_rows(n: int, d: int, seed: int, chunk: int = 1 << 16) -> torch.Tensor:
    """N(0,1) rows scaled to unit Euclidean length (input conditioning only)."""
    g = _gen(seed)
    x = torch.empty(n, d, dtype=torch.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        blk = torch.randn(e - s, d, generator=g, dtype=torch.float32)
        blk.div_(blk.norm(dim=1, keepdim=True))
        x[s:e] = blk
    return x


def uniform_rows(n: int, d: int, seed: int) -> torch.Tensor:
    """i.i.d. U[0,1) entries: non-negative "randomly generated" data, the only thing the
    paper says about its experiment's input (Sect. 7); Hellinger distance needs >= 0."""
    return torch.rand(n, d, generator=_gen(seed), dtype=torch.float32)


def config(which: int, n: Optional[int] = None, nq: Optional[int] = None) -> Workload:
    """The five benchmark/parity configurations; `n` (and `nq` for config 5)
    shrink them for tests while keeping distribution, d, k and metric."""
    seed = BASE_SEED + which
    if which == 1:
        n = n or 4096
        return Workload("c1_gauss_n%d_d64_k10" % n, gaussian(n, 64, seed), n, 0, 10,
                        "sqeuclidean", True)
    if which == 2:
        n = n or 65536
        return Workload("c2_mix64_n%d_d128_k32" % n, mixture(n, 128, 64, seed), n, 0, 32,
                        "sqeuclidean", True)
    if which == 3:
        n = n or (1 << 20)
        return Workload("c3_lowrank32_n%d_d256_k10" % n, low_rank(n, 256, 32, seed), n, 0, 10,
                        "sqeuclidean", True)
    if which == 4:
        n = n or (1 << 18)
        return Workload("c4_unit_n%d_d1024_k100_cos" % n, unit_rows(n, 1024, seed), n, 0, 100,
                        "cosine", True)
    if which == 5:
        n = n or (1 << 23)
        nq = nq or max(1, n // 8)
        return Workload("c5_mix256_nq%d_nr%d_d128_k16" % (nq, n), mixture(n, 128, 256, seed),
                        nq, 0, 16, "sqeuclidean", False)
    if which == 6:
        # the shape of the paper's own experiment (Sect. 7, Table 1): d = 256, k = 100,
        # Hellinger distance, n = 10 000 .. 80 000
        n = n or 80000
        return Workload("paper_table1_n%d_d256_k100_hellinger" % n, uniform_rows(n, 256, seed), n, 0,
                        100, "hellinger", True)
    if which == 7:
        # a distance that is a fold but not an inner product (Sect. 3): Manhattan, on config 2's data
        n = n or 65536
        return Workload("fold_l1_mix64_n%d_d128_k32" % n, mixture(n, 128, 64, BASE_SEED + 2), n, 0, 32,
                        "l1", True)
    if which == 8:
        # a distance that is not symmetric (Sect. 3): Kullback-Leibler on strictly positive rows
        n = n or 65536
        return Workload("kl_uniform_n%d_d128_k32" % n, uniform_rows(n, 128, seed).add_(0.05), n, 0, 32,
                        "kl", True)
    raise ValueError("config must be 1..8")
