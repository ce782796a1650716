"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the oracle-side tests and the HIP-side tests and
benchmark.  It holds none of the method's arithmetic: it only builds test
matrices A = U diag(s) V^T (+ noise) the way the paper's performance
experiment does (random orthogonal factors, prescribed spectrum), at the five
configurations the benchmark names.

Recipe (all configs): thin Gaussian factors from numpy Generator(PCG64(seed))
with seeds 1000+c (U) and 2000+c (V), orthonormalised by a reduced QR on the
host; A assembled as (U diag(s)) V^T in fp64 and cast to the config dtype.
Noise uses seed 3000+c.  With `device` given, the assembly and the noise run
through torch on that device (harness plumbing only) and A is returned as a
torch tensor; otherwise everything is numpy.
"""
from dataclasses import dataclass, replace
from typing import Callable, Optional

import numpy as np


@dataclass(frozen=True)
class Config:
    cid: int
    name: str
    dtype: str            # "f32" or "f64"
    m: int
    n: int
    rank: int             # planted rank (number of nonzero s_i)
    k: int
    p: int
    q: int
    noise: float = 0.0    # std of iid Gaussian noise added to A
    center: bool = False  # subtract column means (PCA-shaped input)
    seed: int = 0         # Philox seed for the sketch
    spectrum: Optional[Callable] = None

    @property
    def l(self):
        return self.k + self.p

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.float64

    def singular_values(self):
        i = np.arange(self.rank, dtype=np.float64)
        return self.spectrum(i)


CONFIGS = {
    1: Config(1, "planted-rank10-512x256", "f64", 512, 256, 10, 10, 10, 2,
              spectrum=lambda i: 10.0 ** (-i / 5.0)),
    2: Config(2, "expdecay-10000x2000", "f32", 10000, 2000, 2000, 64, 16, 2,
              spectrum=lambda i: 0.9 ** i),
    3: Config(3, "pca-100000x1000", "f32", 100000, 1000, 100, 100, 20, 3,
              noise=0.01, center=True, spectrum=lambda i: 100.0 / (1.0 + i)),
    4: Config(4, "polydecay-20000x20000", "f64", 20000, 20000, 2048, 256, 32, 2,
              noise=1e-6, spectrum=lambda i: 1.0 / (1.0 + i)),
    5: Config(5, "mfma-65536x16384", "f32", 65536, 16384, 512, 512, 64, 1,
              noise=1e-3, spectrum=lambda i: np.exp(-i / 128.0)),
}


# The three spectra of the paper's performance comparison (Experiments section), 1-based there, 0-based index i here.
PAPER_SPECTRA = {
    "fast": lambda i: 1.0 / (1.0 + i) ** 2,                                   # sigma_ii = 1 / i^2
    "sharp": lambda i, beta=20.0: 1e-4 + 1.0 / (1.0 + np.exp(np.minimum(i + 2.0 - beta, 700.0))),  # 1e-4 + 1/(1+exp(i+1-beta))
    "slow": lambda i: 1.0 / (1.0 + i) ** 0.1,                                 # sigma_ii = 1 / i^0.1
}


def paper_case(kind: str, n: int, frac: float, dtype: str = "f64", m: int = 2000, p: int = 10, q: int = 2) -> Config:
    """A = U Sigma V^T of size m x n (the paper uses A^{2000 x n}) with one of its spectra, k = ceil(frac * n)."""
    k = int(np.ceil(frac * n))
    return Config(10 + list(PAPER_SPECTRA).index(kind), f"paper-{kind}-{m}x{n}-k{k}", dtype, m, n, min(m, n), k, p, q,
                  spectrum=PAPER_SPECTRA[kind])


def scaled(cfg: Config, m: int, n: int, rank=None, k=None, p=None) -> Config:
    """Same recipe at another size (parity cases and CPU-side replicas)."""
    rank = min(cfg.rank if rank is None else rank, m, n)
    return replace(cfg, m=m, n=n, rank=rank,
                   k=cfg.k if k is None else k, p=cfg.p if p is None else p,
                   name=f"{cfg.name}@{m}x{n}")


def orthonormal_factor(rows: int, cols: int, seed: int) -> np.ndarray:
    g = np.random.Generator(np.random.PCG64(seed)).standard_normal((rows, cols))
    qf, _ = np.linalg.qr(g, mode="reduced")
    return qf


def build(cfg: Config, device=None):
    """Return A for `cfg`: numpy array (device None) or torch tensor on `device`."""
    s = cfg.singular_values()
    U = orthonormal_factor(cfg.m, cfg.rank, 1000 + cfg.cid)
    V = orthonormal_factor(cfg.n, cfg.rank, 2000 + cfg.cid)
    if device is None:
        A = (U * s) @ V.T
        if cfg.noise > 0.0:
            rng = np.random.Generator(np.random.PCG64(3000 + cfg.cid))
            rows = max(1, (1 << 24) // cfg.n)
            for r0 in range(0, cfg.m, rows):
                blk = A[r0:r0 + rows]
                blk += cfg.noise * rng.standard_normal(blk.shape)
        if cfg.center:
            A -= A.mean(axis=0, keepdims=True)
        return np.ascontiguousarray(A.astype(cfg.np_dtype))

    import torch
    tdt = torch.float32 if cfg.dtype == "f32" else torch.float64
    gen = torch.Generator(device=device)
    gen.manual_seed(3000 + cfg.cid)
    Vt = torch.from_numpy(np.ascontiguousarray(V.T)).to(device)
    A = torch.empty((cfg.m, cfg.n), dtype=tdt, device=device)
    rows = max(1, (1 << 26) // cfg.n)
    colsum = torch.zeros(cfg.n, dtype=torch.float64, device=device)
    for r0 in range(0, cfg.m, rows):
        Ub = torch.from_numpy(U[r0:r0 + rows] * s).to(device)
        blk = Ub @ Vt
        if cfg.noise > 0.0:
            blk += cfg.noise * torch.randn(blk.shape, dtype=torch.float64,
                                           device=device, generator=gen)
        if cfg.center:
            colsum += blk.sum(dim=0)
        A[r0:r0 + rows] = blk.to(tdt)
    if cfg.center:
        mean = (colsum / cfg.m)
        for r0 in range(0, cfg.m, rows):
            A[r0:r0 + rows] = (A[r0:r0 + rows].to(torch.float64) - mean).to(tdt)
    return A


def gaussian_matrix(rows: int, cols: int, seed: int, dtype=np.float64) -> np.ndarray:
    """Plain seeded N(0,1) matrix for stage-level parity cases."""
    g = np.random.Generator(np.random.PCG64(seed)).standard_normal((rows, cols))
    return np.ascontiguousarray(g.astype(dtype))


def graded_matrix(rows: int, cols: int, cond: float, seed: int, dtype=np.float64) -> np.ndarray:
    """rows x cols matrix with singular values geometrically spaced from 1 to 1/cond."""
    U = orthonormal_factor(rows, cols, seed)
    V = orthonormal_factor(cols, cols, seed + 1)
    s = cond ** (-np.arange(cols, dtype=np.float64) / max(1, cols - 1))
    return np.ascontiguousarray(((U * s) @ V.T).astype(dtype))
