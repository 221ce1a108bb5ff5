"""Seeded synthetic inputs for the clustering path (inputs only: no k-means arithmetic lives here).

The paper clusters the linear-layer weight matrices of LLaMA-family models (Section 3.1, Section 4.1).
Those weights are not available, so every test and benchmark draws a synthetic matrix with the same
shape and a comparable value distribution: a Gaussian bulk, a small fraction of large-variance
outliers, values rounded to fp16 (the paper keeps all tensors 16-bit) and then held as fp32.
The matrix is split row-major into N = R*C/d sub-vectors of length d (Section 3.1, the reshape that
defines W'), and the initial centroids are a seeded random subset of those vectors.

Both the CPU oracle's tests and the HIP path's tests/bench import this module; it holds nothing
but random draws, a dtype round-trip and a reshape.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20250313


@dataclass(frozen=True)
class Workload:
    name: str
    number: int          # position in the benchmark's config list, 1-based
    rows: int
    cols: int
    d: int               # sub-vector length (paper: g)
    K: int               # number of centroids (paper: n)
    iters: int           # Lloyd iterations
    sigma: float         # std of the Gaussian bulk
    p_out: float         # fraction of entries replaced by outliers
    sigma_out: float     # std of the outliers
    row_lognormal: float = 0.0   # if >0: each row scaled by exp(s * N(0,1)) before fp16 rounding

    @property
    def N(self) -> int:
        return self.rows * self.cols // self.d

    @property
    def code_bits_per_weight(self) -> float:
        return float(np.log2(self.K)) / self.d


WORKLOADS = {
    w.name: w
    for w in (
        Workload("cfg1_512x512_d4_k256", 1, 512, 512, 4, 256, 10, 0.02, 0.005, 0.2),
        Workload("cfg2_4096x4096_d4_k4096", 2, 4096, 4096, 4, 4096, 20, 0.02, 0.005, 0.2),
        Workload("cfg3_4096x11008_d4_k65536", 3, 4096, 11008, 4, 65536, 20, 0.02, 0.005, 0.2, 0.3),
        Workload("cfg4_8192x28672_d8_k65536", 4, 8192, 28672, 8, 65536, 10, 0.015, 0.005, 0.15),
        Workload("cfg5_4096x14336_d16_k65536", 5, 4096, 14336, 16, 65536, 10, 0.02, 0.01, 0.2),
    )
}


def by_number(number: int) -> Workload:
    for w in WORKLOADS.values():
        if w.number == number:
            return w
    raise KeyError(number)


def make_matrix(rows: int, cols: int, sigma: float, p_out: float, sigma_out: float,
                row_lognormal: float, rng: np.random.Generator) -> np.ndarray:
    """Gaussian bulk + sparse outliers (+ optional per-row scale), rounded to fp16, returned as fp32."""
    W = rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(sigma)
    mask = rng.random((rows, cols)) < p_out
    W[mask] = rng.standard_normal(int(mask.sum()), dtype=np.float32) * np.float32(sigma_out)
    if row_lognormal > 0.0:
        scale = np.exp(row_lognormal * rng.standard_normal(rows)).astype(np.float32)
        W *= scale[:, None]
    return W.astype(np.float16).astype(np.float32)


def make_inputs(w: Workload, seed: int | None = None, rows: int | None = None):
    """Return (X[N,d] fp32, C0[K,d] fp32) for a workload.

    `rows` truncates the matrix to its first rows (a smaller problem with the same distribution);
    K is kept, so it must not exceed the reduced N.
    """
    rng = np.random.default_rng(BASE_SEED + w.number if seed is None else seed)
    R = w.rows if rows is None else rows
    W = make_matrix(R, w.cols, w.sigma, w.p_out, w.sigma_out, w.row_lognormal, rng)
    X = W.reshape(-1, w.d)
    if w.K > X.shape[0]:
        raise ValueError("K exceeds the number of sub-vectors")
    sel = rng.choice(X.shape[0], size=w.K, replace=False)
    C0 = np.ascontiguousarray(X[sel])
    return X, C0


def make_small(N: int, d: int, K: int, seed: int, sigma: float = 0.02, p_out: float = 0.005,
               sigma_out: float = 0.2, fp16_round: bool = True):
    """Free-shape problem for tests: N vectors of length d, K seeded-subset initial centroids."""
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((N, d), dtype=np.float32) * np.float32(sigma)
    mask = rng.random((N, d)) < p_out
    W[mask] = rng.standard_normal(int(mask.sum()), dtype=np.float32) * np.float32(sigma_out)
    if fp16_round:
        W = W.astype(np.float16).astype(np.float32)
    sel = rng.choice(N, size=K, replace=False)
    return np.ascontiguousarray(W), np.ascontiguousarray(W[sel])
