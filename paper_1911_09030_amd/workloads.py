"""Seeded synthetic inputs shared by the GPU path and the CPU oracle.

Nothing here is part of the optimizer's arithmetic: this module only draws the
*inputs* (the quadratic's curvature ``a`` and optimum ``xstar``, per-coordinate
noise levels, explicit gradient tensors, Zipf-distributed row sets) with numpy's
seeded generators, so that both sides are fed identical bits.  The random
numbers the method itself consumes inside the fused step (noise and per-worker
offsets from Philox4x32-10) are implemented independently on each side.

The five workloads follow the benchmark configurations of this repository; the
embedding-table one stands in for the state shapes of the paper's LSTM-2048-512
language model on the 1B Word benchmark (Section 6.1), whose data and weights
are not used.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    d: int
    W: int
    H: int
    T: int
    eta: float
    eps: float
    kind: str = "quadratic"            # quadratic | explicit | embedding
    a_dist: str = "uniform"            # uniform U(0.1,10) | loguniform [1e-3,1e2]
    noise_scale: float = 0.1
    off_scale: float = 0.1             # per-worker optimum offsets ~ N(0, 0.1^2) per coordinate
    seed: int = 0
    # embedding workload
    rows: int = 0
    row_len: int = 0
    k: int = 0
    zipf_s: float = 1.1
    val_sigma: float = 0.1
    dense_blocks: tuple = field(default_factory=tuple)
    H_sweep: tuple = field(default_factory=tuple)


WORKLOADS = {
    "c1": Workload("c1", d=1_048_576, W=4, H=4, T=64, eta=0.5, eps=1.0),
    "c2": Workload("c2", d=25_000_000, W=8, H=8, T=256, eta=0.1, eps=1.0, a_dist="loguniform"),
    "c3": Workload("c3", d=100_000_000, W=8, H=16, T=512, eta=0.1, eps=1.0, kind="explicit",
                   H_sweep=(1, 4, 16, 64)),
    "c4": Workload("c4", d=800_000 * 512, W=8, H=16, T=256, eta=0.5, eps=1.0, kind="embedding",
                   rows=800_000, row_len=512, k=8192, dense_blocks=((2048, 8192),) * 4),
    "c5": Workload("c5", d=400_000_000, W=8, H=16, T=1024, eta=0.05, eps=1e-2),
}


# Elements (10 GB) between the arrays of the benchmark's spread layout: 19 arrays then span 190 GB, i.e. every
# part of the 288 GB address range; with 6 or 8 GB the result still depended on where the backing allocation
# happened to start (8.7 to 9.6 ms per step from run to run), with 10 GB it was 8.71-8.73 ms in every run.
SPREAD_ROW_DISTANCE = 2_500_000_000


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def curvature(d: int, seed: int, dist: str = "uniform") -> np.ndarray:
    """``a`` of the diagonal quadratic: U(0.1, 10) or log-uniform on [1e-3, 1e2]."""
    u = _rng(seed, 0).random(d, dtype=np.float32)
    if dist == "uniform":
        return (np.float32(0.1) + np.float32(9.9) * u).astype(np.float32)
    if dist == "loguniform":
        return np.power(np.float32(10.0), np.float32(-3.0) + np.float32(5.0) * u).astype(np.float32)
    raise ValueError(dist)


def optimum(d: int, seed: int) -> np.ndarray:
    """Shared optimum ``xstar ~ N(0, 1)``."""
    return _rng(seed, 1).standard_normal(d, dtype=np.float32)


def offsets(d: int, W: int, seed: int, scale: float = 0.1) -> np.ndarray:
    """Per-worker shifts of the optimum as a stored array [W][d] (the alternative
    to regenerating them inside the kernel)."""
    return (np.float32(scale) * _rng(seed, 2).standard_normal((W, d), dtype=np.float32)).astype(np.float32)


def sigma(d: int, seed: int) -> np.ndarray:
    """Per-coordinate gradient noise level, log-uniform on [1e-4, 1]."""
    u = _rng(seed, 4).random(d, dtype=np.float32)
    return np.power(np.float32(10.0), np.float32(-4.0) * u).astype(np.float32)


def explicit_gradients(d: int, W: int, seed: int, step: int, sig: np.ndarray | None = None) -> np.ndarray:
    """A dense gradient tensor [W][d] for one iteration: N(0, sigma_j^2)."""
    g = _rng(seed, 1000 + step).standard_normal((W, d), dtype=np.float32)
    if sig is not None:
        g *= sig[None, :]
    return g


class ZipfRows:
    """Draws k distinct rows per (worker, step) with P(rank r) ~ r^-s over ``rows`` ranks;
    rank r is row r-1 (a frequency-sorted vocabulary)."""

    def __init__(self, rows: int, s: float = 1.1):
        w = np.arange(1, rows + 1, dtype=np.float64) ** (-s)
        self.cdf = np.cumsum(w)
        self.cdf /= self.cdf[-1]
        self.rows = rows

    def draw(self, k: int, rng: np.random.Generator) -> np.ndarray:
        if k > self.rows:
            raise ValueError("k exceeds the number of rows")
        got = np.empty(0, dtype=np.int64)
        while got.size < k:
            cand = np.searchsorted(self.cdf, rng.random(4 * k), side="left")
            cand = np.minimum(cand, self.rows - 1)
            allr = np.concatenate([got, cand])
            _, first = np.unique(allr, return_index=True)
            got = allr[np.sort(first)]          # keep first occurrences, in draw order
        return got[:k].astype(np.int32)


def sparse_step(zipf: ZipfRows, W: int, k: int, row_len: int, seed: int, step: int, val_sigma: float = 0.1,
                with_vals: bool = True):
    """Row indices [W][k] (distinct within a worker) and values [W][k][row_len] ~ N(0, val_sigma^2)."""
    rng = _rng(seed, 2000 + step)
    idx = np.stack([zipf.draw(k, rng) for _ in range(W)])
    vals = None
    if with_vals:
        vals = (np.float32(val_sigma) * _rng(seed, 5000 + step).standard_normal((W, k, row_len), dtype=np.float32))
    return idx, vals


def column_sample(d: int, n_groups: int, seed: int = 0) -> np.ndarray:
    """Absolute coordinates of ``n_groups`` whole 4-coordinate groups spread over [0, d):
    the first, the last, and a seeded random choice in between.  Columns of the dense
    path are independent, so the oracle can follow any subset of them exactly."""
    ng = d // 4
    n_groups = min(n_groups, ng)
    rng = _rng(seed, 9)
    q = np.unique(np.concatenate([[0, ng - 1], rng.integers(0, ng, size=max(n_groups - 2, 0))]))
    cols = (q[:, None] * 4 + np.arange(4)[None, :]).reshape(-1)
    if d % 4:
        cols = np.concatenate([cols, np.arange(ng * 4, d)])
    return cols.astype(np.int64)
