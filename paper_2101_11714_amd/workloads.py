"""Seeded synthetic workloads shaped like the paper's (Criteo Kaggle / Terabyte).

This module only draws random inputs (cores, indices, offsets, upstream
gradients, access counts).  It contains none of the method's arithmetic: no
digit decoding, no contraction, no pooling.  Both the CPU oracle's tests and
the HIP path's tests and benchmark read their inputs from here, so the two
sides always see the same arrays.

Shapes follow Table 1 of the paper (Kaggle's largest table: 10,131,227 rows,
dimension 16, cores (1,200,2,R) (R,220,2,R) (R,250,4,1)) and the paper's
statements that Criteo has one index per bag (pooling factor 1, Section 6.6),
that row popularity follows a power law (Section 3.1, Section 4.2) and that
the cache holds 0.01 % of the rows (Section 4.2).  The data sets themselves
are not used; all values are synthetic.
"""

from __future__ import annotations

import math
from dataclasses import dataclass, field
from functools import lru_cache
from typing import Dict, List, Optional, Tuple

import numpy as np
from scipy.special import ndtri


@dataclass(frozen=True)
class TableShape:
    """One TT-compressed table: row/column factorisations and ranks (Eq. 2)."""

    num_rows: int
    m: Tuple[int, int, int]
    n: Tuple[int, int, int]
    r: Tuple[int, int, int, int]

    @property
    def dim(self) -> int:
        return self.n[0] * self.n[1] * self.n[2]

    def core_shape(self, k: int) -> Tuple[int, int, int, int]:
        """Storage shape of core k: [m_k][r_{k-1}][n_k][r_k] (slice-major)."""
        return (self.m[k], self.r[k], self.n[k], self.r[k + 1])

    def core_size(self, k: int) -> int:
        s = self.core_shape(k)
        return s[0] * s[1] * s[2] * s[3]


@dataclass(frozen=True)
class Workload:
    name: str
    tables: Tuple[TableShape, ...]
    n_bags: int
    bag_len: Tuple[int, int]            # inclusive range of bag lengths (uniform)
    index_dist: str                     # "uniform" or "zipf"
    zipf_alpha: float
    init: str                           # "normal0.1" or "sampled_gaussian"
    seed: int
    lr: float = 0.1
    cache_fraction: float = 0.0         # fraction of rows held uncompressed
    warmup_batches: int = 0             # batches that feed the access counts
    identity_rank_map: bool = False     # adversarial: hot rows share digits


def _kaggle(R: int) -> TableShape:
    return TableShape(10_131_227, (200, 220, 250), (2, 2, 4), (1, R, R, 1))


def _multihot_tables() -> Tuple[TableShape, ...]:
    out = []
    for rows in (10_000_000, 15_000_000, 20_000_000, 25_000_000,
                 30_000_000, 35_000_000, 40_000_000):
        out.append(TableShape(rows, (200, 200, rows // 40_000), (4, 4, 4), (1, 32, 32, 1)))
    return tuple(out)


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", (TableShape(1000, (10, 10, 10), (2, 2, 4), (1, 8, 8, 1)),),
                     64, (1, 4), "uniform", 0.0, "normal0.1", 1),
    "kaggle_r32": Workload("kaggle_r32", (_kaggle(32),), 2048, (1, 1), "zipf", 1.05,
                           "sampled_gaussian", 2),
    "sweep_r8": Workload("sweep_r8", (_kaggle(8),), 4096, (1, 1), "zipf", 1.05,
                         "sampled_gaussian", 3),
    "sweep_r16": Workload("sweep_r16", (_kaggle(16),), 4096, (1, 1), "zipf", 1.05,
                          "sampled_gaussian", 3),
    "sweep_r32": Workload("sweep_r32", (_kaggle(32),), 4096, (1, 1), "zipf", 1.05,
                          "sampled_gaussian", 3),
    "sweep_r64": Workload("sweep_r64", (_kaggle(64),), 4096, (1, 1), "zipf", 1.05,
                          "sampled_gaussian", 3),
    "terabyte_r64": Workload("terabyte_r64",
                             (TableShape(40_000_000, (200, 200, 1000), (4, 4, 4), (1, 64, 64, 1)),),
                             8192, (1, 1), "zipf", 1.1, "sampled_gaussian", 4),
    "multihot_cache": Workload("multihot_cache", _multihot_tables(), 8192, (20, 20), "zipf", 1.2,
                               "sampled_gaussian", 5, cache_fraction=1e-4, warmup_batches=10),
}


# --------------------------------------------------------------------------
# cores
# --------------------------------------------------------------------------

_TAIL = 2.0  # the sampled Gaussian keeps only |z| > 2 (Alg. 3 as read here)


def _sampled_gaussian(rng: np.random.Generator, size: int) -> np.ndarray:
    """Standard normal conditioned on |z| > 2, drawn by inverting the tail CDF."""
    u = rng.random(size)
    sign = np.where(rng.random(size) < 0.5, -1.0, 1.0)
    p_tail = 0.5 * math.erfc(_TAIL / math.sqrt(2.0))          # P(z > 2)
    z = -ndtri(u * p_tail)                                    # z > 2
    return sign * z


def _sampled_gaussian_second_moment() -> float:
    phi = math.exp(-0.5 * _TAIL * _TAIL) / math.sqrt(2.0 * math.pi)
    p_tail = 0.5 * math.erfc(_TAIL / math.sqrt(2.0))
    return 1.0 + _TAIL * phi / p_tail


def make_cores(shape: TableShape, init: str, seed: int, table: int = 0) -> List[np.ndarray]:
    """Three fp32 cores, core k stored as [m_k][r_{k-1}][n_k][r_k].

    ``normal0.1``: i.i.d. N(0, sigma = 0.1).
    ``sampled_gaussian``: Alg. 3 read as "redraw while |z| <= 2", then one scale
    factor per table so that a reconstructed table entry has variance
    1/(3 num_rows), the N(0, 1/3n) target of Section 3.2.
    """
    cores = []
    for k in range(3):
        rng = np.random.default_rng([seed, table, 100 + k])
        size = shape.core_size(k)
        if init == "normal0.1":
            g = rng.standard_normal(size) * 0.1
        elif init == "sampled_gaussian":
            v = _sampled_gaussian_second_moment()
            scale = (1.0 / (3.0 * shape.num_rows * shape.r[1] * shape.r[2] * v ** 3)) ** (1.0 / 6.0)
            g = _sampled_gaussian(rng, size) * scale
        else:
            raise ValueError(init)
        cores.append(np.ascontiguousarray(g.astype(np.float32).reshape(shape.core_shape(k))))
    return cores


# --------------------------------------------------------------------------
# indices
# --------------------------------------------------------------------------

@lru_cache(maxsize=2)
def _zipf_cdf(num_rows: int, alpha: float) -> np.ndarray:
    w = np.arange(1, num_rows + 1, dtype=np.float64) ** (-alpha)
    c = np.cumsum(w)
    c /= c[-1]
    return c


def _rank_to_row(num_rows: int, seed: int, table: int, identity: bool):
    """A fixed bijection rank -> row id so hot rows are spread over all digits."""
    if identity:
        return 1, 0
    rng = np.random.default_rng([seed, table, 200])
    a = int(0.6180339887 * num_rows) | 1
    a += 2 * int(rng.integers(0, 1000))
    while math.gcd(a, num_rows) != 1:
        a += 2
    b = int(rng.integers(0, num_rows))
    return a, b


def draw_indices(wl: Workload, table: int, count: int, rng: np.random.Generator) -> np.ndarray:
    shape = wl.tables[table]
    if wl.index_dist == "uniform":
        return rng.integers(0, shape.num_rows, size=count, dtype=np.int64)
    cdf = _zipf_cdf(shape.num_rows, wl.zipf_alpha)
    rank0 = np.searchsorted(cdf, rng.random(count), side="left").astype(np.int64)
    rank0 = np.minimum(rank0, shape.num_rows - 1)
    a, b = _rank_to_row(shape.num_rows, wl.seed, table, wl.identity_rank_map)
    return (rank0 * a + b) % shape.num_rows


@dataclass
class Batch:
    indices: np.ndarray                 # int64 [L]
    offsets: np.ndarray                 # int64 [n_bags + 1]
    grad_output: np.ndarray             # float32 [n_bags, N]
    alpha: Optional[np.ndarray] = None  # float32 [L] per-sample weights


def make_batch(wl: Workload, table: int = 0, step: int = 0, with_alpha: bool = False) -> Batch:
    shape = wl.tables[table]
    rng = np.random.default_rng([wl.seed, table, 300, step])
    lo, hi = wl.bag_len
    if lo == hi:
        lens = np.full(wl.n_bags, lo, dtype=np.int64)
    else:
        lens = rng.integers(lo, hi + 1, size=wl.n_bags, dtype=np.int64)
    offsets = np.zeros(wl.n_bags + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    L = int(offsets[-1])
    indices = draw_indices(wl, table, L, rng)
    grad = rng.standard_normal((wl.n_bags, shape.dim)).astype(np.float32)
    alpha = None
    if with_alpha:
        alpha = (0.5 + rng.random(L)).astype(np.float32)
    return Batch(indices, offsets, grad, alpha)


def warmup_counts(wl: Workload, table: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Access counts over ``warmup_batches`` earlier batches of the same sampler.

    Stands in for the paper's warm-up phase that fills the cache (Section 4.2).
    Returns (row ids seen, their counts); the order of the rows is scrambled so
    that a consumer cannot rely on it.
    """
    parts = [make_batch(wl, table, step=1_000_000 + s).indices for s in range(wl.warmup_batches)]
    rows, counts = np.unique(np.concatenate(parts), return_counts=True)
    rng = np.random.default_rng([wl.seed, table, 400])
    p = rng.permutation(rows.size)
    return rows[p].astype(np.int64), counts[p].astype(np.int64)


def cache_size(wl: Workload, table: int = 0) -> int:
    return int(math.ceil(wl.cache_fraction * wl.tables[table].num_rows)) if wl.cache_fraction else 0


def make_hit_rate_batch(shape: TableShape, cached_rows: np.ndarray, n_bags: int, bag_len: int, hit_rate: float,
                        seed: int) -> Batch:
    """A batch whose share of cached positions is controlled (the synthetic samples of the paper's
    hit-rate study, Section 6.7): every position is, with probability hit_rate, a row drawn uniformly
    from cached_rows, else a row drawn uniformly from the rest of the table."""
    rng = np.random.default_rng([seed, 700, n_bags, bag_len, int(round(hit_rate * 10000))])
    L = n_bags * bag_len
    cached_rows = np.asarray(cached_rows, dtype=np.int64)
    idx = rng.integers(0, shape.num_rows, L, dtype=np.int64)
    is_cached = np.isin(idx, cached_rows)
    while is_cached.any():                                   # a miss must really miss
        idx[is_cached] = rng.integers(0, shape.num_rows, int(is_cached.sum()), dtype=np.int64)
        is_cached = np.isin(idx, cached_rows)
    hit = rng.random(L) < hit_rate
    if cached_rows.size:
        idx[hit] = cached_rows[rng.integers(0, cached_rows.size, int(hit.sum()))]
    offsets = np.arange(n_bags + 1, dtype=np.int64) * bag_len
    grad = rng.standard_normal((n_bags, shape.dim)).astype(np.float32)
    return Batch(idx, offsets, grad, None)
