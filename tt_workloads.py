"""Seeded synthetic inputs for the TT embedding-bag hot path.

This module only *draws inputs* (table shapes, TT cores, indices, bag offsets,
output gradients).  It contains none of the method's arithmetic: no index
splitting, no core contraction, no sorting of lookups.  Both the CPU oracle's
tests and the HIP path's tests / benchmark take their inputs from here so that
the two sides see identical bytes.

Workloads.  The paper trains on click-log and grid datasets whose sparse
features follow a power law (Section II-C) with tables of up to 10^7-10^8 rows
and embedding dimensions 16/64/128 (Table II); none of those datasets is
available, so five synthetic configurations with the same table shapes and a
bounded Zipf access law stand in for them.

Recipe (all `numpy.random.default_rng(seed)`):
  seed(cfg, table, what, batch) = 1466800 + 100*cfg + table + what + 1000*batch
  what = 0 indices, 50 cores, 75 bag lengths / output gradients.
  bounded Zipf: P(rank = k) ~ k^-alpha for k = 1..N, sampled by inverse CDF
  (float64 cumulative sum + searchsorted); row = rank-1, or pi[rank-1] with
  pi = rng.permutation(N) when the configuration asks for a row permutation.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from functools import lru_cache

import numpy as np

SEED_BASE = 1466800


@dataclass(frozen=True)
class TableShape:
    """Shape of one TT table: N rows factored n1*n2*n3 (>= N), D = d1*d2*d3 columns."""

    num_rows: int
    n: tuple
    d: tuple
    r: tuple  # (1, R1, R2, 1)

    @property
    def dim(self) -> int:
        return self.d[0] * self.d[1] * self.d[2]

    def core_shape(self, k: int) -> tuple:
        """Core k is stored as [r[k]][n[k]][d[k]][r[k+1]], row-major."""
        return (self.r[k], self.n[k], self.d[k], self.r[k + 1])

    def core_size(self, k: int) -> int:
        return self.r[k] * self.n[k] * self.d[k] * self.r[k + 1]


@dataclass(frozen=True)
class Config:
    cfg: int
    name: str
    tables: tuple  # of TableShape
    sigma: float
    batch: int  # bags per table
    multi_hot: bool  # False: one lookup per bag; True: length ~ U{1..max_len}
    max_len: int
    dist: str  # "uniform" | "zipf"
    alpha: float
    permute_rows: bool
    lr: float
    phases: str


def near_equal_factors(num_rows: int) -> tuple:
    """Three near-equal factors whose product covers num_rows (padding allowed).

    n3 = ceil(N^(1/3)), n2 = ceil(sqrt(N/n3)), n1 = ceil(N/(n2*n3)); rows at or
    beyond num_rows are padding and are never addressed.
    """
    n3 = max(1, int(round(num_rows ** (1.0 / 3.0))) - 2)
    while n3 ** 3 < num_rows:  # smallest n3 with n3^3 >= N (integer arithmetic, no float ceil)
        n3 += 1
    n2 = max(1, math.isqrt(num_rows // n3) - 2)
    while n2 * n2 * n3 < num_rows:  # smallest n2 with n2^2 * n3 >= N
        n2 += 1
    n1 = max(1, -(-num_rows // (n2 * n3)))
    assert n1 * n2 * n3 >= num_rows
    return (n1, n2, n3)


def _cfg5_rows() -> tuple:
    rng = np.random.default_rng(SEED_BASE + 500 + 99)
    u = rng.uniform(3.0, math.log10(4e7), size=26)
    rows = np.round(10.0 ** u).astype(np.int64)
    # make the two ends of the stated range present so the extremes are exercised
    rows[0] = 1000
    rows[1] = 40_000_000
    return tuple(int(x) for x in rows)


def get_config(cfg: int) -> Config:
    if cfg == 1:
        t = TableShape(1000, (10, 10, 10), (2, 2, 4), (1, 4, 4, 1))
        return Config(1, "cfg1", (t,), 0.1, 256, False, 1, "uniform", 0.0, False, 0.01, "fwd+bwd")
    if cfg == 2:
        t = TableShape(1_000_000, (100, 100, 100), (4, 4, 4), (1, 16, 16, 1))
        return Config(2, "cfg2", (t,), 0.05, 4096, False, 1, "zipf", 1.05, True, 0.01, "fwd+bwd")
    if cfg in (3, 4):
        t = TableShape(10_000_000, (200, 250, 200), (4, 8, 4), (1, 32, 32, 1))
        return Config(cfg, "cfg%d" % cfg, (t,) * 8, 0.05, 16384, True, 40, "zipf", 1.2, False, 0.01,
                      "fwd" if cfg == 3 else "bwd+update")
    if cfg == 5:
        tabs = tuple(TableShape(nr, near_equal_factors(nr), (4, 8, 4), (1, 64, 64, 1))
                     for nr in _cfg5_rows())
        return Config(5, "cfg5", tabs, 0.05, 65536, False, 1, "zipf", 1.1, False, 0.01,
                      "reorder||fwd+bwd+update")
    raise ValueError("unknown config %r" % (cfg,))


def _seed(cfg: int, table: int, what: int, batch: int = 0) -> int:
    return SEED_BASE + 100 * cfg + table + what + 1000 * batch


def make_cores(cfg: Config, table: int) -> list:
    """Three fp32 cores ~ N(0, sigma), each flat in [r][n][d][r'] order."""
    shape = cfg.tables[table]
    rng = np.random.default_rng(_seed(cfg.cfg if cfg.cfg != 4 else 3, table, 50))
    return [(rng.standard_normal(shape.core_size(k), dtype=np.float32) * np.float32(cfg.sigma))
            for k in range(3)]


@lru_cache(maxsize=4)
def _zipf_cdf(num_rows: int, alpha: float) -> np.ndarray:
    k = np.arange(1, num_rows + 1, dtype=np.float64)
    w = k ** (-alpha)
    c = np.cumsum(w)
    c /= c[-1]
    return c


def sample_rows(rng, num_rows: int, count: int, dist: str, alpha: float,
                perm: np.ndarray | None = None) -> np.ndarray:
    if dist == "uniform":
        rows = rng.integers(0, num_rows, size=count, dtype=np.int64)
    elif dist == "zipf":
        u = rng.random(count)
        rows = np.searchsorted(_zipf_cdf(num_rows, alpha), u, side="left").astype(np.int64)
        np.minimum(rows, num_rows - 1, out=rows)
    else:
        raise ValueError(dist)
    if perm is not None:
        rows = perm[rows]
    return rows


def make_batch(cfg: Config, table: int, batch: int = 0, permute_rows: bool | None = None,
               num_bags: int | None = None):
    """Return (indices int64[nnz], offsets int64[B+1]) for one table and batch.

    `permute_rows` overrides the configuration (used to report the permuted
    variant of configs 3-5 next to the literal, identity-mapped reading).
    `num_bags` overrides the batch size (bounded samples of the same workload).
    """
    shape = cfg.tables[table]
    base_cfg = cfg.cfg if cfg.cfg != 4 else 3  # config 4 reuses config 3's inputs
    nb = cfg.batch if num_bags is None else int(num_bags)
    rng_len = np.random.default_rng(_seed(base_cfg, table, 75, batch))
    if cfg.multi_hot:
        lens = rng_len.integers(1, cfg.max_len + 1, size=nb, dtype=np.int64)
    else:
        lens = np.ones(nb, dtype=np.int64)
    offsets = np.zeros(nb + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    nnz = int(offsets[-1])
    do_perm = cfg.permute_rows if permute_rows is None else permute_rows
    perm = None
    if do_perm:
        perm = np.random.default_rng(_seed(base_cfg, table, 25)).permutation(shape.num_rows)
    rng = np.random.default_rng(_seed(base_cfg, table, 0, batch))
    indices = sample_rows(rng, shape.num_rows, nnz, cfg.dist, cfg.alpha, perm)
    return indices, offsets


def make_grad(cfg: Config, table: int, batch: int = 0, num_bags: int | None = None) -> np.ndarray:
    """Per-bag output gradients ~ N(0,1), fp32 [B][D] row-major (flat)."""
    shape = cfg.tables[table]
    nb = cfg.batch if num_bags is None else int(num_bags)
    base_cfg = cfg.cfg if cfg.cfg != 4 else 3
    rng = np.random.default_rng(_seed(base_cfg, table, 76, batch))
    return rng.standard_normal(nb * shape.dim, dtype=np.float32)


def small_random_problem(seed: int, n=(3, 4, 5), d=(2, 3, 2), r=(1, 3, 4, 1), num_rows=None,
                         num_bags=7, max_len=5, sigma=0.5):
    """A tiny random table + batch used by unit tests (odd, unequal factors on purpose)."""
    rng = np.random.default_rng(seed)
    nr = n[0] * n[1] * n[2] if num_rows is None else num_rows
    shape = TableShape(nr, tuple(n), tuple(d), tuple(r))
    cores = [(rng.standard_normal(shape.core_size(k)) * sigma).astype(np.float32) for k in range(3)]
    lens = rng.integers(0, max_len + 1, size=num_bags)
    offsets = np.zeros(num_bags + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    indices = rng.integers(0, nr, size=int(offsets[-1]), dtype=np.int64)
    grad = rng.standard_normal(num_bags * shape.dim).astype(np.float32)
    return shape, cores, indices, offsets, grad
