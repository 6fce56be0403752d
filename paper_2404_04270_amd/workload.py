"""Seeded synthetic inputs for the embedding hot path.

This module only *draws inputs* (tables, lookup indices, upstream gradients,
hot-row sets).  It holds none of the method's arithmetic, imports neither the
HIP binding nor the CPU oracle, and is the one piece of code both of them are
fed from, so that a parity failure can never come from two generators
disagreeing.

The lookups stand in for the click-log datasets the paper trains on (its
evaluation section, Table 3): those are heavily skewed (section 2.3.2 reports
hot rows receiving more than 100x the accesses of the others), which a bounded
Zipf law over the rows of a table reproduces.  Shapes follow the five
workloads listed in `CONFIGS`.
"""
from __future__ import annotations

import functools
from dataclasses import dataclass, replace
from typing import Optional

import numpy as np


@dataclass(frozen=True)
class Config:
    """One workload: table geometry, lookup law and the staleness schedule."""

    name: str
    num_tables: int          # T
    rows: int                # R rows per table
    dim: int                 # D floats per row
    batch: int               # B samples per iteration
    bag: int                 # L lookups per sample and table (sum-pooled)
    zipf_alpha: float        # exponent of the bounded Zipf law over ranks
    permute: bool            # rank -> row through a per-table random permutation
    lr: float                # SGD learning rate
    grad_sigma: float        # upstream gradients ~ N(0, grad_sigma)
    hot_frac: float          # hot set = this fraction of rows, by access count
    snapshot_every: int      # K: iterations between snapshots
    threshold: float         # drift threshold T
    iters: int               # iterations of the full run
    seed: int
    init_bound: float = 0.05  # weights ~ uniform(-init_bound, init_bound)

    @property
    def hot_rows(self) -> int:
        return int(round(self.hot_frac * self.rows))

    @property
    def table_bytes(self) -> int:
        return self.num_tables * self.rows * self.dim * 4

    def scaled(self, **kw) -> "Config":
        return replace(self, **kw)


CONFIGS = {
    1: Config("cfg1_tiny", 8, 10_000, 16, 128, 1, 1.05, False, 0.01, 0.01,
              0.01, 10, 1e-3, 100, 0),
    2: Config("cfg2_26x100k_d16", 26, 100_000, 16, 2048, 1, 1.1, True, 0.01,
              0.01, 0.01, 50, 5e-4, 1000, 1),
    3: Config("cfg3_26x1m_d64", 26, 1_000_000, 64, 8192, 1, 1.2, False, 0.01,
              0.01, 0.005, 100, 1e-4, 2000, 2),
    4: Config("cfg4_multihot_8x10m_d128", 8, 10_000_000, 128, 4096, 20, 1.2,
              False, 0.01, 0.01, 0.001, 100, 1e-4, 1000, 3),
    5: Config("cfg5_single_200m_d64", 1, 200_000_000, 64, 65_536, 1, 1.05,
              False, 0.01, 0.01, 0.0005, 200, 1e-4, 1000, 4),
}
CFG5_THRESHOLD_SWEEP = (0.0, 1e-5, 1e-4, 1e-3)


@functools.lru_cache(maxsize=2)
def zipf_cdf(rows: int, alpha: float) -> np.ndarray:
    """Cumulative distribution of P(rank k) ~ k^-alpha, k = 1..rows (fp64).
    Read-only for callers: the last two tables are kept and shared."""
    pmf = np.arange(1, rows + 1, dtype=np.float64) ** (-alpha)
    cdf = np.cumsum(pmf)
    cdf /= cdf[-1]
    cdf[-1] = 1.0
    cdf.setflags(write=False)
    return cdf


class Workload:
    """Draws the arrays of one config, deterministically from its seed."""

    def __init__(self, cfg: Config):
        self.cfg = cfg
        self._cdf: Optional[np.ndarray] = None
        self._perm: Optional[list] = None

    # ---- lookups -------------------------------------------------------
    def _rank_to_row(self, table: int) -> Optional[np.ndarray]:
        if not self.cfg.permute:
            return None
        if self._perm is None:
            self._perm = [
                np.random.default_rng([self.cfg.seed, 3000 + t])
                .permutation(self.cfg.rows).astype(np.int32)
                for t in range(self.cfg.num_tables)
            ]
        return self._perm[table]

    def indices(self, first_iter: int, n_iters: int) -> np.ndarray:
        """int32 [n_iters, T, B, L]: row ids looked up in each iteration."""
        c = self.cfg
        if self._cdf is None:
            self._cdf = zipf_cdf(c.rows, c.zipf_alpha)
        out = np.empty((n_iters, c.num_tables, c.batch, c.bag), dtype=np.int32)
        for k in range(n_iters):
            it = first_iter + k
            for t in range(c.num_tables):
                u = np.random.default_rng([c.seed, 1000 + t, it]).random(
                    c.batch * c.bag)
                rank0 = np.searchsorted(self._cdf, u, side="left")
                np.minimum(rank0, c.rows - 1, out=rank0)
                perm = self._rank_to_row(t)
                rows = rank0 if perm is None else perm[rank0]
                out[k, t] = rows.reshape(c.batch, c.bag)
        return out

    # ---- dense inputs --------------------------------------------------
    def weights(self, table: int) -> np.ndarray:
        """fp32 [R, D] initial values of one table."""
        c = self.cfg
        rng = np.random.default_rng([c.seed, table])
        w = rng.random((c.rows, c.dim), dtype=np.float32)
        w *= np.float32(2.0 * c.init_bound)
        w -= np.float32(c.init_bound)
        return w

    def weights_device(self, table: int, device):
        """Same law as `weights`, drawn on the device (for tables too large to
        draw on the host in reasonable time).  A different stream of numbers
        than `weights`: callers that compare against the CPU copy it back."""
        import torch
        c = self.cfg
        gen = torch.Generator(device=device)
        gen.manual_seed(c.seed * 1000 + table)
        w = torch.empty((c.rows, c.dim), dtype=torch.float32, device=device)
        w.uniform_(-c.init_bound, c.init_bound, generator=gen)
        return w

    def grads(self, it: int) -> np.ndarray:
        """fp32 [T, B, D]: gradient of the loss w.r.t. each pooled vector."""
        c = self.cfg
        rng = np.random.default_rng([c.seed, 2000, it])
        g = rng.standard_normal((c.num_tables, c.batch, c.dim),
                                dtype=np.float32)
        g *= np.float32(c.grad_sigma)
        return g


def hot_set(idx_stream: np.ndarray, rows: int, n_hot: int) -> np.ndarray:
    """Most-accessed rows of each table over a stream of lookups.

    idx_stream: int32 [n_iters, T, B, L].  Returns int32 [T, n_hot], each row
    of it ascending by row id.  Ties in the count go to the lower row id.
    """
    n_tables = idx_stream.shape[1]
    out = np.empty((n_tables, n_hot), dtype=np.int32)
    for t in range(n_tables):
        if n_hot == 0:
            continue
        # The first n_hot rows by (count descending, row ascending), without sorting
        # all rows: c is the n_hot-th largest count; every row above it is in, and
        # the places left go to the rows that have exactly c, lowest ids first.
        flat = idx_stream[:, t].reshape(-1)
        if rows <= max(1, flat.size):
            ids, cnt = None, np.bincount(flat, minlength=rows)       # ids = 0 .. rows-1
        else:
            # far more rows than lookups: count only the rows that occur
            ids, cnt = np.unique(flat, return_counts=True)
            if ids.size < n_hot:       # not enough accessed rows: unaccessed ones, lowest first
                rest = np.setdiff1d(np.arange(min(rows, n_hot + ids.size)), ids)
                out[t] = np.sort(np.concatenate([ids, rest[: n_hot - ids.size]])).astype(np.int32)
                continue
        c = np.partition(cnt, cnt.size - n_hot)[cnt.size - n_hot]
        above = np.flatnonzero(cnt > c)
        ties = np.flatnonzero(cnt == c)[: n_hot - above.size]
        pick = np.sort(np.concatenate([above, ties]))
        out[t] = (pick if ids is None else ids[pick]).astype(np.int32)
    return out


def bitmap_words(rows: int) -> int:
    return (rows + 31) // 32
