"""Seeded synthetic inputs shaped like the paper's workloads.

The paper (Section 5) trains logistic regression on LIBSVM text/tabular sets
and a small network on MNIST; none of those files is used here.  These
generators produce stand-ins with the same shapes, densities and value
distributions.  This module holds data generation only: no loss, gradient,
quantizer, sparsifier or update arithmetic lives here, so that it can feed both
the CPU oracle and the GPU library without coupling them.

Every generator is a pure function of its arguments (numpy ``default_rng``).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass
class Problem:
    """A finite-sum problem instance: features, labels and regularisation weights."""

    n: int
    d: int
    y: np.ndarray                        # float32 [n], entries +1/-1
    l2: float                            # weight of the smooth squared-norm term
    l1: float                            # weight of the nonsmooth 1-norm term
    dense: Optional[np.ndarray] = None   # float32 [n, d] row-major, or None
    indptr: Optional[np.ndarray] = None  # int64 [n+1]   (CSR)
    indices: Optional[np.ndarray] = None  # int32 [nnz]  sorted, unique per row
    values: Optional[np.ndarray] = None  # float32 [nnz]
    meta: dict = field(default_factory=dict)

    @property
    def is_csr(self) -> bool:
        return self.dense is None


def _labels_from_planted(margins: np.ndarray, rng: np.random.Generator, flip: float) -> np.ndarray:
    y = np.where(margins >= 0, 1.0, -1.0).astype(np.float32)
    flips = rng.random(y.shape[0]) < flip
    y[flips] = -y[flips]
    return y


def dense_logistic(n: int, d: int, seed: int = 0, l2: float = 1e-4, l1: float = 0.0,
                   flip: float = 0.05, chunk_rows: int = 16384) -> Problem:
    """Dense features ~ N(0,1)/sqrt(d), labels from a planted N(0,I) vector plus flips.

    Stands in for the paper's dense workloads (the covtype/MNIST-shaped ones).
    """
    rng = np.random.default_rng(seed)
    w_star = rng.standard_normal(d).astype(np.float32)
    X = np.empty((n, d), dtype=np.float32)
    margins = np.empty(n, dtype=np.float64)
    scale = np.float32(1.0 / np.sqrt(d))
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        blk = rng.standard_normal((r1 - r0, d), dtype=np.float32)
        blk *= scale
        X[r0:r1] = blk
        margins[r0:r1] = blk.astype(np.float64) @ w_star.astype(np.float64)
    y = _labels_from_planted(margins, rng, flip)
    return Problem(n=n, d=d, y=y, l2=l2, l1=l1, dense=X, meta={"kind": "dense", "seed": seed})


def sparse_text_logistic(n: int, d: int, mean_nnz: float = 52.0, seed: int = 0,
                         l2: float = 1e-4, l1: float = 1e-5, flip: float = 0.05) -> Problem:
    """CSR features shaped like a bag-of-words corpus (real-sim / rcv1 in the paper).

    Row lengths: a lognormal/Poisson mix with the requested mean; column j is drawn
    with probability proportional to 1/(j+1) without repeats inside a row; values are
    (1+log tf)*log(1+n/df_j) with tf geometric; rows are scaled to unit 2-norm; indices
    are sorted.  Labels come from a planted sparse vector plus flips.
    """
    rng = np.random.default_rng(seed)
    # --- row lengths
    sigma = 0.6
    logn = rng.lognormal(mean=np.log(mean_nnz) - 0.5 * sigma * sigma, sigma=sigma, size=n)
    pois = rng.poisson(mean_nnz, size=n)
    pick = rng.random(n) < 0.5
    lens = np.where(pick, np.rint(logn), pois).astype(np.int64)
    lens = np.clip(lens, 1, min(d, 8 * int(mean_nnz) + 8))
    # --- candidate columns (oversampled), Zipf weights via inverse CDF
    w = 1.0 / (np.arange(d, dtype=np.float64) + 1.0)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    over = lens * 2 + 8
    row_of = np.repeat(np.arange(n, dtype=np.int64), over)
    cols = np.searchsorted(cdf, rng.random(row_of.shape[0]), side="right").astype(np.int64)
    np.minimum(cols, d - 1, out=cols)
    # dedupe (row, col)
    key = row_of * d + cols
    key = np.unique(key)
    row_of = key // d
    cols = key % d
    # keep at most lens[row] of the unique candidates, chosen at random
    tie = rng.random(key.shape[0])
    order = np.lexsort((tie, row_of))
    row_sorted = row_of[order]
    starts = np.searchsorted(row_sorted, np.arange(n))
    rank = np.arange(key.shape[0]) - starts[row_sorted]
    keep = order[rank < lens[row_sorted]]
    keep.sort()                      # back to (row, col) order: key was sorted
    row_of = row_of[keep]
    cols = cols[keep]
    counts = np.bincount(row_of, minlength=n)
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=indptr[1:])
    nnz = int(indptr[-1])
    # --- values
    df = np.bincount(cols, minlength=d).astype(np.float64)
    idf = np.log1p(n / np.maximum(df, 1.0))
    tf = rng.geometric(0.6, size=nnz).astype(np.float64)
    vals = (1.0 + np.log(tf)) * idf[cols]
    sq = np.zeros(n, dtype=np.float64)
    np.add.at(sq, row_of, vals * vals)
    vals = vals / np.sqrt(sq[row_of])
    values = vals.astype(np.float32)
    indices = cols.astype(np.int32)
    # --- labels from a planted sparse vector
    w_star = np.zeros(d, dtype=np.float64)
    support = rng.random(d) < 0.05
    support[: min(d, 64)] = True
    w_star[support] = rng.standard_normal(int(support.sum()))
    margins = np.zeros(n, dtype=np.float64)
    np.add.at(margins, row_of, vals * w_star[cols])
    margins -= np.median(margins)
    y = _labels_from_planted(margins, rng, flip)
    return Problem(n=n, d=d, y=y, l2=l2, l1=l1, indptr=indptr, indices=indices, values=values,
                   meta={"kind": "csr", "seed": seed, "nnz": nnz})


def mixture_vector(N: int, seed: int = 0, p_wide: float = 0.1, sigma_narrow: float = 0.01,
                   sigma_wide: float = 1.0, chunk: int = 1 << 24) -> np.ndarray:
    """Gradient-like vector: each coordinate N(0, sigma_wide^2) w.p. p_wide else N(0, sigma_narrow^2)."""
    rng = np.random.default_rng(seed)
    v = np.empty(N, dtype=np.float32)
    for s in range(0, N, chunk):
        e = min(N, s + chunk)
        z = rng.standard_normal(e - s, dtype=np.float32)
        wide = rng.random(e - s, dtype=np.float32) < np.float32(p_wide)
        z *= np.where(wide, np.float32(sigma_wide), np.float32(sigma_narrow))
        v[s:e] = z
    return v


@dataclass(frozen=True)
class Config:
    """One named workload: problem shape plus algorithm settings."""

    name: str
    algo: str          # "asylpg" | "sparse" | "acc" | "quantizer"
    n: int
    d: int
    M: int
    B: int
    b_x: int
    b: int
    m: int             # rounds per epoch
    S: int             # epochs
    lr: float
    l2: float
    l1: float
    csr: bool
    seed: int = 0


# The five workloads.  lr, m and S for C2..C4 are choices made here (the paper
# tunes lr on a grid and uses m = ceil(n/B)); they are listed in the design notes.
CONFIGS = {
    "C1": Config("C1", "asylpg", n=2000, d=1000, M=4, B=16, b_x=8, b=8, m=500, S=1,
                 lr=0.1, l2=1e-4, l1=0.0, csr=False),
    "C2": Config("C2", "asylpg", n=72000, d=20958, M=8, B=32, b_x=8, b=8, m=282, S=2,
                 lr=0.1, l2=1e-4, l1=1e-5, csr=True),
    "C3": Config("C3", "sparse", n=72000, d=20958, M=16, B=64, b_x=8, b=4, m=71, S=2,
                 lr=0.1, l2=1e-4, l1=1e-5, csr=True),
    "C4": Config("C4", "acc", n=200000, d=4096, M=32, B=256, b_x=8, b=8, m=25, S=2,
                 lr=0.1, l2=1e-4, l1=0.0, csr=False),
    "C5": Config("C5", "quantizer", n=0, d=1 << 28, M=16, B=0, b_x=8, b=8, m=0, S=0,
                 lr=0.0, l2=0.0, l1=0.0, csr=False),
}


def make_problem(cfg: Config, n: Optional[int] = None, d: Optional[int] = None) -> Problem:
    """Build the problem of a config, optionally at reduced n/d (same recipe)."""
    n = cfg.n if n is None else n
    d = cfg.d if d is None else d
    if cfg.csr:
        return sparse_text_logistic(n, d, seed=cfg.seed, l2=cfg.l2, l1=cfg.l1)
    return dense_logistic(n, d, seed=cfg.seed, l2=cfg.l2, l1=cfg.l1)
