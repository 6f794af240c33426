"""Seeded draws the harness hands to both sides as plain inputs: initial rows, per-epoch subsets, radii."""
from __future__ import annotations

import numpy as np


def linear_sigma(a: float, b: float, n_epochs: int) -> np.ndarray:
    """Radius per epoch, linear from ``a`` (epoch 0) to ``b`` (last epoch), both endpoints used."""
    if n_epochs < 1:
        raise ValueError("n_epochs must be >= 1")
    if n_epochs == 1:
        return np.array([float(a)])
    return a + (b - a) * np.arange(n_epochs, dtype=np.float64) / (n_epochs - 1)


def exponential_sigma(a: float, b: float, n_epochs: int) -> np.ndarray:
    """Radius per epoch, geometric from ``a`` (epoch 0) to ``b`` (last epoch): a * (b / a) ** (e / (E - 1)).
    A second decay type next to the linear one (the paper tunes the decay type without listing the choices); the
    radius is an argument of the library either way."""
    if n_epochs < 1 or a <= 0 or b <= 0:
        raise ValueError("need n_epochs >= 1 and positive radii")
    if n_epochs == 1:
        return np.array([float(a)])
    return a * (b / a) ** (np.arange(n_epochs, dtype=np.float64) / (n_epochs - 1))


def draw_initial_rows(seed: int, n: int, k: int) -> np.ndarray:
    """``k`` distinct row numbers in [0, n): the rows whose values become the initial node weights."""
    if k > n:
        raise ValueError("need at least k rows")
    rng = np.random.default_rng([int(seed), 0x1717])
    return np.sort(rng.choice(n, size=k, replace=False)).astype(np.int64)


def draw_subset(seed: int, epoch: int, n: int, m: int) -> np.ndarray:
    """A uniformly drawn size-``m`` subset of [0, n) for one epoch, as a sorted uint32 list.

    Redrawn per epoch from (seed, epoch).  For large n the subset is built by sampling with replacement and
    de-duplicating until exactly m distinct values remain (each size-m subset stays equally likely because
    the procedure is symmetric in the row numbers).
    """
    if not (0 < m <= n):
        raise ValueError("need 0 < m <= n")
    if n > 0xFFFFFFFF:
        raise ValueError("row numbers must fit uint32")
    rng = np.random.default_rng([int(seed), 0x5E1, int(epoch)])
    if n <= (1 << 24):
        return np.sort(rng.choice(n, size=m, replace=False)).astype(np.uint32)
    have = np.empty(0, dtype=np.int64)
    while have.size < m:
        need = m - have.size
        cand = rng.integers(0, n, size=int(need * 1.2) + 16, dtype=np.int64)
        merged = np.unique(np.concatenate([have, cand]))
        if merged.size > m:
            # drop a uniformly chosen surplus of the *new* values only
            new = np.setdiff1d(merged, have, assume_unique=True)
            keep = rng.choice(new.size, size=need, replace=False)
            merged = np.union1d(have, new[keep])
        have = merged
    return have.astype(np.uint32)


def standardise(X: np.ndarray) -> np.ndarray:
    """Feature-wise zero mean and unit variance (float64 statistics, float32 result), the preprocessing of the
    paper's quality protocol (Section 4.1.1); constant features are only centred."""
    mean = X.mean(axis=0, dtype=np.float64)
    std = X.std(axis=0, dtype=np.float64)
    std[std == 0.0] = 1.0
    return ((X - mean) / std).astype(np.float32)


def train_holdout_split(seed: int, n: int, train_fraction: float = 0.7):
    """A seeded permutation of [0, n) cut into a training part and a holdout part (70 / 30 by default, Section
    4.1.1), each returned as a sorted uint32 row list."""
    if not (0.0 < train_fraction < 1.0) or n < 2:
        raise ValueError("need 0 < train_fraction < 1 and n >= 2")
    perm = np.random.default_rng([int(seed), 0x70]).permutation(n)
    cut = min(max(int(round(n * train_fraction)), 1), n - 1)
    return np.sort(perm[:cut]).astype(np.uint32), np.sort(perm[cut:]).astype(np.uint32)
