"""Seeded Gaussian-mixture sample matrices, reproducible however they are chunked.

Rows are produced in fixed blocks of BLOCK_ROWS rows; block ``b`` draws from
``numpy.random.default_rng([seed, 1 + b])`` only, so ``rows(a, c)`` returns the same values whether the
caller asks for the whole matrix, one chunk at a time, or a single row.  Values are cast to float32 once:
that float32 array *is* the dataset handed to both the oracle and the GPU path.
"""
from __future__ import annotations

import numpy as np

BLOCK_ROWS = 1 << 16


class GaussianMixture:
    """Mixture of ``n_comp`` axis-aligned Gaussians in ``d`` dimensions, plus an optional uniform background.

    centres  ~ U[centre_lo, centre_hi]^d
    std      ~ U[std_lo, std_hi], one value per component (isotropic=True) or per component and axis
    weights  equal, or one draw from Dirichlet(1, ..., 1)
    noise    with probability ``noise_frac`` a row is U[noise_lo, noise_hi]^d instead of a mixture draw
    """

    def __init__(self, seed: int, d: int, n_comp: int, *, centre=(-10.0, 10.0), std=(0.2, 3.0),
                 isotropic=False, weights="equal", noise_frac=0.0, noise=(-15.0, 15.0)):
        self.seed = int(seed)
        self.d = int(d)
        self.n_comp = int(n_comp)
        self.noise_frac = float(noise_frac)
        self.noise = (float(noise[0]), float(noise[1]))
        rng = np.random.default_rng([self.seed, 0])
        self.centres = rng.uniform(centre[0], centre[1], size=(n_comp, d))
        if isotropic:
            self.stds = np.repeat(rng.uniform(std[0], std[1], size=(n_comp, 1)), d, axis=1)
        else:
            self.stds = rng.uniform(std[0], std[1], size=(n_comp, d))
        if weights == "equal":
            self.weights = np.full(n_comp, 1.0 / n_comp)
        elif weights == "dirichlet":
            self.weights = rng.dirichlet(np.ones(n_comp))
        else:
            raise ValueError(f"unknown weights rule {weights!r}")

    def _block(self, b: int) -> np.ndarray:
        rng = np.random.default_rng([self.seed, 1 + b])
        comp = rng.choice(self.n_comp, size=BLOCK_ROWS, p=self.weights)
        z = rng.standard_normal(size=(BLOCK_ROWS, self.d), dtype=np.float32)
        out = z * self.stds[comp].astype(np.float32) + self.centres[comp].astype(np.float32)
        if self.noise_frac > 0.0:
            is_noise = rng.random(BLOCK_ROWS) < self.noise_frac
            # one full uniform block is drawn and used where flagged, so the stream never depends on the count
            u = rng.uniform(self.noise[0], self.noise[1], size=(BLOCK_ROWS, self.d)).astype(np.float32)
            out[is_noise] = u[is_noise]
        return out.astype(np.float32, copy=False)

    def rows(self, start: int, stop: int) -> np.ndarray:
        """float32 array of rows ``start`` .. ``stop-1`` (C order, shape (stop-start, d))."""
        start, stop = int(start), int(stop)
        if stop < start or start < 0:
            raise ValueError("bad row range")
        out = np.empty((stop - start, self.d), dtype=np.float32)
        b = start // BLOCK_ROWS
        while b * BLOCK_ROWS < stop:
            lo = max(start, b * BLOCK_ROWS)
            hi = min(stop, (b + 1) * BLOCK_ROWS)
            if hi > lo:
                blk = self._block(b)
                out[lo - start:hi - start] = blk[lo - b * BLOCK_ROWS:hi - b * BLOCK_ROWS]
            b += 1
        return out

    def fill(self, out: np.ndarray, start: int = 0) -> np.ndarray:
        """Write rows ``start`` .. ``start+len(out)-1`` into a caller-provided float32 array (e.g. a memmap)."""
        n = out.shape[0]
        step = BLOCK_ROWS
        for lo in range(0, n, step):
            hi = min(n, lo + step)
            out[lo:hi] = self.rows(start + lo, start + hi)
        return out


def uniform01_rows(seed: int, start: int, stop: int, d: int) -> np.ndarray:
    """U[0,1) float32 rows, block-seeded like GaussianMixture (the distribution of the paper's speed runs)."""
    out = np.empty((stop - start, d), dtype=np.float32)
    b = start // BLOCK_ROWS
    while b * BLOCK_ROWS < stop:
        lo = max(start, b * BLOCK_ROWS)
        hi = min(stop, (b + 1) * BLOCK_ROWS)
        if hi > lo:
            blk = np.random.default_rng([int(seed), 1 + b]).random(size=(BLOCK_ROWS, d), dtype=np.float32)
            out[lo - start:hi - start] = blk[lo - b * BLOCK_ROWS:hi - b * BLOCK_ROWS]
        b += 1
    return out


class Uniform01:
    """U[0,1) rows behind the same interface as GaussianMixture (``rows``, ``fill``)."""

    def __init__(self, seed: int, d: int):
        self.seed, self.d = int(seed), int(d)

    def rows(self, start: int, stop: int) -> np.ndarray:
        return uniform01_rows(self.seed, start, stop, self.d)

    def fill(self, out: np.ndarray, start: int = 0) -> np.ndarray:
        step = BLOCK_ROWS * 16
        for lo in range(0, out.shape[0], step):
            hi = min(out.shape[0], lo + step)
            out[lo:hi] = self.rows(start + lo, start + hi)
        return out
