"""Host-side builder of the K x K neighbourhood-distance matrix G of a regular lattice (paper Section 3.2).

Rectangular and hexagonal maps have a fixed G: the Euclidean distance between node positions.  The data-driven
topologies of Sections 3.2.1-3.2.2 (spanning tree, relative neighbourhood graph) depend on the current weights and
are rebuilt on the GPU by ``Som.som_topology``; there is no host implementation of them in this package.
"""
from __future__ import annotations

import numpy as np


def lattice_distances(n_rows: int, n_cols: int, kind: str = "rect") -> np.ndarray:
    """float32 G for a rectangular ("rect") or hexagonal ("hex") lattice, node k at row k // n_cols."""
    r, c = np.divmod(np.arange(n_rows * n_cols), n_cols)
    if kind == "rect":
        z = c + 1j * r
    elif kind == "hex":
        z = (c + 0.5 * (r & 1)) + 1j * (r * np.sqrt(0.75))
    else:
        raise ValueError(f"unknown lattice {kind!r}")
    return np.abs(z[:, None] - z[None, :]).astype(np.float32)


def graph_distances(kind: str, lattice=None) -> np.ndarray:
    """G of a lattice topology; the graph topologies ("mst", "rng") are served by ``Som.som_topology`` only."""
    if kind in ("rect", "hex"):
        return lattice_distances(lattice[0], lattice[1], kind)
    if kind in ("mst", "rng"):
        raise ValueError(f"{kind!r} distances depend on the weights: use Som.som_topology on the GPU")
    raise ValueError(f"unknown topology {kind!r}")
