"""Host-side builders of the K x K neighbourhood-distance matrix G that the update kernel consumes.

Regular lattices (paper Section 3.2) give Euclidean distances between node positions; the data-driven
topologies (Sections 3.2.1-3.2.2, Algorithms 1-2) give hop counts along a minimum spanning tree or a relative
neighbourhood graph of the current node weights.  Pairwise node distances use the squared-distance Gram
identity in float64, as Section 3.2.1 describes; tree and shortest-path steps use scipy's graph routines.
"""
from __future__ import annotations

import numpy as np
from scipy.sparse import csr_matrix
from scipy.sparse.csgraph import minimum_spanning_tree, shortest_path


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


def _gram_sq_distances(W: np.ndarray) -> np.ndarray:
    W = np.asarray(W, dtype=np.float64)
    sq = (W * W).sum(axis=1)
    d2 = sq[:, None] + sq[None, :] - 2.0 * (W @ W.T)
    np.maximum(d2, 0.0, out=d2)
    np.fill_diagonal(d2, 0.0)
    return 0.5 * (d2 + d2.T)


def _hops(adj: np.ndarray) -> np.ndarray:
    g = shortest_path(csr_matrix(adj), method="D", unweighted=True, directed=False)
    return g.astype(np.float32)          # unreachable pairs stay +inf


def mst_hop_distances(W: np.ndarray) -> np.ndarray:
    """Hop counts along the minimum spanning tree of the node weights (Algorithm 1)."""
    d2 = _gram_sq_distances(W)
    K = d2.shape[0]
    if K == 1:
        return np.zeros((1, 1), dtype=np.float32)
    # scipy treats explicit zeros as missing edges: lift every off-diagonal weight by a tiny constant
    w = np.triu(d2 + np.finfo(np.float64).tiny * 1e10, 1)
    tree = minimum_spanning_tree(csr_matrix(w)).toarray()
    adj = ((tree + tree.T) > 0).astype(np.int8)
    return _hops(adj)


def rng_hop_distances(W: np.ndarray, block: int = 64) -> np.ndarray:
    """Hop counts along the relative neighbourhood graph of the node weights (Algorithm 2).

    Pair (p, q) stays an edge unless a third node is strictly closer to both ends than they are to each other.
    The blocker test runs in chunks of ``block`` rows of p to bound the (block, K, K) temporary.
    """
    d2 = _gram_sq_distances(W)
    K = d2.shape[0]
    keep = np.zeros((K, K), dtype=bool)
    for lo in range(0, K, block):
        hi = min(K, lo + block)
        lune = np.maximum(d2[lo:hi, None, :], d2[None, :, :])      # [p, q, r] = max(d(p, r), d(q, r))
        # r = p and r = q give max = d(p, q) itself, never strictly smaller, so they need no masking
        keep[lo:hi] = ~(lune.min(axis=2) < d2[lo:hi])
    np.fill_diagonal(keep, False)
    keep &= keep.T
    return _hops(keep.astype(np.int8))


def graph_distances(kind: str, W: np.ndarray | None = None, lattice=None) -> np.ndarray:
    if kind in ("rect", "hex"):
        return lattice_distances(lattice[0], lattice[1], kind)
    if kind == "mst":
        return mst_hop_distances(W)
    if kind == "rng":
        return rng_hop_distances(W)
    raise ValueError(f"unknown topology {kind!r}")
