"""Node-to-node neighbourhood distance matrices, float64 CPU.  TEST INFRASTRUCTURE ONLY.

Regular lattices (paper Section 3.2): rectangular grid and hexagonal layout, Euclidean distance between the
node positions.  Data-driven graphs (Sections 3.2.1 and 3.2.2, Algorithms 1 and 2): minimum spanning tree by
Kruskal's method and relative neighbourhood graph by the blocker test over the current node weights, then
all-pairs hop counts along the graph.  The hop counts come from a breadth-first search from every node, which
yields the same matrix as the Floyd-Warshall recurrence the paper names.

Pins (tests/test_oracle_topology.py): closed forms for the lattices, scipy.sparse.csgraph's spanning tree
weight and unweighted shortest paths, an O(K^3) triple loop for the RNG on small K, RNG contains MST.
"""
from __future__ import annotations

from collections import deque

import numpy as np


def rect_lattice_distances(n_rows: int, n_cols: int) -> np.ndarray:
    """Node k sits at (k // n_cols, k % n_cols); G is the Euclidean distance between those positions."""
    k = np.arange(n_rows * n_cols)
    pos = np.stack([k // n_cols, k % n_cols], axis=1).astype(np.float64)
    diff = pos[:, None, :] - pos[None, :, :]
    return np.sqrt((diff * diff).sum(axis=2))


def hex_lattice_positions(n_rows: int, n_cols: int) -> np.ndarray:
    """Hexagonal layout: odd rows shifted half a cell right, rows sqrt(3)/2 apart (six neighbours at 1)."""
    k = np.arange(n_rows * n_cols)
    r, c = k // n_cols, k % n_cols
    return np.stack([c + 0.5 * (r % 2), r * (np.sqrt(3.0) / 2.0)], axis=1)


def hex_lattice_distances(n_rows: int, n_cols: int) -> np.ndarray:
    pos = hex_lattice_positions(n_rows, n_cols)
    diff = pos[:, None, :] - pos[None, :, :]
    return np.sqrt((diff * diff).sum(axis=2))


def node_sq_distances(W: np.ndarray, block: int = 256) -> np.ndarray:
    """Pairwise squared distances between node weight vectors, by direct differences.

    Rows are taken in blocks only to bound the size of the temporary; every entry is the same sum either way."""
    W = np.asarray(W, dtype=np.float64)
    K = W.shape[0]
    d2 = np.empty((K, K), dtype=np.float64)
    for lo in range(0, K, block):
        diff = W[lo:lo + block, None, :] - W[None, :, :]
        d2[lo:lo + block] = np.einsum("pqd,pqd->pq", diff, diff)
    return d2


def mst_edges(W: np.ndarray) -> np.ndarray:
    """Minimum spanning tree over the node weights by Kruskal's method (Algorithm 1, step 8).

    Candidate edges (p < q) are visited in order of (squared distance, p, q); an edge is kept when it joins
    two different components (union-find).  Returns an array of K-1 rows (p, q).
    """
    d2 = node_sq_distances(W)
    K = d2.shape[0]
    p, q = np.triu_indices(K, k=1)
    order = np.lexsort((q, p, d2[p, q]))
    parent = list(range(K))

    def find(a):
        while parent[a] != a:
            parent[a] = parent[parent[a]]
            a = parent[a]
        return a

    edges = []
    for e in order:
        a, c = find(int(p[e])), find(int(q[e]))
        if a != c:
            parent[a] = c
            edges.append((int(p[e]), int(q[e])))
            if len(edges) == K - 1:
                break
    return np.asarray(edges, dtype=np.int64).reshape(-1, 2)


def rng_blocked(d2: np.ndarray, p: int) -> np.ndarray:
    """Blocker test of Algorithm 2 (steps 7-9) for node p against every q at once, on squared distances d2.

    blocked[q] is True when some third node r (r != p, r != q) is strictly closer to both ends than they are to each
    other:  max(d(p, r), d(q, r)) < d(p, q).
    """
    K = d2.shape[0]
    m = np.maximum(d2[p][None, :], d2)          # m[q, r] = max(d2[p, r], d2[q, r])
    m[:, p] = np.inf
    m[np.arange(K), np.arange(K)] = np.inf      # r must differ from q (and from p)
    return m.min(axis=1) < d2[p]


def rng_edges(W: np.ndarray) -> np.ndarray:
    """Relative neighbourhood graph over the node weights (Algorithm 2, steps 7-9).

    The pair (p, q) is an edge unless some third node r blocks it, i.e. is strictly closer to both ends than
    they are to each other:  max(d(p, r), d(q, r)) < d(p, q).
    """
    d2 = node_sq_distances(W)
    K = d2.shape[0]
    edges = []
    for p in range(K):
        blocked = rng_blocked(d2, p)
        for q in range(p + 1, K):
            if not blocked[q]:
                edges.append((p, q))
    return np.asarray(edges, dtype=np.int64).reshape(-1, 2)


def hop_distances(K: int, edges: np.ndarray) -> np.ndarray:
    """All-pairs hop counts of an undirected graph; unreachable pairs are +inf (Algorithms 1/2, step 10)."""
    adj = [[] for _ in range(K)]
    for p, q in np.asarray(edges, dtype=np.int64).reshape(-1, 2):
        adj[int(p)].append(int(q))
        adj[int(q)].append(int(p))
    G = np.full((K, K), np.inf)
    for s in range(K):
        G[s, s] = 0.0
        queue = deque([s])
        while queue:
            u = queue.popleft()
            for v in adj[u]:
                if G[s, v] == np.inf:
                    G[s, v] = G[s, u] + 1.0
                    queue.append(v)
    return G


def graph_distances(kind: str, W: np.ndarray = None, lattice=None) -> np.ndarray:
    """Neighbourhood distance matrix for a named topology ("rect", "hex", "mst", "rng")."""
    if kind == "rect":
        return rect_lattice_distances(*lattice)
    if kind == "hex":
        return hex_lattice_distances(*lattice)
    if kind == "mst":
        return hop_distances(len(W), mst_edges(W))
    if kind == "rng":
        return hop_distances(len(W), rng_edges(W))
    raise ValueError(f"unknown topology {kind!r}")
