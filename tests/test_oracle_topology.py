"""Pins for the oracle's neighbourhood-distance builders: closed forms, scipy's graph routines, brute force."""
import math

import numpy as np
from scipy.sparse import csr_matrix
from scipy.sparse.csgraph import minimum_spanning_tree, shortest_path

import oracle


def _nodes(seed, K=40, D=6):
    return np.random.default_rng(seed).normal(size=(K, D)).astype(np.float32)


def test_rect_lattice_closed_form():
    G = oracle.rect_lattice_distances(3, 4)
    assert G.shape == (12, 12)
    assert G[0, 3] == 3.0 and G[0, 4] == 1.0 and G[0, 11] == math.sqrt(4 + 9)
    assert G[5, 6] == 1.0 and G[5, 10] == math.sqrt(2.0)
    assert (G == G.T).all() and (np.diag(G) == 0).all()


def test_hex_lattice_rings():
    rows, cols = 7, 7
    G = oracle.hex_lattice_distances(rows, cols)
    for centre in (3 * cols + 3, 2 * cols + 3):          # an odd and an even row, interior
        d = np.sort(G[centre])
        assert d[0] == 0.0
        np.testing.assert_allclose(d[1:7], 1.0, rtol=1e-14)           # six nearest neighbours at distance 1
        np.testing.assert_allclose(d[7:13], math.sqrt(3.0), rtol=1e-14)  # next ring
        np.testing.assert_allclose(d[13:19], 2.0, rtol=1e-14)
        assert d[19] > 2.0 + 1e-9
    pos = oracle.hex_lattice_positions(2, 2)
    np.testing.assert_allclose(pos, [[0, 0], [1, 0], [0.5, math.sqrt(3) / 2], [1.5, math.sqrt(3) / 2]])


def test_node_sq_distances_direct():
    W = _nodes(1, K=9, D=4)
    d2 = oracle.node_sq_distances(W)
    for p in range(9):
        for q in range(9):
            assert abs(d2[p, q] - float(((W[p].astype(np.float64) - W[q].astype(np.float64)) ** 2).sum())) < 1e-13


def test_mst_matches_scipy_and_is_a_tree():
    for seed in range(3):
        W = _nodes(seed, K=60)
        E = oracle.mst_edges(W)
        assert E.shape == (59, 2)
        d = np.sqrt(oracle.node_sq_distances(W))
        ref = minimum_spanning_tree(csr_matrix(np.triu(d, 1)))
        assert abs(d[E[:, 0], E[:, 1]].sum() - ref.sum()) < 1e-9
        ours = {tuple(sorted(e)) for e in E.tolist()}
        theirs = {tuple(sorted(e)) for e in zip(*ref.nonzero())}
        assert ours == theirs                                # distinct weights: the tree is unique
        G = oracle.hop_distances(60, E)
        assert np.isfinite(G).all()                          # connected


def test_hop_distances_match_scipy_unweighted_shortest_path():
    W = _nodes(5, K=50)
    for E in (oracle.mst_edges(W), oracle.rng_edges(W)):
        A = np.zeros((50, 50))
        A[E[:, 0], E[:, 1]] = 1
        A[E[:, 1], E[:, 0]] = 1
        ref = shortest_path(csr_matrix(A), method="D", unweighted=True, directed=False)
        G = oracle.hop_distances(50, E)
        assert (G == ref).all()
        assert (G == G.T).all() and (np.diag(G) == 0).all()
    # two components: unreachable pairs are +inf
    G = oracle.hop_distances(4, np.array([[0, 1], [2, 3]]))
    assert G[0, 1] == 1 and np.isinf(G[0, 2]) and np.isinf(G[3, 1])
    # a path graph: hop count is the index difference
    G = oracle.hop_distances(5, np.array([[0, 1], [1, 2], [2, 3], [3, 4]]))
    assert (G == np.abs(np.subtract.outer(np.arange(5), np.arange(5)))).all()


def test_rng_matches_triple_loop_and_contains_mst():
    for seed in range(3):
        W = _nodes(10 + seed, K=24, D=3)
        d2 = oracle.node_sq_distances(W)
        brute = set()
        for p in range(24):
            for q in range(p + 1, 24):
                if not any(max(d2[p, r], d2[q, r]) < d2[p, q] for r in range(24) if r != p and r != q):
                    brute.add((p, q))
        E = {tuple(e) for e in oracle.rng_edges(W).tolist()}
        assert E == brute
        assert {tuple(e) for e in oracle.mst_edges(W).tolist()} <= E


def test_rng_on_a_square_and_a_line():
    # unit square: sides survive, diagonals are blocked by the other two corners
    W = np.array([[0, 0], [1, 0], [1, 1], [0, 1]], dtype=np.float32)
    assert {tuple(e) for e in oracle.rng_edges(W).tolist()} == {(0, 1), (0, 3), (1, 2), (2, 3)}
    # collinear points: only consecutive pairs
    W = np.array([[0.0], [1.0], [2.5], [7.0]], dtype=np.float32)
    assert {tuple(e) for e in oracle.rng_edges(W).tolist()} == {(0, 1), (1, 2), (2, 3)}
    assert {tuple(e) for e in oracle.mst_edges(W).tolist()} == {(0, 1), (1, 2), (2, 3)}


def test_rng_exact_ties_do_not_block():
    """Algorithm 2's blocker test is strict: a third node exactly as far from one end as the ends are from each
    other blocks nothing.  All squared distances below are small integers, exact in any precision."""
    # three mutually equidistant nodes (every squared distance is 2): all three edges
    W = np.array([[1, 0, 0], [0, 1, 0], [0, 0, 1]], dtype=np.float32)
    assert oracle.node_sq_distances(W)[np.triu_indices(3, 1)].tolist() == [2.0, 2.0, 2.0]
    assert {tuple(e) for e in oracle.rng_edges(W).tolist()} == {(0, 1), (0, 2), (1, 2)}
    # isosceles: |pq|^2 = |pr|^2 = 25, |qr|^2 = 20.  r ties with q seen from p, so (p,q) and (p,r) both stay;
    # (q,r) is the shortest side and stays as well
    W = np.array([[0, 0], [5, 0], [3, 4]], dtype=np.float32)
    assert oracle.node_sq_distances(W)[np.triu_indices(3, 1)].tolist() == [25.0, 25.0, 20.0]
    assert {tuple(e) for e in oracle.rng_edges(W).tolist()} == {(0, 1), (0, 2), (1, 2)}
    # the same triangle with its apex pulled one unit closer to p: now r is strictly inside the lune of (p,q)
    W = np.array([[0, 0], [5, 0], [3, 3]], dtype=np.float32)       # |pr|^2 = 18, |qr|^2 = 13 < 25
    assert {tuple(e) for e in oracle.rng_edges(W).tolist()} == {(0, 2), (1, 2)}
    # equally spaced collinear nodes 0, 1, 2, 3: consecutive pairs only (the middle nodes block strictly), and a
    # unit square with its centre: centre-corner edges (1/2) are shorter than the sides (1), the centre is strictly
    # inside every side's lune (max = 1/2 < 1), so only the four spokes stay
    W = np.array([[0.0], [1.0], [2.0], [3.0]], dtype=np.float32)
    assert {tuple(e) for e in oracle.rng_edges(W).tolist()} == {(0, 1), (1, 2), (2, 3)}
    W = np.array([[0, 0], [1, 0], [1, 1], [0, 1], [0.5, 0.5]], dtype=np.float32)
    assert {tuple(e) for e in oracle.rng_edges(W).tolist()} == {(0, 4), (1, 4), (2, 4), (3, 4)}
    # regular unit square alone: the diagonal's ends see the other corners at exactly the side length (1 < 2:
    # blocked), and each side sees the far corners at distances (1, 2): max 2 > 1, not blocked
    W = np.array([[0, 0], [2, 0], [1, 1], [1, -1]], dtype=np.float32)   # a square standing on a corner, side^2 = 2
    assert {tuple(e) for e in oracle.rng_edges(W).tolist()} == {(0, 2), (0, 3), (1, 2), (1, 3)}
    # hop counts of the tie triangle: everything one hop apart
    G = oracle.graph_distances("rng", W=np.array([[1, 0, 0], [0, 1, 0], [0, 0, 1]], dtype=np.float32))
    assert G.tolist() == [[0, 1, 1], [1, 0, 1], [1, 1, 0]]


def test_graph_distances_dispatch():
    W = _nodes(20, K=16)
    assert (oracle.graph_distances("rect", lattice=(4, 4)) == oracle.rect_lattice_distances(4, 4)).all()
    assert (oracle.graph_distances("hex", lattice=(4, 4)) == oracle.hex_lattice_distances(4, 4)).all()
    assert (oracle.graph_distances("mst", W=W) == oracle.hop_distances(16, oracle.mst_edges(W))).all()
    assert (oracle.graph_distances("rng", W=W) == oracle.hop_distances(16, oracle.rng_edges(W))).all()
