"""Pins for the CPU oracle's epoch: hand-worked values, library routines, closed forms and invariants.

Each test is aimed at a plausible slip in oracle/som.py: a dropped term, a wrong sign or index, a transposed
operand, a tie broken the wrong way, a safeguard that fires when it should not.
"""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.spatial.distance import cdist

import oracle
from synth import GaussianMixture


def _rng(seed):
    return np.random.default_rng(seed)


def _random_problem(seed, m=300, K=12, D=5):
    r = _rng(seed)
    X = r.normal(size=(m, D)).astype(np.float32)
    W = r.normal(size=(K, D)).astype(np.float32)
    pos = r.uniform(0, 4, size=(K, 2))
    G = np.sqrt(((pos[:, None] - pos[None]) ** 2).sum(-1))
    return X, W, G


# ---------------------------------------------------------------- hand-worked case
def test_hand_worked_chain3(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "hand_case_chain3.json")))
    X = np.array(g["X"], dtype=np.float32)
    W = np.array(g["W"], dtype=np.float32)
    G = np.array(g["G"], dtype=np.float64)
    sigma = math.sqrt(1.0 / (2.0 * math.log(2.0)))
    out = oracle.epoch_definition(X, None, W, G, sigma)
    assert out["b"].tolist() == g["b"]
    assert out["d2_best"].tolist() == g["d2_best"]
    assert out["d2_second"].tolist() == g["d2_second"]
    den = [float(Fraction(a, b)) for a, b in g["den_fractions"]]
    np.testing.assert_allclose(out["den"], den, rtol=1e-14)
    Wn = [[float(Fraction(a, b)) for a, b in row] for row in g["W_new_fractions"]]
    np.testing.assert_allclose(out["W"], Wn, rtol=1e-14)
    assert abs(out["qe"] - g["qe"]) < 1e-15
    S, n = oracle.accumulate(X, None, out["b"], 3)
    assert S.tolist() == g["S"] and n.tolist() == g["n"]
    out2 = oracle.epoch_grouped(X, None, W, G, sigma)
    assert out2["b"].tolist() == g["b"]
    np.testing.assert_allclose(out2["W"], Wn, rtol=1e-14)


def test_direction_of_G_is_bmu_row_to_updated_column():
    # G[0,1] = 0 (full influence of BMU-0 samples on node 1); G[1,0] = inf (BMU-1 samples never reach node 0)
    X = np.array([[0.0], [1.0], [10.0], [12.0]], dtype=np.float32)
    W = np.array([[0.5], [11.0]], dtype=np.float32)
    G = np.array([[0.0, 0.0], [np.inf, 0.0]])
    out = oracle.epoch_definition(X, None, W, G, 1.0)
    assert out["b"].tolist() == [0, 0, 1, 1]
    np.testing.assert_allclose(out["W"][:, 0], [0.5, 23.0 / 4.0], rtol=1e-15)
    Wn, _, _ = oracle.neighborhood_update(*oracle.accumulate(X, None, out["b"], 2), G, 1.0, W)
    np.testing.assert_allclose(Wn[:, 0], [0.5, 23.0 / 4.0], rtol=1e-15)


# ---------------------------------------------------------------- distances and BMU
def test_sq_distances_match_scipy_cdist():
    X, W, _ = _random_problem(1, m=200, K=17, D=9)
    ref = cdist(X.astype(np.float64), W.astype(np.float64), "sqeuclidean")
    np.testing.assert_allclose(oracle.sq_distances(X, W), ref, rtol=1e-13, atol=1e-13)
    b, best, second = oracle.bmu(X, W, block=37)
    assert (b == ref.argmin(1)).all()
    np.testing.assert_allclose(best, ref.min(1), rtol=1e-13)
    np.testing.assert_allclose(second, np.sort(ref, axis=1)[:, 1], rtol=1e-13)


def test_bmu_brute_force_loops_tiny():
    X, W, _ = _random_problem(2, m=7, K=4, D=3)
    b, best, _ = oracle.bmu(X, W)
    for i in range(7):
        d = [sum((float(X[i, t]) - float(W[k, t])) ** 2 for t in range(3)) for k in range(4)]
        assert b[i] == d.index(min(d))
        assert abs(best[i] - min(d)) < 1e-14


def test_bmu_exact_tie_takes_lowest_index():
    W = np.array([[1.0, 0.0], [-1.0, 0.0], [0.0, 1.0], [0.0, -1.0]], dtype=np.float32)
    X = np.array([[0.0, 0.0], [0.0, 0.5]], dtype=np.float32)
    b, best, second = oracle.bmu(X, W)
    assert b.tolist() == [0, 2]
    assert best.tolist() == [1.0, 0.25] and second.tolist() == [1.0, 1.25]
    # duplicate nodes
    Wd = np.array([[3.0], [1.0], [1.0], [1.0]], dtype=np.float32)
    assert oracle.bmu(np.array([[0.9]], dtype=np.float32), Wd)[0].tolist() == [1]
    assert oracle.bmu_gram(np.array([[0.9]], dtype=np.float32), Wd)[0].tolist() == [1]


def _offset_tie_case(seed):
    """A sample x and the eight nodes x + (+-a, +-b, +-c) in shuffled order, plus one far node.  x and the offsets
    sit on one binary grid per coordinate, so every x_d +- offset_d is again a float32 value and every direct
    difference is exactly +-offset_d: the eight squared distances are the same sum of the same three squares, equal
    bit for bit in any precision.  The three coordinates live at different scales (about 1000, 0.5 and 5), so
    |w|^2 and x.w need more than 53 bits and the order of the eight float64 Gram values |w|^2 - 2 x.w is decided
    by rounding."""
    r = _rng(seed)
    x = np.array([[1024 + r.integers(1, 2 ** 22) / 2.0 ** 13, r.integers(1, 2 ** 22) / 2.0 ** 22,
                   4 + r.integers(1, 2 ** 21) / 2.0 ** 20]])
    off = np.array([r.integers(1, 2 ** 20) / 2.0 ** 13, r.integers(1, 2 ** 21) / 2.0 ** 22, r.integers(1, 2 ** 20) / 2.0 ** 20])
    signs = np.array([[sa, sb, sc] for sa in (1, -1) for sb in (1, -1) for sc in (1, -1)], dtype=np.float64)
    W = np.concatenate([x + signs[r.permutation(8)] * off, x + [[400.0, 3.0, 0.0]]])
    assert (W.astype(np.float32) == W).all() and (x.astype(np.float32) == x).all()
    return x.astype(np.float32), W.astype(np.float32), float((off * off).sum())


def test_bmu_gram_exact_ties_follow_the_definition_not_the_gram_order():
    # known result: eight nodes at exactly the same distance, one far node; index 0 wins, the runner-up ties with it
    low_index_outside_gram_pair = pair_in_descending_order = 0
    for seed in range(40):
        x, W, d2 = _offset_tie_case(seed)
        Wd = W.astype(np.float64)
        g = (Wd * Wd).sum(1) - 2.0 * (x.astype(np.float64) @ Wd.T)[0]
        pair = np.argsort(g, kind="stable")[:2]
        low_index_outside_gram_pair += 0 not in pair
        pair_in_descending_order += pair[0] > pair[1]
        for fn in (oracle.bmu, oracle.bmu_gram):
            b, best, second = fn(x, W)
            assert b.tolist() == [0] and best[0] == second[0] and abs(best[0] - d2) <= 1e-15 * d2, (fn.__name__, seed)
    # the cases really are adverse for a shortlist of two: both situations occurred
    assert low_index_outside_gram_pair > 0 and pair_in_descending_order > 0


def test_bmu_gram_two_way_tie_in_descending_gram_order():
    # two nodes at exactly equal distance whose Gram values put the higher index first: the lower index wins
    hits = 0
    for seed in range(40):
        x, W, d2 = _offset_tie_case(seed)
        W = W[[0, 1, 8]]
        Wd = W.astype(np.float64)
        g = (Wd * Wd).sum(1) - 2.0 * (x.astype(np.float64) @ Wd.T)[0]
        hits += g[1] < g[0]
        b, best, second = oracle.bmu_gram(x, W)
        assert b.tolist() == [0] and best[0] == second[0] and abs(best[0] - d2) <= 1e-15 * d2
    assert hits > 0


def test_bmu_single_node():
    X, _, _ = _random_problem(3)
    b, best, second = oracle.bmu(X, X[:1])
    assert (b == 0).all() and np.isinf(second).all() and best[0] == 0.0


def test_bmu_gram_matches_definition():
    gm = GaussianMixture(5, 50, 6)
    X = gm.rows(0, 3000)
    W = X[_rng(5).choice(3000, 64, replace=False)]
    b0, best0, sec0 = oracle.bmu(X, W)
    b1, best1, sec1 = oracle.bmu_gram(X, W, block=700)
    assert (b0 == b1).all()
    np.testing.assert_allclose(best1, best0, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(sec1, sec0, rtol=1e-12)


def test_near_tie_mask():
    best = np.array([1.0, 1.0, 0.0, 0.0])
    second = np.array([1.0 + 2e-5, 1.0 + 5e-6, 1e-3, 0.0])
    assert oracle.near_tie_mask(best, second).tolist() == [False, True, False, True]


# ---------------------------------------------------------------- closed forms of the update
def test_single_node_gives_data_mean():
    X, _, _ = _random_problem(4)
    for sigma in (0.1, 1.0, 50.0):
        out = oracle.epoch_definition(X, None, np.zeros((1, X.shape[1])), np.zeros((1, 1)), sigma)
        np.testing.assert_allclose(out["W"][0], X.astype(np.float64).mean(0), rtol=1e-13, atol=1e-15)


def test_small_radius_is_one_lloyd_step():
    X, W, G = _random_problem(6, m=400, K=9, D=4)
    G = oracle.rect_lattice_distances(3, 3)          # smallest non-zero distance is 1
    W[8] = 100.0                                      # a node no sample will choose
    out = oracle.epoch_definition(X, None, W, G, 0.05)
    # independent Lloyd step
    lab = cdist(X.astype(np.float64), W.astype(np.float64)).argmin(1)
    for k in range(9):
        if (lab == k).any():
            np.testing.assert_allclose(out["W"][k], X[lab == k].astype(np.float64).mean(0), rtol=1e-12, atol=1e-14)
        else:
            assert out["guarded"][k]
            assert (out["W"][k] == W[k].astype(np.float64)).all()
    assert out["guarded"][8] and out["guarded"].sum() == (np.bincount(lab, minlength=9) == 0).sum()


def test_huge_radius_gives_data_mean_everywhere():
    X, W, G = _random_problem(7)
    out = oracle.epoch_definition(X, None, W, G, 1e6)
    mean = X.astype(np.float64).mean(0)
    np.testing.assert_allclose(out["W"], np.tile(mean, (W.shape[0], 1)), rtol=1e-9, atol=1e-11)


def test_new_weights_are_convex_combinations_of_samples():
    r = _rng(8)
    D, m, K = 5, 6, 4                                # m = D + 1 affinely independent samples: unique coefficients
    X = r.normal(size=(m, D)).astype(np.float32)
    W = r.normal(size=(K, D)).astype(np.float32)
    G = oracle.rect_lattice_distances(2, 2)
    out = oracle.epoch_definition(X, None, W, G, 0.9)
    A = np.vstack([X.astype(np.float64).T, np.ones(m)])
    for j in range(K):
        c = np.linalg.solve(A, np.append(out["W"][j], 1.0))
        assert c.min() > -1e-12 and abs(c.sum() - 1.0) < 1e-12
        expect = oracle.influence(G, 0.9)[out["b"], j]
        np.testing.assert_allclose(c, expect / expect.sum(), rtol=1e-9, atol=1e-12)
    # the weaker per-coordinate statement on a bigger problem
    X, W, G = _random_problem(9)
    out = oracle.epoch_definition(X, None, W, G, 0.7)
    assert (out["W"] <= X.max(0) + 1e-12).all() and (out["W"] >= X.min(0) - 1e-12).all()


def test_displacement_form_of_eq3_equals_ratio_form():
    X, W, G = _random_problem(10, m=40, K=6, D=3)
    out = oracle.epoch_definition(X, None, W, G, 1.3)
    Wd = oracle.displacement_form_update(X, out["b"], W, G, 1.3, eta=1.0)
    np.testing.assert_allclose(Wd, out["W"], rtol=1e-12, atol=1e-13)


def test_grouped_form_equals_definition():
    X, W, G = _random_problem(11, m=1000, K=20, D=7)
    a = oracle.epoch_definition(X, None, W, G, 0.8)
    g = oracle.epoch_grouped(X, None, W, G, 0.8)
    assert (a["b"] == g["b"]).all()
    np.testing.assert_allclose(g["W"], a["W"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g["den"], a["den"], rtol=1e-12)
    assert abs(g["qe"] - a["qe"]) < 1e-12


# ---------------------------------------------------------------- invariances (Eq. 3 is a sum over samples; Eq. 4 over shards)
def test_sample_order_chunk_and_shard_invariance():
    X, W, G = _random_problem(12, m=500, K=10, D=6)
    base = oracle.epoch_definition(X, None, W, G, 1.1, chunk=4096)
    perm = _rng(12).permutation(500)
    p = oracle.epoch_definition(X[perm], None, W, G, 1.1)
    np.testing.assert_allclose(p["W"], base["W"], rtol=1e-12, atol=1e-13)
    c = oracle.epoch_definition(X, None, W, G, 1.1, chunk=37)
    np.testing.assert_allclose(c["W"], base["W"], rtol=1e-12, atol=1e-13)
    # shards: per-shard (S, n) add up to the whole-set (S, n)
    S, n = oracle.accumulate(X, None, base["b"], 10)
    S2 = np.zeros_like(S)
    n2 = np.zeros_like(n)
    for lo, hi in ((0, 123), (123, 124), (124, 500)):
        s, c_ = oracle.accumulate(X[lo:hi], None, base["b"][lo:hi], 10)
        S2 += s
        n2 += c_
    np.testing.assert_allclose(S2, S, rtol=1e-13, atol=1e-13)
    assert (n2 == n).all() and n.sum() == 500


def test_index_list_selects_rows():
    X, W, G = _random_problem(13, m=200)
    idx = np.sort(_rng(13).choice(200, 50, replace=False)).astype(np.uint32)
    a = oracle.epoch_definition(X, idx, W, G, 1.0)
    b = oracle.epoch_definition(X[idx], None, W, G, 1.0)
    assert (a["b"] == b["b"]).all() and (a["W"] == b["W"]).all()
    g = oracle.epoch_grouped(X, idx, W, G, 1.0)
    np.testing.assert_allclose(g["W"], a["W"], rtol=1e-12, atol=1e-13)


def test_node_relabelling_equivariance():
    X, W, G = _random_problem(14)
    perm = _rng(14).permutation(W.shape[0])
    a = oracle.epoch_definition(X, None, W, G, 0.9)
    b = oracle.epoch_definition(X, None, W[perm], G[np.ix_(perm, perm)], 0.9)
    np.testing.assert_allclose(b["W"], a["W"][perm], rtol=1e-12, atol=1e-13)
    assert (perm[b["b"]] == a["b"]).all()


def test_safeguard_threshold_and_empty_epoch():
    # a far node on a chain: its denominator is exp(-g^2/(2 sigma^2)) * count, compare with the threshold
    W = np.array([[0.0], [50.0], [100.0]], dtype=np.float32)
    X = np.array([[0.1], [-0.1]], dtype=np.float32)
    G = np.array([[0.0, 1.0, 2.0], [1.0, 0.0, 1.0], [2.0, 1.0, 0.0]])
    sigma = 0.1                                           # h(1) = e^-50 ~ 2e-22 (kept), h(2) = e^-200 ~ 1e-87 (guarded)
    out = oracle.epoch_definition(X, None, W, G, sigma)
    assert out["guarded"].tolist() == [False, False, True]
    np.testing.assert_allclose(out["W"][:, 0], [0.0, 0.0, 100.0], atol=1e-12)
    assert abs(out["den"][1] - 2 * math.exp(-50.0)) < 1e-30
    empty = oracle.epoch_definition(X, np.empty(0, dtype=np.uint32), W, G, sigma)
    assert empty["guarded"].all() and (empty["W"] == W).all()


def test_infinite_graph_distance_means_no_influence():
    h = oracle.influence(np.array([[0.0, np.inf], [np.inf, 0.0]]), 2.0)
    assert h.tolist() == [[1.0, 0.0], [0.0, 1.0]]
    assert oracle.influence(np.array([[2.0]]), 1.0)[0, 0] == math.exp(-2.0)


# ---------------------------------------------------------------- Eq. 1 / Eq. 2
def test_sampling_budget():
    assert oracle.sampling_budget(1000, rho=0.1) == 100
    assert oracle.sampling_budget(1000, rho=0.0999) == 99
    assert oracle.sampling_budget(5, rho=0.01) == 1
    assert oracle.sampling_budget(1000, m0=64) == 64
    assert oracle.sampling_budget(10, m0=64) == 10          # budget beyond the dataset means the full dataset
    assert oracle.sampling_budget(10, rho=3.0) == 10
    with pytest.raises(ValueError):
        oracle.sampling_budget(10)


def test_training_reduces_quantization_error_on_clustered_data():
    gm = GaussianMixture(21, 8, 5, std=(0.5, 2.0), isotropic=True)
    X = gm.rows(0, 2000)
    W = X[:25].copy()
    G = oracle.rect_lattice_distances(5, 5)
    qe0 = oracle.quantization_error(oracle.bmu(X, W)[1])
    for sigma in np.linspace(2.5, 0.5, 6):
        W = oracle.epoch_grouped(X, None, W, G, sigma)["W"]
    qe1 = oracle.quantization_error(oracle.bmu(X, W)[1])
    assert qe1 < 0.9 * qe0


# ---------------------------------------------------------------- learning rate and momentum (paragraph after Eq. 4)
def test_general_update_reduces_to_the_plain_one():
    X, W, G = _random_problem(30, m=200, K=8, D=3)
    b = oracle.bmu(X, W)[0]
    S, n = oracle.accumulate(X, None, b, 8)
    plain, guarded, _ = oracle.neighborhood_update(S, n, G, 0.9, W)
    Wn, Vn, g2 = oracle.neighborhood_update_momentum(S, n, G, 0.9, W, None, eta=1.0, mu=0.0)
    np.testing.assert_allclose(Wn, plain, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(Vn, plain - W.astype(np.float64), rtol=1e-12, atol=1e-14)
    assert (g2 == guarded).all()


def test_learning_rate_is_the_eta_of_eq3():
    X, W, G = _random_problem(31, m=30, K=5, D=2)
    b = oracle.bmu(X, W)[0]
    S, n = oracle.accumulate(X, None, b, 5)
    for eta in (0.25, 0.7):
        Wn, _, _ = oracle.neighborhood_update_momentum(S, n, G, 1.2, W, None, eta=eta)
        np.testing.assert_allclose(Wn, oracle.displacement_form_update(X, b, W, G, 1.2, eta=eta), rtol=1e-12, atol=1e-13)


def test_momentum_recurrence_single_node():
    # K = 1: w' = w + eta (mean - w) + mu v, v' = w' - w; two steps by hand
    X = np.array([[2.0], [4.0]], dtype=np.float32)
    G = np.zeros((1, 1))
    S, n = np.array([[6.0]]), np.array([2])
    W1, V1, _ = oracle.neighborhood_update_momentum(S, n, G, 1.0, np.array([[1.0]]), np.array([[0.5]]), eta=0.5, mu=0.2)
    assert abs(W1[0, 0] - (1.0 + 0.5 * (3.0 - 1.0) + 0.2 * 0.5)) < 1e-15 and abs(V1[0, 0] - 1.1) < 1e-15
    W2, V2, _ = oracle.neighborhood_update_momentum(S, n, G, 1.0, W1, V1, eta=0.5, mu=0.2)
    assert abs(W2[0, 0] - (2.1 + 0.5 * (3.0 - 2.1) + 0.2 * 1.1)) < 1e-15
    # a node below the denominator threshold only coasts on its velocity
    G2 = np.array([[0.0, np.inf], [np.inf, 0.0]])
    Wn, Vn, guarded = oracle.neighborhood_update_momentum(np.array([[6.0], [0.0]]), np.array([2, 0]), G2, 1.0,
                                                          np.array([[1.0], [9.0]]), np.array([[0.0], [1.0]]), eta=1.0, mu=0.5)
    assert guarded.tolist() == [False, True] and Wn[:, 0].tolist() == [3.0, 9.5] and Vn[:, 0].tolist() == [2.0, 0.5]


# ---------------------------------------------------------------- the shifted-exponent reading of the safeguard
def test_shifted_update_equals_the_plain_one_where_nothing_underflows():
    """exp(m_j / 2 sigma^2) cancels in Num / Den: with a wide radius both readings give the same weights."""
    rng = np.random.default_rng(5)
    K, D = 30, 4
    G = oracle.rect_lattice_distances(5, 6)
    n = rng.integers(0, 9, size=K)
    n[::4] = 0
    S = rng.normal(size=(K, D)) * n[:, None]
    W = rng.normal(size=(K, D))
    plain, guarded, _ = oracle.neighborhood_update(S, n, G, 2.0, W)
    shifted, unchanged = oracle.neighborhood_update_shifted(S, n, G, 2.0, W)
    assert not guarded.any() and not unchanged.any()
    np.testing.assert_allclose(shifted, plain, rtol=1e-12, atol=1e-14)


def test_shifted_update_far_empty_node_follows_its_nearest_occupied_node():
    """Chain 0 - 1 - 2, only node 0 occupied, tiny radius: the threshold reading leaves nodes 1 and 2 where they are
    (their denominators are e^-200 and e^-800 times n_0), the shifted reading moves both onto node 0's sample mean."""
    G = np.array([[0, 1, 2], [1, 0, 1], [2, 1, 0]], dtype=np.float64)
    n = np.array([4, 0, 0])
    S = np.array([[8.0, -4.0], [0.0, 0.0], [0.0, 0.0]])
    W = np.array([[0.0, 0.0], [5.0, 5.0], [9.0, 9.0]])
    plain, guarded, _ = oracle.neighborhood_update(S, n, G, 0.05, W)
    assert guarded.tolist() == [False, True, True] and (plain[1:] == W[1:]).all()
    shifted, unchanged = oracle.neighborhood_update_shifted(S, n, G, 0.05, W)
    assert not unchanged.any()
    np.testing.assert_allclose(shifted, np.array([[2.0, -1.0]] * 3), rtol=1e-14)


def test_shifted_update_equidistant_occupied_nodes_and_unreachable_node():
    """Node 1 sits between two occupied nodes at the same distance: for sigma -> 0 it takes their count-weighted mean.
    Node 3 is in another component of the graph: nothing reaches it, it stays."""
    inf = np.inf
    G = np.array([[0, 1, 2, inf], [1, 0, 1, inf], [2, 1, 0, inf], [inf, inf, inf, 0]])
    n = np.array([1, 0, 3, 0])
    S = np.array([[1.0], [0.0], [9.0], [0.0]])          # means 1 and 3
    W = np.array([[0.0], [7.0], [0.0], [-5.0]])
    shifted, unchanged = oracle.neighborhood_update_shifted(S, n, G, 0.01, W)
    assert unchanged.tolist() == [False, False, False, True]
    np.testing.assert_allclose(shifted[:, 0], [1.0, (1.0 + 9.0) / 4.0, 3.0, -5.0], rtol=1e-12)
