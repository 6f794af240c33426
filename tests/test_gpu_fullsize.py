"""Parity at the benchmark's own size and launch configuration: cfg1, 1,000,000 x 50 samples, 1024 nodes.

The brute-force oracle checks a seeded sample of rows one by one; properties that hold at any size cover the rest
(counts add up to m, the per-node sums add up to the column sums of X, BMU distances reproduce the QE), and one
teacher-forced epoch is compared against the oracle's grouped form on all rows.
"""
import numpy as np
import pytest
import torch

import oracle
from synth import draw_initial_rows, linear_sigma, make_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def som():
    from paper_2604_26555_amd import Som
    s = Som(0)
    yield s
    s.close()


@pytest.fixture(scope="module")
def cfg1():
    wl = make_workload("cfg1")
    X = wl.data().rows(0, wl.n)
    W0 = X[draw_initial_rows(wl.seed, wl.n, wl.k)].copy()
    return wl, X, W0


def bounded_flips(b_gpu, b, mask, best, second, D, what):
    """The oracle's update follows the GPU's unit inside the 1e-5 near-tie mask; that licence is bounded.  The library
    decides near-ties by float32 direct differences ((D + 3) 2^-24 relative error per squared distance), so it may
    differ from the float64 oracle only where the best two distances are closer than (D + 4) 2^-23 relative, and the
    share of such samples stays below 5e-3."""
    flip = b_gpu != b
    assert not (flip & ~mask).any()
    flips = int(flip.sum())
    print(f"{what}: {flips} of {len(b)} samples differ from the oracle's unit inside the mask ({int(mask.sum())} masked), "
          f"share {flips / len(b):.2e}", flush=True)
    gap = (second[flip] - best[flip]) / np.maximum(second[flip], np.finfo(np.float64).tiny)
    assert (gap <= (D + 4) * 2.0 ** -23).all(), f"{what}: a differing unit at relative gap {gap.max():.2e}"
    assert flips <= 5e-3 * len(b)


def trained(som, wl, Xd, W0, epochs):
    """Weights after a few GPU epochs (a spread-out map rather than the initial sample rows)."""
    from paper_2604_26555_amd import topology
    G = torch.from_numpy(topology.graph_distances(wl.topology, lattice=wl.lattice)).cuda()
    Wd = torch.from_numpy(W0).cuda()
    sig = linear_sigma(*wl.sigma, wl.epochs)
    for e in range(epochs):
        som.som_epoch(Xd, Wd, G, float(sig[e]), want_stats=False)
    som.som_sync()
    return Wd, G, sig


@pytest.mark.parametrize("search", ["auto", "float32"])
@pytest.mark.parametrize("epochs", [0, 3, 12])
def test_full_size_bmu_sampled_against_brute_force(som, cfg1, epochs, search):
    wl, X, W0 = cfg1
    Xd = torch.from_numpy(X).cuda()
    Wd, _, _ = trained(som, wl, Xd, W0, epochs)
    som.som_set_search(search)       # bf16 parts on the matrix pipe (the benchmark's configuration), or float32 MFMA
    W = Wd.cpu().numpy()
    d2 = torch.empty(wl.n, dtype=torch.float32, device="cuda")
    qe = torch.zeros(2, dtype=torch.float64, device="cuda")
    b_gpu, _, _ = som.som_bmu(Xd, Wd, d2=d2, qe=qe)
    b_plain = som.som_bmu(Xd, Wd)[0].cpu().numpy()      # as the benchmark's epochs run it: no distances asked for
    som.som_set_search("auto")
    b_gpu, d2 = b_gpu.cpu().numpy(), d2.cpu().numpy()
    rows = np.sort(np.random.default_rng(77 + epochs).choice(wl.n, 4000, replace=False))
    rows = np.unique(np.concatenate([rows, [0, 255, 256, wl.n - 65, wl.n - 1]]))      # tile edges and the ragged tail
    b, best, second = oracle.bmu(X[rows], W)
    mask = oracle.near_tie_mask(best, second)
    assert ((b_gpu[rows] == b) | mask).all()
    assert ((b_plain[rows] == b) | mask).all()
    assert b_plain.min() >= 0 and b_plain.max() < wl.k
    print(f"units with and without distances differ on {int((b_plain != b_gpu).sum())} of {wl.n} samples", flush=True)
    same = b_gpu[rows] == b
    np.testing.assert_allclose(d2[rows][same], best[same], rtol=1e-4, atol=1e-12)
    # properties at full size
    assert b_gpu.min() >= 0 and b_gpu.max() < wl.k
    q = qe.cpu().numpy()
    assert abs(q[1] - d2.astype(np.float64).sum()) <= 1e-6 * q[1]
    assert abs(q[0] - np.sqrt(d2.astype(np.float64)).sum()) <= 1e-6 * q[0]
    # every reported distance is the distance to the reported node
    chk = np.random.default_rng(5).choice(wl.n, 20000, replace=False)
    direct = ((X[chk].astype(np.float64) - W[b_gpu[chk]].astype(np.float64)) ** 2).sum(1)
    np.testing.assert_allclose(d2[chk], direct, rtol=1e-4, atol=1e-12)


def test_full_size_accumulate_properties_and_epoch(som, cfg1):
    wl, X, W0 = cfg1
    Xd = torch.from_numpy(X).cuda()
    Wd, G, sig = trained(som, wl, Xd, W0, 5)
    W = Wd.cpu().numpy()
    b_gpu, _, _ = som.som_bmu(Xd, Wd)
    S = torch.zeros((wl.k, wl.d), dtype=torch.float64, device="cuda")
    n = torch.zeros(wl.k, dtype=torch.int64, device="cuda")
    som.som_accumulate(Xd, b_gpu, wl.k, S, n)
    S, n = S.cpu().numpy(), n.cpu().numpy()
    b_np = b_gpu.cpu().numpy()
    assert n.sum() == wl.n and (n == np.bincount(b_np, minlength=wl.k)).all()
    col = X.astype(np.float64).sum(0)
    # every sample enters one float32 addition whose result is below a few max|x|: at most n * 2^-24 * max|x| in total
    np.testing.assert_allclose(S.sum(0), col, rtol=0, atol=wl.n * 2.0 ** -24 * np.abs(X).max())
    S_or, _ = oracle.accumulate(X, None, b_np, wl.k)
    assert (np.abs(S - S_or) <= 1e-6 * np.abs(X).max() * np.maximum(n, 1)[:, None]).all()
    # one teacher-forced epoch on all rows against the oracle's grouped form
    ref_b, best, second = oracle.bmu_gram(X, W)
    mask = oracle.near_tie_mask(best, second)
    assert ((b_np == ref_b) | mask).all(), f"{((b_np != ref_b) & ~mask).sum()} BMU mismatches outside the near-tie mask"
    b_use = np.where(mask, b_np, ref_b)
    bounded_flips(b_np, ref_b, mask, best, second, wl.d, "full size")
    G_or = oracle.graph_distances(wl.topology, lattice=wl.lattice)
    ref = oracle.epoch_grouped(X, None, W, G_or, float(sig[5]), b=b_use)
    st = som.som_epoch(Xd, Wd, G, float(sig[5]))
    scale = np.abs(ref["W"]).max(axis=1, keepdims=True)
    assert (np.abs(Wd.cpu().numpy() - ref["W"]) <= 1e-4 * scale).all()
    assert abs(st.qe - oracle.quantization_error(best)) <= 1e-4 * oracle.quantization_error(best)
    assert st.n_empty == int((ref["n"] == 0).sum()) and st.m == wl.n


def test_bmu_over_more_rows_than_one_pass(som):
    """More than 2^27 rows (the library's BMU search takes them in passes of that size): sampled rows, among them
    the ones either side of the pass boundary, against the brute-force oracle; sums over all rows."""
    from concurrent.futures import ThreadPoolExecutor
    from synth import Uniform01
    m, D, K = (1 << 27) + 100_003, 4, 500
    gen = Uniform01(4711, D)
    Xd = torch.empty((m, D), dtype=torch.float32, device="cuda")
    piece = 1 << 24
    with ThreadPoolExecutor(8) as pool:
        for lo, rows in zip(range(0, m, piece), pool.map(lambda lo: gen.rows(lo, min(m, lo + piece)), range(0, m, piece))):
            Xd[lo:lo + len(rows)].copy_(torch.from_numpy(rows))
    W = gen.rows(m, m + K).copy()
    Wd = torch.from_numpy(W).cuda()
    d2 = torch.empty(m, dtype=torch.float32, device="cuda")
    qe = torch.zeros(2, dtype=torch.float64, device="cuda")
    b_gpu, _, _ = som.som_bmu(Xd, Wd, d2=d2, qe=qe)
    som.som_sync()
    edge = 1 << 27
    rows = np.unique(np.concatenate([np.random.default_rng(3).choice(m, 5000, replace=False),
                                     [0, edge - 257, edge - 1, edge, edge + 1, edge + 255, edge + 256, m - 1]]))
    rows_d = torch.from_numpy(rows).cuda()
    Xs = Xd[rows_d].cpu().numpy()
    b, best, second = oracle.bmu(Xs, W)
    mask = oracle.near_tie_mask(best, second)
    got = b_gpu[rows_d].cpu().numpy()
    assert ((got == b) | mask).all()
    same = got == b
    np.testing.assert_allclose(d2[rows_d].cpu().numpy()[same], best[same], rtol=1e-4, atol=1e-12)
    assert int(b_gpu.min()) >= 0 and int(b_gpu.max()) < K
    q = qe.cpu().numpy()
    assert abs(q[1] - float(d2.double().sum())) <= 1e-6 * q[1]
    assert abs(q[0] - float(d2.double().sqrt().sum())) <= 1e-6 * q[0]


def test_bmu_wide_rows_in_several_passes(som):
    """D = 8192: the default search writes the samples' bf16 parts into a bounded workspace and takes the rows in
    passes that fit it (262144 rows here); sampled rows around the pass boundary against the brute-force oracle."""
    from concurrent.futures import ThreadPoolExecutor
    from synth import Uniform01
    m, D, K = 300_001, 8192, 400
    gen = Uniform01(815, D)
    Xd = torch.empty((m, D), dtype=torch.float32, device="cuda")
    piece = 1 << 14
    with ThreadPoolExecutor(8) as pool:
        for lo, rows in zip(range(0, m, piece), pool.map(lambda lo: gen.rows(lo, min(m, lo + piece)), range(0, m, piece))):
            Xd[lo:lo + len(rows)].copy_(torch.from_numpy(rows))
    W = gen.rows(m, m + K).copy()
    Wd = torch.from_numpy(W).cuda()
    d2 = torch.empty(m, dtype=torch.float32, device="cuda")
    b_gpu, _, _ = som.som_bmu(Xd, Wd, d2=d2)
    som.som_sync()
    edge = 262_144
    rows = np.unique(np.concatenate([np.random.default_rng(4).choice(m, 300, replace=False),
                                     [0, edge - 129, edge - 1, edge, edge + 1, edge + 127, edge + 128, m - 1]]))
    rows_d = torch.from_numpy(rows).cuda()
    b, best, second = oracle.bmu(Xd[rows_d].cpu().numpy(), W)
    mask = oracle.near_tie_mask(best, second)
    got = b_gpu[rows_d].cpu().numpy()
    assert ((got == b) | mask).all()
    same = got == b
    np.testing.assert_allclose(d2[rows_d].cpu().numpy()[same], best[same], rtol=1e-4, atol=1e-12)
    assert int(b_gpu.min()) >= 0 and int(b_gpu.max()) < K


# ------------------------------------------------------------------------------------------- top of the grid axis
# Supplementary Table S3 takes the map up to 64 x 64 = 4096 nodes; the three tests below put every stage at that size
# against the oracle.

def test_update_at_4096_nodes(som):
    K, D = 4096, 50
    rng = np.random.default_rng(4096)
    W = rng.normal(size=(K, D)).astype(np.float32)
    n = rng.integers(0, 400, size=K).astype(np.int64)
    n[rng.random(K) < 0.3] = 0
    S = rng.normal(size=(K, D)) * n[:, None]
    G = oracle.hex_lattice_distances(64, 64).astype(np.float32)
    for sigma in (32.0, 2.0, 0.4):
        Wd = torch.from_numpy(W).cuda()
        ng = torch.zeros(1, dtype=torch.int32, device="cuda")
        som.som_neighborhood_update(torch.from_numpy(S).cuda(), torch.from_numpy(n).cuda(), torch.from_numpy(G).cuda(), sigma, Wd,
                                    n_guarded=ng)
        W_or, guarded, den = oracle.neighborhood_update(S, n, G.astype(np.float64), sigma, W)
        keep = ~((den > oracle.DEFAULT_EPS_H / 4) & (den < oracle.DEFAULT_EPS_H * 4))
        scale = np.maximum(np.abs(W_or).max(axis=1, keepdims=True), 1e-30)
        err = np.abs(Wd.cpu().numpy() - W_or) / scale
        print(f"update K=4096 sigma={sigma}: max relative error {err[keep].max():.2e}, guarded {int(guarded.sum())}", flush=True)
        assert (err[keep] <= 1e-4).all()
        assert abs(int(ng.item()) - int(guarded.sum())) <= int((~keep).sum())


@pytest.mark.parametrize("search", ["auto", "float32"])
def test_epoch_at_4096_nodes_teacher_forced(som, search):
    """64 x 64 hexagonal map, 2 * 10^5 x 50 samples: units, distances, weights and counters of two epochs (large and small
    radius) against the oracle, each started from the same weights."""
    wl = make_workload("cfg1", n=200_000, k=4096, lattice=(64, 64))
    X = wl.data().rows(0, wl.n)
    W = X[draw_initial_rows(wl.seed, wl.n, wl.k)].copy()
    G_or = oracle.hex_lattice_distances(64, 64)
    Xd, Gd = torch.from_numpy(X).cuda(), torch.from_numpy(G_or.astype(np.float32)).cuda()
    som.som_set_search(search)
    try:
        for sigma in (32.0, 1.5):
            Wd = torch.from_numpy(W).cuda()
            d2 = torch.empty(wl.n, dtype=torch.float32, device="cuda")
            b_gpu, _, _ = som.som_bmu(Xd, Wd, d2=d2)
            b_gpu = b_gpu.cpu().numpy()
            b, best, second = oracle.bmu_gram(X, W, block=16384)
            mask = oracle.near_tie_mask(best, second)
            bad = (b_gpu != b) & ~mask
            assert not bad.any(), f"{int(bad.sum())} units differ outside the near-tie mask"
            bounded_flips(b_gpu, b, mask, best, second, wl.d, f"K=4096 {search} sigma={sigma}")
            same = b_gpu == b
            np.testing.assert_allclose(d2.cpu().numpy()[same], best[same], rtol=1e-4, atol=1e-12)
            ref = oracle.epoch_grouped(X, None, W, G_or, sigma, b=np.where(mask, b_gpu, b))
            st = som.som_epoch(Xd, Wd, Gd, sigma)
            keep = ~((ref["den"] > oracle.DEFAULT_EPS_H / 4) & (ref["den"] < oracle.DEFAULT_EPS_H * 4))
            scale = np.maximum(np.abs(ref["W"]).max(axis=1, keepdims=True), 1e-30)
            err = np.abs(Wd.cpu().numpy() - ref["W"]) / scale
            assert (err[keep] <= 1e-4).all(), f"max relative weight error {err[keep].max():.2e}"
            qe = oracle.quantization_error(best)
            assert abs(st.qe - qe) <= 1e-4 * qe and st.m == wl.n
            assert st.n_empty == int((ref["n"] == 0).sum())
            W = ref["W"].astype(np.float32)          # the second epoch runs on a spread-out map
    finally:
        som.som_set_search("auto")


def test_relative_neighbourhood_graph_at_4096_nodes(som):
    """K = 4096, D = 50.  The oracle's blocker test decides the complete neighbour row of 96 sampled nodes (among them
    the first and the last); the whole graph must be symmetric, contain the oracle's spanning tree, and its hop counts
    from sampled sources must be the unweighted shortest paths of its own edges (the routine the oracle's hop counts
    are pinned to)."""
    from scipy.sparse import csr_matrix
    from scipy.sparse.csgraph import shortest_path
    from synth import GaussianMixture
    K, D = 4096, 50
    W = GaussianMixture(4096, D, 12).rows(0, K)
    R = som.som_topology(torch.from_numpy(W).cuda(), "rng").cpu().numpy()
    adj = R == 1
    assert np.array_equal(R, R.T) and (R.diagonal() == 0).all() and np.isfinite(R).all()
    d2 = oracle.node_sq_distances(W)
    rows = np.unique(np.concatenate([np.random.default_rng(1).choice(K, 94, replace=False), [0, K - 1]]))
    for p in rows:
        expect = ~oracle.rng_blocked(d2, int(p))
        expect[p] = False
        assert np.array_equal(adj[p], expect), f"neighbour row of node {p} differs from the blocker test"
    e = oracle.mst_edges(W)
    assert adj[e[:, 0], e[:, 1]].all()                       # the graph contains the minimum spanning tree
    src = [0, 777, 2048, K - 1]
    hops = shortest_path(csr_matrix(adj.astype(np.int8)), unweighted=True, indices=src)
    assert np.array_equal(R[src], hops.astype(np.float32))
    print(f"RNG K=4096: {int(adj.sum()) // 2} edges, largest hop count {int(R.max())}", flush=True)


def test_streamed_epoch_with_a_chunk_above_4_gib(som):
    """2.5 * 10^7 x 50 rows (5 GB) in host memory, streamed in chunks of 2.2 * 10^7 rows (4.4 GB: byte counts beyond
    32 bits in the staging copies, the transfers and the kernels' row offsets), against the same epoch on resident
    samples; best-matching units of sampled rows on both sides of the chunk boundary against the brute-force oracle."""
    from concurrent.futures import ThreadPoolExecutor
    wl = make_workload("cfg4", n=25_000_000)
    gen = wl.data()
    X = np.empty((wl.n, wl.d), dtype=np.float32)
    piece = 1 << 20
    with ThreadPoolExecutor(8) as pool:
        list(pool.map(lambda lo: gen.fill(X[lo:lo + piece], lo), range(0, wl.n, piece)))
    W0 = X[draw_initial_rows(wl.seed, wl.n, wl.k)].copy()
    G = torch.from_numpy(oracle.rect_lattice_distances(32, 32).astype(np.float32)).cuda()
    chunk = 22_000_000
    assert chunk * wl.d * 4 > 1 << 32
    Wa, Wb = torch.from_numpy(W0).cuda(), torch.from_numpy(W0).cuda()
    print("streaming 2.5e7 rows in chunks of 2.2e7", flush=True)
    sb = som.som_epoch_host(X, Wb, G, 4.0, chunk_rows=chunk)
    Xd = torch.from_numpy(X).cuda()
    sa = som.som_epoch(Xd, Wa, G, 4.0)
    print(f"streamed {sb.ms_bmu_acc:.1f} ms of compute, {sb.ms_h2d:.1f} ms of copies; resident {sa.ms_bmu_acc:.1f} ms", flush=True)
    np.testing.assert_allclose(Wb.cpu().numpy(), Wa.cpu().numpy(), rtol=1e-6, atol=1e-7)
    assert sa.m == sb.m == wl.n and abs(sa.sum_dist - sb.sum_dist) <= 1e-9 * sa.sum_dist and sa.n_empty == sb.n_empty
    b_gpu, _, _ = som.som_bmu(Xd, torch.from_numpy(W0).cuda())
    rows = np.unique(np.concatenate([np.random.default_rng(9).choice(wl.n, 3000, replace=False),
                                     [0, chunk - 1, chunk, chunk + 1, wl.n - 1]]))
    b, best, second = oracle.bmu(X[rows], W0)
    mask = oracle.near_tie_mask(best, second)
    assert ((b_gpu.cpu().numpy()[rows] == b) | mask).all()
    # the streamed statistics are those of the oracle on the sampled rows' scale: mean distance within sampling error
    assert abs(sb.qe - float(np.sqrt(best).mean())) <= 0.05 * sb.qe
