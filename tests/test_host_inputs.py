"""The package's lattice builder against the oracle's closed forms, and the seeded input generators."""
import numpy as np
import pytest

import oracle
from paper_2604_26555_amd import topology as T
from synth import GaussianMixture, draw_initial_rows, draw_subset, linear_sigma, make_workload


@pytest.mark.parametrize("shape", [(1, 1), (3, 4), (10, 10), (7, 5)])
def test_lattices(shape):
    np.testing.assert_allclose(T.lattice_distances(*shape, "rect"), oracle.rect_lattice_distances(*shape), rtol=2e-7)
    np.testing.assert_allclose(T.lattice_distances(*shape, "hex"), oracle.hex_lattice_distances(*shape), rtol=2e-7)


def test_graph_topologies_have_no_host_path():
    for kind in ("mst", "rng"):
        with pytest.raises(ValueError):
            T.graph_distances(kind, lattice=(4, 4))


def test_generators_are_chunk_invariant_and_seeded():
    gm = GaussianMixture(7, 5, 4, weights="dirichlet", noise_frac=0.1)
    whole = gm.rows(0, 150_000)
    assert whole.dtype == np.float32
    np.testing.assert_array_equal(whole[65_000:66_000], gm.rows(65_000, 66_000))
    np.testing.assert_array_equal(whole[131_071:131_073], GaussianMixture(7, 5, 4, weights="dirichlet", noise_frac=0.1).rows(131_071, 131_073))
    assert abs(whole.min()) <= 15.0 + 20 and not np.array_equal(whole[:10], GaussianMixture(8, 5, 4).rows(0, 10))
    s = linear_sigma(16.0, 1.0, 20)
    assert s[0] == 16.0 and s[-1] == 1.0 and len(s) == 20 and linear_sigma(3.0, 1.0, 1).tolist() == [3.0]
    rows = draw_initial_rows(3, 1000, 64)
    assert len(set(rows.tolist())) == 64 and rows.max() < 1000
    a, b = draw_subset(3, 0, 10_000, 1000), draw_subset(3, 1, 10_000, 1000)
    assert a.dtype == np.uint32 and len(set(a.tolist())) == 1000 and (np.diff(a.astype(np.int64)) > 0).all()
    assert not np.array_equal(a, b) and np.array_equal(a, draw_subset(3, 0, 10_000, 1000))
    big = draw_subset(5, 2, 1 << 25, 100_000)
    assert len(big) == 100_000 and (np.diff(big.astype(np.int64)) > 0).all() and big.max() < (1 << 25)
    wl = make_workload("cfg1", n=5000)
    assert wl.n == 5000 and wl.k == 1024 and wl.data().rows(0, 3).shape == (3, 50)
