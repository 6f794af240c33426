"""The seeded input generators: reproducible, of the stated shape, and free of the method's arithmetic."""
import numpy as np

from synth import (draw_initial_rows, draw_subset, exponential_sigma, linear_sigma, make_workload, standardise,
                   train_holdout_split)


def test_draws_are_reproducible_and_well_formed():
    a, b = draw_subset(3, 5, 100_000, 7_000), draw_subset(3, 5, 100_000, 7_000)
    assert np.array_equal(a, b) and a.dtype == np.uint32 and len(np.unique(a)) == 7_000 and (np.diff(a) > 0).all()
    assert not np.array_equal(a, draw_subset(3, 6, 100_000, 7_000))        # redrawn per epoch
    rows = draw_initial_rows(1, 1000, 100)
    assert len(np.unique(rows)) == 100 and rows.max() < 1000
    sig = linear_sigma(16.0, 1.0, 20)
    assert sig[0] == 16.0 and sig[-1] == 1.0 and np.allclose(np.diff(sig), -15.0 / 19)
    geo = exponential_sigma(16.0, 1.0, 5)
    assert np.allclose(geo, [16.0, 8.0, 4.0, 2.0, 1.0]) and exponential_sigma(3.0, 1.0, 1)[0] == 3.0


def test_train_holdout_split_partitions_the_rows():
    train, hold = train_holdout_split(9, 1000)
    assert len(train) == 700 and len(hold) == 300
    assert np.array_equal(np.sort(np.concatenate([train, hold])), np.arange(1000))
    assert np.array_equal(train, train_holdout_split(9, 1000)[0])
    assert not np.array_equal(train, train_holdout_split(10, 1000)[0])


def test_standardise_gives_zero_mean_unit_variance():
    wl = make_workload("cfg0")
    X = wl.data().rows(0, 5000)
    X[:, 3] = 2.5                                                       # a constant feature is only centred
    Z = standardise(X)
    assert Z.dtype == np.float32
    assert np.abs(Z.mean(axis=0)).max() < 1e-5
    std = Z.std(axis=0)
    assert np.abs(np.delete(std, 3) - 1.0).max() < 1e-4 and std[3] == 0.0
