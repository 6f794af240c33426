"""Seeded synthetic input generators shared by the CPU oracle's tests and the GPU path's tests/bench.

This package produces *inputs only*: sample matrices, index lists, initial weights and per-epoch
radius values.  It contains none of the SOM arithmetic (no distances, no best-matching-unit search,
no neighbourhood function, no update) so that the oracle and the HIP path stay independent.
"""
from .mixtures import GaussianMixture, Uniform01, uniform01_rows
from .configs import WORKLOADS, Workload, make_workload
from .draws import linear_sigma, exponential_sigma, draw_initial_rows, draw_subset, standardise, train_holdout_split

__all__ = [
    "GaussianMixture", "Uniform01", "uniform01_rows", "WORKLOADS", "Workload", "make_workload",
    "linear_sigma", "exponential_sigma", "draw_initial_rows", "draw_subset", "standardise", "train_holdout_split",
]
