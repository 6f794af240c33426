"""The synthetic workloads (shapes, distributions, radii) the build is measured and tested on.

Each entry only *describes inputs*: which mixture, how many rows, which lattice shape or graph kind, the
radius endpoints and epoch count.  The distance matrices themselves are built by whoever consumes the
workload (the oracle has its own builders, the GPU package has its own).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

from .mixtures import GaussianMixture, Uniform01


@dataclass(frozen=True)
class Workload:
    name: str
    n: int                      # rows in the dataset
    d: int                      # features
    k: int                      # nodes
    topology: str               # "rect" | "hex" | "mst" | "rng"
    lattice: Optional[Tuple[int, int]]  # (rows, cols) for rect / hex
    sigma: Tuple[float, float]  # radius at first and last epoch (linear in between)
    epochs: int
    rho: float = 1.0            # fraction of rows presented per epoch (1.0 = full selector)
    seed: int = 1000
    mixture: dict = field(default_factory=dict)

    def data(self):
        if self.mixture.get("uniform"):
            return Uniform01(self.seed, self.d)
        return GaussianMixture(self.seed, self.d, **self.mixture)


WORKLOADS = {
    # 10x10 rectangular lattice, 5 isotropic Gaussians in 8-D
    "cfg0": Workload("cfg0", 10_000, 8, 100, "rect", (10, 10), (5.0, 0.5), 10, seed=1000,
                     mixture=dict(n_comp=5, std=(0.5, 2.0), isotropic=True)),
    # 32x32 hexagonal lattice, 20 axis-aligned anisotropic Gaussians in 50-D   (headline workload)
    "cfg1": Workload("cfg1", 1_000_000, 50, 1024, "hex", (32, 32), (16.0, 1.0), 20, seed=1001,
                     mixture=dict(n_comp=20, std=(0.2, 3.0))),
    # 1024-node MST topology, 50 components with Dirichlet(1) weights and 5 % uniform background
    "cfg2": Workload("cfg2", 10_000_000, 50, 1024, "mst", None, (8.0, 0.5), 20, seed=1002,
                     mixture=dict(n_comp=50, std=(0.2, 3.0), weights="dirichlet", noise_frac=0.05)),
    # 1024-node RNG topology, 10 % random subset per epoch of a 1e8-row resident matrix
    "cfg3": Workload("cfg3", 100_000_000, 50, 1024, "rng", None, (8.0, 0.5), 30, rho=0.1, seed=1003,
                     mixture=dict(n_comp=100, std=(0.2, 3.0))),
    # 32x32 rectangular lattice, 1e9 rows streamed from host memory in chunks
    "cfg4": Workload("cfg4", 1_000_000_000, 50, 1024, "rect", (32, 32), (16.0, 1.0), 10, seed=1004,
                     mixture=dict(n_comp=100, std=(0.2, 3.0))),
    # default point of the paper's speed runs (Section 4.2.1): uniform [0,1) matrix, 32x32 grid, 10 iterations;
    # one axis at a time is varied from here (Supplementary Table S3)
    "scale": Workload("scale", 10_000_000, 50, 1024, "hex", (32, 32), (16.0, 1.0), 10, seed=1005,
                      mixture=dict(uniform=True)),
}


def make_workload(name: str, n: Optional[int] = None, **overrides) -> Workload:
    """A named workload, optionally with fewer rows (same distribution) or other fields replaced."""
    base = WORKLOADS[name]
    fields = dict(base.__dict__)
    if n is not None:
        fields["n"] = int(n)
    fields.update(overrides)
    return Workload(**fields)
