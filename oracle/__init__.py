"""CPU float64 oracle for the batch-SOM epoch.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this package: only ``tests/``, ``__graft_entry__.smoke()`` and
the ``cpu_baseline`` leg of ``bench.py`` do.  It shares no code with the HIP library.
"""
from .som import (  # noqa: F401
    sampling_budget, sq_distances, bmu, near_tie_mask, influence, epoch_definition, displacement_form_update,
    accumulate, neighborhood_update, neighborhood_update_momentum, neighborhood_update_shifted, epoch_grouped, bmu_gram, quantization_error, DEFAULT_EPS_H,
)
from .topology import (  # noqa: F401
    rect_lattice_distances, hex_lattice_positions, hex_lattice_distances, node_sq_distances,
    mst_edges, rng_edges, rng_blocked, hop_distances, graph_distances,
)
