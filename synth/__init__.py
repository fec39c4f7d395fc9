"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package holds input recipes only: atom positions, random embeddings and
random weights of given shapes.  It contains none of the method's arithmetic
(no neighbour search, no basis functions, no network layers), so that the
oracle and the HIP library stay independent of each other while still seeing
identical inputs.
"""
from .configs import CONFIGS, BlockDims, Workload, get_workload  # noqa: F401
from .systems import (  # noqa: F401
    cube_positions,
    slab_adsorbate_positions,
    box_positions,
    make_positions,
)
from .tensors import (  # noqa: F401
    glorot,
    weights_D,
    weights_G,
    weights_head,
    weights_out,
    edge_embeddings,
)
