"""Seeded synthetic input generators (graphs, sample pools, evaluation pairs).

This package only manufactures *inputs*: it holds none of the method's
arithmetic (no Philox stream of the trainer, no alias table, no SGD step, no
loss).  Both the CPU oracle's tests and the HIP path's tests and bench take
their graphs and pools from here, so the two sides see identical data without
sharing any code of the method itself.
"""
from .graphs import (  # noqa: F401
    barabasi_albert,
    chung_lu,
    planted_partition,
    degrees,
    csr_from_edges,
    csr_edge_weights,
    split_holdout,
    uniform_negative_pairs,
)
from .pools import walk_pool, marginal_pool  # noqa: F401
from .configs import CONFIGS, expected_degrees, make_graph  # noqa: F401
