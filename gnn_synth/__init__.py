"""Seeded synthetic inputs (graphs, features, weights) for the aggregation path.

This package only draws random structure and random numbers.  It holds none of
the method's arithmetic: no normalisation weights, no aggregation, no
renumbering.  Both the CPU oracle's tests and the GPU path's tests consume the
buffers made here, so the two sides see identical bytes without sharing code.
"""
from .graphs import (  # noqa: F401
    BASE_SEED,
    Graph,
    add_self_loops,
    block_diagonal_batch,
    config_graph,
    config_spec,
    csr_from_undirected_pairs,
    features,
    glorot,
    planted_community_graph,
    power_law_graph,
    replicate,
    rmat_graph,
    shuffle_ids,
)
