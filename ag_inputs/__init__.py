"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This package only *produces inputs* (graphs in CSR form, feature matrices,
labels, weight initialisations).  It holds none of the aggregation method's
arithmetic: no SpMM, no reordering, no splitting.
"""
from .graphs import (  # noqa: F401
    Graph,
    planted_partition,
    chung_lu_communities,
    mixed_density,
    directed_random,
    rmat,
    from_edges,
    gcn_normalise,
    row_normalise,
    features,
    glorot_uniform,
    labels,
    config_graph,
    CONFIGS,
)
