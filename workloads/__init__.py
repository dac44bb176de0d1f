"""Seeded synthetic inputs for the quantized-GNN-layer hot path.

This package only draws random graphs, features and weights.  It holds none of
the method's arithmetic (no quantisation, no bit planes, no products), so both
the CPU oracle's tests and the HIP path's tests can take inputs from it without
sharing any code of the method.
"""
from .graphs import (SubgraphBatch, block_bernoulli_graph, sbm_graph,
                     chung_lu_bfs_graph)
from .configs import CONFIGS, Workload, make_workload

__all__ = ["SubgraphBatch", "block_bernoulli_graph", "sbm_graph",
           "chung_lu_bfs_graph", "CONFIGS", "Workload", "make_workload"]
