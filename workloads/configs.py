"""The five benchmark workloads, as seeded synthetic inputs.

They stand in for the partitioned datasets of the paper's Table 1, which are not
available: shapes, densities and block structure follow the benchmark
description; everything is drawn from numpy Generators seeded with
[0, config id, tensor id].

`n_blocks` can shrink a workload (fewer subgraphs of the same size and density)
so that CPU tests stay fast; the default is the full size.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from .graphs import (SubgraphBatch, block_bernoulli_graph, sbm_graph,
                     chung_lu_bfs_graph)


@dataclass
class Workload:
    cfg: int
    name: str
    model: str                    # "aggregate" | "gcn" | "gin"
    graph: SubgraphBatch
    X: np.ndarray                 # fp32 [N, D]; uint32 when x_is_quantized
    x_is_quantized: bool
    W: list                       # fp32 [D_l, H_l] per layer (empty: no update)
    s: int                        # bits of the node embeddings
    t: int                        # bits of the weights
    storage: str                  # "dense": one N x N adjacency + tile map;
                                  # "compact": N x block (one block per subgraph)
    bit_sweep: tuple = ()
    notes: dict = field(default_factory=dict)

    @property
    def n_layers(self) -> int:
        return len(self.W)


def _rng(cfg: int, tensor: int) -> np.random.Generator:
    return np.random.default_rng([0, cfg, tensor])


def _features(cfg, n, d):
    return _rng(cfg, 1).standard_normal((n, d), dtype=np.float32)


def _weights(cfg, dims):
    return [_rng(cfg, 10 + l).uniform(-0.1, 0.1, size=(dims[l], dims[l + 1]))
            .astype(np.float32) for l in range(len(dims) - 1)]


def make_workload(cfg: int, bits: int | None = None,
                  n_blocks: int | None = None) -> Workload:
    if cfg == 1:
        nb = n_blocks or 4
        g = block_bernoulli_graph(nb, 64, 0.1, True, _rng(1, 0))
        x = _rng(1, 1).integers(0, 4, size=(g.n_nodes, 16)).astype(np.uint32)
        return Workload(1, "tiny aggregation, uint2 features", "aggregate", g,
                        x, True, [], 2, 0, "dense")
    if cfg == 2:
        nb = n_blocks or 16
        g = block_bernoulli_graph(nb, 256, 0.02, True, _rng(2, 0))
        b = bits or 4
        return Workload(2, "one GCN layer, 16 subgraphs of 256", "gcn", g,
                        _features(2, g.n_nodes, 128), False,
                        _weights(2, [128, 16]), b, b, "dense")
    if cfg == 3:
        nb = n_blocks or 8
        g = block_bernoulli_graph(nb, 1024, 0.01, False, _rng(3, 0))
        b = bits or 8
        return Workload(3, "bitwidth sweep, 8 subgraphs of 1024", "gcn", g,
                        _features(3, g.n_nodes, 64), False,
                        _weights(3, [64, 64]), b, b, "dense",
                        bit_sweep=(1, 2, 3, 4, 5, 6, 7, 8, 16, 32))
    if cfg == 4:
        nb = n_blocks or 64
        g = sbm_graph(nb, 1024, 0.008, 1e-5, _rng(4, 0))
        b = bits or 8
        return Workload(4, "5-layer GIN, hidden 64, SBM communities of 1024",
                        "gin", g, _features(4, g.n_nodes, 128), False,
                        _weights(4, [128, 64, 64, 64, 64, 64]), b, b,
                        "compact")
    if cfg == 5:
        nb = n_blocks or 128
        g = chung_lu_bfs_graph(nb * 2048, 2.1, 12.0, 2048, True, _rng(5, 0))
        b = bits or 8
        return Workload(5, "2-layer GCN, hidden 16, power-law graph in "
                        "2048-node subgraphs", "gcn", g,
                        _features(5, g.n_nodes, 512), False,
                        _weights(5, [512, 16, 16]), b, b, "compact",
                        bit_sweep=(1, 2, 4, 8))
    raise ValueError(f"unknown config {cfg}")


CONFIGS = (1, 2, 3, 4, 5)
