"""Random block-diagonal graphs shaped like batched, partitioned subgraphs.

A batch of subgraphs is a block-diagonal adjacency: nodes are numbered so that
subgraph b owns ids [b*block, (b+1)*block) and no edge crosses two subgraphs
(batching after partitioning, Section 4.1 of the paper; the evaluation notes
that the all-zero tiles mostly come from this structure).  Edges are kept as a
CSR pattern in global ids; dense 0/1 views are produced on demand.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class SubgraphBatch:
    n_nodes: int          # N, rows of the block-diagonal adjacency
    block: int            # nodes per subgraph (last one may be shorter)
    indptr: np.ndarray    # int64 [N+1]
    indices: np.ndarray   # int64 [nnz], global column ids, sorted per row
    info: dict            # how it was drawn (probabilities, dropped edges ...)

    @property
    def nnz(self) -> int:
        return int(self.indices.size)

    @property
    def n_blocks(self) -> int:
        return -(-self.n_nodes // self.block)

    def rows(self) -> np.ndarray:
        return np.repeat(np.arange(self.n_nodes, dtype=np.int64),
                         np.diff(self.indptr))

    def scipy_csr(self, dtype=np.uint64):
        import scipy.sparse as sp
        data = np.ones(self.nnz, dtype=dtype)
        return sp.csr_matrix((data, self.indices, self.indptr),
                             shape=(self.n_nodes, self.n_nodes))

    def dense(self) -> np.ndarray:
        """Full N x N uint8 0/1 matrix (small graphs only)."""
        a = np.zeros((self.n_nodes, self.n_nodes), dtype=np.uint8)
        a[self.rows(), self.indices] = 1
        return a

    def dense_compact(self) -> np.ndarray:
        """N x block uint8: row v keeps only the columns of its own subgraph,
        column j standing for node (v // block) * block + j."""
        r = self.rows()
        a = np.zeros((self.n_nodes, self.block), dtype=np.uint8)
        a[r, self.indices - (r // self.block) * self.block] = 1
        return a

    def degrees(self) -> np.ndarray:
        return np.diff(self.indptr).astype(np.int64)


def _from_edges(n: int, block: int, src, dst, info) -> SubgraphBatch:
    """Symmetric pattern from an undirected edge list (deduplicated)."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    r = np.concatenate([src, dst])
    c = np.concatenate([dst, src])
    key = np.unique(r * n + c)
    r, c = key // n, key % n
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(r, minlength=n), out=indptr[1:])
    return SubgraphBatch(n, block, indptr, c.astype(np.int64), info)


def block_bernoulli_graph(n_blocks: int, block: int, p: float,
                          self_loops: bool, rng: np.random.Generator
                          ) -> SubgraphBatch:
    """Each subgraph: upper triangle i<j drawn Bernoulli(p), mirrored; the
    diagonal is all ones when self_loops is set, else all zeros."""
    srcs, dsts = [], []
    for b in range(n_blocks):
        u = rng.random((block, block)) < p
        i, j = np.nonzero(np.triu(u, k=1))
        srcs.append(i + b * block)
        dsts.append(j + b * block)
    n = n_blocks * block
    src = np.concatenate(srcs)
    dst = np.concatenate(dsts)
    if self_loops:
        d = np.arange(n, dtype=np.int64)
        src = np.concatenate([src, d])
        dst = np.concatenate([dst, d])
    return _from_edges(n, block, src, dst,
                       {"kind": "block_bernoulli", "p": p,
                        "self_loops": self_loops})


def sbm_graph(n_comm: int, comm: int, p_in: float, p_out: float,
              rng: np.random.Generator) -> SubgraphBatch:
    """Stochastic block model cut into one subgraph per community.

    Inter-community edges are drawn only as a count (they are dropped when the
    graph is cut into per-community subgraph batches, the usual convention for
    partition-and-batch inference); the dropped fraction is kept in info."""
    g = block_bernoulli_graph(n_comm, comm, p_in, False, rng)
    n = n_comm * comm
    n_pairs_out = n * (n - 1) // 2 - n_comm * (comm * (comm - 1) // 2)
    dropped = int(rng.binomial(n_pairs_out, p_out))
    kept = g.nnz // 2
    g.info = {"kind": "sbm", "p_in": p_in, "p_out": p_out,
              "edges_kept": kept, "edges_dropped": dropped,
              "dropped_fraction": dropped / max(1, kept + dropped)}
    return g


def _bfs_order(n: int, indptr: np.ndarray, indices: np.ndarray,
               start: int) -> np.ndarray:
    """Breadth-first visiting order over all components: first from `start`,
    then restarting at the lowest unvisited id."""
    seen = np.zeros(n, dtype=bool)
    order = np.empty(n, dtype=np.int64)
    pos = 0
    next_restart = 0
    root = start
    while pos < n:
        seen[root] = True
        frontier = np.array([root], dtype=np.int64)
        while frontier.size:
            order[pos:pos + frontier.size] = frontier
            pos += frontier.size
            # neighbours of the whole frontier, in frontier order
            lo, hi = indptr[frontier], indptr[frontier + 1]
            cnt = hi - lo
            if cnt.sum() == 0:
                break
            idx = np.repeat(lo - np.concatenate([[0], np.cumsum(cnt)[:-1]]), cnt) \
                + np.arange(cnt.sum())
            nb = indices[idx]
            nb = nb[~seen[nb]]
            # first occurrence order, without duplicates
            _, first = np.unique(nb, return_index=True)
            frontier = nb[np.sort(first)]
            seen[frontier] = True
        while next_restart < n and seen[next_restart]:
            next_restart += 1
        root = next_restart
    return order


def chung_lu_bfs_graph(n: int, gamma: float, mean_degree: float, block: int,
                       self_loops: bool, rng: np.random.Generator
                       ) -> SubgraphBatch:
    """Chung-Lu power-law graph, relabelled in BFS order, cut into contiguous
    subgraphs of `block` nodes (edges across the cut are dropped).

    Expected degree w_i ~ (i+1)^(-1/(gamma-1)) scaled to `mean_degree`; the fast
    variant draws sum(w)/2 endpoint pairs with probability ~ w and removes
    loops and duplicates."""
    w = (np.arange(n, dtype=np.float64) + 1.0) ** (-1.0 / (gamma - 1.0))
    w *= mean_degree * n / w.sum()
    m = int(round(w.sum() / 2))
    pr = w / w.sum()
    u = rng.choice(n, size=m, p=pr)
    v = rng.choice(n, size=m, p=pr)
    keep = u != v
    g0 = _from_edges(n, n, u[keep], v[keep], {})
    order = _bfs_order(n, g0.indptr, g0.indices,
                       int(np.argmax(np.diff(g0.indptr))))
    new_id = np.empty(n, dtype=np.int64)
    new_id[order] = np.arange(n, dtype=np.int64)
    r = new_id[g0.rows()]
    c = new_id[g0.indices]
    und = r < c
    r, c = r[und], c[und]
    same = (r // block) == (c // block)
    total = int(r.size)
    r, c = r[same], c[same]
    if self_loops:
        d = np.arange(n, dtype=np.int64)
        r = np.concatenate([r, d])
        c = np.concatenate([c, d])
    info = {"kind": "chung_lu_bfs", "gamma": gamma, "mean_degree": mean_degree,
            "edges_total": total, "edges_kept": int(same.sum()),
            "dropped_fraction": 1.0 - float(same.sum()) / max(1, total),
            "self_loops": self_loops}
    return _from_edges(n, block, r, c, info)
