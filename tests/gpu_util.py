"""Helpers shared by the GPU parity tests: move workloads to the device, run the
HIP path through the binding, bring results back as numpy."""
import numpy as np
import torch

import paper_2111_09547_amd as q


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def as_u32(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def pack_adjacency(graph_or_dense, storage="dense"):
    """uint8 0/1 adjacency -> packed Bits (LEFT, 1 bit)."""
    if isinstance(graph_or_dense, np.ndarray):
        return q.qgtc_pack_bits(dev(graph_or_dense.astype(np.uint8)), 1, q.LEFT)
    g = graph_or_dense
    if storage == "dense":
        return q.qgtc_pack_bits(dev(g.dense()), 1, q.LEFT)
    return q.qgtc_pack_bits(dev(g.dense_compact()), 1, q.LEFT, block_rows=g.block)


def words_np(bits: q.Bits) -> np.ndarray:
    """Packed words as the oracle shapes them: LEFT [nbits][rows][ceil(cols/32)],
    RIGHT [nbits][ceil(rows/32)][cols] (strides removed)."""
    c = bits.c
    w = bits.words.cpu().numpy().view(np.uint32)
    k = c.rows if c.layout == q.LEFT else -(-c.rows // 32)
    m = -(-c.cols // 32) if c.layout == q.LEFT else c.cols
    off = (c.data - bits.words.data_ptr()) // 4
    out = np.empty((c.nbits, k, m), dtype=np.uint32)
    for p in range(c.nbits):
        for r in range(k):
            s = off + p * c.plane_stride_words + r * c.ld_words
            out[p, r] = w[s:s + m]
    return out


def sync():
    torch.cuda.synchronize()
