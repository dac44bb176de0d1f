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


def assert_fp32_close(got, ref, what=""):
    """The fp32 parity rule, elementwise: |got - ref| <= 1e-6 * max(|ref|, max|ref|), i.e.
    1e-6 relative with an absolute floor of 1e-6 * max|ref| for entries near zero.  Prints
    the largest error met, relative to max|ref| and (for entries above 1e-3 of the largest)
    relative to the entry itself."""
    got = np.asarray(got, dtype=np.float64)
    ref64 = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref64.shape
    top = float(np.abs(ref64).max()) if ref64.size else 0.0
    err = np.abs(got - ref64)
    worst = float(err.max()) if err.size else 0.0
    big = np.abs(ref64) > 1e-3 * top
    rel = float((err[big] / np.abs(ref64[big])).max()) if big.any() else 0.0
    print(f"fp32 parity {what}: max|err| = {worst:.3e} = {worst / top if top else 0.0:.3e} of max|ref|, "
          f"max relative error on entries above 1e-3 of the largest = {rel:.3e}, "
          f"{int((err == 0).sum())} of {err.size} entries identical")
    assert np.isfinite(got).all()
    assert worst <= 1e-6 * top, (what, worst, top)
