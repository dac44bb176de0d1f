"""Host-side packing (Section 4.6): qgtc_pack_bits_host against the oracle's packing and
quantizer, the compound-buffer layout, argument checks.  No GPU needed."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import qgnn, bitplane as bp


def _b():
    import paper_2111_09547_amd.binding as b
    b.lib()
    return b


def host_pack(b, src: np.ndarray, nbits, layout, quant=None, block_rows=0, threads=3):
    rows, cols = src.shape
    d, words = b.describe(rows, cols, nbits, layout, block_rows)
    buf = np.full(words + 8, 0xDEADBEEF, dtype=np.uint32)            # every word must be written
    base = buf.ctypes.data
    d.data = base + (-base % 16)
    off = (d.data - base) // 4
    dt = {np.dtype(np.float32): b.SRC_F32, np.dtype(np.uint8): b.SRC_U8, np.dtype(np.int32): b.SRC_I32}[src.dtype]
    q = None if quant is None else C.byref(b._QuantC(float(quant[0]), float(quant[1]), nbits))
    st = b.lib().qgtc_pack_bits_host(C.c_void_p(src.ctypes.data), dt, rows, cols, src.strides[0] // src.itemsize,
                                     q, C.byref(d), threads)
    assert st == 0, st
    k = rows if layout == b.LEFT else -(-rows // 32)
    m = -(-cols // 32) if layout == b.LEFT else cols
    out = np.empty((nbits, k, m), dtype=np.uint32)
    for p in range(nbits):
        for r in range(k):
            s = off + p * d.plane_stride_words + r * d.ld_words
            out[p, r] = buf[s:s + m]
    return out, buf, d, off


@pytest.mark.parametrize("layout", ["left", "right"])
@pytest.mark.parametrize("bits", [1, 2, 3, 5, 8, 16, 32])
@pytest.mark.parametrize("shape", [(1, 1), (37, 70), (64, 128), (100, 33)])
def test_host_pack_integers_match_the_oracle(layout, bits, shape):
    b = _b()
    lay = b.LEFT if layout == "left" else b.RIGHT
    rng = np.random.default_rng([51, bits, shape[0], shape[1]])
    v = rng.integers(0, 2 ** bits, size=shape, dtype=np.uint64).astype(np.uint32)
    got, buf, d, off = host_pack(b, v.view(np.int32), bits, lay)
    want = bp.pack(v, bits, bp.LEFT if layout == "left" else bp.RIGHT)
    assert (got == want).all()
    if layout == "left":                      # padding words up to ld are written as zeros
        ld = d.ld_words
        m = -(-shape[1] // 32)
        for r in range(shape[0]):
            assert (buf[off + r * ld + m: off + (r + 1) * ld] == 0).all()


@pytest.mark.parametrize("bits", [1, 4, 8, 11])
def test_host_pack_quantizes_like_eq2(bits):
    b = _b()
    rng = np.random.default_rng([52, bits])
    x = rng.normal(size=(130, 45)).astype(np.float32)
    x[0, 0], x[1, 1] = x.min() - 1.0, x.max() + 1.0          # beyond the range: clamped
    lo, hi = float(np.float32(-2.5)), float(np.float32(3.0))
    want = qgnn.quantize(x, lo, hi, bits)
    for lay, olay in ((b.LEFT, bp.LEFT), (b.RIGHT, bp.RIGHT)):
        got, _, _, _ = host_pack(b, x, bits, lay, quant=(lo, hi), threads=0)
        assert (got == bp.pack(want, bits, olay)).all()


def test_host_pack_u8_adjacency_block_storage_and_threads():
    b = _b()
    rng = np.random.default_rng(53)
    a = (rng.random((96 * 3, 96)) < 0.1).astype(np.uint8)
    ref, _, d, _ = host_pack(b, a, 1, b.LEFT, block_rows=96, threads=1)
    assert d.block_rows == 96 and (ref == bp.pack(a.astype(np.uint32), 1, bp.LEFT)).all()
    for t in (2, 7, 64):
        got, _, _, _ = host_pack(b, a, 1, b.LEFT, block_rows=96, threads=t)
        assert (got == ref).all()


def test_host_pack_argument_checks_and_compound_layout():
    b = _b()
    l = b.lib()
    x = np.zeros((8, 8), dtype=np.float32)
    d, words = b.describe(8, 8, 2, b.RIGHT)
    buf = np.zeros(words + 4, dtype=np.uint32)
    d.data = buf.ctypes.data + (-buf.ctypes.data % 16)
    src = C.c_void_p(x.ctypes.data)
    assert l.qgtc_pack_bits_host(None, 0, 8, 8, 8, None, C.byref(d), 1) == 1
    assert l.qgtc_pack_bits_host(src, 0, 8, 8, 8, None, C.byref(d), 1) == 1          # fp32 needs a quantizer
    q3 = b._QuantC(0.0, 1.0, 3)
    assert l.qgtc_pack_bits_host(src, 0, 8, 8, 8, C.byref(q3), C.byref(d), 1) == 3   # width mismatch
    q2 = b._QuantC(1.0, 1.0, 2)
    assert l.qgtc_pack_bits_host(src, 0, 8, 8, 8, C.byref(q2), C.byref(d), 1) == 2   # empty range
    q2 = b._QuantC(0.0, 1.0, 2)
    assert l.qgtc_pack_bits_host(src, 0, 8, 4, 8, C.byref(q2), C.byref(d), 1) == 2   # shape mismatch
    assert l.qgtc_pack_bits_host(src, 0, 8, 8, 8, C.byref(q2), C.byref(d), -1) == 2
    db, _ = b.describe(8, 8, 2, b.RIGHT_BYTES)
    db.data = d.data
    assert l.qgtc_pack_bits_host(src, 0, 8, 8, 8, C.byref(q2), C.byref(db), 1) == 7  # planes only
    assert l.qgtc_pack_bits_host(src, 0, 8, 8, 8, C.byref(q2), C.byref(d), 1) == 0

    sizes = (C.c_size_t * 3)(1, 256, 1000)
    offs = (C.c_size_t * 3)()
    assert l.qgtc_compound_layout(sizes, 3, offs) == 256 + 256 + 1024
    assert list(offs) == [0, 256, 512]
    assert l.qgtc_compound_layout(None, 2, offs) == 0
    assert l.qgtc_compound_layout(sizes, 0, offs) == 0


def test_subgraph_packet_on_the_host():
    """The compound buffer holds both packed objects where the layout says, and the
    descriptors into it decode to the inputs."""
    from paper_2111_09547_amd.packing import SubgraphPacket
    rng = np.random.default_rng(54)
    n, blk, dcols, s = 192, 96, 40, 4
    a = (rng.random((n, blk)) < 0.2).astype(np.uint8)
    x = rng.normal(size=(n, dcols)).astype(np.float32)
    xr = (float(x.min()), float(x.max()))
    pk = SubgraphPacket(n, blk, dcols, s, block_rows=blk, device=None, pin=False)
    pk.pack(torch.from_numpy(a), torch.from_numpy(x), xr)
    assert pk.offsets[0] == 0 and pk.offsets[1] % 256 == 0 and pk.nbytes >= pk.payload_bytes
    host = pk.host.numpy().view(np.uint32)
    ab, xb = pk.host_bits()
    wa = bp.pack(a.astype(np.uint32), 1, bp.LEFT)
    for r in range(n):
        o = pk.offsets[0] // 4 + r * ab.c.ld_words
        assert (host[o:o + wa.shape[2]] == wa[0, r]).all()
    wx = bp.pack(qgnn.quantize(x, xr[0], xr[1], s), s, bp.RIGHT)
    for p in range(s):
        for kw in range(n // 32):
            o = pk.offsets[1] // 4 + p * xb.c.plane_stride_words + kw * xb.c.ld_words
            assert (host[o:o + dcols] == wx[p, kw]).all()
