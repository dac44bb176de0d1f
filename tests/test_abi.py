"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments on the host before launching
anything (no kernel runs here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2111_09547_amd", "lib", "libqgtc.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB),
                                reason="libqgtc.so not built (run __graft_entry__.build())")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "qgtc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qgtc_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    import paper_2111_09547_amd.binding as b
    lib = C.CDLL(LIB)
    names = declared_symbols()
    assert {"qgtc_pack_bits", "qgtc_build_tile_map", "qgtc_aggregate", "qgtc_update",
            "qgtc_layer"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert b.qgtc_version() >= 100


def test_describe_and_sizes():
    import paper_2111_09547_amd.binding as b
    d, words = b.describe(13, 70, 3, b.LEFT)
    # K padded to 128 bits: ceil(70/128)*4 = 4 words per row
    assert (d.ld_words, d.plane_stride_words, words) == (4, 52, 156)
    d, words = b.describe(45, 77, 2, b.RIGHT)
    assert (d.ld_words, d.plane_stride_words, words) == (77, 154, 308)
    assert b.lib().qgtc_describe(C.byref(d), 4, 4, 0, b.LEFT, 0) == 0
    assert b.lib().qgtc_describe(C.byref(d), 4, 4, 33, b.LEFT, 0) == 0
    nb = b.lib().qgtc_tile_map_bytes(256, 256, 16, 128)
    assert nb >= (16 + 16 * 2 + 1 + 256) * 4
    assert b.lib().qgtc_tile_map_bytes(256, 256, 7, 128) == 0
    words = b.lib().qgtc_describe(C.byref(d), 70, 20, 8, b.RIGHT_BYTES, 0)
    assert (d.ld_words, d.plane_stride_words, words) == (512, 1024, 2048)
    assert b.lib().qgtc_describe(C.byref(d), 70, 20, 7, b.RIGHT_BYTES, 0) == 1024
    assert b.lib().qgtc_describe(C.byref(d), 70, 20, 9, b.RIGHT_BYTES, 0) == 0
    words = b.lib().qgtc_describe(C.byref(d), 10, 70, 8, b.LEFT_BYTES, 0)
    assert (d.ld_words, words) == (20, 200)
    assert b.lib().qgtc_describe(C.byref(d), 10, 70, 9, b.LEFT_BYTES, 0) == 0
    assert b.lib().qgtc_layer_workspace_bytes(100, 70, 16, 4) >= 100 * 3 * 4 * 4 + 100 * 4


def test_status_strings():
    import paper_2111_09547_amd.binding as b
    for s in range(9):
        assert len(b.lib().qgtc_status_string(s)) > 1


def _fake_bits(b, rows, cols, nbits, layout, block_rows=0, addr=0x10000):
    d, _ = b.describe(rows, cols, nbits, layout, block_rows)
    d.data = addr                      # never dereferenced: validation fails first
    return d


def test_argument_validation_happens_before_any_launch():
    import paper_2111_09547_amd.binding as b
    l = b.lib()
    ep = b.Epilogue(mode=b.OUT_I32).to_c()
    out = C.c_void_p(0x20000)
    A = _fake_bits(b, 64, 64, 1, b.LEFT)
    X = _fake_bits(b, 64, 16, 2, b.RIGHT)
    # NULL operands
    assert l.qgtc_aggregate(None, None, C.byref(X), C.byref(ep), out, 16, None) == 1
    assert l.qgtc_aggregate(C.byref(A), None, C.byref(X), C.byref(ep), None, 16, None) == 1
    # adjacency must be 1 bit, LEFT
    A2 = _fake_bits(b, 64, 64, 2, b.LEFT)
    assert l.qgtc_aggregate(C.byref(A2), None, C.byref(X), C.byref(ep), out, 16, None) == 3
    A3 = _fake_bits(b, 64, 64, 1, b.RIGHT)
    assert l.qgtc_aggregate(C.byref(A3), None, C.byref(X), C.byref(ep), out, 16, None) == 5
    # X must be RIGHT
    X2 = _fake_bits(b, 64, 16, 2, b.LEFT)
    assert l.qgtc_aggregate(C.byref(A), None, C.byref(X2), C.byref(ep), out, 16, None) == 5
    # contraction sizes must agree
    X3 = _fake_bits(b, 96, 16, 2, b.RIGHT)
    assert l.qgtc_aggregate(C.byref(A), None, C.byref(X3), C.byref(ep), out, 16, None) == 2
    # leading dimension of the output too small
    assert l.qgtc_aggregate(C.byref(A), None, C.byref(X), C.byref(ep), out, 8, None) == 2
    # misaligned adjacency
    A4 = _fake_bits(b, 64, 64, 1, b.LEFT, addr=0x10004)
    assert l.qgtc_aggregate(C.byref(A4), None, C.byref(X), C.byref(ep), out, 16, None) == 4
    # block-diagonal storage needs a multiple of 32 rows per block
    A5 = _fake_bits(b, 96, 48, 1, b.LEFT, block_rows=48)
    assert l.qgtc_aggregate(C.byref(A5), None, C.byref(X3), C.byref(ep), out, 16, None) == 4
    # bit width out of range
    X4 = _fake_bits(b, 64, 16, 2, b.RIGHT)
    X4.nbits = 40
    assert l.qgtc_aggregate(C.byref(A), None, C.byref(X4), C.byref(ep), out, 16, None) == 3
    # self term needs a square adjacency
    A6 = _fake_bits(b, 32, 64, 1, b.LEFT)
    eps = b.Epilogue(mode=b.OUT_I32, self_term=True).to_c()
    assert l.qgtc_aggregate(C.byref(A6), None, C.byref(X), C.byref(eps), out, 16, None) == 2
    # update: contraction mismatch, wrong layouts
    Y = _fake_bits(b, 64, 32, 3, b.LEFT)
    W = _fake_bits(b, 64, 8, 3, b.RIGHT)
    assert l.qgtc_update(C.byref(Y), C.byref(W), C.byref(ep), out, 8, None) == 2
    assert l.qgtc_update(C.byref(W), C.byref(Y), C.byref(ep), out, 8, None) == 5
    # layer: aggregation epilogue must emit bits; workspace too small
    W2 = _fake_bits(b, 16, 8, 2, b.RIGHT)
    assert l.qgtc_layer(C.byref(A), None, C.byref(X), C.byref(W2), C.byref(ep), C.byref(ep),
                        C.c_void_p(0x30000), 1 << 20, out, 8, None) == 7
    epb = b.Epilogue(mode=b.OUT_BITS, rq_nbits=2, rq_inv_scale=1.0).to_c()
    assert l.qgtc_layer(C.byref(A), None, C.byref(X), C.byref(W2), C.byref(epb), C.byref(ep),
                        C.c_void_p(0x30000), 16, out, 8, None) == 6
    # weights as bytes are for the fused kernel only: a shape it does not cover is refused
    Wby = _fake_bits(b, 16, 300, 2, b.RIGHT_BYTES)
    assert l.qgtc_layer(C.byref(A), None, C.byref(X), C.byref(Wby), C.byref(epb), C.byref(ep),
                        C.c_void_p(0x30000), 1 << 20, out, 300, None) == 7
    Wby = _fake_bits(b, 16, 8, 2, b.RIGHT_BYTES)
    assert l.qgtc_update(C.byref(Y), C.byref(Wby), C.byref(ep), out, 8, None) == 5
    # codes as bytes on the left: only the matrix-core update takes them (<= 8 bits on both sides)
    Yby = _fake_bits(b, 64, 64, 8, b.LEFT_BYTES)
    W9 = _fake_bits(b, 64, 8, 9, b.RIGHT)
    assert l.qgtc_update(C.byref(Yby), C.byref(W9), C.byref(ep), out, 8, None) == 7
    assert l.qgtc_aggregate(C.byref(Yby), None, C.byref(X), C.byref(ep), out, 16, None) == 5
    # per-column affine map: not for int32 outputs, a shift needs a scale, and in
    # qgtc_layer it belongs to the update's epilogue
    epa = b.Epilogue(mode=b.OUT_I32).to_c()
    epa.col_scale = 0x60000
    assert l.qgtc_aggregate(C.byref(A), None, C.byref(X), C.byref(epa), out, 16, None) == 7
    assert l.qgtc_update(C.byref(Y), C.byref(_fake_bits(b, 32, 8, 3, b.RIGHT)), C.byref(epa), out, 8, None) == 7
    epa = b.Epilogue(mode=b.OUT_F32, cc=1.0).to_c()
    epa.col_shift = 0x60000
    assert l.qgtc_aggregate(C.byref(A), None, C.byref(X), C.byref(epa), out, 16, None) == 1
    epb2 = b.Epilogue(mode=b.OUT_BITS, rq_nbits=2, rq_inv_scale=1.0).to_c()
    epb2.col_scale = 0x60000
    assert l.qgtc_layer(C.byref(A), None, C.byref(X), C.byref(W2), C.byref(epb2), C.byref(ep),
                        C.c_void_p(0x30000), 1 << 20, out, 8, None) == 7
    # pack: fp32 source needs a quantizer with hi > lo
    D = _fake_bits(b, 64, 16, 2, b.RIGHT)
    assert l.qgtc_pack_bits(C.c_void_p(0x40000), 0, 64, 16, 16, None, C.byref(D), None) == 1
    assert l.qgtc_pack_bits(C.c_void_p(0x40000), 0, 64, 8, 16, None, C.byref(D), None) == 2
    # tile map: unsupported tile shape for the aggregation
    m = b._TileMapC(8, 128, 8, 1, 0x50000, 0x51000, 0x52000, 0x53000)
    assert l.qgtc_aggregate(C.byref(A), C.byref(m), C.byref(X), C.byref(ep), out, 16, None) == 7


def test_probe_arguments_are_checked():
    import paper_2111_09547_amd.binding as b
    l = b.lib()
    assert l.qgtc_probe_popcount(1, 1, 1, None, None) == 1
    assert l.qgtc_probe_popcount(0, 1, 1, C.c_void_p(0x1000), None) == 2
    assert l.qgtc_probe_popcount(1, 5, 1, C.c_void_p(0x1000), None) == 2


def test_options_are_range_checked():
    import paper_2111_09547_amd.binding as b
    l = b.lib()
    assert l.qgtc_set_option(b.OPT_UPDATE_PATH, 3) == 7
    assert l.qgtc_set_option(b.OPT_UPDATE_PATH, 0) == 0
    assert l.qgtc_set_option(b.OPT_AGG_XCD_RUN, 5000) == 7
    assert l.qgtc_set_option(b.OPT_AGG_XCD_RUN, -1) == 0
    assert l.qgtc_set_option(b.OPT_AGG_XCD_RUN, 0) == 0
    assert l.qgtc_set_option(99, 0) == 7


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2111_09547_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "lib_path", lambda: str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        b.lib()
