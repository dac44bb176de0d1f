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
    """Every function declared in include/*.h (comments stripped)."""
    import glob
    names = set()
    for path in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
        names |= set(re.findall(r"\b(qgtc_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


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


def test_tuning_is_range_checked_before_any_launch():
    """qgtc_tuning comes with the call; values outside its ranges are refused on the host."""
    import paper_2111_09547_amd.binding as b
    l = b.lib()
    Y = _fake_bits(b, 64, 64, 4, b.LEFT)
    W = _fake_bits(b, 64, 16, 4, b.RIGHT)
    for bad in (b._TuningC(3, 0, 0, 0), b._TuningC(0, 5000, 0, 0), b._TuningC(0, 0, 2, 0), b._TuningC(0, 0, 0, 3),
                b._TuningC(-1, 0, 0, 0), b._TuningC(0, 0, 0, 0, 3, 0), b._TuningC(0, 0, 0, 0, -1, 0),
                b._TuningC(0, 0, 0, 0, 0, 3), b._TuningC(0, 0, 0, 0, 0, -1)):
        ep = b.Epilogue(mode=b.OUT_I32).to_c()
        ep.tuning = C.pointer(bad)
        assert l.qgtc_update(C.byref(Y), C.byref(W), C.byref(ep), C.c_void_p(0x20000), 16, None) == 7


def test_layer_static_refuses_oversized_layers_on_the_host():
    """The layer without a workspace argument checks its size limit before any GPU call."""
    import paper_2111_09547_amd.binding as b
    l = b.lib()
    n, d = 70000, 2048
    assert l.qgtc_layer_workspace_bytes(n, d, 16, 16) > b.LAYER_STATIC_MAX_BYTES
    A = _fake_bits(b, n, 128, 1, b.LEFT, block_rows=128)
    X = _fake_bits(b, n, d, 16, b.RIGHT)
    W = _fake_bits(b, d, 16, 16, b.RIGHT)
    agg = b.Epilogue(mode=b.OUT_BITS, rq_nbits=16, rq_inv_scale=1.0).to_c()
    upd = b.Epilogue(mode=b.OUT_I32).to_c()
    st = l.qgtc_layer_static(C.byref(A), None, C.byref(X), C.byref(W), C.byref(agg), C.byref(upd),
                             C.c_void_p(0x30000), 16, None)
    assert st == 6                                       # QGTC_ERR_WORKSPACE
    assert l.qgtc_layer_static(None, None, C.byref(X), C.byref(W), C.byref(agg), C.byref(upd),
                               C.c_void_p(0x30000), 16, None) == 1


def test_selector_and_scalar_helpers_on_the_host():
    """qgtc_plan_layer, qgtc_quant_inv_scale, qgtc_layer_epilogues and qgtc_fold_batchnorm
    are pure host functions: rules and values checked without a GPU."""
    import numpy as np
    import paper_2111_09547_amd.binding as b
    from oracle import qgnn
    # Eq. (2)'s inverse step, rounded once to fp32, as the oracle forms it
    for lo, hi, bits in ((0.0, 8.0, 2), (-1.7, 3.9, 8), (0.0, 12345.0, 5), (-4.0, 4.0, 32)):
        assert b.qgtc_quant_inv_scale(lo, hi, bits) == float(qgnn.inv_scale(lo, hi, bits))
    assert b.qgtc_quant_inv_scale(1.0, 1.0, 4) == 0.0 and b.qgtc_quant_inv_scale(0.0, 1.0, 33) == 0.0
    # selector: narrow tiles only when they skip enough; fused kernel up to 8 bits, 1024 x 256
    plan = b.qgtc_plan_layer(65536, 64, 64, 8, 8, n_tile_rows=4096, a_cols=1024, nnz_tiles=(131072, 65536, 32768))
    assert plan["tile_kbits"] == 128 and plan["fused"] == 1 and plan["update_path"] == 2
    plan = b.qgtc_plan_layer(262144, 512, 16, 8, 8, n_tile_rows=16384, a_cols=2048, nnz_tiles=(60000, 40000, 30000))
    assert plan["tile_kbits"] == 32                      # 60000*32*1.3 < 40000*64 < 30000*128
    assert plan["est_us_update_first"] < plan["est_us_aggregate_first"]      # 512 -> 16 columns
    plan = b.qgtc_plan_layer(8192, 64, 64, 16, 16, n_tile_rows=512, a_cols=8192)
    assert plan["fused"] == 0 and plan["update_path"] == 1 and plan["tile_kbits"] == 128
    assert b.qgtc_plan_layer(8192, 2000, 64, 8, 8)["fused"] == 0
    assert b.qgtc_plan_layer(100, 64, 64, 8, 8, n_tile_rows=7)["ksplit"] == 4         # few tile rows: split the lists
    # zero-word jumping: from 3 planes, when fewer than 70 % (60 % from 5 planes) of the (row, word) pairs of the
    # kept tiles hold a bit
    kw = dict(n_tile_rows=4096, a_cols=1024, nnz_tiles=(131072, 65536, 32768))
    assert b.qgtc_plan_layer(65536, 64, 64, 8, 8, nnz_row_words=480000, **kw)["zero_words"] == 2
    assert b.qgtc_plan_layer(65536, 64, 64, 8, 8, nnz_row_words=2000000, **kw)["zero_words"] == 1      # 95 % present
    assert b.qgtc_plan_layer(65536, 64, 64, 2, 2, nnz_row_words=480000, **kw)["zero_words"] == 1        # too few planes
    assert b.qgtc_plan_layer(65536, 64, 64, 4, 4, nnz_row_words=1363149, **kw)["zero_words"] == 2       # 65 % present
    assert b.qgtc_plan_layer(65536, 64, 64, 5, 5, nnz_row_words=1363149, **kw)["zero_words"] == 1
    assert b.qgtc_plan_layer(65536, 64, 64, 8, 8, **kw)["zero_words"] == 0                              # unknown
    # tile width under zero-word jumping: the same (row, word) pairs are visited at every width, so fewer, wider tiles
    # weigh less than in the visit-all rule (tiles x (words per tile + 5.8)); a power-law batch like config 5
    kw5 = dict(n_tile_rows=16384, a_cols=2048, nnz_tiles=(42346, 34753, 29175), nnz_row_words=361800)
    plan = b.qgtc_plan_layer(262144, 512, 16, 8, 8, **kw5)
    assert (plan["zero_words"], plan["tile_kbits"]) == (2, 64)
    plan = b.qgtc_plan_layer(262144, 512, 16, 2, 2, **kw5)
    assert (plan["zero_words"], plan["tile_kbits"]) == (1, 32)                  # too few planes to jump: least visited bits
    assert b.qgtc_plan_layer(65536, 64, 64, 8, 8, nnz_row_words=480000, **kw)["tile_kbits"] == 128     # all tiles kept
    # independent runs: two for a launch of more than one and at most two rounds of the wave slots over a batch of
    # subgraphs, one otherwise; issue priority by remaining work when the launch has at most one wave per slot
    # (256 compute units: 3072 slots at 8 planes visiting every word, 4096 with zero-word jumping)
    plan = b.qgtc_plan_layer(65536, 64, 64, 8, 8, subgraphs=64, nnz_row_words=2000000, **kw)      # 4096 waves, visit all
    assert (plan["runs"], plan["even_progress"]) == (2, 1)
    plan = b.qgtc_plan_layer(65536, 64, 64, 8, 8, subgraphs=64, nnz_row_words=480000, **kw)       # jumping: one round
    assert (plan["runs"], plan["even_progress"]) == (1, 2)
    plan = b.qgtc_plan_layer(65536, 128, 64, 8, 8, subgraphs=64, nnz_row_words=480000, **kw)      # two column groups: one
    assert (plan["runs"], plan["even_progress"]) == (1, 2)                                        # wave takes both, one round
    kw6 = dict(n_tile_rows=6144, a_cols=1024, nnz_tiles=(196608, 98304, 49152))
    plan = b.qgtc_plan_layer(98304, 64, 64, 8, 8, subgraphs=96, nnz_row_words=720000, **kw6)      # 6144 waves: 1.5 rounds
    assert (plan["runs"], plan["even_progress"]) == (2, 1)
    assert b.qgtc_plan_layer(65536, 64, 64, 8, 8, n_tile_rows=4096, a_cols=1024)["runs"] == 1            # one graph
    assert b.qgtc_plan_layer(65536, 64, 64, 8, 8, n_tile_rows=4096, a_cols=1024, subgraphs=8)["runs"] == 1
    assert b.qgtc_plan_layer(262144, 512, 16, 8, 8, n_tile_rows=16384, a_cols=2048, subgraphs=128)["runs"] == 1   # long launch
    assert b.qgtc_plan_layer(65536, 64, 64, 16, 16, n_tile_rows=4096, a_cols=1024, subgraphs=64)["runs"] == 1     # not fused
    with pytest.raises(b.QgtcError):
        b.qgtc_plan_layer(10, 0, 4, 8, 8)
    # the scalars of a layer: the hand-worked 2-layer network of tests/golden
    e1, e2, zs, nx = b.qgtc_layer_epilogues(2, 2, 2, -2.0, 1.0, (-1.0, 1.0), 8, 8)
    assert (e1.mode, e1.rq_nbits, e1.rq_inv_scale, e1.relu) == (b.OUT_BITS, 2, 0.5, False)
    assert (e2.mode, e2.rq_nbits, e2.rq_inv_scale, e2.relu) == (b.OUT_BITS, 2, 0.5, True)
    assert zs == 1.0 and nx == 2.0
    e1, e2, zs, nx = b.qgtc_layer_epilogues(2, 2, 2, 0.0, 2.0, (-1.0, 1.0), 8, None, last=True)
    assert e2.mode == b.OUT_F32 and (e2.cc, e2.rs, e2.l0a, e2.l0b, e2.ck, e2.cs) == (2.0, -4.0, 0.0, 0.0, -2.0, 0.5)
    assert nx == 0.0
    # one-layer GIN: the zero point of the features enters through l0a / l0b
    e1, e2, _, _ = b.qgtc_layer_epilogues(8, 8, 64, -3.5, 0.03, (-0.1, 0.1), 900, None, self_term=True, last=True)
    assert e1.self_term and not e2.self_term and e2.l0a == -3.5 and e2.l0b == -3.5
    # update first: every code a pure scale
    e1, e2, zs, nx = b.qgtc_layer_epilogues(2, 2, 2, 0.0, 1.0, (-1.0, 1.0), 16, 4, self_term=True, update_first=True)
    assert not e1.self_term and e2.self_term and zs == 2.0 and nx == 2.0
    # batch normalization fold against the oracle's
    rng = np.random.default_rng(3)
    g, be, mu, var = rng.uniform(0.5, 2, 7), rng.uniform(-1, 1, 7), rng.uniform(-1, 1, 7), rng.uniform(0.1, 3, 7)
    a, sh = b.qgtc_fold_batchnorm(g, be, mu, var, 1e-5, 3.1e-4)
    ra, rb = qgnn.fold_batchnorm(g, be, mu, var, 1e-5, 3.1e-4)
    assert (a.numpy() == ra).all() and (sh.numpy() == rb).all()


def test_device_info_rejects_null_and_reports_no_device_without_a_gpu():
    import torch
    import paper_2111_09547_amd.binding as b
    l = b.lib()
    assert l.qgtc_device_info(None) == 1                      # QGTC_ERR_NULL
    if not torch.cuda.is_available():
        d = b._DeviceC()
        assert l.qgtc_device_info(C.byref(d)) != 0        # no device to query: an error, not a crash


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2111_09547_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "lib_path", lambda: str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        b.lib()
