"""GPU parity: each entry point of the C ABI against the CPU oracle, element by
element, on seeded inputs that span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

from oracle import qgnn, bitplane as bp
from workloads import make_workload

pytestmark = pytest.mark.gpu

q = pytest.importorskip("paper_2111_09547_amd")
from gpu_util import assert_fp32_close, dev, as_u32, pack_adjacency, words_np, sync  # noqa: E402


def rand_graph(rng, n, k, p):
    return (rng.random((n, k)) < p).astype(np.uint8)


# ------------------------------------------------------------------ pack / unpack
@pytest.mark.parametrize("bits", [1, 5, 8])
@pytest.mark.parametrize("shape", [(1, 1), (45, 77), (130, 64), (64, 300), (512, 16)])
def test_pack_bytes_layout(bits, shape):
    """Codes as bytes in matrix-core operand order: position of every byte as the
    header states it, 7 + 1 split for 8 bits, zero fill, from fp32 and from integers."""
    rows, cols = shape
    rng = np.random.default_rng([3, bits, rows, cols])
    x = rng.standard_normal((rows, cols)).astype(np.float32)
    lo, hi = float(x.min()), float(x.max()) + 1e-3
    codes = qgnn.quantize(x, lo, hi, bits)
    for src, kw in ((dev(x), dict(quant=(lo, hi))), (dev(codes.view(np.int32)), {})):
        b = q.alloc_bits(rows, cols, bits, q.RIGHT_BYTES)
        b.words.fill_(-1)
        q.qgtc_pack_bits(src, bits, q.RIGHT_BYTES, out=b, **kw)
        assert (as_u32(q.qgtc_unpack_bits(b)) == codes).all()
        raw = b.words.cpu().numpy().view(np.uint8)
        n_nt, n_ks = -(-cols // 16), -(-rows // 64)
        parts = 2 if bits == 8 else 1
        want = np.zeros((parts, n_nt, n_ks, 64, 16), dtype=np.uint8)
        for k in range(rows):
            for c in range(cols):
                lane = c % 16 + 16 * ((k % 64) // 16)
                v = int(codes[k, c])
                want[0, c // 16, k // 64, lane, k % 16] = v & 0x7f if bits == 8 else v
                if bits == 8:
                    want[1, c // 16, k // 64, lane, k % 16] = v >> 7
        assert b.c.ld_words == 256 * n_ks and b.c.plane_stride_words == n_nt * n_ks * 256
        assert (raw[:want.size] == want.ravel()).all()


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("bits", [1, 2, 3, 8, 13, 32])
@pytest.mark.parametrize("shape", [(1, 1), (45, 77), (130, 64), (64, 2100)])
def test_pack_integers_roundtrip(layout, bits, shape):
    rng = np.random.default_rng([1, layout, bits, shape[0]])
    v = rng.integers(0, 2 ** bits, size=shape, dtype=np.uint64).astype(np.uint32)
    b = q.qgtc_pack_bits(dev(v.view(np.int32)), bits, layout)
    sync()
    want = bp.pack(v, bits, layout)
    assert (words_np(b) == want).all()
    if layout == q.LEFT:                      # padding words up to ld are zero
        w = b.words.cpu().numpy().view(np.uint32)[:b.c.plane_stride_words * bits]
        w = w.reshape(bits, shape[0], b.c.ld_words)
        assert (w[:, :, want.shape[2]:] == 0).all()
    assert (as_u32(q.qgtc_unpack_bits(b)) == v).all()


def test_pack_u8_masks_high_bits():
    rng = np.random.default_rng(2)
    v = rng.integers(0, 256, size=(70, 40)).astype(np.uint8)
    b = q.qgtc_pack_bits(dev(v), 3, q.RIGHT)
    assert (as_u32(q.qgtc_unpack_bits(b)) == (v & 7)).all()


@pytest.mark.parametrize("bits", [1, 2, 4, 8, 16, 24, 32])
def test_pack_quantizes_like_eq2(bits):
    rng = np.random.default_rng([3, bits])
    x = rng.standard_normal((333, 50)).astype(np.float32)
    x[0, 0], x[1, 1] = 1e30, -1e30            # far outside the range: clamped
    lo, hi = -2.5, 3.25
    b = q.qgtc_pack_bits(dev(x), bits, q.RIGHT, quant=(lo, hi))
    want = qgnn.quantize(x, lo, hi, bits)
    assert (as_u32(q.qgtc_unpack_bits(b)) == want).all()
    # min-max range of the data itself
    lo, hi = float(x[2:].min()), float(x[2:].max())
    b = q.qgtc_pack_bits(dev(x[2:]), bits, q.LEFT, quant=(lo, hi))
    assert (as_u32(q.qgtc_unpack_bits(b)) == qgnn.quantize(x[2:], lo, hi, bits)).all()


def test_row_and_col_sums():
    rng = np.random.default_rng(4)
    v = rng.integers(0, 64, size=(150, 90)).astype(np.uint32)
    bl = q.qgtc_pack_bits(dev(v.view(np.int32)), 6, q.LEFT)
    br = q.qgtc_pack_bits(dev(v.view(np.int32)), 6, q.RIGHT)
    assert (q.qgtc_row_sums(bl).cpu().numpy() == v.sum(axis=1)).all()
    assert (q.qgtc_col_sums(br).cpu().numpy() == v.sum(axis=0)).all()


# ----------------------------------------------------------------------- tile map
@pytest.mark.parametrize("tile", [(8, 128), (16, 128), (16, 64), (16, 32), (32, 256), (64, 512)])
def test_tile_map_matches_brute_force(tile):
    rng = np.random.default_rng([5, tile[0], tile[1]])
    n, k = 203, 1000
    A = rand_graph(rng, n, k, 0.0008)
    A[40:60] = 0                                 # some all-zero rows of tiles
    Ab = pack_adjacency(A)
    m = q.qgtc_build_tile_map(Ab, tile[0], tile[1])
    sync()
    lists, deg = qgnn.tile_map(A, tile[0], tile[1])
    cnt = m.row_cnt.cpu().numpy()
    idx = m.col_idx.cpu().numpy()
    assert cnt.tolist() == [len(l) for l in lists]
    for tr, l in enumerate(lists):
        assert idx[tr, :len(l)].tolist() == l
    assert int(m.nnz_tiles.cpu()[0]) == sum(len(l) for l in lists)
    assert (m.deg.cpu().numpy() == deg).all()



def test_device_is_what_the_kernels_are_written_for():
    """The launch shapes read the compute-unit count from the device; the workgroup dealing
    is written for 8 XCDs of 32 compute units: check both on the device the tests run on."""
    d = q.qgtc_device_info()
    assert d["is_gfx950"]
    assert d["compute_units"] == torch.cuda.get_device_properties(0).multi_processor_count
    assert d["xcds"] == d["xcds_assumed"] == 8 and d["compute_units"] == 256


@pytest.mark.parametrize("shape", [(1, 1), (100, 300), (257, 257), (1000, 2100), (4100, 640)])
def test_tile_stats_match_the_oracle_at_three_widths(shape):
    """qgtc_tile_stats: non-zero tiles at 16 x 32 / 64 / 128 in one pass, against the brute-force
    tile map of the oracle and against the three maps built one by one."""
    n, k = shape
    rng = np.random.default_rng([5, n, k])
    A = rand_graph(rng, n, k, 0.004)
    if n > 64:
        A[40:90, :] = 0                             # rows of tiles without any edge
    Ab = pack_adjacency(A)
    got = q.qgtc_tile_stats(Ab).cpu().numpy().tolist()
    want = [sum(len(l) for l in qgnn.tile_map(A, 16, kb)[0]) for kb in (32, 64, 128)]
    # (row, 32-bit word) pairs that hold a bit: brute force on the dense matrix
    pad = np.zeros((n, -(-k // 32) * 32), dtype=np.uint8)
    pad[:, :k] = A
    row_words = int(pad.reshape(n, -1, 32).any(axis=2).sum())
    assert got == want + [-(-n // 16), row_words, 0, 0, 0]
    assert q.tile_stats_numbers(q.qgtc_tile_stats(Ab)) == dict(nnz_tiles=want, n_tile_rows=-(-n // 16),
                                                               nnz_row_words=row_words)
    for i, kb in enumerate((32, 64, 128)):
        assert int(q.qgtc_build_tile_map(Ab, 16, kb).nnz_tiles.cpu()[0]) == want[i]
    # a second call into the same buffer starts from zero again
    buf = q.qgtc_tile_stats(Ab)
    assert q.qgtc_tile_stats(Ab, out=buf).cpu().numpy().tolist() == got


def test_tile_stats_on_block_diagonal_storage():
    w = make_workload(5, n_blocks=2)
    g = w.graph
    Ab = pack_adjacency(g, "compact")
    got = q.qgtc_tile_stats(Ab).cpu().numpy().tolist()
    compact = g.dense_compact()
    want = [sum(len(l) for l in qgnn.tile_map(compact, 16, kb)[0]) for kb in (32, 64, 128)]
    row_words = int(compact.reshape(g.n_nodes, -1, 32).any(axis=2).sum())
    assert got == want + [g.n_nodes // 16, row_words, 0, 0, 0]
    assert want[0] > want[1] > want[2]


def expected_run_log2(cnt):
    """The rule stated for nnz_tiles[1] in qgtc.h, on the host."""
    w = np.asarray(cnt, dtype=np.int64) + 1
    for sh in (6, 5, 4):
        load = np.zeros(8, dtype=np.int64)
        np.add.at(load, (np.arange(len(w)) >> sh) & 7, w)
        if load.max() * 8 * 50 <= w.sum() * 51:
            return sh
    return 3


@pytest.mark.parametrize("case", ["uniform", "hubs_first", "mild_skew", "small", "ragged"])
def test_tile_map_run_hint(case):
    """nnz_tiles[1]: long runs for evenly spread tiles, short ones when a few tile rows
    hold most tiles or when there are too few tile rows for eight long runs."""
    rng = np.random.default_rng(17)
    n = {"small": 100 * 16, "ragged": 1000 * 16 + 5}.get(case, 1024 * 16)
    k = 2048
    A = np.zeros((n, k), dtype=np.uint8)
    rows = np.arange(n)
    A[rows, rows % k] = 1                                     # one tile per tile row at least
    if case == "hubs_first":
        A[:64 * 16:16, ::128] = 1                             # the first 64 tile rows hold every tile
    if case == "mild_skew":
        for tr in range(0, 1024, 4):
            A[tr * 16, rng.integers(0, k, size=3)] = 1
    Ab = pack_adjacency(A)
    m = q.qgtc_build_tile_map(Ab, 16, 128)
    sync()
    cnt = m.row_cnt.cpu().numpy()
    total, run = m.nnz_tiles.cpu().numpy().tolist()
    assert total == cnt.sum()
    assert run == expected_run_log2(cnt)
    if case == "uniform":
        assert run == 6
    if case in ("hubs_first", "small"):
        assert run == 3


# ---------------------------------------------------------------------- aggregate
def run_aggregate(A, X, s, tile_kbits=None, block=0, ep=None):
    if block:
        n = A.shape[0]
        compact = np.zeros((n, block), dtype=np.uint8)
        for r in range(n):
            b0 = (r // block) * block
            seg = A[r, b0:b0 + block]
            compact[r, :seg.size] = seg
        Ab = q.qgtc_pack_bits(dev(compact), 1, q.LEFT, block_rows=block)
    else:
        Ab = pack_adjacency(A)
    Xb = q.qgtc_pack_bits(dev(X.view(np.int32)), s, q.RIGHT)
    m = q.qgtc_build_tile_map(Ab, 16, tile_kbits) if tile_kbits else None
    return q.qgtc_aggregate(Ab, m, Xb, ep or q.Epilogue(mode=q.OUT_I32)), m


def test_config1_tiny_aggregation():
    w = make_workload(1)
    A = w.graph.dense()
    want = qgnn.aggregate(A, w.X)
    for kb in (None, 128, 64, 32):
        got, _ = run_aggregate(A, w.X, w.s, kb)
        assert (as_u32(got) == want).all(), kb
    # 1-bit all-ones features give the node degrees
    ones = np.ones((A.shape[0], 16), dtype=np.uint32)
    got, m = run_aggregate(A, ones, 1, 128)
    assert (as_u32(got) == w.graph.degrees()[:, None]).all()
    assert (m.deg.cpu().numpy() == w.graph.degrees()).all()


@pytest.mark.parametrize("s", [1, 2, 3, 4, 5, 6, 7, 8, 11, 16, 32])
@pytest.mark.parametrize("shape", [(100, 100, 70), (257, 257, 16), (96, 300, 33), (40, 40, 130)])
def test_aggregate_int32_ragged(s, shape):
    n, k, d = shape
    rng = np.random.default_rng([6, s, n, d])
    A = rand_graph(rng, n, k, 0.05)
    X = rng.integers(0, 2 ** s, size=(k, d), dtype=np.uint64).astype(np.uint32)
    want = qgnn.aggregate(A, X)
    for kb in (None, 128, 32):
        got, _ = run_aggregate(A, X, s, kb)
        assert (as_u32(got) == want).all(), kb


@pytest.mark.parametrize("d", [16, 70, 200])
def test_aggregate_does_not_depend_on_xcd_run(d):
    """The way workgroups are dealt to the XCDs is a scheduling choice only."""
    rng = np.random.default_rng([8, d])
    n, s = 2100, 3                       # 132 tile rows: several runs per XCD and a ragged tail
    A = rand_graph(rng, n, n, 0.01)
    X = rng.integers(0, 2 ** s, size=(n, d)).astype(np.uint32)
    want = qgnn.aggregate(A, X)
    for run in (-1, 0, 1, 3, 64, 4096):
        ep = q.Epilogue(mode=q.OUT_I32, tuning=q.Tuning(agg_xcd_run=run))
        got, _ = run_aggregate(A, X, s, 128, ep=ep)
        assert (as_u32(got) == want).all(), run
    with pytest.raises(q.QgtcError) as e:                  # out of range: refused, nothing launched
        run_aggregate(A, X, s, 128, ep=q.Epilogue(mode=q.OUT_I32, tuning=q.Tuning(agg_xcd_run=5000)))
    assert e.value.status == 7


@pytest.mark.parametrize("d", [16, 32, 64, 200])
def test_aggregate_block_diagonal_compact_and_self_term(d):
    rng = np.random.default_rng([7, d])
    n, block, s = 330, 96, 5
    A = np.zeros((n, n), dtype=np.uint8)
    for b0 in range(0, n, block):
        b1 = min(n, b0 + block)
        A[b0:b1, b0:b1] = rand_graph(rng, b1 - b0, b1 - b0, 0.08)
    X = rng.integers(0, 2 ** s, size=(n, d)).astype(np.uint32)
    for self_term in (False, True):
        want = qgnn.aggregate(A, X, self_term)
        ep = q.Epilogue(mode=q.OUT_I32, self_term=self_term)
        for kb in (None, 128, 64):
            got, _ = run_aggregate(A, X, s, kb, block=block, ep=ep)
            assert (as_u32(got) == want).all(), (self_term, kb)
        got, _ = run_aggregate(A, X, s, 128, ep=ep)          # same graph, dense storage
        assert (as_u32(got) == want).all()


@pytest.mark.parametrize("d", [16, 24, 64, 100])
@pytest.mark.parametrize("rq_bits", [1, 3, 8, 12])
def test_aggregate_bits_and_f32_epilogues(d, rq_bits):
    rng = np.random.default_rng([8, d, rq_bits])
    n, s = 150, 4
    A = rand_graph(rng, n, n, 0.1)
    X = rng.integers(0, 2 ** s, size=(n, d)).astype(np.uint32)
    Y = qgnn.aggregate(A, X)
    rq_lo, inv = 3, qgnn.inv_scale(3.0, float(Y.max()), rq_bits)
    ep = q.Epilogue(mode=q.OUT_BITS, rq_nbits=rq_bits, rq_lo=rq_lo, rq_inv_scale=float(inv))
    got, _ = run_aggregate(A, X, s, 128, ep=ep)
    want = qgnn.requantize(Y, rq_lo, inv, rq_bits)
    assert (words_np(got) == bp.pack(want, rq_bits, bp.LEFT)).all()
    assert (as_u32(q.qgtc_unpack_bits(got)) == want).all()
    # a destination with the default LEFT strides (rows padded to 128 bits), poisoned: the
    # zero padding is part of what the epilogue writes, so the result can serve as the left
    # operand of a kernel that reads whole 128-bit rows
    dst = q.alloc_bits(n, d, rq_bits, q.LEFT)
    assert dst.c.ld_words % 4 == 0 and dst.c.ld_words >= -(-d // 32)
    dst.words.fill_(-1)
    Ab = pack_adjacency(A)
    q.qgtc_aggregate(Ab, q.qgtc_build_tile_map(Ab, 16, 128), q.qgtc_pack_bits(dev(X.view(np.int32)), s, q.RIGHT),
                     ep, out=dst)
    raw = dst.words.cpu().numpy().view(np.uint32)[:rq_bits * n * dst.c.ld_words].reshape(rq_bits, n, -1)
    kw = -(-d // 32)
    assert (raw[:, :, :kw] == bp.pack(want, rq_bits, bp.LEFT)).all()
    assert (raw[:, :, kw:] == 0).all()
    # fp32: sx * Y + lo_x * deg
    deg = A.sum(axis=1).astype(np.int32)
    ep = q.Epilogue(mode=q.OUT_F32, cc=0.37, rs=-1.25, row_i=dev(deg))
    got, _ = run_aggregate(A, X, s, 128, ep=ep)
    ref = qgnn.dequantize(Y, cc=0.37, rs=-1.25, row_i=deg)
    assert_fp32_close(got.cpu().numpy(), ref, '')
    # int32 with ReLU on the signed accumulator (wrapped values count as negative)
    Xbig = np.full((n, d), 2 ** 31 - 1, dtype=np.uint32)
    ep = q.Epilogue(mode=q.OUT_I32, relu=True)
    got, _ = run_aggregate(A, Xbig, 32, 128, ep=ep)
    assert (got.cpu().numpy() == qgnn.int_output(qgnn.aggregate(A, Xbig), relu=True)).all()


# ------------------------------------------------------------------------- update
@pytest.mark.parametrize("st", [(1, 1), (2, 3), (4, 4), (8, 8), (8, 2), (3, 7), (16, 16), (32, 32), (12, 5)])
@pytest.mark.parametrize("shape", [(100, 64, 64), (257, 128, 16), (70, 40, 5), (1000, 512, 16), (64, 300, 70)])
def test_update_int32(st, shape):
    s, t = st
    n, d, h = shape
    rng = np.random.default_rng([9, s, t, n])
    Yq = rng.integers(0, 2 ** s, size=(n, d), dtype=np.uint64).astype(np.uint32)
    Wq = rng.integers(0, 2 ** t, size=(d, h), dtype=np.uint64).astype(np.uint32)
    Yb = q.qgtc_pack_bits(dev(Yq.view(np.int32)), s, q.LEFT)
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT)
    got = q.qgtc_update(Yb, Wb, q.Epilogue(mode=q.OUT_I32))
    assert (as_u32(got) == qgnn.update(Yq, Wq)).all()


@pytest.mark.parametrize("rq_bits", [1, 4, 8, 10])
def test_update_bits_and_f32_epilogues(rq_bits):
    rng = np.random.default_rng([10, rq_bits])
    n, d, h, s, t = 300, 64, 24, 4, 3
    Yq = rng.integers(0, 2 ** s, size=(n, d)).astype(np.uint32)
    Wq = rng.integers(0, 2 ** t, size=(d, h)).astype(np.uint32)
    Yb = q.qgtc_pack_bits(dev(Yq.view(np.int32)), s, q.LEFT)
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT)
    Z = qgnn.update(Yq, Wq)
    inv = qgnn.inv_scale(0.0, float(Z.max()), rq_bits)
    ep = q.Epilogue(mode=q.OUT_BITS, relu=True, rq_nbits=rq_bits, rq_lo=0, rq_inv_scale=float(inv))
    got = q.qgtc_update(Yb, Wb, ep)
    want = qgnn.requantize(Z, 0, inv, rq_bits, relu=True)
    assert (words_np(got) == bp.pack(want, rq_bits, bp.RIGHT)).all()
    rs = Yq.sum(axis=1).astype(np.int32)
    cs = Wq.sum(axis=0).astype(np.int32)
    rl = rng.integers(1, 30, size=n).astype(np.int32)
    kw = dict(cc=1.7e-3, rs=-0.031, l0a=0.4, l0b=-0.9, ck=-6.4, cs=0.0125)
    for relu in (False, True):
        ep = q.Epilogue(mode=q.OUT_F32, relu=relu, row_i=dev(rs), row_l=dev(rl), col_i=dev(cs), **kw)
        got = q.qgtc_update(Yb, Wb, ep).cpu().numpy()
        ref = qgnn.dequantize(Z, row_i=rs, row_l=rl, col_i=cs, relu=relu, **kw)
        assert_fp32_close(got, ref, '')


# -------------------------------------------------------------------------- layer
@pytest.mark.parametrize("cfg,bits,nb", [(2, 4, None), (3, 1, 2), (3, 3, 2), (3, 8, 2), (3, 16, 1), (3, 32, 1)])
def test_layer_matches_oracle(cfg, bits, nb):
    w = make_workload(cfg, bits=bits, n_blocks=nb)
    A = w.graph.dense()
    xr = (float(w.X.min()), float(w.X.max()))
    wr = (float(w.W[0].min()), float(w.W[0].max()))
    Xq = qgnn.quantize(w.X, xr[0], xr[1], w.s)
    Wq = qgnn.quantize(w.W[0], wr[0], wr[1], w.t)
    Y, Yq, Z, (rq_lo, rq_inv) = qgnn.layer(A, Xq, Wq, w.s)
    Ab = pack_adjacency(A)
    m = q.qgtc_build_tile_map(Ab)
    Xb = q.qgtc_pack_bits(dev(w.X), w.s, q.RIGHT, quant=xr)
    Wb = q.qgtc_pack_bits(dev(w.W[0]), w.t, q.RIGHT, quant=wr)
    assert (as_u32(q.qgtc_unpack_bits(Xb)) == Xq).all()
    assert (as_u32(q.qgtc_unpack_bits(Wb)) == Wq).all()
    agg_ep = q.Epilogue(mode=q.OUT_BITS, rq_nbits=w.s, rq_lo=rq_lo, rq_inv_scale=float(rq_inv))
    got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, q.Epilogue(mode=q.OUT_I32))
    assert (as_u32(got) == Z).all()
    # the two halves on their own
    y32 = q.qgtc_aggregate(Ab, m, Xb, q.Epilogue(mode=q.OUT_I32))
    assert (as_u32(y32) == Y).all()
    yb = q.qgtc_aggregate(Ab, m, Xb, agg_ep)
    assert (as_u32(q.qgtc_unpack_bits(yb)) == Yq).all()
    # running twice gives the same bytes (no races)
    again = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, q.Epilogue(mode=q.OUT_I32))
    assert torch.equal(got, again)


# ------------------------------------------------- update on the matrix cores
def test_popcount_probe_runs_and_leaves_its_sink_alone():
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    q.qgtc_probe_popcount(64, 4, 10, sink)
    sync()
    assert int(sink.abs().sum()) == 0


@pytest.mark.parametrize("d", [16, 64, 130])
def test_degenerate_graphs(d):
    """Empty tile lists: an adjacency without any edge, one with edges in a single tile
    row only, and isolated nodes with the GIN self term; aggregation and fused layer."""
    rng = np.random.default_rng([13, d])
    n, s, t, h = 200, 4, 3, 24
    Xq = rng.integers(0, 2 ** s, size=(n, d)).astype(np.uint32)
    Wq = rng.integers(0, 2 ** t, size=(d, h)).astype(np.uint32)
    Xb = q.qgtc_pack_bits(dev(Xq.view(np.int32)), s, q.RIGHT)
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT_BYTES)
    one_row = np.zeros((n, n), dtype=np.uint8)
    one_row[37, [3, 150, 199]] = 1
    for A in (np.zeros((n, n), dtype=np.uint8), one_row):
        for self_term in (False, True):
            Ab = pack_adjacency(A)
            for kb in (128, 32):
                m = q.qgtc_build_tile_map(Ab, 16, kb)
                assert int(m.nnz_tiles.cpu()[0]) == (0 if A.sum() == 0 else len({c // kb for c in (3, 150, 199)}))
                want = qgnn.aggregate(A, Xq, self_term)
                got = q.qgtc_aggregate(Ab, m, Xb, q.Epilogue(mode=q.OUT_I32, self_term=self_term))
                assert (as_u32(got) == want).all(), (self_term, kb)
                Yq = qgnn.requantize(want, 0, np.float32(0.5), s)
                agg_ep = q.Epilogue(mode=q.OUT_BITS, rq_nbits=s, rq_lo=0, rq_inv_scale=0.5, self_term=self_term)
                got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, q.Epilogue(mode=q.OUT_I32))
                assert (as_u32(got) == qgnn.update(Yq, Wq)).all(), (self_term, kb)


def test_empty_operands_launch_nothing():
    Ab = q.alloc_bits(0, 64, 1, q.LEFT)
    Xb = q.alloc_bits(64, 16, 2, q.RIGHT)
    out = q.qgtc_aggregate(Ab, None, Xb, q.Epilogue(mode=q.OUT_I32))
    sync()
    assert tuple(out.shape) == (0, 16)
    Yb = q.alloc_bits(0, 64, 2, q.LEFT)
    Wb = q.alloc_bits(64, 8, 2, q.RIGHT)
    out = q.qgtc_update(Yb, Wb, q.Epilogue(mode=q.OUT_I32))
    sync()
    assert tuple(out.shape) == (0, 8)


@pytest.mark.parametrize("st", [(8, 8), (8, 3), (5, 8), (1, 1)])
@pytest.mark.parametrize("shape", [(100, 64, 64), (257, 130, 16), (70, 40, 5), (1000, 512, 16), (33, 7, 70)])
def test_update_from_bytes(st, shape):
    """Left operand as one byte per code (QGTC_LEFT_BYTES): layout as the header states
    it, zero fill, and the update on it against the oracle in all three output modes."""
    n, d, h = shape
    s, t = st
    rng = np.random.default_rng([12, n, d, h, s, t])
    x = rng.standard_normal((n, d)).astype(np.float32)
    lo, hi = float(x.min()), float(x.max()) + 1e-3
    Yq = qgnn.quantize(x, lo, hi, s)
    Wq = rng.integers(0, 2 ** t, size=(d, h)).astype(np.uint32)
    Yb = q.alloc_bits(n, d, s, q.LEFT_BYTES)
    Yb.words.fill_(-1)
    q.qgtc_pack_bits(dev(x), s, q.LEFT_BYTES, quant=(lo, hi), out=Yb)
    ld = Yb.c.ld_words * 4
    assert ld % 16 == 0 and ld >= d
    raw = Yb.words.cpu().numpy().view(np.uint8)[:n * ld].reshape(n, ld)
    assert (raw[:, :d] == Yq).all() and (raw[:, d:] == 0).all()
    assert (as_u32(q.qgtc_unpack_bits(Yb)) == Yq).all()
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT)
    Z = qgnn.update(Yq, Wq)
    assert (as_u32(q.qgtc_update(Yb, Wb, q.Epilogue(mode=q.OUT_I32))) == Z).all()
    inv = qgnn.inv_scale(0.0, float(max(1, Z.max())), 4)
    got = q.qgtc_update(Yb, Wb, q.Epilogue(mode=q.OUT_BITS, relu=True, rq_nbits=4, rq_lo=1, rq_inv_scale=float(inv)))
    assert (words_np(got) == bp.pack(qgnn.requantize(Z, 1, inv, 4, relu=True), 4, bp.RIGHT)).all()
    got = q.qgtc_update(Yb, Wb, q.Epilogue(mode=q.OUT_F32, cc=0.37)).cpu().numpy()
    ref = qgnn.dequantize(Z, cc=0.37)
    assert_fp32_close(got, ref, '')


# ------------------------------------------------------------------- fused layer
def _compact_rows(A, block):
    """Block-diagonal storage: row r keeps the columns of its own diagonal block."""
    n = A.shape[0]
    out = np.zeros((n, block), dtype=np.uint8)
    for r in range(n):
        b0 = (r // block) * block
        seg = A[r, b0:b0 + block]
        out[r, :seg.size] = seg
    return out


def _layer_case(rng, n, d, h, s, t, block, self_term, p_edge=0.06):
    A = np.zeros((n, n), dtype=np.uint8)
    if block:
        for b0 in range(0, n, block):
            b1 = min(n, b0 + block)
            A[b0:b1, b0:b1] = rand_graph(rng, b1 - b0, b1 - b0, p_edge)
    else:
        A = rand_graph(rng, n, n, p_edge)
    if self_term:
        A[np.arange(n), np.arange(n)] = 0
    Xq = rng.integers(0, 2 ** s, size=(n, d)).astype(np.uint32)
    Wq = rng.integers(0, 2 ** t, size=(d, h)).astype(np.uint32)
    return A, Xq, Wq


@pytest.mark.parametrize("shape", [(200, 5, 3), (300, 16, 16), (100, 24, 40), (64, 32, 8),
                                   (40, 33, 5), (100, 64, 64), (330, 70, 16), (257, 128, 100),
                                   (530, 200, 256), (96, 512, 16), (200, 600, 40), (64, 1024, 24)])
@pytest.mark.parametrize("st", [(8, 8), (8, 3), (4, 8), (7, 7), (1, 1), (2, 5)])
def test_fused_layer_all_outputs(shape, st):
    """qgtc_layer as one kernel: int32, packed low-bit and fp32 outputs against the
    oracle, and against the same call run as two kernels, for every way of
    splitting the tile lists between waves."""
    n, d, h = shape
    s, t = st
    rng = np.random.default_rng([11, n, d, h, s, t])
    block = 96 if n % 2 == 0 else 0
    self_term = (n + s) % 2 == 0
    A, Xq, Wq = _layer_case(rng, n, d, h, s, t, block, self_term)
    Y = qgnn.aggregate(A, Xq, self_term)
    rq_inv = qgnn.inv_scale(0.0, float(max(1, qgnn.as_signed(Y).max())), s)
    Yq = qgnn.requantize(Y, 0, rq_inv, s)
    Z = qgnn.update(Yq, Wq)

    Xb = q.qgtc_pack_bits(dev(Xq.view(np.int32)), s, q.RIGHT)
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT)
    Wbytes = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT_BYTES)
    assert (as_u32(q.qgtc_unpack_bits(Wbytes)) == Wq).all()
    assert (as_u32(q.qgtc_col_sums(Wbytes)) == Wq.sum(axis=0, dtype=np.uint64).astype(np.uint32)).all()
    agg_ep = q.Epilogue(mode=q.OUT_BITS, rq_nbits=s, rq_lo=0, rq_inv_scale=float(rq_inv),
                        self_term=self_term)
    out_bits = min(s, 6)
    z_inv = qgnn.inv_scale(0.0, float(max(1, qgnn.as_signed(Z).max())), out_bits)
    want_bits = bp.pack(qgnn.requantize(Z, 3, z_inv, out_bits, relu=True), out_bits, bp.RIGHT)
    rl = rng.integers(1, 30, size=n).astype(np.int32)
    cs = Wq.sum(axis=0).astype(np.int32)
    kw = dict(cc=1.7e-3, rs=-0.031, l0a=0.4, l0b=-0.9, ck=-6.4, cs=0.0125)
    want_f32 = qgnn.dequantize(Z, row_i=Yq.sum(axis=1, dtype=np.int64), row_l=rl, col_i=cs, **kw)

    storages = [(pack_adjacency(A), 128), (pack_adjacency(A), None)]
    if block:
        compact = np.zeros((n, block), dtype=np.uint8)
        for r in range(n):
            b0 = (r // block) * block
            seg = A[r, b0:b0 + block]
            compact[r, :seg.size] = seg
        storages.append((q.qgtc_pack_bits(dev(compact), 1, q.LEFT, block_rows=block), 32))
    for Ab, kb in storages:
        m = q.qgtc_build_tile_map(Ab, 16, kb) if kb else None
        for path, ksplit in ((q.LAYER_FUSED, 0), (q.LAYER_FUSED, 1), (q.LAYER_FUSED, 2),
                             (q.LAYER_FUSED, 4), (q.LAYER_TWO_KERNELS, 0)):
            tn = q.Tuning(layer_path=path, layer_ksplit=ksplit)
            tag = (kb, path, ksplit)
            q.qgtc_prof_enable(True)
            q.qgtc_prof_reset()
            got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, q.Epilogue(mode=q.OUT_I32, tuning=tn))
            fused_launches = q.qgtc_prof_read(q.KERNEL_LAYER)[1]
            q.qgtc_prof_enable(False)
            q.qgtc_prof_reset()
            assert fused_launches == (1 if path == q.LAYER_FUSED else 0), tag
            assert (as_u32(got) == Z).all(), tag
            # weights cached as bytes in operand order: always the fused kernel
            got = q.qgtc_layer(Ab, m, Xb, Wbytes, agg_ep, q.Epilogue(mode=q.OUT_I32, tuning=tn))
            assert (as_u32(got) == Z).all(), tag
            ep = q.Epilogue(mode=q.OUT_BITS, relu=True, rq_nbits=out_bits, rq_lo=3,
                            rq_inv_scale=float(z_inv), tuning=tn)
            # poison the destination: every word, padding included, must be written
            dst = q.alloc_bits(n, h, out_bits, q.RIGHT)
            dst.words.fill_(-1)
            got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, ep, out=dst)
            assert (words_np(got) == want_bits).all(), tag
            ep = q.Epilogue(mode=q.OUT_F32, row_i=None, row_l=dev(rl), col_i=dev(cs), tuning=tn, **kw)
            got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, ep).cpu().numpy()
            assert_fp32_close(got, want_f32, str(tag))


# ------------------------------------------------- folded batch normalization
@pytest.mark.parametrize("shape", [(200, 24, 40), (330, 70, 16), (257, 128, 100), (96, 512, 16), (64, 64, 64)])
@pytest.mark.parametrize("st", [(8, 8), (4, 4), (3, 5), (11, 11)])
def test_column_affine_epilogue(shape, st):
    """A per-column affine map in front of the activation (a batch normalization folded
    into the kernel): low-bit and fp32 outputs of qgtc_aggregate, of both update kernels
    and of qgtc_layer as one and as two kernels, against the oracle."""
    n, d, h = shape
    s, t = st
    rng = np.random.default_rng([29, n, d, h, s, t])
    block = 96 if n % 2 == 0 else 0
    A, Xq, Wq = _layer_case(rng, n, d, h, s, t, block, False)
    Y = qgnn.aggregate(A, Xq)
    rq_bits = min(s, 8)
    y_inv = qgnn.inv_scale(0.0, float(max(1, qgnn.as_signed(Y).max())), rq_bits)
    Yq = qgnn.requantize(Y, 0, y_inv, rq_bits)
    Z = qgnn.update(Yq, Wq)
    out_bits = min(s, 8)

    def bn_params(C, cols, value_scale):
        x = value_scale * qgnn.as_signed(C).astype(np.float64)
        gamma = rng.uniform(0.5, 2.0, size=cols)
        beta = rng.uniform(-1.0, 1.0, size=cols)
        return qgnn.fold_batchnorm(gamma, beta, x.mean(axis=0), x.var(axis=0) + 1e-3, 1e-5, value_scale), \
            qgnn.fold_batchnorm(gamma, beta, x.mean(axis=0), x.var(axis=0) + 1e-3, 1e-5, 1.0)

    Ab = pack_adjacency(A)
    m = q.qgtc_build_tile_map(Ab, 16, 128)
    Xb = q.qgtc_pack_bits(dev(Xq.view(np.int32)), s, q.RIGHT)

    # aggregation: codes along the columns (LEFT) and fp32
    (a, b), (a1, b1) = bn_params(Y, d, 2.0e-3)
    v = qgnn.as_signed(Y) * a[None, :].astype(np.float64) + b[None, :]
    inv = qgnn.inv_scale(0.0, float(max(1e-3, v.max())), out_bits)
    want = qgnn.requantize_affine(Y, a, b, 0, inv, out_bits, relu=True)
    ep = q.Epilogue(mode=q.OUT_BITS, relu=True, rq_nbits=out_bits, rq_lo=0, rq_inv_scale=float(inv),
                    col_scale=dev(a), col_shift=dev(b))
    got = q.qgtc_aggregate(Ab, m, Xb, ep)
    assert (words_np(got) == bp.pack(want, out_bits, bp.LEFT)).all()
    ep = q.Epilogue(mode=q.OUT_F32, cc=2.0e-3, relu=True, col_scale=dev(a1), col_shift=dev(b1))
    got = q.qgtc_aggregate(Ab, m, Xb, ep).cpu().numpy()
    ref = qgnn.dequantize(Y, cc=2.0e-3, relu=True, col_a=a1, col_b=b1)
    assert_fp32_close(got, ref, '')

    # update and layer: codes along the rows (RIGHT) and fp32; the shift may be absent
    (a, b), (a1, b1) = bn_params(Z, h, 1.0e-4)
    v = qgnn.as_signed(Z) * a[None, :].astype(np.float64) + b[None, :]
    inv = qgnn.inv_scale(0.0, float(max(1e-3, v.max())), out_bits)
    want_bits = bp.pack(qgnn.requantize_affine(Z, a, b, 0, inv, out_bits, relu=True), out_bits, bp.RIGHT)
    want_noshift = bp.pack(qgnn.requantize_affine(Z, a, None, 0, inv, out_bits, relu=False), out_bits, bp.RIGHT)
    rs = Yq.sum(axis=1, dtype=np.int64)
    kw = dict(cc=1.0e-4, rs=-2.0e-3)
    want_f32 = qgnn.dequantize(Z, row_i=rs, relu=True, col_a=a1, col_b=b1, **kw)
    ep_bits = q.Epilogue(mode=q.OUT_BITS, relu=True, rq_nbits=out_bits, rq_lo=0, rq_inv_scale=float(inv),
                         col_scale=dev(a), col_shift=dev(b))
    ep_noshift = q.Epilogue(mode=q.OUT_BITS, rq_nbits=out_bits, rq_lo=0, rq_inv_scale=float(inv),
                            col_scale=dev(a))
    Yb = q.qgtc_pack_bits(dev(Yq.view(np.int32)), rq_bits, q.LEFT)
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT)
    for path in (q.UPDATE_POPCOUNT, q.UPDATE_MATRIX_CORES):
        ep_bits.tuning = ep_noshift.tuning = q.Tuning(update_path=path)
        assert (words_np(q.qgtc_update(Yb, Wb, ep_bits)) == want_bits).all(), path
        assert (words_np(q.qgtc_update(Yb, Wb, ep_noshift)) == want_noshift).all(), path
        ep = q.Epilogue(mode=q.OUT_F32, row_i=dev(rs.astype(np.int32)), relu=True,
                        col_scale=dev(a1), col_shift=dev(b1), tuning=q.Tuning(update_path=path), **kw)
        got = q.qgtc_update(Yb, Wb, ep).cpu().numpy()
        assert_fp32_close(got, want_f32, str(path))
    agg_ep = q.Epilogue(mode=q.OUT_BITS, rq_nbits=rq_bits, rq_lo=0, rq_inv_scale=float(y_inv))
    for path in (q.LAYER_FUSED, q.LAYER_TWO_KERNELS):
        ep_bits.tuning = ep_noshift.tuning = q.Tuning(layer_path=path)
        dst = q.alloc_bits(n, h, out_bits, q.RIGHT)
        dst.words.fill_(-1)
        assert (words_np(q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, ep_bits, out=dst)) == want_bits).all(), path
        assert (words_np(q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, ep_noshift)) == want_noshift).all(), path
        ep = q.Epilogue(mode=q.OUT_F32, row_i=None, relu=True, col_scale=dev(a1), col_shift=dev(b1),
                        tuning=q.Tuning(layer_path=path), **kw)
        got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, ep).cpu().numpy()
        assert_fp32_close(got, want_f32, str(path))


@pytest.mark.parametrize("st", [(1, 1), (2, 3), (4, 4), (7, 7), (8, 8), (8, 2), (3, 8), (8, 7)])
@pytest.mark.parametrize("shape", [(100, 64, 64), (257, 128, 16), (70, 40, 5), (1000, 512, 16), (64, 300, 70),
                                   (4096, 64, 64), (33, 16, 130)])
def test_update_matrix_core_path_equals_popcount_and_oracle(st, shape):
    s, t = st
    n, d, h = shape
    rng = np.random.default_rng([11, s, t, n])
    Yq = rng.integers(0, 2 ** s, size=(n, d), dtype=np.uint64).astype(np.uint32)
    Wq = rng.integers(0, 2 ** t, size=(d, h), dtype=np.uint64).astype(np.uint32)
    Yq[0, :] = 2 ** s - 1                      # extreme codes (top bit set at 8 bits)
    Wq[:, 0] = 2 ** t - 1
    Yb = q.qgtc_pack_bits(dev(Yq.view(np.int32)), s, q.LEFT)
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT)
    Z = qgnn.update(Yq, Wq)
    inv = qgnn.inv_scale(0.0, float(Z.max()), 5)
    rs = Yq.sum(axis=1).astype(np.int32)
    cs = Wq.sum(axis=0).astype(np.int32)
    kw = dict(cc=1.7e-3, rs=-0.031, l0a=0.4, l0b=-0.9, ck=-6.4, cs=0.0125)
    outs = {}
    for path in (q.UPDATE_POPCOUNT, q.UPDATE_MATRIX_CORES):
        tn = q.Tuning(update_path=path)
        z = q.qgtc_update(Yb, Wb, q.Epilogue(mode=q.OUT_I32, tuning=tn))
        bits = q.qgtc_update(Yb, Wb, q.Epilogue(mode=q.OUT_BITS, relu=True, rq_nbits=5, rq_lo=0,
                                                rq_inv_scale=float(inv), tuning=tn))
        f = q.qgtc_update(Yb, Wb, q.Epilogue(mode=q.OUT_F32, row_i=dev(rs), row_l=dev(rs),
                                             col_i=dev(cs), tuning=tn, **kw))
        outs[path] = (as_u32(z), words_np(bits), f.cpu().numpy())
    for path, (z, bits, f) in outs.items():
        assert (z == Z).all(), path
        assert (bits == bp.pack(qgnn.requantize(Z, 0, inv, 5, relu=True), 5, bp.RIGHT)).all(), path
        ref = qgnn.dequantize(Z, row_i=rs, row_l=rs, col_i=cs, **kw)
        assert_fp32_close(f, ref, str(path))


# ------------------------------------------------------------ zero-word jumping
@pytest.mark.parametrize("s", [3, 4, 8, 11])
@pytest.mark.parametrize("shape,p_edge", [((300, 64), 0.01), ((300, 64), 0.6), ((130, 20), 0.03), ((257, 130), 0.002),
                                          ((64, 16), 1.0), ((515, 300), 0.0)])
def test_zero_word_jumping_gives_the_same_integers(s, shape, p_edge):
    """The aggregation with every word of a kept tile visited and with the zero words
    jumped over (qgtc_tuning.zero_words), with and without a map, at the three tile widths,
    stand-alone and inside the fused layer: the same integers as the oracle."""
    n, d = shape
    rng = np.random.default_rng([83, s, n, d, int(p_edge * 1000)])
    A = rand_graph(rng, n, n, p_edge)
    if n > 100:
        A[33:70, :] = 0                                     # rows of tiles without a bit
        A[:, 64:160] = 0                                    # whole word columns without a bit
    Xq = rng.integers(0, 2 ** s, size=(n, d), dtype=np.uint64).astype(np.uint32)
    Y = qgnn.aggregate(A, Xq, True)
    Ab = pack_adjacency(A)
    Xb = q.qgtc_pack_bits(dev(Xq.view(np.int32)), s, q.RIGHT)
    h, t = 24, 5
    Wq = rng.integers(0, 2 ** t, size=(d, h)).astype(np.uint32)
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT)
    rq_bits = min(s, 8)
    inv = qgnn.inv_scale(0.0, float(max(1, qgnn.as_signed(Y).max())), rq_bits)
    Z = qgnn.update(qgnn.requantize(Y, 0, inv, rq_bits), Wq)
    for kb in (None, 32, 64, 128):
        m = q.qgtc_build_tile_map(Ab, 16, kb) if kb else None
        for zw in (q.ZERO_WORDS_AUTO, q.ZERO_WORDS_VISIT, q.ZERO_WORDS_SKIP):
            tn = q.Tuning(zero_words=zw)
            got = q.qgtc_aggregate(Ab, m, Xb, q.Epilogue(mode=q.OUT_I32, self_term=True, tuning=tn))
            assert (as_u32(got) == Y).all(), (kb, zw)
            agg_ep = q.Epilogue(mode=q.OUT_BITS, rq_nbits=rq_bits, rq_inv_scale=float(inv), self_term=True)
            got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, q.Epilogue(mode=q.OUT_I32, tuning=tn))
            assert (as_u32(got) == Z).all(), (kb, zw)
            # the issue priority inside the tile loop (qgtc_tuning.even_progress) is scheduling only
            for evp in (1, 2):
                tn2 = q.Tuning(zero_words=zw, even_progress=evp)
                got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, q.Epilogue(mode=q.OUT_I32, tuning=tn2))
                assert (as_u32(got) == Z).all(), (kb, zw, evp)


@pytest.mark.parametrize("s", [5, 6, 8])
@pytest.mark.parametrize("k_words", [2047, 2048, 2049])
def test_jumping_with_counts_at_the_16_bit_limit(s, k_words):
    """From five planes on the jumping form keeps two rows of a tile in one register, 16 bits
    each, while a row of A has at most 2047 words (a count is at most 65504); one word more
    and a count could be 65536, which takes the form with full-width accumulators.  Rows of
    ones against columns of ones reach the largest count on both sides of that limit, in a
    lower and an upper row of a tile, next to sparse rows."""
    k = 32 * k_words
    n, d, h, t = 40, 20, 24, 4
    rng = np.random.default_rng([97, s, k_words])
    A = (rng.random((n, k)) < 0.002).astype(np.uint8)
    A[3, :] = 1                                             # lower half of a tile (rows 0 - 7)
    A[12, :] = 1                                            # upper half (rows 8 - 15): the shifted counts
    A[27, :] = 1
    A[21, : k // 2] = 1
    A[16:20, :] = 0
    Xq = rng.integers(0, 2 ** s, size=(k, d), dtype=np.uint64).astype(np.uint32)
    Xq[:, 0] = 2 ** s - 1                                   # every plane: a count of k
    Xq[:, 7] = 2 ** (s - 1)
    Y = qgnn.aggregate(A, Xq, False)
    assert Y[12, 0] == k * (2 ** s - 1)
    Wq = rng.integers(0, 2 ** t, size=(d, h)).astype(np.uint32)
    inv = qgnn.inv_scale(0.0, float(Y.max()), s)
    Z = qgnn.update(qgnn.requantize(Y, 0, inv, s), Wq)
    Ab = pack_adjacency(A)
    Xb = q.qgtc_pack_bits(dev(Xq.view(np.int32)), s, q.RIGHT)
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT)
    for kb in (32, 64, 128):
        m = q.qgtc_build_tile_map(Ab, 16, kb)
        for zw in (q.ZERO_WORDS_SKIP, q.ZERO_WORDS_VISIT):
            tn = q.Tuning(zero_words=zw)
            got = q.qgtc_aggregate(Ab, m, Xb, q.Epilogue(mode=q.OUT_I32, tuning=tn))
            assert (as_u32(got) == Y).all(), (kb, zw)
            agg_ep = q.Epilogue(mode=q.OUT_BITS, rq_nbits=s, rq_inv_scale=float(inv))
            got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, q.Epilogue(mode=q.OUT_I32, tuning=tn))
            assert (as_u32(got) == Z).all(), (kb, zw)


# ------------------------------------------------------------ seeded random shapes
@pytest.mark.parametrize("seed", range(48))
def test_layer_on_random_shapes(seed):
    """qgtc_layer on shapes and bit widths drawn from a seeded generator (single rows and
    columns, ragged tails, widths above 8 bits that leave the fused kernel, every storage
    and tile width), int32 and low-bit outputs against the oracle."""
    rng = np.random.default_rng([61, seed])
    n = int(rng.choice([1, 2, 15, 16, 17, 31, 33, 64, 100, 129, 255, 400]))
    d = int(rng.choice([1, 2, 7, 16, 17, 32, 33, 63, 64, 65, 130, 260]))
    h = int(rng.choice([1, 3, 15, 16, 17, 40, 64, 100, 256, 260]))
    s = int(rng.choice([1, 2, 3, 5, 8, 8, 8, 9, 12]))
    t = int(rng.choice([1, 2, 4, 7, 8, 8, 10]))
    block = int(rng.choice([0, 0, 32, 64, 96]))
    kb = [None, 32, 64, 128][int(rng.integers(0, 4))]
    self_term = bool(rng.integers(0, 2))
    A, Xq, Wq = _layer_case(rng, n, d, h, s, t, block, self_term, p_edge=float(rng.choice([0.0, 0.02, 0.3])))
    Y = qgnn.aggregate(A, Xq, self_term)
    rq_bits = min(s, int(rng.choice([s, 8, 4])))
    rq_inv = qgnn.inv_scale(0.0, float(max(1, qgnn.as_signed(Y).max())), rq_bits)
    Yq = qgnn.requantize(Y, 0, rq_inv, rq_bits)
    Z = qgnn.update(Yq, Wq)
    out_bits = int(rng.choice([1, 3, 8, min(s, 8)]))
    z_inv = qgnn.inv_scale(0.0, float(max(1, qgnn.as_signed(Z).max())), out_bits)
    want_bits = bp.pack(qgnn.requantize(Z, 1, z_inv, out_bits, relu=True), out_bits, bp.RIGHT)

    if block:
        Ab = q.qgtc_pack_bits(dev(_compact_rows(A, block)), 1, q.LEFT, block_rows=block)
    else:
        Ab = pack_adjacency(A)
    m = q.qgtc_build_tile_map(Ab, 16, kb) if kb else None
    Xb = q.qgtc_pack_bits(dev(Xq.view(np.int32)), s, q.RIGHT)
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT)
    agg_ep = q.Epilogue(mode=q.OUT_BITS, rq_nbits=rq_bits, rq_lo=0, rq_inv_scale=float(rq_inv),
                        self_term=self_term)
    tag = dict(n=n, d=d, h=h, s=s, t=t, block=block, kb=kb, self_term=self_term, rq_bits=rq_bits, out_bits=out_bits)
    got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, q.Epilogue(mode=q.OUT_I32))
    assert (as_u32(got) == Z).all(), tag
    ep = q.Epilogue(mode=q.OUT_BITS, relu=True, rq_nbits=out_bits, rq_lo=1, rq_inv_scale=float(z_inv))
    dst = q.alloc_bits(n, h, out_bits, q.RIGHT)
    dst.words.fill_(-1)
    got = q.qgtc_layer(Ab, m, Xb, Wb, agg_ep, ep, out=dst)
    assert (words_np(got) == want_bits).all(), tag
    if s <= 8 and t <= 8 and d <= 1024 and h <= 256:            # weights as bytes: the fused kernel only
        Wby = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT_BYTES)
        got = q.qgtc_layer(Ab, m, Xb, Wby, agg_ep, q.Epilogue(mode=q.OUT_I32))
        assert (as_u32(got) == Z).all(), tag


@pytest.mark.parametrize("seed", range(40))
def test_aggregate_and_update_on_random_shapes(seed):
    """qgtc_aggregate and qgtc_update by themselves on seeded random shapes and bit widths
    up to 32 (results modulo 2^32), every output mode, against the oracle."""
    rng = np.random.default_rng([67, seed])
    n = int(rng.choice([1, 5, 16, 31, 48, 65, 128, 200, 333]))
    k = n
    d = int(rng.choice([1, 3, 16, 20, 32, 50, 64, 70, 129, 300]))
    h = int(rng.choice([1, 2, 15, 16, 33, 64, 90]))
    s = int(rng.choice([1, 2, 4, 7, 8, 9, 13, 16, 24, 32]))
    t = int(rng.choice([1, 3, 8, 8, 11, 16, 32]))
    self_term = bool(rng.integers(0, 2))
    kb = [None, 32, 64, 128][int(rng.integers(0, 4))]
    A = rand_graph(rng, n, k, float(rng.choice([0.0, 0.05, 0.5])))
    Xq = rng.integers(0, 2 ** s, size=(k, d), dtype=np.uint64).astype(np.uint32)
    tag = dict(n=n, d=d, h=h, s=s, t=t, self_term=self_term, kb=kb)
    Y = qgnn.aggregate(A, Xq, self_term)
    Ab = pack_adjacency(A)
    m = q.qgtc_build_tile_map(Ab, 16, kb) if kb else None
    Xb = q.qgtc_pack_bits(dev(Xq.view(np.int32)), s, q.RIGHT)
    got = q.qgtc_aggregate(Ab, m, Xb, q.Epilogue(mode=q.OUT_I32, self_term=self_term))
    assert (as_u32(got) == Y).all(), tag
    rq_bits = int(rng.choice([1, 4, 8, 12]))
    hi = float(max(1, qgnn.as_signed(Y).max()))
    inv = qgnn.inv_scale(0.0, hi, rq_bits)
    Yq = qgnn.requantize(Y, 0, inv, rq_bits, relu=True)
    ep = q.Epilogue(mode=q.OUT_BITS, relu=True, rq_nbits=rq_bits, rq_lo=0, rq_inv_scale=float(inv),
                    self_term=self_term)
    Yb = q.qgtc_aggregate(Ab, m, Xb, ep)
    assert (words_np(Yb) == bp.pack(Yq, rq_bits, bp.LEFT)).all(), tag
    got = q.qgtc_aggregate(Ab, m, Xb, q.Epilogue(mode=q.OUT_F32, cc=0.013, self_term=self_term)).cpu().numpy()
    ref = qgnn.dequantize(Y, cc=0.013)
    assert_fp32_close(got, ref, str(tag))

    Wq = rng.integers(0, 2 ** t, size=(d, h), dtype=np.uint64).astype(np.uint32)
    Z = qgnn.update(Yq, Wq)
    Wb = q.qgtc_pack_bits(dev(Wq.view(np.int32)), t, q.RIGHT)
    got = q.qgtc_update(Yb, Wb, q.Epilogue(mode=q.OUT_I32, relu=True))
    assert (as_u32(got) == qgnn.int_output(Z, relu=True).view(np.uint32)).all(), tag
    out_bits = int(rng.choice([1, 5, 8, 16]))
    z_inv = qgnn.inv_scale(0.0, float(max(1, qgnn.as_signed(Z).max())), out_bits)
    got = q.qgtc_update(Yb, Wb, q.Epilogue(mode=q.OUT_BITS, rq_nbits=out_bits, rq_lo=0, rq_inv_scale=float(z_inv)))
    assert (words_np(got) == bp.pack(qgnn.requantize(Z, 0, z_inv, out_bits), out_bits, bp.RIGHT)).all(), tag
