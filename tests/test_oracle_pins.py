"""Pins for the CPU oracle: what the paper prints, closed forms, invariants,
brute force on tiny inputs.  None of these calls the HIP path."""
import itertools

import numpy as np
import pytest

from oracle import qgnn, bitplane as bp
from conftest import load_golden


# ---------------------------------------------------------------- brute force
def py_matmul(L, R):
    """Textbook triple loop on Python integers (no wrap)."""
    n, k, m = len(L), len(R), len(R[0])
    return [[sum(int(L[i][x]) * int(R[x][j]) for x in range(k))
             for j in range(m)] for i in range(n)]


def py_bit_matmul(L, R, lb, rb):
    """sum_i sum_j 2^(i+j) popcnt(plane_i(L row) & plane_j(R col)), Python ints."""
    n, k, m = len(L), len(R), len(R[0])
    out = [[0] * m for _ in range(n)]
    for r in range(n):
        for c in range(m):
            acc = 0
            for i in range(lb):
                lw = sum(((int(L[r][x]) >> i) & 1) << x for x in range(k))
                for j in range(rb):
                    rw = sum(((int(R[x][c]) >> j) & 1) << x for x in range(k))
                    acc += bin(lw & rw).count("1") << (i + j)
            out[r][c] = acc
    return out


# ------------------------------------------------------- the paper's examples
def test_paper_popcnt_example():
    g = load_golden("paper_examples.txt")
    assert bp.popcnt(g["popcnt_arg"][0]) == g["popcnt_val"][0]
    assert g["popcnt_arg"][0] == 0b1011


def test_paper_eq5_expansion_exhaustive():
    """Eq. (5): the printed 3-bit x 2-bit expansion equals a*b for all 32 pairs,
    and so do the oracle's product and the literal bit-plane product."""
    terms = load_golden("paper_examples.txt")["eq5_terms"]
    for a, b in itertools.product(range(8), range(4)):
        printed = sum(((a >> ai) & 1) * ((b >> bi) & 1) << sh
                      for ai, bi, sh in terms)
        assert printed == a * b
        L = np.array([[a]], dtype=np.uint32)
        R = np.array([[b]], dtype=np.uint32)
        assert int(qgnn.matmul_mod32(L, R)[0, 0]) == a * b
        assert int(bp.any_bit_matmul(L, R, 3, 2)[0, 0]) == a * b


def test_eq6_vector_form():
    """Eq. (6)/(7): 3-bit . 2-bit vectors of length k via shifted popcounts."""
    rng = np.random.default_rng(1)
    for k in (1, 5, 33, 70):
        vi = rng.integers(0, 8, size=(1, k))
        vj = rng.integers(0, 4, size=(k, 1))
        want = int((vi.astype(np.int64) @ vj.astype(np.int64))[0, 0])
        assert py_bit_matmul(vi.tolist(), vj.tolist(), 3, 2)[0][0] == want
        assert int(bp.any_bit_matmul(vi, vj, 3, 2)[0, 0]) == want
        assert int(qgnn.matmul_mod32(vi, vj)[0, 0]) == want


# -------------------------------------------------------- hand-computed layer
def test_hand_computed_layer():
    g = load_golden("layer_4x4.txt")
    A = np.array(g["A"], dtype=np.uint8)
    X = np.array(g["X"], dtype=np.uint32)
    W = np.array(g["W"], dtype=np.uint32)
    Y = qgnn.aggregate(A, X)
    assert Y.tolist() == g["Y"]
    assert qgnn.aggregate(A, X, self_term=True).tolist() == g["Y_gin"]
    assert qgnn.update(Y, W).tolist() == g["Z"]
    assert qgnn.degrees(A).tolist() == g["deg"]
    # sparse adjacency input gives the same
    import scipy.sparse as sp
    assert qgnn.aggregate(sp.csr_matrix(A), X).tolist() == g["Y"]
    # Algorithm 1 taken literally
    xn, z = bp.algorithm1_layer(A, X, W, g["s"][0], g["t"][0])
    assert xn.tolist() == g["Y"] and z.tolist() == g["Z"]
    # requantize
    inv = qgnn.inv_scale(g["rq_lo"][0], g["rq_hi"][0], g["rq_bits"][0])
    assert float(inv) == 0.25
    assert qgnn.requantize(Y, g["rq_lo"][0], inv, g["rq_bits"][0]).tolist() == g["Yq2"]
    # dequantize the aggregation
    sx = qgnn.scale(g["lo_x"][0], g["hi_x"][0], g["s"][0])
    yh = qgnn.dequantize(Y, cc=sx, rs=g["lo_x"][0], row_i=g["deg"])
    assert yh.tolist() == g["Yhat"]


# ------------------------------------------------ brute force on tiny inputs
@pytest.mark.parametrize("s,t", [(s, t) for s in range(1, 9) for t in range(1, 9)])
def test_layer_vs_brute_force_small_bits(s, t):
    rng = np.random.default_rng([7, s, t])
    n, d, h = 9, 7, 5
    A = (rng.random((n, n)) < 0.35).astype(np.uint8)
    X = rng.integers(0, 2 ** s, size=(n, d)).astype(np.uint32)
    W = rng.integers(0, 2 ** t, size=(d, h)).astype(np.uint32)
    Yb = py_matmul(A.tolist(), X.tolist())
    assert py_bit_matmul(A.tolist(), X.tolist(), 1, s) == Yb
    Y = qgnn.aggregate(A, X)
    assert Y.tolist() == Yb
    # exact chain (identity requant): (A.Xq).Wq
    Zb = py_matmul(Yb, W.tolist())
    assert qgnn.update(Y, W).tolist() == Zb
    _, z1 = bp.algorithm1_layer(A, X, W, s, t)
    assert z1.tolist() == Zb
    # requantized chain, s-bit Yq
    Yr, Yq, Z, rq = qgnn.layer(A, X, W, s)
    assert Yr.tolist() == Yb and int(Yq.max()) < 2 ** s
    assert Z.tolist() == py_bit_matmul(Yq.tolist(), W.tolist(), s, t)


@pytest.mark.parametrize("bits", [16, 32])
def test_wrap_mod_2_32_vs_bigints(bits):
    rng = np.random.default_rng([9, bits])
    n, d, h = 6, 40, 4
    A = (rng.random((n, n)) < 0.6).astype(np.uint8)
    X = rng.integers(0, 2 ** bits, size=(n, d), dtype=np.uint64).astype(np.uint32)
    W = rng.integers(0, 2 ** bits, size=(d, h), dtype=np.uint64).astype(np.uint32)
    # force extreme values too
    X[0, :] = 2 ** bits - 1
    W[:, 0] = 2 ** bits - 1
    Yb = py_matmul(A.tolist(), X.tolist())
    Y = qgnn.aggregate(A, X)
    assert Y.tolist() == [[v % 2 ** 32 for v in r] for r in Yb]
    Z = qgnn.update(X, W)
    Zb = py_matmul(X.tolist(), W.tolist())
    assert max(max(r) for r in Zb) >= 2 ** 32 or bits == 16
    assert Z.tolist() == [[v % 2 ** 32 for v in r] for r in Zb]
    # shifted popcounts, truncated to 32 bits, agree (terms with i+j >= 32 vanish)
    Zp = py_bit_matmul(X.tolist(), W.tolist(), bits, bits)
    assert [[v % 2 ** 32 for v in r] for r in Zp] == Z.tolist()


def test_matmul_float64_and_uint64_paths_agree():
    rng = np.random.default_rng(3)
    L = rng.integers(0, 2 ** 32, size=(5, 33), dtype=np.uint64).astype(np.uint32)
    R = rng.integers(0, 2 ** 32, size=(33, 4), dtype=np.uint64).astype(np.uint32)
    want = [[v % 2 ** 32 for v in r] for r in py_matmul(L.tolist(), R.tolist())]
    assert qgnn.matmul_mod32(L, R).tolist() == want            # uint64 path
    Ls, Rs = L >> 20, R >> 20                                   # float64 path
    want = [[v % 2 ** 32 for v in r] for r in py_matmul(Ls.tolist(), Rs.tolist())]
    assert qgnn.matmul_mod32(Ls, Rs).tolist() == want


# ------------------------------------------------------ aggregation invariants
def _rand_graph(rng, n, p, sym=True):
    u = rng.random((n, n)) < p
    if sym:
        u = np.triu(u, 1)
        u = u | u.T
    return u.astype(np.uint8)


def test_one_bit_all_ones_gives_degrees():
    rng = np.random.default_rng(4)
    A = _rand_graph(rng, 50, 0.2)
    X = np.ones((50, 3), dtype=np.uint32)
    Y = qgnn.aggregate(A, X)
    assert (Y == A.sum(axis=1, dtype=np.int64)[:, None]).all()
    assert (qgnn.degrees(A) == Y[:, 0]).all()


def test_identity_and_all_ones_adjacency():
    rng = np.random.default_rng(5)
    X = rng.integers(0, 16, size=(20, 6)).astype(np.uint32)
    assert (qgnn.aggregate(np.eye(20, dtype=np.uint8), X) == X).all()
    Y = qgnn.aggregate(np.ones((20, 20), dtype=np.uint8), X)
    assert (Y == X.sum(axis=0, dtype=np.int64)[None, :]).all()


def test_symmetric_sum_identity_and_permutation_equivariance():
    rng = np.random.default_rng(6)
    n = 40
    A = _rand_graph(rng, n, 0.15)
    X = rng.integers(0, 256, size=(n, 5)).astype(np.uint32)
    Y = qgnn.aggregate(A, X).astype(np.int64)
    deg = A.sum(axis=1, dtype=np.int64)
    assert (Y.sum(axis=0) == (deg[:, None] * X).sum(axis=0)).all()
    p = rng.permutation(n)
    Yp = qgnn.aggregate(A[np.ix_(p, p)], X[p])
    assert (Yp == Y[p]).all()


def test_transposed_operand_would_fail():
    """A directed (asymmetric) example: row v sums in-row neighbours only."""
    A = np.array([[0, 1, 1], [0, 0, 0], [1, 0, 0]], dtype=np.uint8)
    X = np.array([[1], [10], [100]], dtype=np.uint32)
    assert qgnn.aggregate(A, X).ravel().tolist() == [110, 0, 1]


def test_extra_zero_planes_change_nothing():
    rng = np.random.default_rng(8)
    A = _rand_graph(rng, 12, 0.3)
    X = rng.integers(0, 8, size=(12, 4)).astype(np.uint32)
    a = bp.any_bit_matmul(A, X, 1, 3)
    b = bp.any_bit_matmul(A, X, 1, 7)
    assert (a == b).all()


# ------------------------------------------------------------- quantization
def test_quantize_hand_grid():
    g = load_golden("quantize_2bit.txt")
    q = qgnn.quantize(np.array(g["x"], dtype=np.float32), g["lo"][0], g["hi"][0],
                      g["bits"][0])
    assert q.tolist() == g["q"]


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 5, 8, 12, 16, 24])
def test_quantize_closed_form_on_grid(bits):
    """x = lo + (k + 1/2) * scale quantizes to k when lo and scale are powers of
    two (every operation is then exact in fp32)."""
    lo, hi = -4.0, 4.0
    sc = 8.0 / 2 ** bits
    ks = np.unique(np.linspace(0, 2 ** bits - 1, 97).astype(np.int64))
    half = 0.5 if bits <= 20 else 0.0      # keep x exactly representable in fp32
    x64 = lo + (ks + half) * sc
    x = x64.astype(np.float32)
    assert (x.astype(np.float64) == x64).all()
    assert qgnn.quantize(x, lo, hi, bits).tolist() == ks.tolist()
    assert int(qgnn.quantize(np.float32(hi), lo, hi, bits)) == 2 ** bits - 1
    assert int(qgnn.quantize(np.float32(lo), lo, hi, bits)) == 0
    assert int(qgnn.quantize(np.float32(-100), lo, hi, bits)) == 0
    assert int(qgnn.quantize(np.float32(100), lo, hi, bits)) == 2 ** bits - 1


@pytest.mark.parametrize("bits", [1, 2, 4, 8, 16, 32])
def test_quantize_monotone_bounded_and_close(bits):
    rng = np.random.default_rng([10, bits])
    x = np.sort(rng.standard_normal(4000).astype(np.float32))
    lo, hi = float(x.min()), float(x.max())
    q = qgnn.quantize(x, lo, hi, bits).astype(np.int64)
    assert (np.diff(q) >= 0).all() and q.min() == 0 and q.max() <= 2 ** bits - 1
    # above 24 bits fp32 cannot hit the top code exactly
    assert q.max() == 2 ** bits - 1 if bits <= 16 else q.max() >= (2 ** bits - 1) * (1 - 1e-6)
    xh = qgnn.dequantize_values(q, lo, hi, bits)
    sx = qgnn.scale(lo, hi, bits)
    err = x.astype(np.float64) - xh
    # floor: the value lies in [xh, xh + sx) up to fp32 rounding; the top code
    # also absorbs x = hi
    tol = 1e-6 * (hi - lo)
    assert (err > -tol).all() and (err <= sx + tol).all()


def test_requantize_rule():
    c = np.array([[0, 1, 5, 6, 11, 12, 2 ** 31 - 1, 2 ** 32 - 3]], dtype=np.uint32)
    inv = np.float32(0.5)
    # signed reading: 2^32-3 is -3 -> below rq_lo -> 0 ; big value clamps
    assert qgnn.requantize(c, 1, inv, 3).tolist() == [[0, 0, 2, 2, 5, 5, 7, 0]]
    assert qgnn.requantize(c, -4, inv, 3, relu=True).tolist() == [[2, 2, 4, 5, 7, 7, 7, 2]]
    assert qgnn.requantize(c, -4, inv, 3, relu=False).tolist() == [[2, 2, 4, 5, 7, 7, 7, 0]]
    # identity requant reproduces the value when it fits
    v = np.array([[0, 3, 200, 65535]], dtype=np.uint32)
    assert (qgnn.requantize(v, 0, np.float32(1.0), 16) == v).all()
    # 32 bits: no overflow at the top
    big = np.array([[2 ** 31 - 1]], dtype=np.uint32)
    assert int(qgnn.requantize(big, 0, np.float32(4.0), 32)[0, 0]) == 2 ** 32 - 1


# --------------------------------------------------------------- dequantize
@pytest.mark.parametrize("self_term", [False, True])
def test_dequantized_layer_equals_real_product(self_term):
    """The affine-corrected fp32 outputs equal the products of the dequantized
    operands taken directly in float64."""
    rng = np.random.default_rng([11, int(self_term)])
    n, d, h, s, t = 60, 24, 7, 5, 4
    A = _rand_graph(rng, n, 0.1)
    X = rng.standard_normal((n, d)).astype(np.float32)
    W = rng.uniform(-0.1, 0.1, size=(d, h)).astype(np.float32)
    lox, hix = float(X.min()), float(X.max())
    low, hiw = float(W.min()), float(W.max())
    Xq = qgnn.quantize(X, lox, hix, s)
    Wq = qgnn.quantize(W, low, hiw, t)
    sx, sw = qgnn.scale(lox, hix, s), qgnn.scale(low, hiw, t)
    Xh = lox + sx * Xq.astype(np.float64)
    Wh = low + sw * Wq.astype(np.float64)
    Ad = A.astype(np.float64) + (np.eye(n) if self_term else 0.0)
    deg = Ad.sum(axis=1)
    Y, Yq, Z, (rq_lo, rq_inv) = qgnn.layer(A, Xq, Wq, s, self_term=self_term)
    # aggregation output
    yh = qgnn.dequantize(Y, cc=sx, rs=lox, row_i=deg)
    ref = Ad @ Xh
    assert np.allclose(yh, ref, rtol=0, atol=1e-6 * np.abs(ref).max())
    # update output: Yq stands for y ~ rq_lo + Yq / rq_inv in accumulator units
    sl = sx / float(rq_inv)
    l0 = sx * rq_lo + lox * deg               # per-row offset of the left operand
    Yqh = l0[:, None] + sl * Yq.astype(np.float64)
    ref = Yqh @ Wh
    zh = qgnn.dequantize(Z, cc=sl * sw, rs=sl * low, row_i=Yq.sum(axis=1, dtype=np.int64),
                         l0a=sx * rq_lo, l0b=lox, row_l=deg,
                         ck=low * d, cs=sw, col_i=Wq.sum(axis=0, dtype=np.int64))
    assert np.allclose(zh, ref, rtol=0, atol=2e-6 * np.abs(ref).max())
    # ReLU on the real value
    zr = qgnn.dequantize(Z, cc=sl * sw, rs=sl * low, row_i=Yq.sum(axis=1, dtype=np.int64),
                         l0a=sx * rq_lo, l0b=lox, row_l=deg,
                         ck=low * d, cs=sw, col_i=Wq.sum(axis=0, dtype=np.int64), relu=True)
    assert (zr == np.maximum(zh, 0)).all()


# ------------------------------------------------------------------ packing
def test_pack_hand_vector_and_sizes():
    g = load_golden("quantize_2bit.txt")
    v = np.zeros((1, 64), dtype=np.uint32)
    v[0, g["ones_at"]] = 1
    assert bp.pack(v, 1, bp.LEFT)[0, 0].tolist() == g["words"]
    assert bp.pack(v.T, 1, bp.RIGHT)[0, :, 0].tolist() == g["words"]
    q = np.zeros((13, 70), dtype=np.uint32)
    assert bp.pack(q, 3, bp.LEFT).shape == (3, 13, 3)      # ceil(70/32) words per row
    assert bp.pack(q, 3, bp.RIGHT).shape == (3, 1, 70)     # ceil(13/32) word rows


@pytest.mark.parametrize("layout", [bp.LEFT, bp.RIGHT])
@pytest.mark.parametrize("bits", [1, 3, 8, 17, 32])
def test_pack_roundtrip_and_zero_padding(layout, bits):
    rng = np.random.default_rng([12, layout, bits])
    q = rng.integers(0, 2 ** bits, size=(45, 77), dtype=np.uint64).astype(np.uint32)
    w = bp.pack(q, bits, layout)
    assert (bp.unpack(w, 45, 77, layout) == q).all()
    if layout == bp.LEFT:      # bits past column 77 in the last word are zero
        assert (w[:, :, -1] >> np.uint32(77 - 64) == 0).all()
    else:                      # bits past row 45 in the last word row are zero
        assert (w[:, -1, :] >> np.uint32(45 - 32) == 0).all()
    # plane i really is bit i
    plane0 = bp.unpack(w[:1], 45, 77, layout)
    assert (plane0 == (q & 1)).all()


def test_packed_popcount_product_equals_matmul():
    """AND + popcount on the packed words reproduces the integer product."""
    rng = np.random.default_rng(13)
    n, k, m, lb, rb = 10, 75, 6, 2, 3
    L = rng.integers(0, 2 ** lb, size=(n, k)).astype(np.uint32)
    R = rng.integers(0, 2 ** rb, size=(k, m)).astype(np.uint32)
    lw = bp.pack(L, lb, bp.LEFT)
    rw = bp.pack(R, rb, bp.RIGHT)
    out = np.zeros((n, m), dtype=np.int64)
    for i in range(lb):
        for j in range(rb):
            for r in range(n):
                for c in range(m):
                    cnt = sum(bin(int(lw[i, r, w]) & int(rw[j, w, c])).count("1")
                              for w in range(lw.shape[2]))
                    out[r, c] += cnt << (i + j)
    assert (out == L.astype(np.int64) @ R.astype(np.int64)).all()
    assert (qgnn.matmul_mod32(L, R) == out).all()


# ----------------------------------------------------------------- tile map
def test_tile_map_brute_force_and_block_structure():
    from workloads import make_workload
    w = make_workload(1)
    A = w.graph.dense()
    lists, deg = qgnn.tile_map(A, 8, 128)
    assert (deg == w.graph.degrees()).all()
    for tr, nz in enumerate(lists):
        for tc in range(2):
            want = bool(A[tr * 8:(tr + 1) * 8, tc * 128:(tc + 1) * 128].any())
            assert (tc in nz) == want
    # 64-node blocks aligned to 16 x 64 tiles: non-zero tiles lie on the diagonal
    lists, _ = qgnn.tile_map(A, 16, 64)
    for tr, nz in enumerate(lists):
        assert nz == [tr * 16 // 64]
    # the product does not depend on skipping zero tiles
    X = w.X
    Y = qgnn.aggregate(A, X)
    Yt = np.zeros_like(Y, dtype=np.int64)
    for tr, nz in enumerate(lists):
        for tc in nz:
            Yt[tr * 16:(tr + 1) * 16] += A[tr * 16:(tr + 1) * 16, tc * 64:(tc + 1) * 64].astype(np.int64) \
                @ X[tc * 64:(tc + 1) * 64].astype(np.int64)
    assert (Yt == Y).all()


# -------------------------------------------------------------- multi-layer
def test_update_first_equals_aggregate_first_without_requantization():
    """A (X W) = (A X) W: with an identity requantization in between (range wide
    enough, scale 1) the two orders of the layer give the same integers."""
    rng = np.random.default_rng(77)
    n, d, h, s, t = 40, 24, 7, 3, 2
    A = (rng.random((n, n)) < 0.2).astype(np.uint8)
    Xq = rng.integers(0, 2 ** s, size=(n, d)).astype(np.uint32)
    Wq = rng.integers(0, 2 ** t, size=(d, h)).astype(np.uint32)
    ident = (0, np.float32(1.0))
    for self_term in (False, True):
        _, Yq, Z1, _ = qgnn.layer(A, Xq, Wq, 20, rq=ident, self_term=self_term)
        _, Pq, Z2, _ = qgnn.layer_update_first(A, Xq, Wq, 20, rq=ident, self_term=self_term)
        assert (Yq == qgnn.aggregate(A, Xq, self_term)).all() and (Pq == qgnn.update(Xq, Wq)).all()
        assert (Z1 == Z2).all()
        want = (A.astype(np.int64) + (np.eye(n, dtype=np.int64) if self_term else 0)) @ Xq.astype(np.int64) \
            @ Wq.astype(np.int64)
        assert (Z2 == want.astype(np.uint32)).all()
    # with a real requantization the orders differ (the rounding happens elsewhere)
    _, _, Z1, _ = qgnn.layer(A, Xq, Wq, 2)
    _, _, Z2, _ = qgnn.layer_update_first(A, Xq, Wq, 2)
    assert (Z1 != Z2).any()


def test_forward_chain_is_layerwise_consistent():
    from workloads import make_workload
    w = make_workload(4, n_blocks=1)
    A = w.graph.scipy_csr()
    xr = (float(w.X.min()), float(w.X.max()))
    wr = [(float(W.min()), float(W.max())) for W in w.W]
    trace, rqs = qgnn.forward(A, w.X, xr, w.W, wr, w.s, w.t, self_term=True)
    assert len(trace) == 5
    for l, tr in enumerate(trace):
        Y = qgnn.aggregate(A, tr["Xq"], self_term=True)
        assert (Y == tr["Y"]).all()
        assert int(tr["Yq"].max()) == 2 ** w.s - 1     # calibrated range is used fully
        if l + 1 < len(trace):
            assert (trace[l + 1]["Xq"] == tr["Xq_next"]).all()
    # giving the calibrated ranges back reproduces the same integers
    trace2, _ = qgnn.forward(A, w.X, xr, w.W, wr, w.s, w.t, True, rqs=rqs)
    assert all((a["Z"] == b["Z"]).all() for a, b in zip(trace, trace2))


# ---------------------------------------------------- folded batch normalization
def test_affine_requantize_reduces_to_requantize():
    """a = 1, b = 0: the affine path is the integer rule (all values below 2^24, where
    fp32(C) - fp32(lo) and the integer difference agree)."""
    rng = np.random.default_rng(41)
    C = rng.integers(-5000, 200000, size=(40, 9)).astype(np.int64)
    c_u32 = (C & 0xFFFFFFFF).astype(np.uint32)
    ones = np.ones(9, dtype=np.float32)
    for bits, lo, relu in ((4, 0, True), (8, 17, False), (3, 0, False), (8, 1000, True)):
        inv = qgnn.inv_scale(float(lo), 180000.0, bits)
        want = qgnn.requantize(c_u32, lo, inv, bits, relu=relu)
        got = qgnn.requantize_affine(c_u32, ones, None, lo, inv, bits, relu=relu)
        assert (got == want).all()
        got = qgnn.requantize_affine(c_u32, ones, np.zeros(9, dtype=np.float32), lo, inv, bits, relu=relu)
        assert (got == want).all()


def test_batchnorm_fold_matches_the_definition():
    """Section 4.5: codes produced behind the folded affine map stand for
    ReLU(BN(x)) computed from its definition (batch statistics, gamma, beta, eps) to
    within one quantization step; a dropped shift, a missing sqrt or a swapped
    gamma / beta would be off by far more."""
    rng = np.random.default_rng(43)
    n, h, bits = 500, 12, 8
    C = rng.integers(-30000, 90000, size=(n, h)).astype(np.int64)
    value_scale = 3.1e-4                                   # x = value_scale * C
    x = value_scale * C.astype(np.float64)
    gamma = rng.uniform(0.5, 2.0, size=h)
    beta = rng.uniform(-1.0, 1.0, size=h)
    eps = 1e-5
    mean, var = x.mean(axis=0), x.var(axis=0)
    bn = (x - mean[None, :]) / np.sqrt(var[None, :] + eps) * gamma[None, :] + beta[None, :]
    want = np.maximum(bn, 0.0)
    a, b = qgnn.fold_batchnorm(gamma, beta, mean, var, eps, value_scale)
    hi = float(want.max())
    inv = qgnn.inv_scale(0.0, hi, bits)
    c_u32 = (C & 0xFFFFFFFF).astype(np.uint32)
    q = qgnn.requantize_affine(c_u32, a, b, 0, inv, bits, relu=True)
    step = hi / 2 ** bits
    back = q.astype(np.float64) * step
    inside = want < hi - step                               # the top code also holds the clamp
    assert np.all(back[inside] <= want[inside] + 1e-4 * hi)
    assert np.all(want[inside] - back[inside] < step * (1 + 1e-3) + 1e-4 * hi)
    assert (q[want == 0.0] == 0).all() and q.max() == 2 ** bits - 1
    # fp32 output: the affine map acts on the real value, in front of the ReLU
    base = qgnn.dequantize(c_u32, cc=value_scale)
    a1, b1 = qgnn.fold_batchnorm(gamma, beta, mean, var, eps, 1.0)
    got = qgnn.dequantize(c_u32, cc=value_scale, col_a=a1, col_b=b1, relu=True)
    assert np.allclose(got, want, rtol=1e-5, atol=1e-5 * hi)
    assert np.allclose(qgnn.dequantize(c_u32, cc=value_scale, col_a=a1, col_b=None),
                       base.astype(np.float64) * a1[None, :].astype(np.float64), rtol=1e-6, atol=1e-9)


# ------------------------------------------- int32 output, calibration, sparse inputs
def test_int_output_reads_the_accumulator_as_signed():
    """bitMM2Int: the 32-bit accumulator is handed out as int32; ReLU acts on that
    signed value, so a wrapped (negative) accumulator becomes 0, not a large positive."""
    c = np.array([[0, 7, 2 ** 31 - 1, 2 ** 31, 2 ** 32 - 3, 2 ** 32 - 1]], dtype=np.uint32)
    got = qgnn.int_output(c)
    assert got.dtype == np.int32
    assert got.tolist() == [[0, 7, 2 ** 31 - 1, -2 ** 31, -3, -1]]
    relu = qgnn.int_output(c, relu=True)
    assert relu.dtype == np.int32
    assert relu.tolist() == [[0, 7, 2 ** 31 - 1, 0, 0, 0]]
    assert c.tolist() == [[0, 7, 2 ** 31 - 1, 2 ** 31, 2 ** 32 - 3, 2 ** 32 - 1]]     # input untouched
    assert qgnn.as_signed(c).tolist() == got.tolist()


def test_calibrated_ranges_by_hand():
    """Range a user would set from observed values: lower bound 0, upper bound the largest
    signed accumulator (Eq. (2)'s empirical bounds) - a wrapped value is negative and never
    the maximum; behind a per-column affine map, the largest mapped value."""
    c = np.array([[5, 2 ** 32 - 5], [12, 3]], dtype=np.uint32)      # signed: 5, -5, 12, 3
    lo, inv = qgnn.calibrate_requant(c, 3)
    assert lo == 0 and inv == np.float32(8.0 / 12.0) and isinstance(inv, np.float32)
    assert qgnn.calibrate_requant(np.array([[2 ** 32 - 1]], dtype=np.uint32), 4) == (0, np.float32(16.0))
    # v = C * a + b per column: [[5*0.5+1, -5*2-30], [12*0.5+1, 3*2-30]] = [[3.5, -40], [7, -24]]
    a, b = np.array([0.5, 2.0], dtype=np.float32), np.array([1.0, -30.0], dtype=np.float32)
    lo, inv = qgnn.calibrate_requant_affine(c, a, b, 4)
    assert lo == 0 and inv == np.float32(16.0 / 7.0)
    # no shift: [[2.5, -10], [6, 6]]
    assert qgnn.calibrate_requant_affine(c, a, None, 4)[1] == np.float32(16.0 / 6.0)
    # a swapped scale / shift would give 12 * 1 + 0.5 = 12.5
    assert qgnn.calibrate_requant_affine(c, a, b, 4)[1] != np.float32(16.0 / 12.5)
    # nothing positive: the floor of 1e-6 keeps the scale finite
    neg = np.array([[2 ** 32 - 4, 2 ** 32 - 9]], dtype=np.uint32)
    assert qgnn.calibrate_requant_affine(neg, np.ones(2, dtype=np.float32), None, 2)[1] == np.float32(4.0 / 1e-6)
    # the range it returns is used fully by the codes it is made for
    rng = np.random.default_rng(5)
    C = rng.integers(-1000, 50000, size=(30, 6)).astype(np.int64)
    cu = (C & 0xFFFFFFFF).astype(np.uint32)
    ca = rng.uniform(0.5, 2.0, size=6).astype(np.float32)
    cb = rng.uniform(-3.0, 3.0, size=6).astype(np.float32)
    lo, inv = qgnn.calibrate_requant_affine(cu, ca, cb, 5)
    assert qgnn.requantize_affine(cu, ca, cb, lo, inv, 5, relu=True).max() == 31


@pytest.mark.parametrize("self_term", [False, True])
def test_sparse_adjacency_branches_against_brute_force(self_term):
    """A scipy sparse adjacency goes through its own product: against the textbook triple
    loop on Python integers (directed graph, so a transposed product fails), with the GIN
    self term, and with 32-bit features whose neighbour sums pass 2^32 (wrap)."""
    import scipy.sparse as sp
    rng = np.random.default_rng([21, int(self_term)])
    n, d = 23, 5
    A = (rng.random((n, n)) < 0.3).astype(np.uint8)
    A[3, :] = 0                                             # an isolated row
    assert (A != A.T).any()
    for bits in (3, 32):
        X = rng.integers(0, 2 ** bits, size=(n, d), dtype=np.uint64).astype(np.uint32)
        if bits == 32:
            X[:, 0] = 2 ** 32 - 1                           # every neighbour sum of column 0 wraps
        ref = py_matmul(A.tolist(), X.tolist())
        if self_term:
            ref = [[v + int(X[i][j]) for j, v in enumerate(r)] for i, r in enumerate(ref)]
        want = [[v % 2 ** 32 for v in r] for r in ref]
        if bits == 32:
            assert max(max(r) for r in ref) >= 2 ** 32
        for fmt in (sp.csr_matrix, sp.coo_matrix, sp.csc_matrix):
            As = fmt(A.astype(np.uint64))
            got = qgnn.aggregate(As, X, self_term=self_term)
            assert got.dtype == np.uint32 and got.tolist() == want
        assert qgnn.aggregate(A, X, self_term=self_term).tolist() == want        # dense branch agrees
    deg = [sum(int(v) for v in row) for row in A.tolist()]
    assert deg[3] == 0
    for fmt in (sp.csr_matrix, sp.coo_matrix):
        assert qgnn.degrees(fmt(A)).tolist() == deg         # row sums, not column sums
        assert qgnn.degrees(fmt(A.astype(np.uint64))).tolist() == deg
    assert qgnn.degrees(A).tolist() == deg
    assert qgnn.degrees(sp.csr_matrix(A)).tolist() != qgnn.degrees(sp.csr_matrix(A.T)).tolist()


# ----------------------------------------------------- end-to-end fp32 output
def _golden_net():
    g = load_golden("gcn_2layer_3nodes.txt")
    A = np.array(g["A"], dtype=np.uint8)
    X = np.array(g["X"], dtype=np.float32)
    Ws = [np.array(g["W1"], dtype=np.float32), np.array(g["W2"], dtype=np.float32).reshape(2, 1)]
    xr = (g["x_lo"][0], g["x_hi"][0])
    wr = [(g["w_lo"][0], g["w_hi"][0])] * 2
    return g, A, X, Ws, xr, wr


def test_two_layer_network_worked_by_hand():
    """Every integer of a 2-layer GCN, the scale each stands for and the fp32 output,
    against a hand calculation (tests/golden/gcn_2layer_3nodes.txt), in both orders of the
    two products, with calibrated and with given ranges."""
    g, A, X, Ws, xr, wr = _golden_net()
    s, t = g["s"][0], g["t"][0]
    col = lambda key: np.array(g[key]).reshape(-1, 1).tolist()
    # the ranges of the hand calculation, given by the user
    inv = lambda hi: qgnn.inv_scale(0.0, float(hi), s)
    rqs = [((0, inv(g["agg1_hi"][0])), (0, inv(g["out1_hi"][0]))), ((0, inv(g["agg2_hi"][0])), None)]
    out, trace, used = qgnn.forward_dequantized(A, X, xr, Ws, wr, s, t, False, rqs=rqs)
    assert trace[0]["Xq"].tolist() == g["Xq"] and trace[0]["Wq"].tolist() == g["W1q"]
    assert trace[0]["Y"].tolist() == g["Y1"] and trace[0]["Yq"].tolist() == g["Y1q"]
    assert trace[0]["Z"].tolist() == g["Z1"] and trace[0]["Xq_next"].tolist() == g["X1q"]
    assert trace[0]["x_scale"] == 1.0 and trace[0]["z_scale"] == g["z1_scale"][0]
    assert trace[1]["x_scale"] == g["x1_scale"][0]
    assert trace[1]["Y"].tolist() == g["Y2"] and trace[1]["Yq"].tolist() == g["Y2q"]
    assert trace[1]["Wq"].tolist() == col("W2q") and trace[1]["Z"].tolist() == col("Z2")
    assert out.dtype == np.float32 and out.tolist() == col("out")
    # the other order of the two products
    rqs_u = [((0, inv(g["p1_hi"][0])), (0, inv(g["zu1_hi"][0]))), ((0, inv(g["p2_hi"][0])), None)]
    out_u, tr_u, _ = qgnn.forward_dequantized(A, X, xr, Ws, wr, s, t, False, rqs=rqs_u, update_first=True)
    assert tr_u[0]["Y"].tolist() == g["P1"] and tr_u[0]["Yq"].tolist() == g["P1q"]
    assert tr_u[0]["Z"].tolist() == g["ZU1"] and tr_u[0]["Xq_next"].tolist() == g["XU1q"]
    assert tr_u[1]["Y"].tolist() == col("P2") and tr_u[1]["Yq"].tolist() == col("P2q")
    assert tr_u[1]["Z"].tolist() == col("ZU2")
    assert out_u.tolist() == col("out_update_first")
    # forward() alone gives the same integers
    tr2, _ = qgnn.forward(A, X, xr, Ws, wr, s, t, False, rqs=rqs)
    assert all((a["Z"] == b["Z"]).all() for a, b in zip(trace, tr2))


@pytest.mark.parametrize("self_term", [False, True])
def test_one_layer_network_output_is_the_real_product(self_term):
    """One layer: the fp32 output is the product of the dequantized operands, zero points
    included, taken directly in float64 (A.(lo_x + sx Xq) requantized, times lo_w + sw Wq)."""
    rng = np.random.default_rng([31, int(self_term)])
    n, d, h, s, t = 40, 12, 5, 6, 3
    A = _rand_graph(rng, n, 0.15)
    X = rng.standard_normal((n, d)).astype(np.float32)
    W = rng.uniform(-0.1, 0.1, size=(d, h)).astype(np.float32)
    xr, wr = (float(X.min()), float(X.max())), (float(W.min()), float(W.max()))
    out, trace, used = qgnn.forward_dequantized(A, X, xr, [W], [wr], s, t, self_term)
    tr = trace[0]
    sx, sw = qgnn.scale(*xr, s), qgnn.scale(*wr, t)
    deg = A.sum(axis=1).astype(np.float64) + (1.0 if self_term else 0.0)
    (rq_lo, rq_inv), _ = used[0]
    Yh = (sx * rq_lo + xr[0] * deg)[:, None] + (sx / float(rq_inv)) * tr["Yq"].astype(np.float64)
    ref = Yh @ (wr[0] + sw * tr["Wq"].astype(np.float64))
    assert np.allclose(out, ref, rtol=0, atol=2e-6 * np.abs(ref).max())
    # and Yh is the requantized image of the real aggregation: within one step of it
    Xh = xr[0] + sx * tr["Xq"].astype(np.float64)
    Yreal = (A.astype(np.float64) + (np.eye(n) if self_term else 0.0)) @ Xh
    step = sx / float(rq_inv)
    below = tr["Yq"] < 2 ** s - 1
    assert (np.abs(Yh - Yreal)[below] <= step * (1 + 1e-6)).all()


@pytest.mark.parametrize("update_first", [False, True])
@pytest.mark.parametrize("self_term", [False, True])
def test_scale_chain_of_a_deep_network(update_first, self_term):
    """The pure-scale reading of hidden codes, layer by layer, against a float64 pass over
    real values: with x~ = x_scale * Xq the real aggregation, its requantized image, the real
    update and the next layer's real activations each lie within one quantization step of
    what the integers stand for.  A wrong factor anywhere in the chain (a dropped weight
    step, an inverted scale) is off by far more than a step.  The last layer's output is
    then the exact float64 product."""
    rng = np.random.default_rng([37, int(update_first), int(self_term)])
    n, dims, s, t = 50, [10, 8, 6, 4], 7, 6
    A = _rand_graph(rng, n, 0.12)
    Ad = A.astype(np.float64) + (np.eye(n) if self_term else 0.0)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    Ws = [rng.uniform(-0.1, 0.1, size=(dims[l], dims[l + 1])).astype(np.float32) for l in range(3)]
    xr = (float(X.min()), float(X.max()))
    wr = [(float(W.min()), float(W.max())) for W in Ws]
    out, trace, used = qgnn.forward_dequantized(A, X, xr, Ws, wr, s, t, self_term, update_first=update_first)
    top = 2 ** s - 1
    x_real = qgnn.scale(*xr, s) * trace[0]["Xq"].astype(np.float64)        # pure scale: no zero point
    for l, tr in enumerate(trace):
        sw = qgnn.scale(*wr[l], t)
        w_real = sw * tr["Wq"].astype(np.float64)                          # hidden layers: pure scale
        (rq_lo, inv_mid), out_rq = used[l]
        assert rq_lo == 0
        first = (x_real @ w_real) if update_first else (Ad @ x_real)       # P or Y, real
        unit_mid = (tr["x_scale"] * sw if update_first else tr["x_scale"]) / float(inv_mid)
        mid_real = unit_mid * tr["Yq"].astype(np.float64)
        ok = tr["Yq"] < top
        assert (np.abs(mid_real - np.maximum(first, 0))[ok] <= unit_mid * (1 + 1e-6)).all(), l
        assert np.isclose(tr["z_scale"], unit_mid if update_first else unit_mid * sw, rtol=1e-12)
        if l == len(trace) - 1:
            if update_first:
                ref = Ad @ mid_real
            else:
                ref = mid_real @ (wr[l][0] + w_real)                       # last layer: W with its zero point
            assert np.allclose(out, ref, rtol=0, atol=2e-6 * np.abs(ref).max())
            break
        second = (Ad @ mid_real) if update_first else (mid_real @ w_real)  # Z, real
        assert np.allclose(second, tr["z_scale"] * qgnn.as_signed(tr["Z"]), rtol=1e-9, atol=1e-12)
        unit_out = tr["z_scale"] / float(out_rq[1])
        assert np.isclose(trace[l + 1]["x_scale"], unit_out, rtol=1e-12)
        x_real = unit_out * tr["Xq_next"].astype(np.float64)
        ok = tr["Xq_next"] < top
        assert (np.abs(x_real - np.maximum(second, 0))[ok] <= unit_out * (1 + 1e-6)).all(), l


def test_network_with_batchnorm_layers_against_the_definition():
    """batchnorms given to the oracle are folded per layer with the real value of one
    accumulator unit: the hidden codes then stand for ReLU(BN(z_scale * Z)) computed from
    the definition of batch normalization, within one step; the last layer's normalization
    acts on the real fp32 value."""
    rng = np.random.default_rng(47)
    n, dims, s, t = 60, [9, 7, 5], 8, 8
    A = _rand_graph(rng, n, 0.1)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    Ws = [rng.uniform(-0.1, 0.1, size=(dims[l], dims[l + 1])).astype(np.float32) for l in range(2)]
    xr = (float(X.min()), float(X.max()))
    wr = [(float(W.min()), float(W.max())) for W in Ws]
    bns = [dict(gamma=rng.uniform(0.5, 1.5, size=dims[l + 1]), beta=rng.uniform(-0.2, 0.5, size=dims[l + 1]),
                mean=rng.uniform(-0.3, 0.3, size=dims[l + 1]), var=rng.uniform(0.5, 2.0, size=dims[l + 1]),
                eps=1e-5) for l in range(2)]
    out, trace, used = qgnn.forward_dequantized(A, X, xr, Ws, wr, s, t, True, batchnorms=bns)
    plain, trace0, _ = qgnn.forward_dequantized(A, X, xr, Ws, wr, s, t, True)
    assert (trace[0]["Z"] == trace0[0]["Z"]).all()                         # same first accumulators
    bn = bns[0]
    z_real = trace[0]["z_scale"] * qgnn.as_signed(trace[0]["Z"])
    want = np.maximum((z_real - bn["mean"]) / np.sqrt(bn["var"] + bn["eps"]) * bn["gamma"] + bn["beta"], 0.0)
    unit = 1.0 / float(used[0][1][1])
    assert np.isclose(trace[1]["x_scale"], unit, rtol=1e-12)
    got = unit * trace[0]["Xq_next"].astype(np.float64)
    ok = trace[0]["Xq_next"] < 2 ** s - 1
    assert (np.abs(got - want)[ok] <= unit * (1 + 1e-3) + 1e-5 * want.max()).all()
    # last layer: BN of the real product, from the definition
    tr = trace[1]
    sl = tr["x_scale"] / float(used[1][0][1])
    real = (sl * tr["Yq"].astype(np.float64)) @ (wr[1][0] + qgnn.scale(*wr[1], t) * tr["Wq"].astype(np.float64))
    bn = bns[1]
    ref = (real - bn["mean"]) / np.sqrt(bn["var"] + bn["eps"]) * bn["gamma"] + bn["beta"]
    assert np.allclose(out, ref, rtol=1e-5, atol=1e-5 * np.abs(ref).max())
