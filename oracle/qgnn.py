"""Plain CPU definition of what the quantized GNN layer computes.

TEST INFRASTRUCTURE: slow, obviously-correct numpy, independent of the HIP path.

The paper composes every product out of 1-bit products (Section 3.1, Eq. 3-7):
    a . b = sum_i sum_j 2^(i+j) * popcnt(a_i & b_j)
which is an exact identity for unsigned integers.  The result therefore has a
plain definition - ordinary integer matrix multiplication of the quantized
integers - and that definition, written out, is this oracle.  (The literal
bit-plane form of Algorithm 1 lives in oracle/bitplane.py and is checked
against this file by the CPU tests.)

One layer (Algorithm 1 and Section 3.2; Sections 4.5 and 5 for the outputs):
    Xq = quantize(X, s bits)                      Eq. (2)
    Y  = A @ Xq  (+ Xq for GIN with eps = 0)      neighbour aggregation, 1-bit x s-bit
    Yq = requantize(Y, s bits)                    low-bit output of a fused kernel ("bitMM2Bit")
    Z  = Yq @ Wq                                  node update, s-bit x t-bit
    out = Z as int32 ("bitMM2Int"), or dequantized fp32 (last layer),
          or ReLU + requantize (hidden layer: next layer's Xq)

Readings taken where the paper is silent (each also listed in the design notes):
  * Eq. (2) maps alpha_max to 2^q, which needs q+1 bits: the result is clamped
    to [0, 2^q - 1].  inv_scale = fp32(2^q / (hi - lo)) is formed once in
    float64 and rounded once; (x - lo) and the multiply are single fp32
    operations, then floor.
  * Accumulators are 32-bit (Section 2.3 / 3.2): every integer result is
    defined modulo 2^32.
  * Requantizing an integer result: r = clamp(floor(fp32(y - rq_lo) * inv), 0,
    2^bits - 1), integer subtraction first (negative -> 0), one int->fp32
    conversion (round to nearest even), one fp32 multiply.  y is the accumulator
    read as a signed 32-bit value.
  * Dequantization (the paper multiplies raw integers and never mentions zero
    points): with L^ = l0[i] + sl*L and R^ = r0 + sr*R the exact real product is
        out[i,j] = (sl*sr)*C[i,j] + (sl*r0)*rowsum(L)[i]
                   + l0[i]*(r0*K + sr*colsum(R)[j]),   l0[i] = l0a + l0b*lv[i]
    evaluated in float64 in exactly this order:
        t1 = cc*C + rs*row_i[i];  t2 = (l0a + l0b*row_l[i]) * (ck + cs*col_i[j])
        out = fp32(t1 + t2)
    with cc = sl*sr, rs = sl*r0, ck = r0*K, cs = sr formed by the caller.
  * ReLU acts on the value a mode emits: the signed accumulator for integer and
    low-bit outputs, the real value for fp32 output.
"""
from __future__ import annotations

import numpy as np

MASK32 = np.uint64(0xFFFFFFFF)


# --------------------------------------------------------------------------
# Eq. (2): quantization
# --------------------------------------------------------------------------
def inv_scale(lo: float, hi: float, nbits: int) -> np.float32:
    """fp32(2^nbits / (hi - lo)), formed in float64 and rounded once."""
    return np.float32(float(2 ** nbits) / (float(hi) - float(lo)))


def scale(lo: float, hi: float, nbits: int) -> float:
    """Real width of one quantization step, (hi - lo) / 2^nbits (float64)."""
    return (float(hi) - float(lo)) / float(2 ** nbits)


def quantize(x, lo: float, hi: float, nbits: int) -> np.ndarray:
    """Eq. (2): floor((x - lo) / scale), clamped to [0, 2^nbits - 1].

    x is fp32; `lo` is rounded to fp32; the subtraction and the multiplication by
    inv_scale are single fp32 operations."""
    x = np.asarray(x, dtype=np.float32)
    lo32 = np.float32(lo)
    inv = inv_scale(lo, hi, nbits)
    t = np.floor((x - lo32) * inv)          # fp32 - fp32, fp32 * fp32, floor
    assert t.dtype == np.float32
    qmax = float(2 ** nbits - 1)
    # compare in float64 so that 2^32 - 1 is exact; NaN never occurs for finite x
    t64 = t.astype(np.float64)
    q = np.where(t64 <= 0.0, 0.0, np.where(t64 >= qmax, qmax, t64))
    return q.astype(np.uint32)


def dequantize_values(q, lo: float, hi: float, nbits: int) -> np.ndarray:
    """Real value a code stands for: lo + scale * q (float64)."""
    return float(np.float32(lo)) + scale(float(np.float32(lo)), hi, nbits) * \
        np.asarray(q, dtype=np.float64)


# --------------------------------------------------------------------------
# integer products modulo 2^32
# --------------------------------------------------------------------------
def _wrap32(c_u64: np.ndarray) -> np.ndarray:
    return (c_u64 & MASK32).astype(np.uint32)


def matmul_mod32(L, R) -> np.ndarray:
    """L @ R modulo 2^32 for unsigned integer matrices.

    numpy's uint64 matmul wraps modulo 2^64; reducing modulo 2^32 afterwards is
    exact because Z/2^64 -> Z/2^32 is a ring homomorphism.  When every partial
    sum is below 2^53 the same product is taken with the float64 BLAS routine,
    which is then exact as well (and much faster)."""
    L = np.asarray(L)
    R = np.asarray(R)
    k = L.shape[1]
    assert R.shape[0] == k
    lmax = int(L.max()) if L.size else 0
    rmax = int(R.max()) if R.size else 0
    if k * lmax * rmax < 2 ** 53:
        c = L.astype(np.float64) @ R.astype(np.float64)
        return _wrap32(c.astype(np.uint64))
    return _wrap32(L.astype(np.uint64) @ R.astype(np.uint64))


def aggregate(A, Xq, self_term: bool = False) -> np.ndarray:
    """Neighbour aggregation Y = A @ Xq (mod 2^32), plus Xq itself when
    `self_term` (GIN with eps = 0).  A is a dense 0/1 array or a scipy sparse
    0/1 matrix (its uint64 sparse-times-dense product wraps modulo 2^64)."""
    Xq = np.asarray(Xq)
    if hasattr(A, "tocsr"):
        y = _wrap32(np.asarray(A.astype(np.uint64) @ Xq.astype(np.uint64)))
    else:
        A = np.asarray(A)
        assert ((A == 0) | (A == 1)).all(), "adjacency must be binary"
        y = matmul_mod32(A, Xq)
    if self_term:
        y = _wrap32(y.astype(np.uint64) + Xq.astype(np.uint64))
    return y


def update(Yq, Wq) -> np.ndarray:
    """Node update Z = Yq @ Wq (mod 2^32)."""
    return matmul_mod32(Yq, Wq)


def degrees(A) -> np.ndarray:
    if hasattr(A, "tocsr"):
        return np.asarray(A.astype(np.int64).sum(axis=1)).ravel()
    return np.asarray(A, dtype=np.int64).sum(axis=1)


# --------------------------------------------------------------------------
# epilogues
# --------------------------------------------------------------------------
def as_signed(c_u32) -> np.ndarray:
    return np.asarray(c_u32, dtype=np.uint32).view(np.int32).astype(np.int64)


def int_output(c_u32, relu: bool = False) -> np.ndarray:
    """int32 output ("bitMM2Int"); ReLU acts on the signed accumulator."""
    c = np.asarray(c_u32, dtype=np.uint32).view(np.int32)
    return np.maximum(c, 0) if relu else c.copy()


def requantize(c_u32, rq_lo: int, rq_inv_scale, nbits: int,
               relu: bool = False) -> np.ndarray:
    """Low-bit output of a fused kernel ("bitMM2Bit", Section 4.5)."""
    c = as_signed(c_u32)
    if relu:
        c = np.maximum(c, 0)
    d = c - int(rq_lo)                                   # int64, exact
    f = np.maximum(d, 0).astype(np.float32)              # one int->fp32 rounding
    t = np.floor(f * np.float32(rq_inv_scale))           # one fp32 multiply
    assert t.dtype == np.float32
    qmax = float(2 ** nbits - 1)
    t64 = t.astype(np.float64)
    q = np.where(t64 >= qmax, qmax, t64)
    return q.astype(np.uint32)


def fold_batchnorm(gamma, beta, mean, var, eps: float, value_scale: float = 1.0):
    """Section 4.5: BN(x)_j = (x - mean_j) / sqrt(var_j + eps) * gamma_j + beta_j is the
    per-column affine map a_j x + b_j; with x = value_scale * C the kernel applies
    (a_j * value_scale) C + b_j.  Returns (col_a, col_b) as fp32 vectors."""
    g = np.asarray(gamma, dtype=np.float64) / np.sqrt(np.asarray(var, dtype=np.float64) + float(eps))
    a = g * float(value_scale)
    b = np.asarray(beta, dtype=np.float64) - g * np.asarray(mean, dtype=np.float64)
    return a.astype(np.float32), b.astype(np.float32)


def requantize_affine(c_u32, col_a, col_b, rq_lo: int, rq_inv_scale, nbits: int,
                      relu: bool = False) -> np.ndarray:
    """Low-bit output behind a per-column affine map (a batch normalization folded
    into the kernel, Section 4.5): v = fp32(C) * a_j, v = v + b_j (two fp32
    operations), ReLU, then Eq. (2) with lower bound rq_lo and the clamp."""
    c = as_signed(c_u32).astype(np.float32)              # one int->fp32 rounding
    a = np.asarray(col_a, dtype=np.float32)[None, :]
    b = (np.zeros_like(a) if col_b is None else np.asarray(col_b, dtype=np.float32)[None, :])
    v = c * a
    v = v + b
    assert v.dtype == np.float32
    if relu:
        v = np.where(v > 0, v, np.float32(0))
    t = np.floor((v - np.float32(rq_lo)) * np.float32(rq_inv_scale))
    assert t.dtype == np.float32
    qmax = float(2 ** nbits - 1)
    t64 = t.astype(np.float64)
    q = np.where(t64 <= 0.0, 0.0, np.where(t64 >= qmax, qmax, t64))
    return q.astype(np.uint32)


def dequantize(c_u32, cc: float, rs: float = 0.0, row_i=None,
               l0a: float = 0.0, l0b: float = 0.0, row_l=None,
               ck: float = 0.0, cs: float = 0.0, col_i=None,
               relu: bool = False, col_a=None, col_b=None) -> np.ndarray:
    """fp32 output of the last layer: the exact real product of the two
    dequantized operands (see the module docstring), float64 then one rounding.
    col_a / col_b: a per-column affine map (folded batch normalization) applied to
    that real value before the ReLU."""
    c = as_signed(c_u32).astype(np.float64)
    n, m = c.shape
    ri = np.zeros(n) if row_i is None else np.asarray(row_i, dtype=np.float64)
    rl = np.zeros(n) if row_l is None else np.asarray(row_l, dtype=np.float64)
    ci = np.zeros(m) if col_i is None else np.asarray(col_i, dtype=np.float64)
    t1 = np.float64(cc) * c + (np.float64(rs) * ri)[:, None]
    l0 = np.float64(l0a) + np.float64(l0b) * rl
    t2 = l0[:, None] * (np.float64(ck) + np.float64(cs) * ci)[None, :]
    v = t1 + t2
    if col_a is not None:
        cb = np.zeros(m) if col_b is None else np.asarray(col_b, dtype=np.float32).astype(np.float64)
        v = v * np.asarray(col_a, dtype=np.float32).astype(np.float64)[None, :] + cb[None, :]
    if relu:
        v = np.maximum(v, 0.0)
    return v.astype(np.float32)


# --------------------------------------------------------------------------
# zero-tile map (Section 4.3) and the tile statistics of the evaluation
# --------------------------------------------------------------------------
def tile_map(A_dense, tile_rows: int, tile_kbits: int):
    """Per tile-row, the sorted list of tile columns holding at least one edge.

    A tile is tile_rows x tile_kbits entries of the (dense 0/1) adjacency; the
    paper's Tensor-Core tile is 8 x 128.  Returns (lists, degrees)."""
    A = np.asarray(A_dense)
    n, k = A.shape
    ntr = -(-n // tile_rows)
    ntc = -(-k // tile_kbits)
    lists = []
    for tr in range(ntr):
        rows = A[tr * tile_rows:(tr + 1) * tile_rows]
        nz = [tc for tc in range(ntc)
              if rows[:, tc * tile_kbits:(tc + 1) * tile_kbits].any()]
        lists.append(nz)
    return lists, A.astype(np.int64).sum(axis=1)


# --------------------------------------------------------------------------
# one layer and whole models
# --------------------------------------------------------------------------
def calibrate_requant(c_u32, nbits: int):
    """Range a user would set from observed values (Eq. (2): 'empirical bounds'):
    rq_lo = 0, hi = max observed accumulator (at least 1)."""
    hi = max(1, int(as_signed(c_u32).max()))
    return 0, inv_scale(0.0, float(hi), nbits)


def layer(A, Xq, Wq, s: int, rq=None, self_term: bool = False):
    """Aggregate -> requantize to s bits -> update.  Returns (Y, Yq, Z, rq)
    where rq = (rq_lo, rq_inv_scale) is calibrated from Y when not given."""
    Y = aggregate(A, Xq, self_term)
    if rq is None:
        rq = calibrate_requant(Y, s)
    Yq = requantize(Y, rq[0], rq[1], s)
    Z = update(Yq, Wq)
    return Y, Yq, Z, rq


def layer_update_first(A, Xq, Wq, s: int, rq=None, self_term: bool = False):
    """The other order of the two products (Section 6.1 of the paper has GIN update the
    nodes before it aggregates; it pays when the update shrinks the feature dimension):
    P = Xq @ Wq -> requantize to s bits -> Z = A @ Pq (+ Pq with the GIN self term).
    Without the requantization in between, Z equals the aggregate-first result
    (associativity).  Returns (P, Pq, Z, rq), rq calibrated from P when not given."""
    P = update(Xq, Wq)
    if rq is None:
        rq = calibrate_requant(P, s)
    Pq = requantize(P, rq[0], rq[1], s)
    Z = aggregate(A, Pq, self_term)
    return P, Pq, Z, rq


def calibrate_requant_affine(c_u32, col_a, col_b, nbits: int):
    """calibrate_requant for an output behind a per-column affine map and a ReLU:
    rq_lo = 0, hi = largest value met (at least 1e-6)."""
    v = as_signed(c_u32).astype(np.float64) * np.asarray(col_a, dtype=np.float64)[None, :]
    if col_b is not None:
        v = v + np.asarray(col_b, dtype=np.float64)[None, :]
    hi = max(1e-6, float(v.max()))
    return 0, inv_scale(0.0, hi, nbits)


def forward(A, X, x_range, Ws, w_ranges, s: int, t: int, self_term: bool,
            rqs=None, update_first: bool = False, affines=None, batchnorms=None):
    """Multi-layer forward pass: every hidden layer ends in ReLU + requantize
    to s bits (the next layer's Xq); the last layer's integer result is
    returned as it is, together with everything needed to dequantize it.

    update_first: every layer runs as layer_update_first; the trace then holds the
    intermediate product P = Xq @ Wq and its codes under "Y" and "Yq".

    x_range / w_ranges are (lo, hi) pairs for Eq. (2).  rqs, when given, is a
    list of (agg_rq, out_rq) per layer; otherwise ranges are calibrated from the
    values met on the way and returned.  affines: per layer None or (col_a, col_b),
    the per-column affine map in front of a hidden layer's ReLU.  batchnorms: per
    layer None or a dict(gamma, beta, mean, var, eps); a hidden layer's entry is folded
    into that layer's affine map here (fold_batchnorm with the real value of one unit
    of the layer's accumulator), so give either affines or batchnorms for a layer.

    Scales (the reading of low-bit activations between layers): the codes a hidden layer
    emits are read as pure scales, value = x_scale * code with no zero point.  Each trace
    entry carries "x_scale", the real value of one unit of its Xq, and "z_scale", the real
    value of one unit of its accumulator Z under that reading:
        aggregate first:  z_scale = (x_scale / inv_agg) * sw          (Yq = floor(Y * inv_agg))
        update first:     z_scale = (x_scale * sw) / inv_p            (Pq = floor(P * inv_p))
        next x_scale   =  z_scale / inv_out,  or 1 / inv_out behind a folded batch
                          normalization (its codes quantize the normalized value itself)."""
    Xq = quantize(X, x_range[0], x_range[1], s)
    x_scale = scale(float(x_range[0]), float(x_range[1]), s)
    trace = []
    used = []
    for l, W in enumerate(Ws):
        Wq = quantize(W, w_ranges[l][0], w_ranges[l][1], t)
        sw = scale(float(w_ranges[l][0]), float(w_ranges[l][1]), t)
        rq_in = None if rqs is None else rqs[l][0]
        one_layer = layer_update_first if update_first else layer
        Y, Yq, Z, agg_rq = one_layer(A, Xq, Wq, s, rq_in, self_term)
        z_scale = (x_scale / float(agg_rq[1])) * sw if not update_first else (x_scale * sw) / float(agg_rq[1])
        last = l == len(Ws) - 1
        affine = None if affines is None else affines[l]
        if not last and batchnorms is not None and batchnorms[l] is not None:
            assert affine is None
            bn = batchnorms[l]
            affine = fold_batchnorm(bn["gamma"], bn["beta"], bn["mean"], bn["var"], bn["eps"], z_scale)
        if last:
            out_rq = None
            nxt = None
            x_next = None
        elif affine is not None:
            # a batch normalization folded into the layer's epilogue (Section 4.5)
            ca, cb = affine
            out_rq = calibrate_requant_affine(Z, ca, cb, s) if rqs is None else rqs[l][1]
            nxt = requantize_affine(Z, ca, cb, out_rq[0], out_rq[1], s, relu=True)
            x_next = 1.0 / float(out_rq[1])
        else:
            out_rq = calibrate_requant(Z, s) if rqs is None else rqs[l][1]
            nxt = requantize(Z, out_rq[0], out_rq[1], s, relu=True)
            x_next = z_scale / float(out_rq[1])
        trace.append({"Xq": Xq, "Wq": Wq, "Y": Y, "Yq": Yq, "Z": Z,
                      "Xq_next": nxt, "x_scale": x_scale, "z_scale": z_scale, "affine": affine})
        used.append((agg_rq, out_rq))
        Xq = nxt
        x_scale = x_next
    return trace, used


def forward_dequantized(A, X, x_range, Ws, w_ranges, s: int, t: int, self_term: bool,
                        rqs=None, update_first: bool = False, affines=None, batchnorms=None):
    """forward(), then the fp32 output of the last layer (Section 4.5: hidden layers
    emit low-bit codes, the last one full precision).  Returns (out, trace, rqs).

    Aggregate first: the exact real product (see dequantize) of
        left operand   Y^[i, :] = l0[i] + sl * Yq[i, :],  sl = x_scale / inv_agg,
                       l0[i] = x_scale * rq_lo + x_lo * (deg[i] + 1 if self_term else deg[i])
        right operand  W^ = lo_w + sw * Wq
    where x_lo is the zero point of the features the last layer reads: the lower bound of
    x_range for a one-layer network, 0 behind a hidden layer (pure-scale reading, see
    forward).  A batch normalization given for the last layer acts on that real value
    (fold_batchnorm with value scale 1).
    Update first: out = z_scale * Z (every code a pure scale; zero points do not factor
    through the aggregation that follows the update)."""
    trace, used = forward(A, X, x_range, Ws, w_ranges, s, t, self_term, rqs=rqs,
                          update_first=update_first, affines=affines, batchnorms=batchnorms)
    L = len(Ws) - 1
    tr = trace[L]
    col_a = col_b = None
    if batchnorms is not None and batchnorms[L] is not None:
        bn = batchnorms[L]
        col_a, col_b = fold_batchnorm(bn["gamma"], bn["beta"], bn["mean"], bn["var"], bn["eps"], 1.0)
    elif affines is not None and affines[L] is not None:
        col_a, col_b = affines[L]
    if update_first:
        return dequantize(tr["Z"], cc=tr["z_scale"], col_a=col_a, col_b=col_b), trace, used
    rq_lo, inv_agg = used[L][0]
    lo_w = float(w_ranges[L][0])
    sw = scale(lo_w, float(w_ranges[L][1]), t)
    sl = tr["x_scale"] / float(inv_agg)
    x_lo = float(x_range[0]) if L == 0 else 0.0
    out = dequantize(tr["Z"], cc=sl * sw, rs=sl * lo_w,
                     row_i=tr["Yq"].sum(axis=1, dtype=np.int64),
                     l0a=tr["x_scale"] * int(rq_lo) + (x_lo if self_term else 0.0), l0b=x_lo,
                     row_l=degrees(A),
                     ck=lo_w * np.asarray(Ws[L]).shape[0], cs=sw,
                     col_i=tr["Wq"].sum(axis=0, dtype=np.int64), col_a=col_a, col_b=col_b)
    return out, trace, used
