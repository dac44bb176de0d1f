"""Bit planes on the CPU: decomposition, Algorithm 1 taken literally, and the
packed layouts.  TEST INFRASTRUCTURE, independent of the HIP path.

* bit_decompose / bmm / algorithm1_layer follow Algorithm 1 of the paper step by
  step (bitDecompose, one 1-bit product per plane or plane pair, shift-left by
  the plane-index sum, elementwise reduction), with the 1-bit product written as
  Eq. (7): popcnt(row & column).  Plane 0 is the least significant bit.  The
  weight matrix is D x H and the output N x H (the listing's shapes for W and
  X-hat are misprints).  It is slow (Python loops) and only meant for small
  inputs; the CPU tests check oracle/qgnn.py against it.
* pack / unpack define the packed storage ("3D-stacked bit compression",
  Section 4.2): one 1-bit matrix per plane, 32 consecutive entries along the
  contraction dimension K in one 32-bit word, entry 32*w + b in bit b of word w
  (least significant bit = lowest index), zero fill past the end.
    LEFT  operand (A, Y), shape rows x K : words[plane][row][ceil(K/32)]
    RIGHT operand (X, W), shape K x cols : words[plane][ceil(K/32)][col]
"""
from __future__ import annotations

import numpy as np


def bit_decompose(M, nbits: int) -> list:
    """List of 0/1 matrices, entry i holding bit i of every element."""
    M = np.asarray(M, dtype=np.uint64)
    return [((M >> np.uint64(i)) & np.uint64(1)).astype(np.uint8)
            for i in range(nbits)]


def _row_words(bits_1d) -> int:
    """A 0/1 vector as one Python integer (entry k in bit k)."""
    v = 0
    for k, b in enumerate(bits_1d):
        if b:
            v |= 1 << k
    return v


def popcnt(v: int) -> int:
    return bin(v).count("1")


def bmm(Lbits, Rbits) -> np.ndarray:
    """1-bit matrix product, Eq. (7): out[i, j] = popcnt(L[i, :] & R[:, j])."""
    Lbits = np.asarray(Lbits)
    Rbits = np.asarray(Rbits)
    lrows = [_row_words(r) for r in Lbits]
    rcols = [_row_words(c) for c in Rbits.T]
    out = np.zeros((len(lrows), len(rcols)), dtype=object)
    for i, a in enumerate(lrows):
        for j, b in enumerate(rcols):
            out[i, j] = popcnt(a & b)
    return out


def any_bit_matmul(L, R, lbits: int, rbits: int) -> np.ndarray:
    """Shift-and-add of all plane-pair products, as exact Python integers."""
    Ls = bit_decompose(L, lbits)
    Rs = bit_decompose(R, rbits)
    acc = np.zeros((np.asarray(L).shape[0], np.asarray(R).shape[1]), dtype=object)
    for i, Li in enumerate(Ls):
        for j, Rj in enumerate(Rs):
            acc = acc + bmm(Li, Rj) * (1 << (i + j))
    return acc


def algorithm1_layer(A, Xq, Wq, s: int, t: int) -> np.ndarray:
    """Algorithm 1 with an exact (never requantized) intermediate:
    X_new = sum_x (A_bin (*) X_x) << x, then sum over (x, w) of
    (X_new plane x (*) W_w) << (x + w).  Exact Python integers, no wrap."""
    a_bin = bit_decompose(A, 1)[0]
    x_planes = bit_decompose(Xq, s)
    x_new = np.zeros((np.asarray(A).shape[0], np.asarray(Xq).shape[1]),
                     dtype=object)
    for x_idx, xp in enumerate(x_planes):
        x_new = x_new + bmm(a_bin, xp) * (1 << x_idx)
    width = max(1, max(int(v).bit_length() for v in x_new.ravel()))
    return x_new, any_bit_matmul(x_new.astype(np.uint64), Wq, width, t)


# --------------------------------------------------------------------------
# packed storage
# --------------------------------------------------------------------------
LEFT, RIGHT = 0, 1


def _pack_along_last(bits01) -> np.ndarray:
    """0/1 array [..., K] -> uint32 [..., ceil(K/32)], entry 32*w+b in bit b."""
    bits01 = np.asarray(bits01, dtype=np.uint8)
    k = bits01.shape[-1]
    kw = -(-k // 32)
    pad = np.zeros(bits01.shape[:-1] + (kw * 32,), dtype=np.uint8)
    pad[..., :k] = bits01
    by = np.packbits(pad, axis=-1, bitorder="little")      # 8 entries per byte
    return np.ascontiguousarray(by).view("<u4")


def pack(Q, nbits: int, layout: int) -> np.ndarray:
    """Unsigned integers -> packed planes.  LEFT: [nbits][rows][ceil(cols/32)];
    RIGHT: [nbits][ceil(rows/32)][cols].  Bits above nbits are dropped."""
    planes = bit_decompose(Q, nbits)
    if layout == LEFT:
        return np.stack([_pack_along_last(p) for p in planes])
    return np.stack([np.ascontiguousarray(_pack_along_last(p.T).T)
                     for p in planes])


def unpack(words, rows: int, cols: int, layout: int) -> np.ndarray:
    """Packed planes -> uint32 values (inverse of pack)."""
    words = np.asarray(words, dtype=np.uint32)
    out = np.zeros((rows, cols), dtype=np.uint64)
    for i in range(words.shape[0]):
        w = words[i] if layout == LEFT else words[i].T
        by = np.ascontiguousarray(w).astype("<u4").view(np.uint8)
        bits = np.unpackbits(by, axis=-1, bitorder="little")
        if layout == LEFT:
            plane = bits[:rows, :cols]
        else:
            plane = bits[:cols, :rows].T
        out |= plane.astype(np.uint64) << np.uint64(i)
    return out.astype(np.uint32)
