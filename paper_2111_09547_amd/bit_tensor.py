"""The paper's PyTorch-level surface (Section 5): bit tensors and the two any-bitwidth
products, under the names the paper gives them.  Thin wrappers: a bit tensor is the
library's packed operand (`Bits`: an int32 torch tensor as the vehicle plus the
descriptor), the products are qgtc_aggregate (1-bit left operand) and qgtc_update.

    Ab = to_bit(adj_u8, 1, side="left")             # Tensor.to_bit(nbits)
    Xb = to_bit(x_f32, 4, side="right")             # min-max Eq. (2) unless quant=(lo, hi)
    Y = bitMM2Int(Ab, Xb)                           # int32 [N, D]
    Yb = bitMM2Bit(Ab, Xb, 4, inv_scale=...)        # 4-bit result, packed for the next product
    to_val(Yb)                                      # Tensor.to_val(): int32 codes
"""
from __future__ import annotations

import torch

from . import binding as B

_SIDES = {"left": B.LEFT, "right": B.RIGHT}


def to_bit(x: torch.Tensor, nbits: int, side: str = "right", quant=None, block_rows: int = 0) -> B.Bits:
    """Quantize (float input: Eq. (2) with quant = (lo, hi), default the tensor's min and
    max) or take integer codes as they are (uint8 / int32), and pack into bit planes.
    side: "left" for the left operand of a product (A, Y), "right" for the right one (X, W)."""
    assert x.dim() == 2 and x.is_cuda
    if x.dtype == torch.float32 and quant is None:
        quant = (float(x.min()), float(x.max()))
    if x.dtype not in (torch.float32, torch.uint8, torch.int32):
        raise TypeError("to_bit takes float32, uint8 or int32 tensors")
    return B.qgtc_pack_bits(x.contiguous(), nbits, _SIDES[side], quant=quant, block_rows=block_rows)


def to_val(b: B.Bits) -> torch.Tensor:
    """Decode a bit tensor to one int32 code per entry."""
    return B.qgtc_unpack_bits(b)


def _product(A: B.Bits, Bm: B.Bits, ep: B.Epilogue, tile_map):
    if A.layout not in (B.LEFT, B.LEFT_BYTES):
        raise ValueError("the left operand must be packed with side='left'")
    if A.nbits == 1 and A.layout == B.LEFT:
        # a binary left operand is an adjacency: the aggregation kernel, with zero-tile jumping
        if tile_map is None and A.c.ld_words % 4 == 0:
            tile_map = B.qgtc_build_tile_map(A, 16, 128)
        return B.qgtc_aggregate(A, tile_map, Bm, ep)
    return B.qgtc_update(A, Bm, ep)


def bitMM2Int(A: B.Bits, Bm: B.Bits, tile_map=None) -> torch.Tensor:
    """Any-bitwidth product with int32 output (modulo 2^32)."""
    return _product(A, Bm, B.Epilogue(mode=B.OUT_I32), tile_map)


def bitMM2Bit(A: B.Bits, Bm: B.Bits, bit_C: int, inv_scale: float | None = None, rq_lo: int = 0,
              relu: bool = False, tile_map=None) -> B.Bits:
    """Any-bitwidth product with a bit_C-bit output, packed for the next product: as a
    left operand after an aggregation (binary A), as a right operand after an update.
    inv_scale = 2^bit_C / (hi - rq_lo) of Eq. (2); by default hi is the largest accumulator
    of this product (one extra int32 pass to find it)."""
    if inv_scale is None:
        c = bitMM2Int(A, Bm, tile_map)
        hi = max(int(c.max()), rq_lo + 1)
        inv_scale = float(torch.tensor(float(2 ** bit_C) / float(hi - rq_lo), dtype=torch.float64).to(torch.float32))
    ep = B.Epilogue(mode=B.OUT_BITS, relu=relu, rq_nbits=bit_C, rq_lo=rq_lo, rq_inv_scale=float(inv_scale))
    return _product(A, Bm, ep, tile_map)
