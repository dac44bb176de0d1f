"""The paper's PyTorch-level surface (Section 5): a bit-Tensor type carried by an
ordinary int32 tensor, `Tensor.to_bit(nbits)` / `.to_val()`, and the two any-bitwidth
products `bitMM2Int` / `bitMM2Bit`.  Thin wrappers: the storage is the library's packed
operand, the products are qgtc_aggregate (binary left operand that meets the adjacency
contract) and qgtc_update.

    enable_tensor_methods()                  # once: adds Tensor.to_bit, as the paper writes it
    Ab = adj_u8.to_bit(1, side="left")       # or to_bit(adj_u8, 1, side="left")
    Xb = x_f32.to_bit(4)                     # min-max Eq. (2) unless quant=(lo, hi)
    Y  = bitMM2Int(Ab, Xb)                   # int32 [N, D]
    Yb = bitMM2Bit(Ab, Xb, 4, inv_scale=s)   # 4-bit result, a BitTensor for the next product
    Yb.to_val()                              # int32 codes
"""
from __future__ import annotations

import torch

from . import binding as B

_SIDES = {"left": B.LEFT, "right": B.RIGHT}


class BitTensor:
    """An nbits-bit matrix as stacked 1-bit planes packed into 32-bit words (Section 4.2),
    held in an int32 tensor (`storage`, the "vehicle" of Section 5).  `side` says which
    operand of a product it is packed for: "left" (A, Y: packed along the columns) or
    "right" (X, W: packed along the rows)."""

    def __init__(self, bits: B.Bits):
        self.bits = bits

    @property
    def storage(self) -> torch.Tensor:
        return self.bits.words

    @property
    def nbits(self) -> int:
        return self.bits.nbits

    @property
    def shape(self):
        return (self.bits.rows, self.bits.cols)

    @property
    def side(self) -> str:
        return "left" if self.bits.layout in (B.LEFT, B.LEFT_BYTES) else "right"

    def to_val(self) -> torch.Tensor:
        """Decode to one int32 code per entry (Tensor.to_val of Section 5)."""
        return B.qgtc_unpack_bits(self.bits)

    def is_adjacency(self) -> bool:
        """A binary left operand laid out as the aggregation kernel reads it: one plane, rows
        padded to 128 bits (with zeros: every producer in the library writes the padding),
        16-byte aligned."""
        c = self.bits.c
        return (c.layout == B.LEFT and c.nbits == 1 and c.cols >= 1 and c.ld_words % 4 == 0 and
                c.ld_words >= 4 * (-(-c.cols // 128)) and c.data % 16 == 0)

    def __repr__(self):
        return f"BitTensor({self.shape[0]}x{self.shape[1]}, {self.nbits} bit, {self.side})"


def to_bit(x: torch.Tensor, nbits: int, side: str = "right", quant=None, block_rows: int = 0) -> BitTensor:
    """Quantize (float input: Eq. (2) with quant = (lo, hi), default the tensor's min and
    max) or take integer codes as they are (uint8 / int32), and pack into bit planes.
    side: "left" for the left operand of a product (A, Y), "right" for the right one (X, W)."""
    assert x.dim() == 2 and x.is_cuda
    if x.dtype not in (torch.float32, torch.uint8, torch.int32):
        raise TypeError("to_bit takes float32, uint8 or int32 tensors")
    if x.dtype == torch.float32 and quant is None:
        quant = (float(x.min()), float(x.max()))
    return BitTensor(B.qgtc_pack_bits(x.contiguous(), nbits, _SIDES[side], quant=quant, block_rows=block_rows))


def to_val(b: BitTensor) -> torch.Tensor:
    return b.to_val()


def enable_tensor_methods():
    """Adds `Tensor.to_bit(nbits, side="right", quant=None)` to torch.Tensor, the spelling
    of Section 5.  Opt-in: nothing is patched on import."""
    if not hasattr(torch.Tensor, "to_bit"):
        torch.Tensor.to_bit = lambda self, nbits, side="right", quant=None, block_rows=0: \
            to_bit(self, nbits, side=side, quant=quant, block_rows=block_rows)


def _product(A: BitTensor, Bm: BitTensor, ep: B.Epilogue, tile_map):
    if A.side != "left" or Bm.side != "right":
        raise ValueError("the left operand must be packed with side='left', the right one with side='right'")
    if A.is_adjacency():
        # a binary left operand in adjacency form: the aggregation kernel, with zero-tile jumping
        if tile_map is None:
            tile_map = B.qgtc_build_tile_map(A.bits, 16, 128)
        return B.qgtc_aggregate(A.bits, tile_map, Bm.bits, ep)
    # any other left operand (several bits, or a 1-bit result without the row padding)
    return B.qgtc_update(A.bits, Bm.bits, ep)


def bitMM2Int(A: BitTensor, Bm: BitTensor, tile_map=None) -> torch.Tensor:
    """Any-bitwidth product with int32 output (modulo 2^32)."""
    return _product(A, Bm, B.Epilogue(mode=B.OUT_I32), tile_map)


def calibrate_inv_scale(A: BitTensor, Bm: BitTensor, bit_C: int, rq_lo: int = 0, tile_map=None) -> float:
    """inv_scale = 2^bit_C / (hi - rq_lo) of Eq. (2) with hi the largest accumulator of A.B:
    runs the product once with int32 output to find it (a full extra pass - do it once per
    layer, outside the loop that calls bitMM2Bit)."""
    c = bitMM2Int(A, Bm, tile_map)
    hi = max(int(c.max()), rq_lo + 1)
    return B.qgtc_quant_inv_scale(float(rq_lo), float(hi), bit_C)


def bitMM2Bit(A: BitTensor, Bm: BitTensor, bit_C: int, inv_scale: float, rq_lo: int = 0,
              relu: bool = False, tile_map=None) -> BitTensor:
    """Any-bitwidth product with a bit_C-bit output, packed for the next product: as a
    left operand after an aggregation (adjacency A), as a right operand after an update.
    inv_scale = 2^bit_C / (hi - rq_lo) of Eq. (2), set by the caller ("empirical bounds");
    calibrate_inv_scale finds it from the data."""
    ep = B.Epilogue(mode=B.OUT_BITS, relu=relu, rq_nbits=bit_C, rq_lo=rq_lo, rq_inv_scale=float(inv_scale))
    return BitTensor(_product(A, Bm, ep, tile_map))
