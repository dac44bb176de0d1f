"""Bandwidth-optimized subgraph packing (Section 4.6 of the paper): a batch is packed to
bit planes on the host - adjacency and node features side by side in one pinned buffer -
and crosses to the GPU in one copy of low-bit data.  Argument set-up only: the packing is
qgtc_pack_bits_host in the library, the copy is one asynchronous memcpy on the current
stream."""
from __future__ import annotations

import ctypes as C

import torch

from . import binding as B


class SubgraphPacket:
    """One compound buffer, on the host (pinned) and on the device, holding the packed
    adjacency (1 bit, LEFT, optionally block-diagonal storage) and the packed features
    (s bits, RIGHT) of a batch of subgraphs.

        pk = SubgraphPacket(n, a_cols, d, s, block_rows)     # once per batch shape
        pk.pack(A_host_u8, X_host_f32, x_range)              # CPU, synchronous
        A_bits, X_bits = pk.upload()                         # one H2D copy, asynchronous
    """

    def __init__(self, rows: int, a_cols: int, x_cols: int, s: int, block_rows: int = 0,
                 device: str = "cuda", pin: bool = True):
        self.rows, self.a_cols, self.x_cols, self.s = rows, a_cols, x_cols, s
        self.a_desc, a_words = B.describe(rows, a_cols, 1, B.LEFT, block_rows)
        self.x_desc, x_words = B.describe(rows, x_cols, s, B.RIGHT)
        sizes = (C.c_size_t * 2)(a_words * 4, x_words * 4)
        offs = (C.c_size_t * 2)()
        total = B.lib().qgtc_compound_layout(sizes, 2, offs)
        self.offsets = (int(offs[0]), int(offs[1]))
        self.nbytes = int(total)
        self.payload_bytes = int(a_words * 4 + x_words * 4)
        self.host = torch.zeros(self.nbytes // 4, dtype=torch.int32, pin_memory=pin)
        self.device = torch.empty(self.nbytes // 4, dtype=torch.int32, device=device) if device else None

    def _bits(self, buf: torch.Tensor):
        out = []
        for desc, off in ((self.a_desc, self.offsets[0]), (self.x_desc, self.offsets[1])):
            d = B._BitsC.from_buffer_copy(desc)
            d.data = buf.data_ptr() + off
            out.append(B.Bits(buf, d))
        return out

    def host_bits(self):
        """(A, X) descriptors into the host buffer."""
        return self._bits(self.host)

    def pack(self, A: torch.Tensor, X: torch.Tensor, x_range, threads: int = 0):
        """A: uint8 0/1 host tensor [rows, a_cols]; X: float32 host tensor [rows, x_cols]
        (or int32 / uint8 codes with x_range None)."""
        assert not A.is_cuda and not X.is_cuda and A.stride(1) == 1 and X.stride(1) == 1
        assert tuple(A.shape) == (self.rows, self.a_cols) and tuple(X.shape) == (self.rows, self.x_cols)
        a_bits, x_bits = self.host_bits()
        dt = {torch.float32: B.SRC_F32, torch.uint8: B.SRC_U8, torch.int32: B.SRC_I32}
        B._check(B.lib().qgtc_pack_bits_host(C.c_void_p(A.data_ptr()), dt[A.dtype], self.rows, self.a_cols,
                                             A.stride(0), None, C.byref(a_bits.c), threads),
                 "qgtc_pack_bits_host")
        q = None
        if x_range is not None:
            q = C.byref(B._QuantC(float(x_range[0]), float(x_range[1]), self.s))
        B._check(B.lib().qgtc_pack_bits_host(C.c_void_p(X.data_ptr()), dt[X.dtype], self.rows, self.x_cols,
                                             X.stride(0), q, C.byref(x_bits.c), threads),
                 "qgtc_pack_bits_host")

    def upload(self):
        """One copy of the whole buffer on the current stream; (A, X) descriptors into the
        device buffer (valid for work queued on that stream after this call)."""
        self.device.copy_(self.host, non_blocking=True)
        return self._bits(self.device)
