"""Host-side driver of the layer path: packs the operands once, then runs the
layers of a quantized GCN / GIN through the library (Algorithm 1 of the paper
per layer; hidden layers hand low-bit planes to the next layer, the last one
emits fp32, Section 4.5).  Only argument set-up happens here; the arithmetic is
in the kernels."""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding as B


def inv_scale(lo: float, hi: float, nbits: int) -> float:
    """fp32(2^nbits / (hi - lo)) as the library forms it for Eq. (2)."""
    return float(torch.tensor(float(2 ** nbits) / (float(hi) - float(lo)),
                              dtype=torch.float64).to(torch.float32))


@dataclass
class LayerRanges:
    agg_hi: int          # requantization range [0, agg_hi) of the aggregation result
    out_hi: int | None   # range [0, out_hi) of the update result (hidden layers)


def fused_layer_applies(d: int, h: int, s: int, t: int) -> bool:
    """The shapes and bit widths qgtc_layer runs as one kernel (see qgtc.h)."""
    return 33 <= d <= 1024 and 1 <= h <= 256 and s <= 8 and t <= 8


class QuantGNN:
    """A stack of quantized layers on one batch of subgraphs.

    A_src: uint8 0/1 device tensor, [N, N] (block_rows = 0) or [N, block_rows]
           (one row of diagonal blocks, see qgtc_bits.block_rows), or an already
           packed adjacency (Bits)
    Ws:    list of fp32 device tensors [D_l, H_l]; quantized to t bits by min-max
    """

    def __init__(self, A_src, Ws, s: int, t: int, self_term: bool,
                 tile_kbits: int = 128, use_map: bool = True, block_rows: int = 0,
                 weights_as_bytes: bool = True):
        self.s, self.t = s, t
        self.self_term = self_term
        self.tile_kbits = tile_kbits
        self.use_map = use_map
        self.Ws = [W.contiguous() for W in Ws]
        self.w_ranges = [(float(W.min()), float(W.max())) for W in Ws]
        self.dims = [(W.shape[0], W.shape[1]) for W in Ws]
        if isinstance(A_src, B.Bits):
            self.A_src, self.A = None, A_src
        else:
            self.A_src = A_src
            self.A = B.alloc_bits(A_src.shape[0], A_src.shape[1], 1, B.LEFT, block_rows)
        self.map = None
        # Weights are cached in the form their layer's kernel reads: bytes in
        # matrix-core operand order where the fused layer kernel applies, bit planes
        # for the two-kernel path.
        self.w_layout = [B.RIGHT_BYTES if weights_as_bytes and fused_layer_applies(d, h, s, t) else B.RIGHT
                         for d, h in self.dims]
        self.W = [B.alloc_bits(d, h, t, lay) for (d, h), lay in zip(self.dims, self.w_layout)]
        self._W_planes = None
        n = self.A.rows
        dmax = max(d for d, _ in self.dims)
        ws_bytes = max(B.lib().qgtc_layer_workspace_bytes(n, d, h, s) for d, h in self.dims)
        self.workspace = torch.empty(ws_bytes // 4 + 1, dtype=torch.int32, device=self.A.words.device)
        # ping-pong buffers for the low-bit activations between layers
        hmax = max(h for _, h in self.dims)
        self.x_bufs = [B.alloc_bits(n, max(dmax, hmax), s, B.RIGHT) for _ in range(2)]
        self.pack_static()

    def pack_static(self):
        """Everything that does not depend on the features: pack A, build its
        zero-tile map, quantize and pack the weights (the paper caches these
        across layers and subgraphs, end of Section 3.2)."""
        if self.A_src is not None:
            B.qgtc_pack_bits(self.A_src, 1, B.LEFT, out=self.A)
        if self.use_map:
            self.map = B.qgtc_build_tile_map(self.A, 16, self.tile_kbits, out=self.map)
            self.deg = self.map.deg
        else:
            self.deg = B.qgtc_row_sums(self.A)
        for W, r, dst, lay in zip(self.Ws, self.w_ranges, self.W, self.w_layout):
            B.qgtc_pack_bits(W, self.t, lay, quant=r, out=dst)
        # only the last layer dequantizes, so only its column sums are needed
        self.w_colsum = [None] * (len(self.W) - 1) + [B.qgtc_col_sums(self.W[-1])]

    # -- helpers -----------------------------------------------------------------
    def _x_view(self, which: int, cols: int) -> B.Bits:
        """A [N, cols] RIGHT-packed view on one of the activation buffers."""
        buf = self.x_bufs[which]
        d, _ = B.describe(self.A.rows, cols, self.s, B.RIGHT)
        d.data = buf.words.data_ptr()
        return B.Bits(buf.words, d)

    def pack_input(self, X: torch.Tensor, x_range) -> B.Bits:
        return B.qgtc_pack_bits(X, self.s, B.RIGHT, quant=x_range,
                                out=self._x_view(0, X.shape[1]))

    def _agg_ep(self, agg_hi: int) -> B.Epilogue:
        return B.Epilogue(mode=B.OUT_BITS, rq_nbits=self.s, rq_lo=0,
                          rq_inv_scale=inv_scale(0.0, float(agg_hi), self.s),
                          self_term=self.self_term)

    # -- calibration: integer maxima per layer, from int32 outputs ---------------------
    def calibrate(self, X: torch.Tensor, x_range):
        """Runs the stack once with int32 outputs and returns LayerRanges per
        layer (range = [0, max observed accumulator], at least 1)."""
        ranges = []
        xb = self.pack_input(X, x_range)
        if self._W_planes is None:          # qgtc_update reads bit planes
            self._W_planes = [B.qgtc_pack_bits(W, self.t, B.RIGHT, quant=r)
                              for W, r in zip(self.Ws, self.w_ranges)]
        for l, W in enumerate(self._W_planes):
            y32 = B.qgtc_aggregate(self.A, self.map, xb,
                                   B.Epilogue(mode=B.OUT_I32, self_term=self.self_term))
            agg_hi = max(1, int(y32.max()))
            yb = B.qgtc_aggregate(self.A, self.map, xb, self._agg_ep(agg_hi))
            z32 = B.qgtc_update(yb, W, B.Epilogue(mode=B.OUT_I32))
            last = l == len(self.W) - 1
            out_hi = None if last else max(1, int(z32.max()))
            ranges.append(LayerRanges(agg_hi, out_hi))
            if not last:
                ep = B.Epilogue(mode=B.OUT_BITS, relu=True, rq_nbits=self.s, rq_lo=0,
                                rq_inv_scale=inv_scale(0.0, float(out_hi), self.s))
                xb = B.qgtc_update(yb, W, ep, out=self._x_view((l + 1) & 1, self.dims[l][1]))
        return ranges

    # -- forward ---------------------------------------------------------------------
    def last_layer_dequant(self, l: int, x_lo: float, x_scale: float, agg_hi: int,
                           yq_rowsum: torch.Tensor) -> B.Epilogue:
        """Epilogue that turns the last update's accumulators into the real
        product of the dequantized operands: Y^ = l0[v] + sl*Yq, W^ = lo_w + sw*Wq."""
        d = self.dims[l][0]
        lo_w, hi_w = self.w_ranges[l]
        sw = (hi_w - lo_w) / float(2 ** self.t)
        inv = inv_scale(0.0, float(agg_hi), self.s)
        sl = x_scale / inv
        return B.Epilogue(mode=B.OUT_F32, cc=sl * sw, rs=sl * lo_w, row_i=yq_rowsum,
                          l0a=(x_lo if self.self_term else 0.0), l0b=x_lo, row_l=self.deg,
                          ck=lo_w * d, cs=sw, col_i=self.w_colsum[l])

    def forward(self, X: torch.Tensor, x_range, ranges, out: torch.Tensor | None = None,
                want_int: bool = False):
        """fp32 [N, H_last] (or the last int32 accumulators when want_int)."""
        xb = self.pack_input(X, x_range)
        n_layers = len(self.W)
        x_lo = float(x_range[0])
        x_scale = (float(x_range[1]) - float(x_range[0])) / float(2 ** self.s)
        for l, W in enumerate(self.W):
            r = ranges[l]
            agg_ep = self._agg_ep(r.agg_hi)
            if l < n_layers - 1:
                ep = B.Epilogue(mode=B.OUT_BITS, relu=True, rq_nbits=self.s, rq_lo=0,
                                rq_inv_scale=inv_scale(0.0, float(r.out_hi), self.s))
                xb = B.qgtc_layer(self.A, self.map, xb, W, agg_ep, ep, self.workspace,
                                  out=self._x_view((l + 1) & 1, self.dims[l][1]))
                # hidden activations are read as pure scales: x^ = Xq * step
                lo_w, hi_w = self.w_ranges[l]
                sw = (hi_w - lo_w) / float(2 ** self.t)
                x_scale = (x_scale / inv_scale(0.0, float(r.agg_hi), self.s)) * sw \
                    / inv_scale(0.0, float(r.out_hi), self.s)
                x_lo = 0.0
            elif want_int:
                return B.qgtc_layer(self.A, self.map, xb, W, agg_ep, B.Epilogue(mode=B.OUT_I32),
                                    self.workspace, out=out)
            else:
                # row_i = None: the layer takes the row sums of its own requantized Y
                ep = self.last_layer_dequant(l, x_lo, x_scale, r.agg_hi, None)
                return B.qgtc_layer(self.A, self.map, xb, W, agg_ep, ep, self.workspace, out=out)
