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
    return B.qgtc_quant_inv_scale(lo, hi, nbits)


@dataclass
class LayerRanges:
    agg_hi: int          # requantization range [0, agg_hi) of the aggregation result
    out_hi: float | None # range [0, out_hi) of the update result (hidden layers): in units of
                         # the accumulator, or of the real value behind a batch normalization


@dataclass
class BatchNorm:
    """Inference-time batch normalization after a layer (Section 4.5): per output
    column gamma, beta and the running mean / variance, as sequences of floats."""
    gamma: object
    beta: object
    mean: object
    var: object
    eps: float = 1e-5


def plan_adjacency(A: "B.Bits", d: int = 64, h: int = 64, s: int = 8, t: int = 8) -> dict:
    """The library's selector on a packed adjacency: one pass over A counts its non-zero
    tiles at the three widths and its non-zero (row, word) pairs (qgtc_tile_stats), the host
    reads the numbers back once (this synchronizes) and qgtc_plan_layer picks the tile width
    with the least executed work and says whether jumping over the zero words inside kept
    tiles pays.  Narrow tiles skip more zeros (the paper's second kind of zero tiles, gaps
    inside a subgraph, Section 6.3) but cost more per bit."""
    st = B.tile_stats_numbers(B.qgtc_tile_stats(A))
    plan = B.qgtc_plan_layer(A.rows, d, h, s, t, n_tile_rows=st["n_tile_rows"], a_cols=A.cols,
                             nnz_tiles=st["nnz_tiles"], nnz_row_words=st["nnz_row_words"])
    plan.update(st)
    return plan


def choose_tile_kbits(A: "B.Bits", d: int = 64, h: int = 64, s: int = 8, t: int = 8) -> int:
    """Tile width for the zero-tile map of a packed adjacency (plan_adjacency)."""
    return plan_adjacency(A, d, h, s, t)["tile_kbits"]


def fused_layer_applies(d: int, h: int, s: int, t: int) -> bool:
    """The shapes and bit widths qgtc_layer runs as one kernel (the selector's rule)."""
    return bool(B.qgtc_plan_layer(16, d, h, s, t)["fused"])


class QuantGNN:
    """A stack of quantized layers on one batch of subgraphs.

    A_src: uint8 0/1 device tensor, [N, N] (block_rows = 0) or [N, block_rows]
           (one row of diagonal blocks, see qgtc_bits.block_rows), or an already
           packed adjacency (Bits)
    Ws:    list of fp32 device tensors [D_l, H_l]; quantized to t bits by min-max
    """

    def __init__(self, A_src, Ws, s: int, t: int, self_term: bool,
                 tile_kbits: int | str = 128, use_map: bool = True, block_rows: int = 0,
                 weights_as_bytes: bool = True, update_first: bool = False, batchnorm=None,
                 tuning: "B.Tuning | None" = None):
        self.s, self.t = s, t
        self.tuning = tuning           # per-call speed choices handed to qgtc_layer (None: the library's)
        # batchnorm: per layer None or a BatchNorm; it is folded into the layer's output
        # epilogue as a per-column affine map (no kernel of its own)
        self.batchnorm = list(batchnorm) if batchnorm is not None else [None] * len(Ws)
        assert len(self.batchnorm) == len(Ws)
        assert not (update_first and any(b is not None for b in self.batchnorm))
        self._bn_cache = {}
        # update_first: every layer computes A.(X.W) instead of (A.X).W (Section 6.1: GIN
        # updates before it aggregates); it runs as qgtc_update + qgtc_aggregate on planes
        self.update_first = update_first
        if update_first:
            weights_as_bytes = False
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
        # The selector's choices that depend on the adjacency (tile width when "auto", zero-word
        # jumping unless the caller's tuning says which): pack A now, read its statistics once.
        self.plan = None
        if tile_kbits == "auto" or tuning is None or tuning.zero_words == 0:
            if self.A_src is not None:
                B.qgtc_pack_bits(self.A_src, 1, B.LEFT, out=self.A)
            self.plan = plan_adjacency(self.A, self.dims[0][0], self.dims[0][1], s, t)
            if tile_kbits == "auto":
                self.tile_kbits = self.plan["tile_kbits"]
            base = tuning or B.Tuning()
            self.tuning = B.Tuning(update_path=base.update_path, agg_xcd_run=base.agg_xcd_run,
                                   layer_path=base.layer_path, layer_ksplit=base.layer_ksplit,
                                   zero_words=base.zero_words or self.plan["zero_words"],
                                   even_progress=base.even_progress)
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
        if update_first:                 # activations between layers as left operands of the update
            self.xl_bufs = [B.alloc_bits(n, max(dmax, hmax), s, B.LEFT) for _ in range(2)]
        self.pack_static()

    def pack_static(self, X: torch.Tensor | None = None, x_range=None):
        """Everything that does not depend on the features: pack A, build its
        zero-tile map, quantize and pack the weights (the paper caches these
        across layers and subgraphs, end of Section 3.2).  With X: the input features
        of the coming forward pass are quantized and packed as well, after the weights
        on their stream (forward(..., x_packed=True) then skips that step)."""
        # The weights are a handful of small launches that do not depend on the adjacency:
        # they go to a second stream (forked from and joined to the current one, also
        # inside a HIP graph) and run beside the HBM-bound packing of A and its map.
        cur = torch.cuda.current_stream()
        if getattr(self, "_w_stream", None) is None:
            self._w_stream = torch.cuda.Stream()
            self._w_colsum_buf = torch.empty(self.dims[-1][1], dtype=torch.int32, device=self.A.words.device)
        self._w_stream.wait_stream(cur)
        with torch.cuda.stream(self._w_stream):
            for W, r, dst, lay in zip(self.Ws, self.w_ranges, self.W, self.w_layout):
                B.qgtc_pack_bits(W, self.t, lay, quant=r, out=dst)
            # only the last layer dequantizes, so only its column sums are needed
            self.w_colsum = [None] * (len(self.W) - 1) + [B.qgtc_col_sums(self.W[-1], out=self._w_colsum_buf)]
            if X is not None and not self.update_first:
                self.pack_input(X, x_range)
        if self.A_src is not None:
            B.qgtc_pack_bits(self.A_src, 1, B.LEFT, out=self.A)
        if self.use_map:
            self.map = B.qgtc_build_tile_map(self.A, 16, self.tile_kbits, out=self.map)
            self.deg = self.map.deg
        else:
            self.deg = B.qgtc_row_sums(self.A)
        cur.wait_stream(self._w_stream)

    # -- helpers -----------------------------------------------------------------
    def _x_view(self, which: int, cols: int) -> B.Bits:
        """A [N, cols] RIGHT-packed view on one of the activation buffers.  Every view has
        the strides of the widest layer, so that a range of rows is the same range of
        words whatever the layer (independent runs of rows work on the buffers at once)."""
        buf = self.x_bufs[which]
        d, _ = B.describe(self.A.rows, cols, self.s, B.RIGHT)
        d.ld_words = buf.c.ld_words
        d.plane_stride_words = buf.c.plane_stride_words
        d.data = buf.words.data_ptr()
        return B.Bits(buf.words, d)

    # -- independent batches of subgraphs -------------------------------------------------
    def _chunks(self, n_chunks: int):
        """Splits the batch into runs of whole subgraphs (block-diagonal storage only):
        per run the row range, a view of A and a view of the tile map.  Subgraphs share
        no edge (Section 4.1), so the runs are independent from the first layer to the
        last and can be issued on different streams."""
        key = (str(n_chunks), self.map.c.row_cnt if self.map is not None else 0)
        if getattr(self, "_chunk_cache", (None, None))[0] == key:
            return self._chunk_cache[1]
        br = self.A.c.block_rows
        assert br > 0 and br % 32 == 0, "independent runs need the block-diagonal storage"
        n = self.A.rows
        n_blocks = -(-n // br)
        if isinstance(n_chunks, int):                 # equal runs
            per = -(-n_blocks // n_chunks)
            sizes = [per] * n_chunks
        else:                                         # subgraphs per run, in order
            sizes = list(n_chunks)
            assert sum(sizes) >= n_blocks
        bounds, b0 = [], 0
        for sz in sizes:
            if b0 < n_blocks and sz > 0:
                bounds.append((b0 * br, min(n, (b0 + sz) * br)))
            b0 += sz
        out = []
        for r0, r1 in bounds:
            a = B._BitsC.from_buffer_copy(self.A.c)
            a.data = self.A.c.data + r0 * self.A.c.ld_words * 4
            a.rows = r1 - r0
            m = None
            if self.map is not None:
                mc = B._TileMapC.from_buffer_copy(self.map.c)
                t0 = r0 // mc.tile_rows
                mc.n_tile_rows = -(-(r1 - r0) // mc.tile_rows)
                mc.row_cnt = self.map.c.row_cnt + 4 * t0
                mc.col_idx = self.map.c.col_idx + 4 * t0 * mc.n_tile_cols
                mc.deg = self.map.c.deg + 4 * r0
                m = B.TileMap(self.map.buffer, mc, r1 - r0)
            out.append((r0, r1, B.Bits(self.A.words, a), m))
        self._chunk_cache = (key, out)
        return out

    def _x_rows(self, which: int, cols: int, r0: int, r1: int) -> B.Bits:
        """Rows [r0, r1) (r0 a multiple of 32) of the [N, cols] view of an activation buffer."""
        full = self._x_view(which, cols)
        d = B._BitsC.from_buffer_copy(full.c)
        d.data = full.c.data + (r0 // 32) * full.c.ld_words * 4
        d.rows = r1 - r0
        return B.Bits(full.words, d)

    def pack_input(self, X: torch.Tensor, x_range) -> B.Bits:
        return B.qgtc_pack_bits(X, self.s, B.RIGHT, quant=x_range,
                                out=self._x_view(0, X.shape[1]))

    def _agg_ep(self, agg_hi: int) -> B.Epilogue:
        return B.Epilogue(mode=B.OUT_BITS, rq_nbits=self.s, rq_lo=0,
                          rq_inv_scale=inv_scale(0.0, float(agg_hi), self.s),
                          self_term=self.self_term)

    def _layer_eps(self, l: int, x_lo: float, x_scale: float, agg_hi, out_hi, last: bool):
        """The two epilogues of layer l and the scales around it, from the library's helper."""
        return B.qgtc_layer_epilogues(self.s, self.t, self.dims[l][0], x_lo, x_scale, self.w_ranges[l],
                                      agg_hi, out_hi, self_term=self.self_term, last=last,
                                      batchnorm=self.batchnorm[l] is not None and not last,
                                      update_first=self.update_first)

    # -- update first ---------------------------------------------------------------------
    def _xl_view(self, which: int, cols: int) -> B.Bits:
        buf = self.xl_bufs[which]
        d, _ = B.describe(self.A.rows, cols, self.s, B.LEFT)
        d.plane_stride_words = buf.c.plane_stride_words
        d.data = buf.words.data_ptr()
        return B.Bits(buf.words, d)

    def _forward_update_first(self, X, x_range, ranges, out, want_int):
        """Per layer: P = X.W (qgtc_update, planes packed along the nodes out) ->
        A.P (qgtc_aggregate; hidden layers emit planes packed along the features, the
        left operand of the next update).  With ranges = None the int32 maxima are
        collected on the way and returned as LayerRanges (agg_hi: range of P)."""
        calibrating = ranges is None
        found = []
        if self.s <= 8 and self.t <= 8:
            # the input goes straight to the int8 matrix cores: codes as bytes, no bit planes
            if getattr(self, "_x_bytes", None) is None:
                self._x_bytes = B.alloc_bits(X.shape[0], X.shape[1], self.s, B.LEFT_BYTES)
            xl = B.qgtc_pack_bits(X, self.s, B.LEFT_BYTES, quant=x_range, out=self._x_bytes)
        else:
            xl = B.qgtc_pack_bits(X, self.s, B.LEFT, quant=x_range, out=self._xl_view(0, X.shape[1]))
        n_layers = len(self.W)
        x_scale = (float(x_range[1]) - float(x_range[0])) / float(2 ** self.s)
        for l, W in enumerate(self.W):
            d, h = self.dims[l]
            last = l == n_layers - 1
            if calibrating:
                p32 = B.qgtc_update(xl, W, B.Epilogue(mode=B.OUT_I32))
                p_hi = max(1, int(p32.max()))
            else:
                p_hi = ranges[l].agg_hi
            # epilogue of X.W (requantize to s bits) - only its range is known while calibrating
            upd_ep, _, _, _ = self._layer_eps(l, 0.0, x_scale, p_hi, 1.0, last=False)
            pb = B.qgtc_update(xl, W, upd_ep, out=self._x_view(l & 1, h))
            out_hi = None
            if calibrating or (last and want_int):
                z32 = B.qgtc_aggregate(self.A, self.map, pb,
                                       B.Epilogue(mode=B.OUT_I32, self_term=self.self_term),
                                       out=out if (last and want_int and not calibrating) else None)
                if calibrating and not last:
                    out_hi = max(1, int(z32.max()))
            if calibrating:
                found.append(LayerRanges(p_hi, out_hi))
            else:
                out_hi = ranges[l].out_hi
            if last:
                if calibrating:
                    return found
                if not want_int:
                    # codes read as pure scales (no zero points): out = z_scale * (A.Pq)
                    _, agg_ep, _, _ = self._layer_eps(l, 0.0, x_scale, p_hi, None, last=True)
                    agg_ep.tuning = self.tuning
                    B.qgtc_aggregate(self.A, self.map, pb, agg_ep, out=out)
                return out
            _, agg_ep, _, x_scale = self._layer_eps(l, 0.0, x_scale, p_hi, out_hi, last=False)
            agg_ep.tuning = self.tuning
            xl = B.qgtc_aggregate(self.A, self.map, pb, agg_ep, out=self._xl_view((l + 1) & 1, h))

    def _bn_fold(self, l: int, value_scale: float):
        """(col_scale, col_shift) of layer l's batch normalization acting on value_scale * C
        (qgtc_fold_batchnorm).  Cached per scale so that a recorded pass allocates nothing."""
        key = (l, float(value_scale))
        if key not in self._bn_cache:
            bn = self.batchnorm[l]
            a, b = B.qgtc_fold_batchnorm(bn.gamma, bn.beta, bn.mean, bn.var, bn.eps, value_scale)
            dv = self.A.words.device
            self._bn_cache[key] = (a.to(dv), b.to(dv))
        return self._bn_cache[key]

    # -- calibration: integer maxima per layer, from int32 outputs ---------------------
    def calibrate(self, X: torch.Tensor, x_range):
        """Runs the stack once with int32 outputs and returns LayerRanges per
        layer (range = [0, max observed accumulator], at least 1)."""
        if self.update_first:
            return self._forward_update_first(X, x_range, None, None, False)
        ranges = []
        xb = self.pack_input(X, x_range)
        if self._W_planes is None:          # qgtc_update reads bit planes
            self._W_planes = [B.qgtc_pack_bits(W, self.t, B.RIGHT, quant=r)
                              for W, r in zip(self.Ws, self.w_ranges)]
        x_scale = (float(x_range[1]) - float(x_range[0])) / float(2 ** self.s)
        for l, W in enumerate(self._W_planes):
            y32 = B.qgtc_aggregate(self.A, self.map, xb,
                                   B.Epilogue(mode=B.OUT_I32, self_term=self.self_term))
            agg_hi = max(1, int(y32.max()))
            yb = B.qgtc_aggregate(self.A, self.map, xb, self._agg_ep(agg_hi))
            z32 = B.qgtc_update(yb, W, B.Epilogue(mode=B.OUT_I32))
            last = l == len(self.W) - 1
            if last:
                ranges.append(LayerRanges(agg_hi, None))
                break
            _, _, z_scale, _ = self._layer_eps(l, 0.0, x_scale, agg_hi, 1.0, last=False)
            ca = cb = None
            if self.batchnorm[l] is not None:
                # range of the normalized value, [0, max(a_j * z + b_j)]
                ca, cb = self._bn_fold(l, z_scale)
                v = z32.to(torch.float64) * ca.to(torch.float64)[None, :] + cb.to(torch.float64)[None, :]
                out_hi = max(1e-6, float(v.max()))
            else:
                out_hi = max(1, int(z32.max()))
            ranges.append(LayerRanges(agg_hi, out_hi))
            _, ep, _, x_scale = self._layer_eps(l, 0.0, x_scale, agg_hi, out_hi, last=False)
            ep.col_scale, ep.col_shift = ca, cb
            xb = B.qgtc_update(yb, W, ep, out=self._x_view((l + 1) & 1, self.dims[l][1]))
        return ranges

    # -- forward ---------------------------------------------------------------------
    def forward(self, X: torch.Tensor, x_range, ranges, out: torch.Tensor | None = None,
                want_int: bool = False, streams: int = 1, x_packed: bool = False,
                x_bits: B.Bits | None = None):
        """fp32 [N, H_last] (or the last int32 accumulators when want_int).

        streams > 1 (block-diagonal storage): the subgraphs are cut into that many
        independent runs, each issued on a stream of its own, so that the start and the
        drain of one run's kernels overlap with the other runs' work.  A list gives the
        number of subgraphs of each run instead ([48, 16]: the first 48, then 16); "auto"
        takes auto_runs() (resolve it before recording a graph: it reads the tile map back).
        x_packed: the features are already packed (pack_static(X, x_range)).
        x_bits: the features as packed planes that live elsewhere (a SubgraphPacket's,
        packed on the host with the same x_range); X is then not read (single run only)."""
        n = self.A.rows
        if streams == "auto":
            streams = self.auto_runs()
        if out is None:
            out = torch.empty((n, self.dims[-1][1]), dtype=torch.int32 if want_int else torch.float32,
                              device=self.A.words.device)
        if self.update_first:
            return self._forward_update_first(X, x_range, ranges, out, want_int)
        if x_bits is not None:
            assert isinstance(streams, int) and streams <= 1
            xb = x_bits
        else:
            xb = self._x_view(0, X.shape[1]) if x_packed else self.pack_input(X, x_range)
        if (isinstance(streams, int) and streams <= 1) or self.A.c.block_rows == 0:
            self._run_layers(0, n, self.A, self.map, self.deg, xb, x_range, ranges, out, want_int,
                             self.workspace)
            return out
        chunks = self._chunks(streams)
        if getattr(self, "_streams", None) is None or len(self._streams) < len(chunks):
            self._streams = [torch.cuda.Stream() for _ in chunks]
            ws_words = self.workspace.numel()
            self._chunk_ws = [torch.empty(ws_words, dtype=torch.int32, device=self.A.words.device)
                              for _ in chunks]
        cur = torch.cuda.current_stream()
        packed = torch.cuda.Event()
        packed.record(cur)
        for (r0, r1, a, m), st, ws in zip(chunks, self._streams, self._chunk_ws):
            st.wait_event(packed)
            with torch.cuda.stream(st):
                x0 = self._x_rows(0, X.shape[1], r0, r1)
                self._run_layers(r0, r1, a, m, self.deg[r0:r1], x0, x_range, ranges, out[r0:r1],
                                 want_int, ws)
            done = torch.cuda.Event()
            done.record(st)
            cur.wait_event(done)
        return out

    def capture(self, X: torch.Tensor, x_range, ranges, out: torch.Tensor, streams: int = 1,
                with_static: bool = False, want_int: bool = False) -> torch.cuda.CUDAGraph:
        """Records one pass (optionally with pack_static in front) into a HIP graph; replay()
        runs it again on the same buffers: X and out are read and written in place.  The
        library's launches are plain kernel launches on the current stream (no memset, no
        synchronization), the runs on side streams fork from and join the capturing stream
        through events, so the whole pass is one graph launch for the host."""
        if streams == "auto":
            streams = self.auto_runs()

        def run():
            if with_static:
                self.pack_static(X, x_range)
            self.forward(X, x_range, ranges, out=out, want_int=want_int, streams=streams,
                         x_packed=with_static and not self.update_first)

        cur = torch.cuda.current_stream()
        side = torch.cuda.Stream()
        side.wait_stream(cur)
        with torch.cuda.stream(side):      # warm-up outside the capture: allocations, code loading
            run()
            run()
        cur.wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run()
        return graph

    def auto_runs(self) -> int:
        """Independent runs of subgraphs to issue a forward pass as: the selector's `runs` of
        the layers that hold most of the aggregation work (each layer's answer weighted by the
        columns it aggregates), 1 unless the adjacency is stored block-diagonally and the two
        halves of the batch hold the same work within 15 % (the tile counts are read back
        once: this synchronizes; call it at set-up)."""
        if getattr(self, "_auto_runs", None) is not None:
            return self._auto_runs
        runs = 1
        br = self.A.c.block_rows
        if br > 0 and br % 32 == 0 and self.map is not None and not self.update_first:
            n_blocks = -(-self.A.rows // br)
            votes = {1: 0, 2: 0}
            for l, (d, _) in enumerate(self.dims):
                votes[self._batch_plan(l, n_blocks)["runs"]] += d
            runs = 2 if votes[2] > votes[1] else 1
            if runs > 1:
                cnt = self.map.row_cnt.cpu().to(torch.int64) + 1       # a tile row: its tiles plus a fixed part
                half = (n_blocks // 2) * br // 16
                a, b = int(cnt[:half].sum()), int(cnt[half:].sum())
                if max(a, b) > 1.15 * min(a, b):
                    runs = 1
        self._auto_runs = runs
        return runs

    def _batch_plan(self, l: int, subgraphs: int = 0) -> dict:
        """The selector on layer l over the whole batch, with the adjacency's statistics when
        the constructor read them."""
        d, h = self.dims[l]
        st = self.plan or {}
        tiles = st.get("nnz_tiles", (0, 0, 0))
        row_words = st.get("nnz_row_words", 0)
        if self.tuning is not None and self.tuning.zero_words == B.ZERO_WORDS_VISIT and row_words:
            # the caller fixed the form that visits every word: plan as for an adjacency whose
            # words all hold a bit
            row_words = 16 * max(tiles[0], 2 * tiles[1], 4 * tiles[2])
        return B.qgtc_plan_layer(self.A.rows, d, h, self.s, self.t, n_tile_rows=-(-self.A.rows // 16),
                                 a_cols=self.A.cols, nnz_tiles=tiles, nnz_row_words=row_words, subgraphs=subgraphs)

    def _run_tuning(self, l: int, whole_batch: bool):
        """Tuning of layer l.  A run that covers part of the batch shares the device with the
        other runs: it takes the K split and the issue-priority choice the whole batch would
        get from the selector, not the ones its own (smaller) number of tile rows suggests -
        those would split the tile lists to fill a device the other runs are already filling,
        and treat a launch as alone on the device that is not."""
        if whole_batch or (self.tuning is not None and self.tuning.layer_ksplit):
            return self.tuning
        plan = self._batch_plan(l)
        base = self.tuning or B.Tuning()
        # (the selector's wave-slot count assumes its own choice of kernel form: where the
        # caller fixed another one, the priority scheme stays off)
        same_form = plan["zero_words"] == 0 or base.zero_words in (0, plan["zero_words"])
        return B.Tuning(update_path=base.update_path, agg_xcd_run=base.agg_xcd_run, layer_path=base.layer_path,
                        layer_ksplit=plan["ksplit"], zero_words=base.zero_words,
                        even_progress=base.even_progress or (plan["even_progress"] if same_form else 1))

    def _run_layers(self, r0, r1, A, tmap, deg, xb, x_range, ranges, out, want_int, workspace):
        """All layers on rows [r0, r1) (whole subgraphs), on the current stream."""
        n_layers = len(self.W)
        whole = r0 == 0 and r1 == self.A.rows
        # the first layer's codes stand for x_lo + x_scale * code; behind a hidden layer the
        # codes are read as pure scales (x_lo = 0)
        x_lo = float(x_range[0])
        x_scale = (float(x_range[1]) - float(x_range[0])) / float(2 ** self.s)
        for l, W in enumerate(self.W):
            r = ranges[l]
            last = l == n_layers - 1
            agg_ep, ep, z_scale, x_next = self._layer_eps(l, x_lo, x_scale, r.agg_hi, r.out_hi, last)
            tuning = self._run_tuning(l, whole)
            ep.tuning = tuning
            if not last:
                if self.batchnorm[l] is not None:
                    ep.col_scale, ep.col_shift = self._bn_fold(l, z_scale)
                xb = B.qgtc_layer(A, tmap, xb, W, agg_ep, ep, workspace,
                                  out=self._x_rows((l + 1) & 1, self.dims[l][1], r0, r1))
                x_lo, x_scale = 0.0, x_next
            elif want_int:
                B.qgtc_layer(A, tmap, xb, W, agg_ep, B.Epilogue(mode=B.OUT_I32, tuning=tuning), workspace,
                             out=out)
            else:
                # row_i = None: the layer takes the row sums of its own requantized Y
                ep.row_l, ep.col_i = deg, self.w_colsum[l]
                if self.batchnorm[l] is not None:      # acts on the real output value
                    ep.col_scale, ep.col_shift = self._bn_fold(l, 1.0)
                B.qgtc_layer(A, tmap, xb, W, agg_ep, ep, workspace, out=out)
