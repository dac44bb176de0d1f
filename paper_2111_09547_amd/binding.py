"""ctypes binding of libqgtc.so: argument marshalling only.

The functions carry the names of the C entry points (see include/qgtc.h).
Device buffers are torch tensors; the current torch stream is passed to every
call.  The library is loaded on first use and the import fails loudly if it has
not been built (python -m paper_2111_09547_amd.build)."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field

import torch  # first: the HIP runtime PyTorch ships must be the one libqgtc binds to

LEFT, RIGHT, RIGHT_BYTES, LEFT_BYTES = 0, 1, 2, 3
SRC_F32, SRC_U8, SRC_I32 = 0, 1, 2
OUT_I32, OUT_F32, OUT_BITS = 0, 1, 2
KERNEL_PACK, KERNEL_TILE_MAP, KERNEL_AGGREGATE, KERNEL_UPDATE, KERNEL_SUMS, KERNEL_LAYER = range(6)

_STATUS = ["ok", "null pointer", "shape mismatch", "bit width out of range",
           "misaligned pointer or leading dimension", "wrong packed layout",
           "workspace too small", "unsupported request", "HIP runtime error"]


class QgtcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = _STATUS[status] if 0 <= status < len(_STATUS) else "unknown"
        super().__init__(f"{where}: status {status} ({name})")


class _BitsC(C.Structure):
    _fields_ = [("data", C.c_void_p), ("nbits", C.c_int32), ("rows", C.c_int32),
                ("cols", C.c_int32), ("layout", C.c_int32), ("block_rows", C.c_int32),
                ("reserved", C.c_int32), ("ld_words", C.c_int64),
                ("plane_stride_words", C.c_int64)]


class _QuantC(C.Structure):
    _fields_ = [("lo", C.c_double), ("hi", C.c_double), ("nbits", C.c_int32)]


class _TileMapC(C.Structure):
    _fields_ = [("tile_rows", C.c_int32), ("tile_kbits", C.c_int32),
                ("n_tile_rows", C.c_int32), ("n_tile_cols", C.c_int32),
                ("row_cnt", C.c_void_p), ("col_idx", C.c_void_p),
                ("nnz_tiles", C.c_void_p), ("deg", C.c_void_p)]


class _TuningC(C.Structure):
    _fields_ = [("update_path", C.c_int32), ("agg_xcd_run", C.c_int32),
                ("layer_path", C.c_int32), ("layer_ksplit", C.c_int32),
                ("zero_words", C.c_int32), ("even_progress", C.c_int32)]


class _EpilogueC(C.Structure):
    _fields_ = [("mode", C.c_int32), ("relu", C.c_int32), ("self_term", C.c_int32),
                ("rq_nbits", C.c_int32), ("rq_lo", C.c_int32), ("rq_inv_scale", C.c_float),
                ("cc", C.c_double), ("rs", C.c_double), ("l0a", C.c_double),
                ("l0b", C.c_double), ("ck", C.c_double), ("cs", C.c_double),
                ("row_i", C.c_void_p), ("row_l", C.c_void_p), ("col_i", C.c_void_p),
                ("col_scale", C.c_void_p), ("col_shift", C.c_void_p),
                ("tuning", C.POINTER(_TuningC))]


class _PlanInC(C.Structure):
    _fields_ = [("rows", C.c_int32), ("in_cols", C.c_int32), ("out_cols", C.c_int32),
                ("s", C.c_int32), ("t", C.c_int32), ("n_tile_rows", C.c_int32),
                ("a_cols", C.c_int32), ("subgraphs", C.c_int32), ("nnz_tiles", C.c_int64 * 3),
                ("nnz_row_words", C.c_int64)]


class _PlanOutC(C.Structure):
    _fields_ = [("tile_kbits", C.c_int32), ("fused", C.c_int32), ("update_path", C.c_int32),
                ("ksplit", C.c_int32), ("est_us_aggregate_first", C.c_double),
                ("est_us_update_first", C.c_double), ("runs", C.c_int32), ("zero_words", C.c_int32),
                ("even_progress", C.c_int32), ("reserved", C.c_int32)]


class _LayerSpecC(C.Structure):
    _fields_ = [("s", C.c_int32), ("t", C.c_int32), ("in_cols", C.c_int32), ("order", C.c_int32),
                ("self_term", C.c_int32), ("last", C.c_int32), ("batchnorm", C.c_int32),
                ("reserved", C.c_int32), ("x_lo", C.c_double), ("x_scale", C.c_double),
                ("w_lo", C.c_double), ("w_hi", C.c_double), ("agg_hi", C.c_double),
                ("out_hi", C.c_double)]


class _DeviceC(C.Structure):
    _fields_ = [("compute_units", C.c_int32), ("xcds", C.c_int32), ("is_gfx950", C.c_int32),
                ("xcds_assumed", C.c_int32)]


_lib = None


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libqgtc.so")


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with "
                          "`python -m paper_2111_09547_amd.build` (needs hipcc)")
    l = C.CDLL(path)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    P = C.POINTER
    sig = {
        "qgtc_status_string": (C.c_char_p, [C.c_int]),
        "qgtc_version": (i32, []),
        "qgtc_describe": (sz, [P(_BitsC), i32, i32, i32, i32, i32]),
        "qgtc_pack_bits": (C.c_int, [vp, i32, i32, i32, i64, P(_QuantC), P(_BitsC), vp]),
        "qgtc_unpack_bits": (C.c_int, [P(_BitsC), vp, i64, vp]),
        "qgtc_pack_bits_host": (C.c_int, [vp, i32, i32, i32, i64, P(_QuantC), P(_BitsC), i32]),
        "qgtc_compound_layout": (sz, [P(sz), i32, P(sz)]),
        "qgtc_row_sums": (C.c_int, [P(_BitsC), vp, vp]),
        "qgtc_col_sums": (C.c_int, [P(_BitsC), vp, vp]),
        "qgtc_tile_map_bytes": (sz, [i32, i32, i32, i32]),
        "qgtc_tile_map_carve": (C.c_int, [P(_TileMapC), vp, i32, i32, i32, i32]),
        "qgtc_build_tile_map": (C.c_int, [P(_BitsC), P(_TileMapC), vp]),
        "qgtc_aggregate": (C.c_int, [P(_BitsC), P(_TileMapC), P(_BitsC), P(_EpilogueC), vp, i64, vp]),
        "qgtc_update": (C.c_int, [P(_BitsC), P(_BitsC), P(_EpilogueC), vp, i64, vp]),
        "qgtc_layer_workspace_bytes": (sz, [i32, i32, i32, i32]),
        "qgtc_layer": (C.c_int, [P(_BitsC), P(_TileMapC), P(_BitsC), P(_BitsC), P(_EpilogueC),
                                 P(_EpilogueC), vp, sz, vp, i64, vp]),
        "qgtc_layer_static": (C.c_int, [P(_BitsC), P(_TileMapC), P(_BitsC), P(_BitsC), P(_EpilogueC),
                                        P(_EpilogueC), vp, i64, vp]),
        "qgtc_tile_stats": (C.c_int, [P(_BitsC), vp, vp]),
        "qgtc_plan_layer": (C.c_int, [P(_PlanInC), P(_PlanOutC)]),
        "qgtc_quant_inv_scale": (C.c_float, [C.c_double, C.c_double, i32]),
        "qgtc_layer_epilogues": (C.c_int, [P(_LayerSpecC), P(_EpilogueC), P(_EpilogueC),
                                          P(C.c_double), P(C.c_double)]),
        "qgtc_fold_batchnorm": (C.c_int, [P(C.c_double), P(C.c_double), P(C.c_double), P(C.c_double),
                                         C.c_double, C.c_double, i32, P(C.c_float), P(C.c_float)]),
        "qgtc_device_info": (C.c_int, [P(_DeviceC)]),
        "qgtc_probe_popcount": (C.c_int, [i32, i32, i32, C.c_void_p, C.c_void_p]),
        "qgtc_prof_enable": (C.c_int, [i32]),
        "qgtc_prof_reset": (C.c_int, []),
        "qgtc_prof_read": (C.c_int, [i32, P(C.c_double), P(i64)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(l, name)          # AttributeError if the symbol is missing
        fn.restype = res
        fn.argtypes = args
    _lib = l
    return l


def _check(status: int, where: str):
    if status != 0:
        raise QgtcError(status, where)


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


# ---------------------------------------------------------------- descriptors
@dataclass
class Bits:
    """Packed bit planes on the device: the words (a torch int32 tensor that owns
    the memory) plus the descriptor the library takes."""
    words: torch.Tensor
    c: _BitsC

    @property
    def rows(self): return self.c.rows
    @property
    def cols(self): return self.c.cols
    @property
    def nbits(self): return self.c.nbits
    @property
    def layout(self): return self.c.layout


@dataclass
class TileMap:
    buffer: torch.Tensor
    c: _TileMapC
    rows: int

    def _view(self, ptr, n):
        off = (ptr - self.buffer.data_ptr()) // 4
        return self.buffer[off:off + n]

    @property
    def row_cnt(self): return self._view(self.c.row_cnt, self.c.n_tile_rows)
    @property
    def col_idx(self):
        return self._view(self.c.col_idx, self.c.n_tile_rows * self.c.n_tile_cols) \
            .view(self.c.n_tile_rows, self.c.n_tile_cols)
    @property
    def nnz_tiles(self): return self._view(self.c.nnz_tiles, 2)
    @property
    def deg(self): return self._view(self.c.deg, self.rows)


@dataclass
class Tuning:
    """Per-call choices that only affect speed (qgtc_tuning); zeros leave them to the library."""
    update_path: int = 0      # UPDATE_AUTO / UPDATE_POPCOUNT / UPDATE_MATRIX_CORES
    agg_xcd_run: int = 0
    layer_path: int = 0       # LAYER_FUSED / LAYER_TWO_KERNELS
    layer_ksplit: int = 0
    zero_words: int = 0       # ZERO_WORDS_AUTO / ZERO_WORDS_VISIT / ZERO_WORDS_SKIP
    even_progress: int = 0    # 0 automatic, 1 off, 2 on (issue priority by remaining work in the fused kernel's tile loop)


@dataclass
class Epilogue:
    mode: int = OUT_I32
    relu: bool = False
    self_term: bool = False
    rq_nbits: int = 0
    rq_lo: int = 0
    rq_inv_scale: float = 0.0
    cc: float = 0.0
    rs: float = 0.0
    l0a: float = 0.0
    l0b: float = 0.0
    ck: float = 0.0
    cs: float = 0.0
    row_i: torch.Tensor | None = None
    row_l: torch.Tensor | None = None
    col_i: torch.Tensor | None = None
    col_scale: torch.Tensor | None = None      # fp32 [cols]: per-column affine (folded batch norm)
    col_shift: torch.Tensor | None = None
    tuning: Tuning | None = None

    def to_c(self) -> _EpilogueC:
        def ptr(t):
            if t is None:
                return None
            assert t.dtype == torch.int32 and t.is_contiguous() and t.is_cuda
            return t.data_ptr()
        def fptr(t):
            if t is None:
                return None
            assert t.dtype == torch.float32 and t.is_contiguous() and t.is_cuda
            return t.data_ptr()
        tn = None
        if self.tuning is not None:
            t = self.tuning
            tn = C.pointer(_TuningC(t.update_path, t.agg_xcd_run, t.layer_path, t.layer_ksplit, t.zero_words, t.even_progress))
        # (the structure keeps the pointed-to tuning alive)
        return _EpilogueC(self.mode, int(self.relu), int(self.self_term), self.rq_nbits,
                          self.rq_lo, self.rq_inv_scale, self.cc, self.rs, self.l0a,
                          self.l0b, self.ck, self.cs, ptr(self.row_i), ptr(self.row_l),
                          ptr(self.col_i), fptr(self.col_scale), fptr(self.col_shift), tn)

    @staticmethod
    def from_c(c: "_EpilogueC") -> "Epilogue":
        """The scalar fields of a C epilogue (pointer fields stay unset)."""
        return Epilogue(mode=c.mode, relu=bool(c.relu), self_term=bool(c.self_term), rq_nbits=c.rq_nbits,
                        rq_lo=c.rq_lo, rq_inv_scale=c.rq_inv_scale, cc=c.cc, rs=c.rs, l0a=c.l0a, l0b=c.l0b,
                        ck=c.ck, cs=c.cs)


def describe(rows: int, cols: int, nbits: int, layout: int, block_rows: int = 0):
    d = _BitsC()
    words = lib().qgtc_describe(C.byref(d), rows, cols, nbits, layout, block_rows)
    if words == 0 and rows > 0 and cols > 0:
        raise QgtcError(2, "qgtc_describe")
    return d, int(words)


def alloc_bits(rows, cols, nbits, layout, block_rows=0, ld_words=None, device="cuda") -> Bits:
    d, words = describe(rows, cols, nbits, layout, block_rows)
    if ld_words is not None:
        assert layout in (LEFT, RIGHT)
        d.ld_words = ld_words
        k = rows if layout == LEFT else -(-rows // 32)
        d.plane_stride_words = k * ld_words
        words = d.plane_stride_words * nbits
    buf = torch.empty(max(int(words), 4), dtype=torch.int32, device=device)
    d.data = buf.data_ptr()
    return Bits(buf, d)


# ---------------------------------------------------------------- entry points
def qgtc_version() -> int:
    return int(lib().qgtc_version())


def qgtc_pack_bits(src: torch.Tensor, nbits: int, layout: int, quant=None,
                   block_rows: int = 0, out: Bits | None = None) -> Bits:
    """src: 2-D device tensor, float32 (quant = (lo, hi) required), uint8 or int32."""
    assert src.dim() == 2 and src.is_cuda and src.stride(1) == 1
    rows, cols = src.shape
    dt = {torch.float32: SRC_F32, torch.uint8: SRC_U8, torch.int32: SRC_I32}[src.dtype]
    dst = out if out is not None else alloc_bits(rows, cols, nbits, layout, block_rows)
    q = None
    if quant is not None:
        q = C.byref(_QuantC(float(quant[0]), float(quant[1]), nbits))
    ld_src = src.stride(0) if rows > 1 else max(cols, 1)
    _check(lib().qgtc_pack_bits(C.c_void_p(src.data_ptr()), dt, rows, cols, ld_src, q,
                                C.byref(dst.c), _stream()), "qgtc_pack_bits")
    return dst


def qgtc_unpack_bits(bits: Bits) -> torch.Tensor:
    out = torch.empty((bits.rows, bits.cols), dtype=torch.int32, device=bits.words.device)
    _check(lib().qgtc_unpack_bits(C.byref(bits.c), C.c_void_p(out.data_ptr()), max(bits.cols, 1),
                                  _stream()), "qgtc_unpack_bits")
    return out


def qgtc_row_sums(bits: Bits) -> torch.Tensor:
    out = torch.empty(bits.rows, dtype=torch.int32, device=bits.words.device)
    _check(lib().qgtc_row_sums(C.byref(bits.c), C.c_void_p(out.data_ptr()), _stream()),
           "qgtc_row_sums")
    return out


def qgtc_col_sums(bits: Bits, out: torch.Tensor | None = None) -> torch.Tensor:
    if out is None:
        out = torch.empty(bits.cols, dtype=torch.int32, device=bits.words.device)
    assert out.dtype == torch.int32 and out.is_contiguous() and out.numel() >= bits.cols
    _check(lib().qgtc_col_sums(C.byref(bits.c), C.c_void_p(out.data_ptr()), _stream()),
           "qgtc_col_sums")
    return out


def qgtc_build_tile_map(A: Bits, tile_rows: int = 16, tile_kbits: int = 128,
                        out: TileMap | None = None) -> TileMap:
    if out is None:
        nbytes = lib().qgtc_tile_map_bytes(A.rows, A.cols, tile_rows, tile_kbits)
        if nbytes == 0:
            raise QgtcError(7, "qgtc_tile_map_bytes")
        buf = torch.empty(nbytes // 4, dtype=torch.int32, device=A.words.device)
        m = _TileMapC()
        _check(lib().qgtc_tile_map_carve(C.byref(m), C.c_void_p(buf.data_ptr()), A.rows, A.cols,
                                         tile_rows, tile_kbits), "qgtc_tile_map_carve")
        out = TileMap(buf, m, A.rows)
    _check(lib().qgtc_build_tile_map(C.byref(A.c), C.byref(out.c), _stream()),
           "qgtc_build_tile_map")
    return out


def _out_arg(ep: Epilogue, rows, cols, out, bits_layout, device):
    """Allocates (when out is None) and returns (object to hand back, void* argument, ld)."""
    if ep.mode == OUT_BITS:
        if out is None:
            ld = -(-cols // 32) if bits_layout == LEFT else None
            out = alloc_bits(rows, cols, ep.rq_nbits, bits_layout, ld_words=ld, device=device)
        return out, C.cast(C.pointer(out.c), C.c_void_p), 0
    if out is None:
        dt = torch.int32 if ep.mode == OUT_I32 else torch.float32
        out = torch.empty((rows, cols), dtype=dt, device=device)
    assert out.is_contiguous() or out.stride(1) == 1
    return out, C.c_void_p(out.data_ptr()), (out.stride(0) if rows > 1 else max(cols, 1))


def qgtc_aggregate(A: Bits, tmap: TileMap | None, X: Bits, ep: Epilogue, out=None):
    res, ptr, ld = _out_arg(ep, A.rows, X.cols, out, LEFT, X.words.device)
    epc = ep.to_c()
    m = C.byref(tmap.c) if tmap is not None else None
    _check(lib().qgtc_aggregate(C.byref(A.c), m, C.byref(X.c), C.byref(epc), ptr, ld, _stream()),
           "qgtc_aggregate")
    return res


def qgtc_update(Y: Bits, W: Bits, ep: Epilogue, out=None):
    res, ptr, ld = _out_arg(ep, Y.rows, W.cols, out, RIGHT, Y.words.device)
    epc = ep.to_c()
    _check(lib().qgtc_update(C.byref(Y.c), C.byref(W.c), C.byref(epc), ptr, ld, _stream()),
           "qgtc_update")
    return res


def qgtc_layer(A: Bits, tmap: TileMap | None, X: Bits, W: Bits, agg_ep: Epilogue,
               upd_ep: Epilogue, workspace: torch.Tensor | None = None, out=None):
    if workspace is None:
        nbytes = lib().qgtc_layer_workspace_bytes(A.rows, X.cols, W.cols, max(agg_ep.rq_nbits, 1))
        workspace = torch.empty(nbytes // 4 + 1, dtype=torch.int32, device=X.words.device)
    res, ptr, ld = _out_arg(upd_ep, A.rows, W.cols, out, RIGHT, X.words.device)
    a, u = agg_ep.to_c(), upd_ep.to_c()
    m = C.byref(tmap.c) if tmap is not None else None
    _check(lib().qgtc_layer(C.byref(A.c), m, C.byref(X.c), C.byref(W.c), C.byref(a), C.byref(u),
                            C.c_void_p(workspace.data_ptr()), workspace.numel() * 4, ptr, ld,
                            _stream()), "qgtc_layer")
    return res


LAYER_STATIC_MAX_BYTES = 16 * 1024 * 1024


def qgtc_layer_static(A: Bits, tmap: TileMap | None, X: Bits, W: Bits, agg_ep: Epilogue,
                      upd_ep: Epilogue, out=None):
    """qgtc_layer without a workspace argument (the library's own static device array
    serves); pass `out` to keep the whole call free of allocations."""
    res, ptr, ld = _out_arg(upd_ep, A.rows, W.cols, out, RIGHT, X.words.device)
    a, u = agg_ep.to_c(), upd_ep.to_c()
    m = C.byref(tmap.c) if tmap is not None else None
    _check(lib().qgtc_layer_static(C.byref(A.c), m, C.byref(X.c), C.byref(W.c), C.byref(a),
                                   C.byref(u), ptr, ld, _stream()), "qgtc_layer_static")
    return res


LAYER_FUSED, LAYER_TWO_KERNELS = 0, 1
UPDATE_AUTO, UPDATE_POPCOUNT, UPDATE_MATRIX_CORES = 0, 1, 2
ZERO_WORDS_AUTO, ZERO_WORDS_VISIT, ZERO_WORDS_SKIP = 0, 1, 2


def qgtc_tile_stats(A: Bits, out: torch.Tensor | None = None) -> torch.Tensor:
    """Device int32[8]: non-zero tiles of A at 16 x 32, 16 x 64, 16 x 128, its rows of tiles,
    and (two words, low half first) its (row, 32-bit word) pairs that hold a bit; see
    tile_stats_numbers."""
    if out is None:
        out = torch.empty(8, dtype=torch.int32, device=A.words.device)
    assert out.dtype == torch.int32 and out.is_contiguous() and out.numel() >= 8
    _check(lib().qgtc_tile_stats(C.byref(A.c), C.c_void_p(out.data_ptr()), _stream()), "qgtc_tile_stats")
    return out


def tile_stats_numbers(counts: torch.Tensor) -> dict:
    """The numbers of qgtc_tile_stats on the host (this synchronizes)."""
    c = [int(v) for v in counts.cpu()]
    return {"nnz_tiles": c[:3], "n_tile_rows": c[3],
            "nnz_row_words": (c[4] & 0xFFFFFFFF) | ((c[5] & 0xFFFFFFFF) << 32)}


def qgtc_plan_layer(rows: int, in_cols: int, out_cols: int, s: int, t: int, n_tile_rows: int = 0,
                    a_cols: int = 0, nnz_tiles=(0, 0, 0), subgraphs: int = 0, nnz_row_words: int = 0) -> dict:
    """The library's selector for one layer (host-only); nnz_tiles: the first three numbers
    of qgtc_tile_stats."""
    pin = _PlanInC(rows, in_cols, out_cols, s, t, n_tile_rows, a_cols, int(subgraphs),
                   (C.c_int64 * 3)(*[int(v) for v in nnz_tiles]), int(nnz_row_words))
    pout = _PlanOutC()
    _check(lib().qgtc_plan_layer(C.byref(pin), C.byref(pout)), "qgtc_plan_layer")
    return {k: getattr(pout, k) for k, _ in _PlanOutC._fields_}


def qgtc_quant_inv_scale(lo: float, hi: float, nbits: int) -> float:
    """fp32(2^nbits / (hi - lo)) as the library forms it for Eq. (2)."""
    return float(lib().qgtc_quant_inv_scale(float(lo), float(hi), int(nbits)))


def qgtc_layer_epilogues(s: int, t: int, in_cols: int, x_lo: float, x_scale: float, w_range, agg_hi: float,
                         out_hi: float | None, self_term: bool = False, last: bool = False,
                         batchnorm: bool = False, update_first: bool = False):
    """(first_ep, second_ep, z_scale, next_x_scale) of one layer of a stack: the scalar
    fields of the two epilogues as the library's helper sets them; the caller adds the
    device vectors (row_l, col_i, col_scale, col_shift)."""
    spec = _LayerSpecC(s, t, in_cols, int(update_first), int(self_term), int(last), int(batchnorm), 0,
                       float(x_lo), float(x_scale), float(w_range[0]), float(w_range[1]), float(agg_hi),
                       float(out_hi) if out_hi is not None else 0.0)
    e1, e2 = _EpilogueC(), _EpilogueC()
    zs, nx = C.c_double(0.0), C.c_double(0.0)
    _check(lib().qgtc_layer_epilogues(C.byref(spec), C.byref(e1), C.byref(e2), C.byref(zs), C.byref(nx)),
           "qgtc_layer_epilogues")
    return Epilogue.from_c(e1), Epilogue.from_c(e2), zs.value, nx.value


def qgtc_fold_batchnorm(gamma, beta, mean, var, eps: float, value_scale: float):
    """(col_scale, col_shift) as host float32 tensors: a batch normalization folded into a
    per-column affine map acting on value_scale * accumulator."""
    n = len(gamma)
    arr = lambda v: (C.c_double * n)(*[float(x) for x in v])
    cs, ch = (C.c_float * n)(), (C.c_float * n)()
    _check(lib().qgtc_fold_batchnorm(arr(gamma), arr(beta), arr(mean), arr(var), float(eps), float(value_scale),
                                     n, cs, ch), "qgtc_fold_batchnorm")
    return torch.tensor(list(cs), dtype=torch.float32), torch.tensor(list(ch), dtype=torch.float32)


def qgtc_device_info() -> dict:
    """Compute units and XCDs of the current device, and whether it is the gfx950 part the
    kernels are written for (raises QgtcError when it is not)."""
    d = _DeviceC()
    _check(lib().qgtc_device_info(C.byref(d)), "qgtc_device_info")
    return {"compute_units": d.compute_units, "xcds": d.xcds, "is_gfx950": bool(d.is_gfx950),
            "xcds_assumed": d.xcds_assumed}


def qgtc_probe_popcount(workgroups: int, waves_per_workgroup: int, iters: int, sink: torch.Tensor):
    _check(lib().qgtc_probe_popcount(workgroups, waves_per_workgroup, iters,
                                     C.c_void_p(sink.data_ptr()), _stream()), "qgtc_probe_popcount")


def qgtc_prof_enable(on: bool):
    _check(lib().qgtc_prof_enable(int(on)), "qgtc_prof_enable")


def qgtc_prof_reset():
    _check(lib().qgtc_prof_reset(), "qgtc_prof_reset")


def qgtc_prof_read(kind: int):
    ms, n = C.c_double(0.0), C.c_int64(0)
    _check(lib().qgtc_prof_read(kind, C.byref(ms), C.byref(n)), "qgtc_prof_read")
    return ms.value, n.value
