/*
 * qgtc.h - C ABI of the any-bitwidth quantized GNN layer for AMD MI355X (gfx950).
 *
 * The layer follows QGTC (arXiv 2111.09547): neighbour aggregation Y = A.X of a
 * binary adjacency with s-bit node embeddings, then the node update Y.W with
 * t-bit weights (Algorithm 1, Section 3.2).  Both products are sums of 1-bit
 * products, sum_i sum_j 2^(i+j) popcnt(plane_i & plane_j) (Section 3.1,
 * Eq. 3-7), taken over bit planes packed into 32-bit words (Section 4.2).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or keeps them.  Descriptor structs (qgtc_bits,
 *     qgtc_tile_map, qgtc_epilogue, qgtc_quant) are HOST structs read during
 *     the call only.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it; no entry point synchronizes.
 *   - Arguments are validated on the host before anything is launched; a
 *     failed call launches nothing and returns a status other than QGTC_OK.
 *   - Integer results are defined modulo 2^32 (32-bit accumulators,
 *     Sections 2.3 and 3.2).
 *   - Empty operands (no rows, or no output columns) are valid: the call returns
 *     QGTC_OK without launching, and the output pointer may then be NULL.
 */
#ifndef QGTC_H
#define QGTC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  QGTC_OK = 0,
  QGTC_ERR_NULL = 1,        /* a required pointer is NULL */
  QGTC_ERR_SHAPE = 2,       /* shapes of the operands do not fit each other */
  QGTC_ERR_BITWIDTH = 3,    /* nbits outside [1, 32] (adjacency: != 1) */
  QGTC_ERR_ALIGN = 4,       /* pointer or leading dimension not aligned as required */
  QGTC_ERR_LAYOUT = 5,      /* operand packed in the wrong layout */
  QGTC_ERR_WORKSPACE = 6,   /* workspace too small */
  QGTC_ERR_UNSUPPORTED = 7, /* valid request this build has no kernel for */
  QGTC_ERR_HIP = 8          /* the HIP runtime reported an error on launch */
} qgtc_status;

const char* qgtc_status_string(qgtc_status s);

/* ---------------------------------------------------------------------------
 * Packed bit planes ("3D-stacked bit compression", Section 4.2 and Figure 4).
 *
 * An nbits-bit unsigned matrix is stored as nbits stacked 1-bit matrices; 32
 * consecutive entries along the contraction dimension K share one 32-bit word,
 * entry 32*w + b in bit b of word w (least significant bit = lowest index),
 * zero fill past the end of the matrix.
 *
 *   QGTC_LEFT  (left operands A, Y; rows x K):  word(p, r, w) =
 *              data[p*plane_stride_words + r*ld_words + w],  w < ceil(cols/32)
 *   QGTC_RIGHT (right operands X, W; K x cols): word(p, w, c) =
 *              data[p*plane_stride_words + w*ld_words + c],  w < ceil(rows/32)
 *
 * LEFT buffers: ld_words is a multiple of 4 and every word in [ceil(cols/32),
 * ld_words) of a row is zero (the paper pads K to 128 bits for its 8x128
 * tiles; the kernels here read adjacency rows 128 bits at a time as well).
 * data must be 16-byte aligned.
 *
 * block_rows (LEFT, adjacency only): 0 for an ordinary rows x cols matrix.  A
 * positive value describes a block-diagonal matrix of batched subgraphs
 * (Section 4.1) stored without its all-zero off-diagonal blocks: row r keeps
 * only the cols == block_rows entries of its own diagonal block, entry j
 * standing for column (r / block_rows) * block_rows + j.  block_rows must be a
 * multiple of 32.
 *
 * QGTC_RIGHT_BYTES (weights W of qgtc_layer only; K x cols, nbits <= 8): the codes
 * themselves, one byte each, in the operand order of the int8 matrix instruction
 * that the fused layer kernel feeds (the paper caches the decomposed W across
 * subgraphs, end of Section 3.2; this is the form to cache here).  Columns are
 * taken in tiles of 16 and K in steps of 64; the 1 KiB block of (tile nt, step ks)
 * holds, for lane l = c % 16 + 16 * ((k % 64) / 16), the 16 consecutive bytes
 * k % 16 = 0..15 of column c, row k:
 *   byte(k, c) = bytes[part * 4 * plane_stride_words + (c / 16) * 4 * ld_words +
 *                      (k / 64) * 1024 + l * 16 + k % 16]
 * with ld_words = 256 * ceil(rows / 64) and plane_stride_words = ceil(cols / 16) *
 * ld_words.  8-bit codes are stored as two parts, their low 7 bits (part 0) and
 * their top bit (part 1), because the instruction multiplies signed bytes;
 * narrower codes have part 0 only.  Zero fill.  data must be 16-byte aligned.
 *
 * QGTC_LEFT_BYTES (left operand Y of qgtc_update only; rows x K, nbits <= 8): the
 * codes themselves, one byte each, row-major: byte(r, k) = bytes[r * 4 * ld_words + k],
 * ld_words a multiple of 4 with 4 * ld_words >= cols, zero fill up to the end of
 * the row.  16 consecutive K positions of a row are one operand register group
 * of the int8 matrix instruction, so the update reads this form without putting
 * bit planes back together.  data must be 16-byte aligned.
 * ------------------------------------------------------------------------- */
enum { QGTC_LEFT = 0, QGTC_RIGHT = 1, QGTC_RIGHT_BYTES = 2, QGTC_LEFT_BYTES = 3 };

typedef struct qgtc_bits {
  uint32_t* data;
  int32_t nbits;
  int32_t rows;
  int32_t cols;
  int32_t layout;
  int32_t block_rows;
  int32_t reserved;
  int64_t ld_words;
  int64_t plane_stride_words;
} qgtc_bits;

/* Fills ld_words / plane_stride_words (and the scalar fields) with the default
 * strides and returns the number of 32-bit words the buffer needs:
 *   LEFT : ld = 4*ceil(cols/128), plane stride = rows*ld
 *   RIGHT: ld = cols,             plane stride = ceil(rows/32)*ld
 *   RIGHT_BYTES: as stated above; the return value covers both parts for 8 bits
 *   LEFT_BYTES: ld = 4*ceil(cols/16) words, plane stride = rows*ld (one "plane")
 * d->data is left untouched.  Returns 0 on invalid arguments. */
size_t qgtc_describe(qgtc_bits* d, int32_t rows, int32_t cols, int32_t nbits,
                     int32_t layout, int32_t block_rows);

/* ---------------------------------------------------------------------------
 * Eq. (2): code = floor((x - lo) / scale), scale = (hi - lo) / 2^nbits.
 * The result is clamped to [0, 2^nbits - 1] (x = hi would need nbits+1 bits).
 * Arithmetic: lo is rounded to fp32; inv_scale = fp32(2^nbits / (hi - lo)) is
 * formed in double; (x - lo) and the multiplication are single fp32 operations.
 * ------------------------------------------------------------------------- */
typedef struct qgtc_quant {
  double lo;
  double hi;
  int32_t nbits;
} qgtc_quant;

enum { QGTC_SRC_F32 = 0, QGTC_SRC_U8 = 1, QGTC_SRC_I32 = 2 };

/* Quantize (fp32 source, q != NULL) or take integers as they are (u8 / i32
 * source, q == NULL; bits above dst->nbits are dropped), decompose into bit
 * planes and pack into dst ("Tensor.to_bit", Sections 4.2 and 5).
 * src: device, row-major rows x cols with leading dimension ld_src (elements).
 * dst: descriptor filled by the caller (qgtc_describe) with rows/cols equal to
 * the arguments; every word of the packed matrix, padding included, is written.
 * Any of the four layouts. */
qgtc_status qgtc_pack_bits(const void* src, int32_t src_dtype, int32_t rows,
                           int32_t cols, int64_t ld_src, const qgtc_quant* q,
                           const qgtc_bits* dst, void* stream);

/* Bandwidth-optimized subgraph packing (Section 4.6): the same packing on the CPU,
 * so that a batch crosses the host-device link as low-bit planes in one transfer.
 * src and dst->data are HOST memory; dst is a LEFT or RIGHT descriptor (others:
 * QGTC_ERR_UNSUPPORTED).  Same arguments, checks and arithmetic as qgtc_pack_bits,
 * and the same words in dst.  threads: worker threads to use (0: one per hardware
 * thread).  Synchronous; never touches the GPU. */
qgtc_status qgtc_pack_bits_host(const void* src, int32_t src_dtype, int32_t rows,
                                int32_t cols, int64_t ld_src, const qgtc_quant* q,
                                const qgtc_bits* dst, int32_t threads);
/* Places n objects of bytes[i] bytes one after the other in one buffer, each at a
 * multiple of 256 bytes: writes their offsets and returns the size of the buffer
 * (the "compound memory object" of Section 4.6: allocate it once in pinned host
 * memory and once on the device, point the descriptors of the packed adjacency and
 * features into it, pack on the host, copy once).  Host-only. */
size_t qgtc_compound_layout(const size_t* bytes, int32_t n, size_t* offsets);

/* Decode a packed matrix (any layout) back to one uint32 per entry
 * ("Tensor.to_val", Section 5).  dst: device, row-major rows x cols, leading
 * dimension ld_dst. */
qgtc_status qgtc_unpack_bits(const qgtc_bits* src, uint32_t* dst, int64_t ld_dst,
                             void* stream);

/* Value sums of a packed matrix, sum_p 2^p * popcnt, modulo 2^32:
 * per row of a LEFT operand (out: rows entries) or per column of a RIGHT or
 * RIGHT_BYTES operand (out: cols entries).  They feed the dequantizing epilogue below. */
qgtc_status qgtc_row_sums(const qgtc_bits* m, int32_t* out, void* stream);
qgtc_status qgtc_col_sums(const qgtc_bits* m, int32_t* out, void* stream);

/* ---------------------------------------------------------------------------
 * Zero-tile map (zero-tile jumping, Section 4.3).  The paper tests every 8x128
 * tile of A inside the product kernel; here the test is done once per
 * adjacency (A is reused by every layer, end of Section 3.2) and kept as, per
 * row of tiles, the ascending list of tile columns that hold at least one edge.
 *   row_cnt[tr]                      number of non-zero tiles in tile row tr
 *   col_idx[tr*n_tile_cols + i]      their tile-column indices, i < row_cnt[tr]
 *   nnz_tiles[0]                     total number of non-zero tiles
 *   nnz_tiles[1]                     log2 of the run of consecutive tile rows the
 *                                    product kernels keep on one XCD, 3..6: the
 *                                    longest run of 8..64 tile rows for which the
 *                                    busiest of the 8 XCDs (runs dealt round-robin,
 *                                    a tile row weighing its tiles + 1) carries at
 *                                    most 2 % more than the mean.  A hint that only
 *                                    affects speed; nnz_tiles[2..3] are reserved.
 *   deg[r]                           popcount of row r of A (node degree)
 * Any tile shape with tile_rows in {8, 16, 32, 64} and tile_kbits in {32, 64,
 * 128, 256, 512} can be built (8 x 128 reproduces the statistic of the paper's
 * Figure 8); qgtc_aggregate takes tile_rows == 16 and tile_kbits in
 * {32, 64, 128}.
 * ------------------------------------------------------------------------- */
typedef struct qgtc_tile_map {
  int32_t tile_rows;
  int32_t tile_kbits;
  int32_t n_tile_rows;  /* ceil(A.rows / tile_rows) */
  int32_t n_tile_cols;  /* ceil(A.cols / tile_kbits) */
  int32_t* row_cnt;     /* [n_tile_rows] */
  int32_t* col_idx;     /* [n_tile_rows * n_tile_cols] */
  int32_t* nnz_tiles;   /* [4] */
  int32_t* deg;         /* [A.rows] */
} qgtc_tile_map;

/* Bytes of one device buffer large enough for all four arrays of a map. */
size_t qgtc_tile_map_bytes(int32_t rows, int32_t kbits, int32_t tile_rows,
                           int32_t tile_kbits);
/* Sets the scalar fields and points the four arrays into `buffer` (device,
 * 16-byte aligned, qgtc_tile_map_bytes long).  Host-only; launches nothing. */
qgtc_status qgtc_tile_map_carve(qgtc_tile_map* map, void* buffer, int32_t rows,
                                int32_t kbits, int32_t tile_rows,
                                int32_t tile_kbits);
/* Scans the packed adjacency A (LEFT, 1 bit) and fills the map. */
qgtc_status qgtc_build_tile_map(const qgtc_bits* A, const qgtc_tile_map* map,
                                void* stream);

/* ---------------------------------------------------------------------------
 * Epilogue fused into the product kernels (inter-layer kernel fusion,
 * Section 4.5).  C is the 32-bit accumulator of entry (i, j), read as signed.
 *
 *   QGTC_OUT_I32  ("bitMM2Int", Section 5): out[i*ld_out + j] = C
 *                 (max(C, 0) with relu).  out: int32_t*.
 *   QGTC_OUT_F32  (last layer, Section 4.5): the real product of the two
 *                 dequantized operands.  With left operand l0[i] + sl*L and
 *                 right operand r0 + sr*R,
 *                   t1  = cc*C + rs*row_i[i]
 *                   t2  = (l0a + l0b*row_l[i]) * (ck + cs*col_i[j])
 *                   out = fp32(t1 + t2)           (max(., 0) first with relu)
 *                 evaluated in fp64 in exactly this order, where the caller
 *                 sets cc = sl*sr, rs = sl*r0, ck = r0*K, cs = sr, row_i =
 *                 row sums of L, col_i = column sums of R and l0[i] = l0a +
 *                 l0b*row_l[i].  NULL vectors read as zeros.  out: float*.
 *   QGTC_OUT_BITS ("bitMM2Bit", Section 5): requantize to rq_nbits bits and
 *                 emit packed planes for the next product:
 *                   d = C - rq_lo (64-bit; C -> max(C, 0) first with relu)
 *                   code = min(floor(fp32(max(d, 0)) * rq_inv_scale), 2^rq_nbits - 1)
 *                 out: const qgtc_bits* describing the destination
 *                 (qgtc_aggregate: LEFT; qgtc_update: RIGHT; nbits == rq_nbits).
 *                 Every word of the destination is written, the zero words
 *                 between the end of a LEFT row and its ld_words included.
 *
 * self_term (qgtc_aggregate only): adds X[i, j] itself to C, i.e. the GIN
 * aggregation (1 + eps).X + A.X with eps = 0; needs a square adjacency.
 *
 * col_scale / col_shift (device, one float per output column, or both NULL): a
 * per-column affine map in front of the activation, which is how a batch
 * normalization that follows the layer folds into the kernel (Section 4.5:
 * BN(x) = (x - E_j) / sqrt(Var_j + eps) * gamma_j + beta_j = a_j x + b_j).
 * col_shift alone may be NULL (zeros).  With col_scale set,
 *   QGTC_OUT_BITS: v = fp32(C) * col_scale[j]        (C signed; one rounded multiply)
 *                  v = v + col_shift[j]              (one rounded add, no fused multiply-add)
 *                  v = max(v, 0) with relu (NaN -> 0)
 *                  code = Eq. (2) of v with lower bound fp32(rq_lo) and rq_inv_scale,
 *                         clamped to [0, 2^rq_nbits - 1] as in qgtc_quant
 *                  (the caller puts the scale of C into col_scale);
 *   QGTC_OUT_F32:  out = fp32((t1 + t2) * col_scale[j] + col_shift[j]) in fp64,
 *                  max(., 0) first with relu;
 *   QGTC_OUT_I32:  QGTC_ERR_UNSUPPORTED.
 * ------------------------------------------------------------------------- */
enum { QGTC_OUT_I32 = 0, QGTC_OUT_F32 = 1, QGTC_OUT_BITS = 2 };

/* Optional choices of a call that only affect speed, never results.  A NULL pointer or
 * zeros leave every choice to the library (the rules of qgtc_plan_layer below).
 *   update_path   which kernel qgtc_update (and the two-kernel path of qgtc_layer) uses
 *                 when both operands have at most 8 bits.  The paper composes every product
 *                 from 1-bit products (Section 3.1) because its matrix unit is 1-bit;
 *                 CDNA4's matrix cores start at int8, where one instruction covers up to
 *                 8 x 8 bit planes, so the update can re-assemble the planes into bytes in
 *                 registers and run there.  0 = automatic, 1 = popcount kernel,
 *                 2 = matrix cores whenever the operands fit.
 *   agg_xcd_run   how qgtc_aggregate deals its workgroups to the 8 XCDs (each with an L2
 *                 of its own): runs of that many consecutive tile rows go to one XCD, the
 *                 next run to the next XCD.  0 = the run length the tile-map build chose
 *                 (8 tile rows without a map), > 0 = that many tile rows (at most 4096),
 *                 < 0 = one contiguous range per XCD.
 *   layer_path    0 = qgtc_layer uses its fused kernel whenever it applies, 1 = always
 *                 aggregate and update as two kernels.
 *   layer_ksplit  waves of a workgroup of the fused kernel that split one tile list:
 *                 0 = automatic (more when the grid is small), 1, 2 or 4.
 *   zero_words    zero-word jumping inside the tiles the map keeps: the aggregation's unit
 *                 of work is one row of a tile times one 32-bit word, and the word of a row
 *                 is wave-uniform, so rows whose word is zero can be jumped over (the
 *                 paper's zero-tile jumping, Section 4.3, at the granularity of the vector
 *                 ALUs instead of the Tensor-Core tile).  Results are the same either way.
 *                 0 = automatic: on when a tile map is passed (a sparse adjacency) and X
 *                 has at least 3 planes; 1 = visit every word of a kept tile (faster when
 *                 most words hold a bit: a row that is present costs one scalar branch
 *                 more in the jumping form); 2 = jump whenever X has at least 3 planes.
 *                 qgtc_plan_layer says which from the statistics of the adjacency.
 *                 From 5 planes on, and while a row of A (of a diagonal block, for block
 *                 storage), rounded up to whole tiles, has at most 2047 words of 32 bits, the
 *                 jumping form keeps two rows of a tile per accumulator register, 16 bits
 *                 each (no count can reach 65536), which lets a fourth wave per SIMD run;
 *                 wider adjacencies take the same form with full-width accumulators.  The
 *                 caller sees no difference but the speed.
 *   even_progress issue priority inside the fused kernel's tile loop by the share of the
 *                 tile list that is left, so that the waves of a SIMD move through their
 *                 lists side by side instead of the oldest finishing long before the
 *                 youngest (which then runs alone).  It pays when every wave of the launch
 *                 is resident from the start - at most one wave per wave slot of the device -
 *                 and costs when there are more, because then the oldest waves should
 *                 finish first and hand their slots on.  0 = automatic: on when this
 *                 launch alone has at most one wave per slot; 1 = off; 2 = on.  A caller
 *                 that runs several launches side by side (runs of a batch on several
 *                 streams) passes what qgtc_plan_layer says for the whole batch.
 * Values outside these ranges: QGTC_ERR_UNSUPPORTED. */
typedef struct qgtc_tuning {
  int32_t update_path;
  int32_t agg_xcd_run;
  int32_t layer_path;
  int32_t layer_ksplit;
  int32_t zero_words;
  int32_t even_progress;
} qgtc_tuning;

typedef struct qgtc_epilogue {
  int32_t mode;
  int32_t relu;
  int32_t self_term;
  int32_t rq_nbits;
  int32_t rq_lo;
  float rq_inv_scale;
  double cc, rs, l0a, l0b, ck, cs;
  const int32_t* row_i; /* [rows] or NULL */
  const int32_t* row_l; /* [rows] or NULL */
  const int32_t* col_i; /* [cols] or NULL */
  const float* col_scale; /* [cols] or NULL */
  const float* col_shift; /* [cols] or NULL */
  const qgtc_tuning* tuning; /* HOST pointer or NULL; qgtc_layer reads upd_ep's */
} qgtc_epilogue;

/* Neighbour aggregation C = A.X (first half of Algorithm 1; zero-tile jumping
 * and non-zero tile reuse, Sections 4.3 and 4.4).
 * A: LEFT, 1 bit, rows x K (or block-diagonal, see block_rows).
 * map: tile map of A, or NULL to visit every tile.
 * X: RIGHT, s bits, K x cols.  X must span less than 4 GiB.
 * out / ld_out: per epilogue mode (ld_out in elements; ignored for BITS). */
qgtc_status qgtc_aggregate(const qgtc_bits* A, const qgtc_tile_map* map,
                           const qgtc_bits* X, const qgtc_epilogue* ep,
                           void* out, int64_t ld_out, void* stream);

/* Node update C = Y.W (second half of Algorithm 1).
 * Y: LEFT, s bits, rows x K, or LEFT_BYTES (then s, t <= 8: the product runs on the
 * int8 matrix cores).  W: RIGHT, t bits, K x cols. */
qgtc_status qgtc_update(const qgtc_bits* Y, const qgtc_bits* W,
                        const qgtc_epilogue* ep, void* out, int64_t ld_out,
                        void* stream);

/* One layer (Algorithm 1): aggregate, requantize the result to agg_ep->rq_nbits
 * bits (agg_ep must be QGTC_OUT_BITS; its output is internal to the call), then
 * update with upd_ep into out.
 * When all operands have at most 8 bits, X has at most 1024 columns and W at most
 * 256, the whole layer runs as ONE kernel (inter-layer fusion, Section 4.5,
 * extended across the two products): the requantized aggregation tile goes
 * through LDS as bytes straight into the int8 matrix cores.  Otherwise the
 * call runs qgtc_aggregate into packed planes in `workspace`, then qgtc_update.
 * Both give the same integers.
 * W: RIGHT (planes; the fused kernel is preceded by a small kernel that re-orders
 * them) or RIGHT_BYTES (taken as it is; QGTC_ERR_UNSUPPORTED when the fused
 * kernel does not apply).
 * upd_ep in QGTC_OUT_F32 mode: with row_i == NULL and rs != 0 the row sums of
 * the requantized aggregation result (the left operand of the update, which only
 * exists inside the call) are taken for row_i.
 * workspace: device, 16-byte aligned, at least qgtc_layer_workspace_bytes(rows
 * of A, columns of X, columns of W, agg_ep->rq_nbits) bytes. */
size_t qgtc_layer_workspace_bytes(int32_t rows, int32_t in_cols, int32_t out_cols,
                                  int32_t nbits);
qgtc_status qgtc_layer(const qgtc_bits* A, const qgtc_tile_map* map,
                       const qgtc_bits* X, const qgtc_bits* W,
                       const qgtc_epilogue* agg_ep, const qgtc_epilogue* upd_ep,
                       void* workspace, size_t workspace_bytes, void* out,
                       int64_t ld_out, void* stream);

/* qgtc_layer for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * checks and results as qgtc_layer, without the workspace: the layer's intermediate
 * data (see qgtc_layer) lives in a device array of QGTC_LAYER_STATIC_MAX_BYTES that
 * is part of the library's code object; every GPU the process uses holds one copy
 * until the process ends.  The call allocates and frees nothing (with the optional
 * kernel timing of qgtc_bench.h switched off, its default).
 * Limit: QGTC_ERR_WORKSPACE when qgtc_layer_workspace_bytes(rows of A, columns of X,
 * columns of W, agg_ep->rq_nbits) exceeds QGTC_LAYER_STATIC_MAX_BYTES.  The fused
 * kernel (all operands <= 8 bits) needs at most 512 KiB and always fits; the
 * two-kernel path needs rows * ceil(columns of X / 32) * rq_nbits * 4 + rows * 4
 * bytes.
 * All calls on one GPU share that GPU's array: calls that overlap in time on the same
 * GPU (different streams or threads) race; calls on one stream are ordered and safe.
 * The address of the array is looked up on the first call on each device (with that
 * device current, hipGetSymbolAddress) and kept. */
#define QGTC_LAYER_STATIC_MAX_BYTES (16 * 1024 * 1024)
qgtc_status qgtc_layer_static(const qgtc_bits* A, const qgtc_tile_map* map,
                              const qgtc_bits* X, const qgtc_bits* W,
                              const qgtc_epilogue* agg_ep, const qgtc_epilogue* upd_ep,
                              void* out, int64_t ld_out, void* stream);

/* ---------------------------------------------------------------------------
 * Non-zero tiles of A at the three tile widths qgtc_aggregate takes, in one pass over
 * the packed adjacency (the second kind of zero tiles of the paper's Section 6.3, gaps
 * inside a subgraph, shows as fewer non-zero tiles at narrower widths):
 *   counts[0..2] = number of non-zero 16 x 32, 16 x 64 and 16 x 128 tiles,
 *   counts[3]    = number of rows of tiles, ceil(A.rows / 16),
 *   counts[4..5] = low and high half of the 64-bit number of (row, 32-bit word) pairs of
 *                  A that hold a bit: the work zero-word jumping really visits
 *                  (qgtc_tuning.zero_words), and the selector's measure of how sparse the
 *                  kept tiles are,
 *   counts[6..7] = 0.
 * counts: device, 8 x int32, 8-byte aligned, written by the call (no need to clear it).
 * The host reads it when it plans (qgtc_plan_layer), once per adjacency.
 * ------------------------------------------------------------------------- */
qgtc_status qgtc_tile_stats(const qgtc_bits* A, int32_t* counts, void* stream);

/* ---------------------------------------------------------------------------
 * The selector: which tile width, which kernels and which launch shape the library
 * takes for one layer (the paper leaves such a heuristic as future work, end of its
 * Section 6.3).  A pure host function over the shape, the bit widths and the tile
 * statistics; qgtc_update and qgtc_layer make their automatic choices through it, so
 * the rules exist once.  Every rule is a measured crossover on MI355X.
 *   in:  rows (nodes), in_cols (D), out_cols (H), s, t,
 *        nnz_tiles[3] from qgtc_tile_stats (all zero: unknown, 128-bit tiles assumed,
 *        every tile of a row counted), n_tile_rows, a_cols (columns of A as stored),
 *        subgraphs (diagonal blocks of a batched adjacency, Section 4.1; 0: unknown or one),
 *        nnz_row_words from qgtc_tile_stats (0: unknown)
 *   out: tile_kbits     32, 64 or 128: least executed work.  Where every word of a kept tile
 *                       is visited: tiles x width x cost per bit.  Where the kernels jump
 *                       over zero words (zero_words = 2 below) the same non-zero words are
 *                       visited at every width, and the word steps to test and the tiles to
 *                       fetch decide: tiles x (words per tile + 5.8).  A narrower tile must
 *                       win by 2 %
 *        fused          1: qgtc_layer runs as one kernel (s, t <= 8, D <= 1024, H <= 256)
 *        update_path    1 popcount, 2 int8 matrix cores: the stand-alone update's kernel
 *        ksplit         waves of a fused workgroup that split a tile list (1, 2, 4)
 *        runs           independent runs of whole subgraphs to issue the layer as, one stream
 *                       each (1 or 2): subgraphs share no edge, so a batch can be cut between
 *                       them; 2 when the fused launch takes more than one and at most two
 *                       rounds of the device's wave slots, where the drain of one run's
 *                       launch then overlaps the other run's work (measured on config 4,
 *                       five layers, visiting every word - 4096 waves on 3072 slots: 434
 *                       against 464 us); 1 otherwise (with zero-word jumping the same
 *                       batch is one round of 4096 slots, and one run with even_progress
 *                       measures 230 against 233 us for two).  A run is then launched with
 *                       the K split and the even_progress of the whole batch
 *                       (qgtc_tuning.layer_ksplit = ksplit, .even_progress = even_progress)
 *        even_progress  the qgtc_tuning.even_progress to pass: 2 when the whole batch's
 *                       fused launch has at most one wave per wave slot, 1 otherwise
 *        zero_words     the qgtc_tuning.zero_words to pass: 2 (jump over zero words inside
 *                       kept tiles) when X has at least 3 planes and fewer than 70 % of the
 *                       (row, word) pairs of the kept tiles hold a bit (60 % from 5 planes
 *                       on) - a present row costs about one instruction pair more in that
 *                       form, and from 5 planes on half of the rows a third instruction per
 *                       plane, so it pays below 10 - 12 present rows out of 16 -, 1 (visit
 *                       all) otherwise; 0 when
 *                       nnz_row_words is unknown (the library then assumes a sparse
 *                       adjacency whenever a tile map is passed)
 *        est_us_aggregate_first, est_us_update_first
 *                       rough times of (A.X).W and A.(X.W) from the measured rates; the two
 *                       orders are different quantized networks (the requantization sits
 *                       elsewhere), so the order stays the caller's choice
 * ------------------------------------------------------------------------- */
typedef struct qgtc_plan_in {
  int32_t rows, in_cols, out_cols;
  int32_t s, t;
  int32_t n_tile_rows;
  int32_t a_cols;
  int32_t subgraphs;
  int64_t nnz_tiles[3];
  int64_t nnz_row_words;
} qgtc_plan_in;

typedef struct qgtc_plan_out {
  int32_t tile_kbits;
  int32_t fused;
  int32_t update_path;
  int32_t ksplit;
  double est_us_aggregate_first;
  double est_us_update_first;
  int32_t runs;
  int32_t zero_words;
  int32_t even_progress;
  int32_t reserved;
} qgtc_plan_out;

qgtc_status qgtc_plan_layer(const qgtc_plan_in* in, qgtc_plan_out* out);

/* ---------------------------------------------------------------------------
 * Host-side scalar algebra around a stack of layers, so that a caller sets up the
 * epilogues without redoing it.  Pure functions; no GPU.
 * ------------------------------------------------------------------------- */

/* fp32(2^nbits / (hi - lo)), formed in double and rounded once: the inverse step of
 * Eq. (2) as qgtc_pack_bits forms it, and rq_inv_scale for a range [lo, hi).
 * 0 when the range is empty or nbits is outside [1, 32]. */
float qgtc_quant_inv_scale(double lo, double hi, int32_t nbits);

/* One layer of a stack.  Activations between layers are low-bit codes (Section 4.5);
 * the codes a hidden layer emits are read as pure scales, value = x_scale * code, the
 * input features of the first layer as x_lo + x_scale * code (Eq. (2)).
 *   order          0: aggregate, requantize, update (Algorithm 1); 1: update first,
 *                  A.(X.W) (Section 6.1)
 *   last           1: this layer emits fp32, 0: ReLU + requantization to s bits
 *   batchnorm      1: col_scale / col_shift of the output epilogue hold a folded batch
 *                  normalization (qgtc_fold_batchnorm); out_hi is then in units of the
 *                  normalized real value
 *   agg_hi         requantization range [0, agg_hi) of the first product's result, in
 *                  accumulator units ("empirical bounds ... determined by users", Eq. (2))
 *   out_hi         hidden layers: range [0, out_hi) of the second product's result */
typedef struct qgtc_layer_spec {
  int32_t s, t;
  int32_t in_cols;
  int32_t order;
  int32_t self_term;
  int32_t last;
  int32_t batchnorm;
  int32_t reserved;
  double x_lo, x_scale;
  double w_lo, w_hi;
  double agg_hi;
  double out_hi;
} qgtc_layer_spec;

/* Fills the scalar fields of the two epilogues of the layer (the pointer fields - row_l =
 * degrees, col_i = column sums of W, col_scale / col_shift, tuning - stay the caller's):
 *   first_ep   epilogue of the first product: QGTC_OUT_BITS to s bits over [0, agg_hi)
 *              (agg_ep of qgtc_layer / qgtc_aggregate; with order 1: of qgtc_update)
 *   second_ep  epilogue of the second product: hidden layer QGTC_OUT_BITS with ReLU over
 *              [0, out_hi); last layer QGTC_OUT_F32 with cc, rs, l0a, l0b, ck, cs set for the
 *              exact real product of the dequantized operands (order 0) or cc alone (order 1)
 *   z_scale    real value of one unit of the second product's accumulator under the
 *              pure-scale reading (what a batch normalization is folded with)
 *   next_x_scale   x_scale of the next layer's codes (0 for the last layer) */
qgtc_status qgtc_layer_epilogues(const qgtc_layer_spec* spec, qgtc_epilogue* first_ep,
                                 qgtc_epilogue* second_ep, double* z_scale,
                                 double* next_x_scale);

/* Batch normalization folded into a per-column affine map (Section 4.5):
 * a_j = gamma_j / sqrt(var_j + eps); col_scale_j = fp32(a_j * value_scale),
 * col_shift_j = fp32(beta_j - a_j * mean_j).  Host arrays of n entries. */
qgtc_status qgtc_fold_batchnorm(const double* gamma, const double* beta, const double* mean,
                                const double* var, double eps, double value_scale, int32_t n,
                                float* col_scale, float* col_shift);

/* What the library found on the current device, against what its kernels are written
 * for: code objects for gfx950 only, workgroups dealt over 8 XCDs of 32 compute units
 * each (Section 4.3's tile rows are spread so that a subgraph's rows share an XCD's L2),
 * launch shapes sized by the compute-unit count read from the device.
 *   compute_units   of the current device (multiprocessor count)
 *   xcds            compute_units / 32
 *   is_gfx950       1 when the device's architecture name starts with "gfx950"
 *   xcds_assumed    8
 * QGTC_OK when the device is gfx950 (a partition with fewer XCDs runs correctly: the
 * dealing is a permutation of workgroup ids whatever the hardware), QGTC_ERR_UNSUPPORTED
 * otherwise, QGTC_ERR_HIP when no device can be queried.  Host call, no launch. */
typedef struct qgtc_device {
  int32_t compute_units;
  int32_t xcds;
  int32_t is_gfx950;
  int32_t xcds_assumed;
} qgtc_device;
qgtc_status qgtc_device_info(qgtc_device* out);

/* Library version, major*10000 + minor*100 + patch. */
int32_t qgtc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QGTC_H */
