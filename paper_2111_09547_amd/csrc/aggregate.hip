// Neighbour aggregation C = A.X on packed bit planes (first half of Algorithm 1;
// zero-tile jumping and non-zero tile reuse, Sections 4.3 and 4.4 of the paper),
// written for gfx950.
//
// CDNA4 has no 1-bit matrix instruction, so the 1-bit products run on the
// vector ALUs: one v_and_b32 plus one v_bcnt_u32_b32 (popcount-accumulate) per
// 32 bit-products and lane.
//
// Work split.  A wave owns a 16-row tile of A and up to 64 output columns:
//   lane <-> output column c (feature index), so words X[plane][kw][c] load
//   fully coalesced, and the adjacency word of row j is broadcast from lane j
//   of each 16-lane DPP row inside the v_and itself (row_newbcast), costing no
//   instruction.  A tile therefore stays in 1..4 VGPRs and is reused for every
//   plane and every column - the "non-zero tile reuse" of the paper, in
//   registers instead of shared memory.
//   With fewer than 64 columns the four DPP rows hold four different row
//   tiles (CW = 16) or two (CW = 32), so no lane idles.
// Zero-tile jumping: the loop runs over the precomputed list of non-zero tile
// columns of the tile row (or over all of them without a map).
// Small grids: the 1..4 waves of a workgroup split the tile list and add their
// partial sums through LDS.
#include "qgtc_internal.h"

namespace qgtc {
namespace {

#include "popc_blocks.inc"

struct AggParams {
  const uint32_t* A;
  int64_t lda;            // words per row of A
  int32_t rows;           // rows of A (= output rows)
  int32_t block_rows;     // 0, or rows per diagonal block
  const uint32_t* X;
  uint32_t ldx4, psx4;    // bytes between word rows / planes of X
  uint32_t x_bytes;       // bytes spanned by X
  int32_t x_kwords;       // word rows of X
  int32_t s;              // planes of X
  int32_t cols;           // columns of X (= output columns)
  const int32_t* row_cnt; // tile map (NULL: all tiles)
  const int32_t* col_idx;
  int32_t n_tile_rows, n_tile_cols;
  int32_t tile_words;     // 1, 2 or 4 words (32/64/128 bits) per tile row
  int32_t cw_shift;       // log2 of columns per wave: 4, 5 or 6
  int32_t n_cg;           // column groups
  int32_t n_rt;           // groups of 64/CW row tiles
  int32_t ksplit;         // waves per workgroup
  int32_t chunk_shift;    // log2 of the run of consecutive workgroups one XCD takes
  uint32_t nblocks;
  EpiParams ep;
};

template <int S>
__device__ __forceinline__ void zero_acc(uint32_t (&acc)[16][S]) {
#pragma unroll
  for (int j = 0; j < 16; ++j)
#pragma unroll
    for (int i = 0; i < S; ++i) acc[j][i] = 0u;
}

// S planes of one word row of X for this lane's column.
// UNI: the word row is wave-uniform (scalar offset); otherwise per lane.
template <int S, bool UNI, bool MULTI>
__device__ __forceinline__ void load_x(uint32_t (&x)[S], __amdgpu_buffer_rsrc_t rx, uint32_t kw,
                                       uint32_t col4, const AggParams& p, int plane0) {
  if constexpr (UNI) {
    const uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)kw) * p.ldx4;
#pragma unroll
    for (int i = 0; i < S; ++i) {
      if (MULTI && plane0 + i >= p.s) {
        x[i] = 0u;
      } else {
        x[i] = __builtin_amdgcn_raw_buffer_load_b32(rx, col4, base + (uint32_t)(plane0 + i) * p.psx4, 0);
      }
    }
  } else {
    const uint32_t voff = kw * p.ldx4 + col4;
#pragma unroll
    for (int i = 0; i < S; ++i) {
      if (MULTI && plane0 + i >= p.s) {
        x[i] = 0u;
      } else {
        x[i] = __builtin_amdgcn_raw_buffer_load_b32(rx, voff, (uint32_t)(plane0 + i) * p.psx4, 0);
      }
    }
  }
}

// The four adjacency words (one per word step) of loop iteration `it` for this
// lane's row, and the word rows of X they meet.  An iteration covers 4 word
// steps: one 128-bit tile, two 64-bit tiles or four 32-bit tiles.
struct Step4 {
  uint32_t a[4];
  uint32_t kw[4];
};

template <bool UNI>
__device__ __forceinline__ Step4 load_steps(const AggParams& p, const uint32_t* arow, bool row_ok,
                                            const int32_t* ci, int n, int it, uint32_t kw_base,
                                            uint32_t kw_max) {
  Step4 r;
  const int tw = p.tile_words;
  const int per_it = 4 / tw;            // tiles per iteration
#pragma unroll
  for (int q = 0; q < 4; ++q) { r.a[q] = 0u; r.kw[q] = 0u; }
  if (tw == 4) {
    const int t = it;
    const bool ok = t < n;
    int tc = ok ? (ci ? ci[t] : t) : 0;
    if (UNI) tc = __builtin_amdgcn_readfirstlane(tc);
    const uint4 v = (ok && row_ok) ? *reinterpret_cast<const uint4*>(arow + (int64_t)tc * 4)
                                   : make_uint4(0u, 0u, 0u, 0u);
    r.a[0] = v.x; r.a[1] = v.y; r.a[2] = v.z; r.a[3] = v.w;
#pragma unroll
    for (int q = 0; q < 4; ++q) r.kw[q] = min(kw_base + (uint32_t)tc * 4u + q, kw_max);
  } else if (tw == 2) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int t = it * per_it + h;
      const bool ok = t < n;
      int tc = ok ? (ci ? ci[t] : t) : 0;
      if (UNI) tc = __builtin_amdgcn_readfirstlane(tc);
      const uint2 v = (ok && row_ok) ? *reinterpret_cast<const uint2*>(arow + (int64_t)tc * 2)
                                     : make_uint2(0u, 0u);
      r.a[2 * h] = v.x; r.a[2 * h + 1] = v.y;
      r.kw[2 * h] = min(kw_base + (uint32_t)tc * 2u, kw_max);
      r.kw[2 * h + 1] = min(kw_base + (uint32_t)tc * 2u + 1u, kw_max);
    }
  } else {
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const int t = it * per_it + h;
      const bool ok = t < n;
      int tc = ok ? (ci ? ci[t] : t) : 0;
      if (UNI) tc = __builtin_amdgcn_readfirstlane(tc);
      r.a[h] = (ok && row_ok) ? arow[tc] : 0u;
      r.kw[h] = min(kw_base + (uint32_t)tc, kw_max);
    }
  }
  return r;
}

// The words that the ballots of bit (p0 + i) of q, i < S, give for one output
// row of the wave.  CWS >= 5: the two halves of the 64-bit ballot (CW = 64: two
// consecutive words of the row; CW = 32: the words of the two row groups);
// CWS == 4: its four 16-bit fields (the words of the four row groups).
template <int S, int CWS>
__device__ __forceinline__ void ballot_words(uint32_t q, int p0, uint32_t (&w)[S][4]) {
#pragma unroll
  for (int i = 0; i < S; ++i) {
    const unsigned long long m = __builtin_amdgcn_ballot_w64(((q >> (p0 + i)) & 1u) != 0u);
    if constexpr (CWS >= 5) {
      w[i][0] = (uint32_t)m;
      w[i][1] = (uint32_t)(m >> 32);
      w[i][2] = 0u;
      w[i][3] = 0u;
    } else {
      w[i][0] = (uint32_t)(m & 0xffffull);
      w[i][1] = (uint32_t)((m >> 16) & 0xffffull);
      w[i][2] = (uint32_t)((m >> 32) & 0xffffull);
      w[i][3] = (uint32_t)((m >> 48) & 0xffffull);
    }
  }
}

// Generic path: planes pg .. pg+7 of the rows the wave owns; lane 4*J + k keeps
// word k of row J.  Planes past qbits give q >> plane == 0 and are not stored.
template <int J, int CWS>
__device__ __forceinline__ void gather_rows(const uint32_t (&q)[16], uint32_t (&ow)[8], int pg,
                                            int km, int wave) {
  if ((J & km) == wave) {
    uint32_t w[8][4];
    ballot_words<8, CWS>(pg < 32 ? q[J] : 0u, pg, w);
    lane_pack<8, (CWS >= 5 ? 2 : 4)>::template run<4 * J>(w, ow);
  }
  if constexpr (J + 1 < 16) gather_rows<J + 1, CWS>(q, ow, pg, km, wave);
}

// Fast path of the requantize-and-pack epilogue: as many output planes as
// feature planes (the layer case), one wave per workgroup, everything unrolled.
template <int J, int S, int CWS>
__device__ __forceinline__ void pack_rows_fast(const uint32_t (&q)[16], uint32_t (&ow)[S]) {
  uint32_t w[S][4];
  ballot_words<S, CWS>(q[J], 0, w);
  lane_pack<S, (CWS >= 5 ? 2 : 4)>::template run<4 * J>(w, ow);
  if constexpr (J + 1 < 16) pack_rows_fast<J + 1, S, CWS>(q, ow);
}

template <int S, int CWS, bool MULTI>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void aggregate_kernel(const AggParams p) {
  constexpr bool UNI = CWS == 6;
  extern __shared__ uint32_t lds[];   // [ksplit][16][64] partial sums when ksplit > 1

  const unsigned bid = xcd_deal(blockIdx.x, p.chunk_shift);
  if (bid >= p.nblocks) return;       // whole workgroup leaves together
  const int rt = (int)(bid / (unsigned)p.n_cg);
  const int cg = (int)(bid % (unsigned)p.n_cg);

  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int lane = threadIdx.x & 63;
  constexpr int cw = 1 << CWS;
  const int rg = UNI ? 0 : (lane >> CWS);
  constexpr int rgs = 64 >> CWS;                 // row tiles per wave
  const int tr = rt * rgs + rg;                     // this lane's tile row
  const bool tr_ok = tr < p.n_tile_rows;
  const int c = cg * cw + (lane & (cw - 1));        // this lane's output column
  const bool c_ok = c < p.cols;
  const uint32_t col4 = (uint32_t)(c_ok ? c : p.cols - 1) * 4u;
  const int arow_idx = tr * 16 + (lane & 15);       // adjacency row whose words this lane fetches
  const bool row_ok = tr_ok && arow_idx < p.rows;
  const uint32_t* arow = p.A + (int64_t)(row_ok ? arow_idx : 0) * p.lda;

  int n = 0;
  if (tr_ok) n = p.row_cnt ? p.row_cnt[tr] : p.n_tile_cols;
  const int32_t* ci = p.col_idx ? p.col_idx + (int64_t)(tr_ok ? tr : 0) * p.n_tile_cols : nullptr;
  if (UNI) n = __builtin_amdgcn_readfirstlane(n);
  const int per_it = 4 / p.tile_words;
  const int n_it = (n + per_it - 1) / per_it;       // loop iterations this lane needs

  uint32_t kw_base = 0u;
  if (p.block_rows > 0 && tr_ok) kw_base = (uint32_t)((tr * 16) / p.block_rows) * (uint32_t)(p.block_rows >> 5);
  const uint32_t kw_max = (uint32_t)(p.x_kwords - 1);

  __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)p.X, 0, (int)p.x_bytes, 0x00020000);

  uint32_t y[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) y[j] = 0u;

  const int n_chunks = MULTI ? (p.s + S - 1) / S : 1;
  for (int chunk = 0; chunk < n_chunks; ++chunk) {
    const int plane0 = chunk * S;
    uint32_t acc[16][S];
    zero_acc<S>(acc);

    int it = wave;
    if (__builtin_amdgcn_ballot_w64(it < n_it) != 0ull) {
      Step4 cur = load_steps<UNI>(p, arow, row_ok, ci, n, it, kw_base, kw_max);
      uint32_t x0[S], x1[S];
      load_x<S, UNI, MULTI>(x0, rx, cur.kw[0], col4, p, plane0);
      while (true) {
        const int it_next = it + p.ksplit;
        const bool more = __builtin_amdgcn_ballot_w64(it_next < n_it) != 0ull;
        Step4 nxt = cur;
        if (more) nxt = load_steps<UNI>(p, arow, row_ok, ci, n, it_next, kw_base, kw_max);
        load_x<S, UNI, MULTI>(x1, rx, cur.kw[1], col4, p, plane0);
        popc_rows<S>::run(cur.a[0], x0, acc);
        load_x<S, UNI, MULTI>(x0, rx, cur.kw[2], col4, p, plane0);
        popc_rows<S>::run(cur.a[1], x1, acc);
        load_x<S, UNI, MULTI>(x1, rx, cur.kw[3], col4, p, plane0);
        popc_rows<S>::run(cur.a[2], x0, acc);
        load_x<S, UNI, MULTI>(x0, rx, nxt.kw[0], col4, p, plane0);
        popc_rows<S>::run(cur.a[3], x1, acc);
        if (!more) break;
        cur = nxt;
        it = it_next;
      }
    }
    // shift-and-add of the per-plane popcounts (Algorithm 1, elementwise reduction)
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      uint32_t v = 0u;
#pragma unroll
      for (int i = 0; i < S; ++i) v += acc[j][i] << i;
      y[j] += v << plane0;
    }
  }

  // ---- epilogue: wave w finishes the rows j with j % ksplit == w ---------------
  const int km = p.ksplit - 1;                      // ksplit is 1, 2 or 4
  if (p.ksplit > 1) {
#pragma unroll
    for (int j = 0; j < 16; ++j) lds[(wave * 16 + j) * 64 + lane] = y[j];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if ((j & km) != wave) continue;               // wave-uniform
      uint32_t v = 0u;
      for (int w = 0; w < p.ksplit; ++w) v += lds[(w * 16 + j) * 64 + lane];
      y[j] = v;
    }
  }

  const EpiParams& e = p.ep;
  const int out_row0 = tr * 16;

  // GIN self term: bit (row % 32) of word row (row / 32) of every plane of X
  if (e.self_term != 0) {
    const uint32_t srow = min((uint32_t)(out_row0 >> 5), kw_max);
    const uint32_t voff = srow * p.ldx4 + col4;
    const int bit0 = out_row0 & 31;
    for (int pg = 0; pg < p.s; pg += 8) {
      uint32_t xs[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        xs[i] = 0u;
        if (pg + i < p.s)
          xs[i] = __builtin_amdgcn_raw_buffer_load_b32(rx, voff, (uint32_t)(pg + i) * p.psx4, 0);
      }
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        if ((j & km) != wave) continue;
        uint32_t sv = 0u;
#pragma unroll
        for (int i = 0; i < 8; ++i) sv += ((xs[i] >> (bit0 + j)) & 1u) << i;
        y[j] += sv << pg;
      }
    }
  }

  if (e.mode == QGTC_OUT_I32) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if ((j & km) != wave) continue;
      const int row = out_row0 + j;
      int32_t o = (int32_t)y[j];
      if (e.relu && o < 0) o = 0;
      if (tr_ok && c_ok && row < p.rows) reinterpret_cast<int32_t*>(e.out)[(int64_t)row * e.ld_out + c] = o;
    }
  } else if (e.mode == QGTC_OUT_F32) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if ((j & km) != wave) continue;
      const int row = out_row0 + j;
      if (tr_ok && c_ok && row < p.rows)
        reinterpret_cast<float*>(e.out)[(int64_t)row * e.ld_out + c] = dequantize_f64(y[j], row, c, e);
    }
  } else {
    const int qbits = e.rq_nbits;
    const uint32_t qmax = qbits >= 32 ? 0xffffffffu : ((1u << qbits) - 1u);
    const float qmaxf = (float)qmax;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const bool ok = tr_ok && c_ok && (out_row0 + j) < p.rows;
      y[j] = ok ? requantize_i32(y[j], e, qmax, qmaxf) : 0u;
    }
    if (!MULTI && qbits == S && p.ksplit == 1) {
      uint32_t ow[S];
#pragma unroll
      for (int i = 0; i < S; ++i) ow[i] = 0u;
      pack_rows_fast<0, S, CWS>(y, ow);
      const int sj = lane >> 2;
      const int sk = lane & 3;
      int srow_out, sword;
      bool mine;
      if constexpr (CWS == 6) {
        srow_out = rt * 16 + sj;
        sword = cg * 2 + sk;
        mine = sk < 2;
      } else {
        srow_out = (rt * rgs + sk) * 16 + sj;
        sword = 0;
        mine = sk < rgs;
      }
      mine = mine && srow_out < p.rows && sword < ((p.cols + 31) >> 5);
      if (mine) {
        uint32_t* dst = reinterpret_cast<uint32_t*>(e.out) + (int64_t)srow_out * e.ld_out + sword;
#pragma unroll
        for (int i = 0; i < S; ++i) dst[(int64_t)i * e.ps_out] = ow[i];
      }
      return;
    }
    // lane 4*j + k will store word k of row j.  CW = 64: k = 0, 1 are the two
    // words of the column group; CW = 32 / 16: k is the row group and every
    // row has a single word.
    const int sj = lane >> 2;
    const int sk = lane & 3;
    bool mine = (sj & km) == wave;
    int srow_out, sword;
    if (CWS == 6) {
      srow_out = rt * 16 + sj;
      sword = cg * 2 + sk;
      mine = mine && sk < 2;
    } else {
      srow_out = (rt * rgs + sk) * 16 + sj;
      sword = 0;
      mine = mine && sk < rgs;
    }
    mine = mine && srow_out < p.rows && sword < ((p.cols + 31) >> 5);
    uint32_t* dst = reinterpret_cast<uint32_t*>(e.out) + (mine ? (int64_t)srow_out * e.ld_out + sword : 0);

    for (int pg = 0; pg < qbits; pg += 8) {
      uint32_t ow[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) ow[i] = 0u;
      gather_rows<0, CWS>(y, ow, pg, km, wave);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (mine && pg + i < qbits) dst[(int64_t)(pg + i) * e.ps_out] = ow[i];
    }
  }
}

template <int S, int CWS, bool MULTI>
qgtc_status launch(const AggParams& p, hipStream_t stream) {
  const unsigned grid = xcd_deal_grid(p.nblocks, p.chunk_shift);
  const size_t lds = p.ksplit > 1 ? (size_t)p.ksplit * 16 * 64 * sizeof(uint32_t) : 0;
  hipLaunchKernelGGL((aggregate_kernel<S, CWS, MULTI>), dim3(grid), dim3(64 * p.ksplit), lds, stream, p);
  return launch_status();
}

template <int CWS>
qgtc_status dispatch(const AggParams& p, hipStream_t stream) {
  switch (p.s) {
    case 1: return launch<1, CWS, false>(p, stream);
    case 2: return launch<2, CWS, false>(p, stream);
    case 3: return launch<3, CWS, false>(p, stream);
    case 4: return launch<4, CWS, false>(p, stream);
    case 5: return launch<5, CWS, false>(p, stream);
    case 6: return launch<6, CWS, false>(p, stream);
    case 7: return launch<7, CWS, false>(p, stream);
    case 8: return launch<8, CWS, false>(p, stream);
    default: return launch<8, CWS, true>(p, stream);
  }
}

}  // namespace
}  // namespace qgtc

using namespace qgtc;

extern "C" qgtc_status qgtc_aggregate(const qgtc_bits* A, const qgtc_tile_map* map, const qgtc_bits* X,
                                      const qgtc_epilogue* ep, void* out, int64_t ld_out, void* stream) {
  if (!A || !X || !ep || !out) return QGTC_ERR_NULL;
  qgtc_status st = check_adjacency(A);
  if (st != QGTC_OK) return st;
  st = check_bits(X, QGTC_RIGHT);
  if (st != QGTC_OK) return st;
  if (A->block_rows > 0) {
    if (A->rows != X->rows) return QGTC_ERR_SHAPE;
  } else if (A->cols != X->rows) {
    return QGTC_ERR_SHAPE;
  }
  const int64_t x_words = span_words(X);
  if (x_words * 4 >= (int64_t)1 << 32 || X->ld_words * 4 >= (int64_t)1 << 31 ||
      X->plane_stride_words * 4 >= (int64_t)1 << 31)
    return QGTC_ERR_UNSUPPORTED;

  AggParams p{};
  p.A = A->data;
  p.lda = A->ld_words;
  p.rows = A->rows;
  p.block_rows = A->block_rows;
  p.X = X->data;
  p.ldx4 = (uint32_t)(X->ld_words * 4);
  p.psx4 = (uint32_t)(X->plane_stride_words * 4);
  p.x_bytes = (uint32_t)(x_words * 4);
  p.x_kwords = cdiv(X->rows, 32);
  p.s = X->nbits;
  p.cols = X->cols;
  if (map) {
    if (!map->row_cnt || !map->col_idx) return QGTC_ERR_NULL;
    if (map->tile_rows != 16 ||
        (map->tile_kbits != 32 && map->tile_kbits != 64 && map->tile_kbits != 128))
      return QGTC_ERR_UNSUPPORTED;
    if (map->n_tile_rows != cdiv(A->rows, 16) || map->n_tile_cols != cdiv(A->cols, map->tile_kbits))
      return QGTC_ERR_SHAPE;
    p.row_cnt = map->row_cnt;
    p.col_idx = map->col_idx;
    p.n_tile_rows = map->n_tile_rows;
    p.n_tile_cols = map->n_tile_cols;
    p.tile_words = map->tile_kbits / 32;
  } else {
    p.n_tile_rows = cdiv(A->rows, 16);
    p.n_tile_cols = cdiv(A->cols, 128);
    p.tile_words = 4;
  }
  const bool square = A->block_rows > 0 || A->rows == A->cols;
  st = make_epilogue(ep, out, ld_out, A->rows, X->cols, QGTC_LEFT, square, &p.ep);
  if (st != QGTC_OK) return st;
  if (A->rows == 0 || X->cols == 0) return QGTC_OK;

  p.cw_shift = X->cols > 32 ? 6 : (X->cols > 16 ? 5 : 4);
  const int cw = 1 << p.cw_shift;
  const int rgs = 64 / cw;
  p.n_cg = cdiv(X->cols, cw);
  p.n_rt = cdiv(p.n_tile_rows, rgs);
  p.nblocks = (uint32_t)p.n_cg * (uint32_t)p.n_rt;
  // few waves: let the four waves of a workgroup split each tile list
  p.ksplit = p.nblocks >= 4096u ? 1 : 4;
  // Each XCD takes runs of `chunk` consecutive workgroups, run k going to XCD
  // k % 8.  A run covers all column groups of a few neighbouring tile rows, which
  // read the same word rows of X from the XCD's L2 (with few tiles per row these
  // are the diagonal tiles); dealing short runs round-robin spreads the rows of
  // one subgraph over all XCDs, so a subgraph that holds far more tiles than the
  // others (the hubs of a power-law graph) does not leave seven XCDs idle.
  {
    const int opt = agg_chunk_option();
    int64_t chunk = (int64_t)(opt > 0 ? opt : 8) * p.n_cg;
    if (opt < 0) chunk = (p.nblocks + 7u) / 8u;          // one run per XCD
    int sh = 0;
    while (((int64_t)1 << sh) < chunk && sh < 30) ++sh;
    p.chunk_shift = sh;
  }

  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  ProfScope prof(QGTC_KERNEL_AGGREGATE, s);
  if (p.cw_shift == 6) return dispatch<6>(p, s);
  return p.cw_shift == 5 ? dispatch<5>(p, s) : dispatch<4>(p, s);
}
