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
//   With at most 32 (16) columns the lanes form 2 (4) groups that take different
//   words of the same tile at once (K slices) and are summed at the end, so no
//   lane idles and the tile list stays uniform over the wave.
// Zero-tile jumping: the loop runs over the precomputed list of non-zero tile
// columns of the tile row (or over all of them without a map).
// Small grids: the 1..4 waves of a workgroup split the tile list and add their
// partial sums through LDS.
#include "qgtc_internal.h"

namespace qgtc {
namespace {

#include "agg_core.inc"

// The two words that the ballots of bit (p0 + i) of q, i < S, give for one output
// row of the wave: columns 0..31 and 32..63 of the column group.
template <int S>
__device__ __forceinline__ void ballot_words(uint32_t q, int p0, uint32_t (&w)[S][4]) {
#pragma unroll
  for (int i = 0; i < S; ++i) {
    const unsigned long long m = __builtin_amdgcn_ballot_w64(((q >> (p0 + i)) & 1u) != 0u);
    w[i][0] = (uint32_t)m;
    w[i][1] = (uint32_t)(m >> 32);
    w[i][2] = 0u;
    w[i][3] = 0u;
  }
}

// Generic path: planes pg .. pg+7 of the rows the wave owns; lane 4*J + k keeps
// word k of row J.  Planes past qbits give q >> plane == 0 and are not stored.
template <int J>
__device__ __forceinline__ void gather_rows(const uint32_t (&q)[16], uint32_t (&ow)[8], int pg,
                                            int km, int wave) {
  if ((J & km) == wave) {
    uint32_t w[8][4];
    ballot_words<8>(pg < 32 ? q[J] : 0u, pg, w);
    lane_pack<8, 2>::template run<4 * J>(w, ow);
  }
  if constexpr (J + 1 < 16) gather_rows<J + 1>(q, ow, pg, km, wave);
}

// Fast path of the requantize-and-pack epilogue: as many output planes as
// feature planes (the layer case), one wave per workgroup, everything unrolled.
template <int J, int S>
__device__ __forceinline__ void pack_rows_fast(const uint32_t (&q)[16], uint32_t (&ow)[S]) {
  uint32_t w[S][4];
  ballot_words<S>(q[J], 0, w);
  lane_pack<S, 2>::template run<4 * J>(w, ow);
  if constexpr (J + 1 < 16) pack_rows_fast<J + 1, S>(q, ow);
}

// TW: words per tile (1, 2, 4); KS: K slices per wave (1, 2, 4; KS <= TW).
// PK: the jumping form with two rows per accumulator register (agg_core.inc).
template <int S, bool MULTI, int TW, int KS, bool SKIP, bool PK = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(PK ? kPack16Waves : agg_waves_per_simd(S)))) void aggregate_kernel(const AggParams p) {
  extern __shared__ uint32_t lds[];   // [ksplit][16][64] partial sums when ksplit > 1

  const unsigned bid = agg_logical_id(p);
  if (bid >= p.nblocks) return;       // whole workgroup leaves together
  const int tr = (int)(bid / (unsigned)p.n_cg);     // tile row
  const int cg = (int)(bid % (unsigned)p.n_cg);     // group of 64 columns

  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int lane = threadIdx.x & 63;
  constexpr int CW = 64 / KS;                       // columns per wave
  const int c = cg * 64 + (lane & (CW - 1));        // this lane's output column
  const bool c_ok = c < p.cols && (KS == 1 || lane < CW);   // lanes of slice 0 write the results
  const uint32_t col4 = (uint32_t)min(c, p.cols - 1) * 4u;
  uint32_t va_off, xoff;
  agg_lane_offsets<TW, KS>(p, lane, col4, &va_off, &xoff);

  int n = p.row_cnt ? p.row_cnt[tr] : p.n_tile_cols;
  n = __builtin_amdgcn_readfirstlane(n);
  // (a list that holds every tile of the row is not read: one dependent load less before the first tile)
  const int32_t* ci = (p.col_idx && n < p.n_tile_cols) ? p.col_idx + (int64_t)tr * p.n_tile_cols : nullptr;

  uint32_t kw_base = 0u;
  if (p.block_rows > 0) kw_base = (uint32_t)((tr * 16) / p.block_rows) * (uint32_t)(p.block_rows >> 5);
  const uint32_t kw_max = (uint32_t)(p.x_kwords - 1);

  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)p.X, 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t ra = agg_row_tile_rsrc(p, tr);

  uint32_t y[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) y[j] = 0u;

  const int n_chunks = MULTI ? (p.s + S - 1) / S : 1;
  for (int chunk = 0; chunk < n_chunks; ++chunk) {
    const int plane0 = chunk * S;
    constexpr int AR = PK ? 8 : 16;
    uint32_t acc[AR][S];
    zero_acc<S, AR>(acc);
    agg_loop_uniform<S, TW, KS, MULTI, SKIP, AR>(acc, p, ra, va_off, rx, xoff, ci, n, wave, p.ksplit, kw_base, kw_max,
                                                 plane0);
    uint32_t v[16];
    agg_shift_add<S>(acc, v);
#pragma unroll
    for (int j = 0; j < 16; ++j) y[j] += v[j] << plane0;
  }
  if constexpr (KS > 1) {
#pragma unroll
    for (int j = 0; j < 16; ++j) y[j] = agg_slice_sum<KS>(y[j]);
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
      if (c_ok && row < p.rows) reinterpret_cast<int32_t*>(e.out)[(int64_t)row * e.ld_out + c] = o;
    }
  } else if (e.mode == QGTC_OUT_F32) {
    // the per-row vectors of the 16 rows: one load per wave (lane j holds row j), read back
    // lane by lane in the row loop
    const int rj = min(out_row0 + (lane & 15), p.rows - 1);
    const int32_t ri_lane = e.row_i ? e.row_i[rj] : 0;
    const int32_t rl_lane = e.row_l ? e.row_l[rj] : 0;
    const int cc_ = min(c, p.cols - 1);
    const double colterm = e.ck + e.cs * (e.col_i ? (double)e.col_i[cc_] : 0.0);
    const float ca = e.col_a ? e.col_a[cc_] : 1.0f;
    const float cb = (e.col_a && e.col_b) ? e.col_b[cc_] : 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const double ri = (double)__builtin_amdgcn_readlane(ri_lane, j);
      const double rl = (double)__builtin_amdgcn_readlane(rl_lane, j);
      if ((j & km) != wave) continue;
      const int row = out_row0 + j;
      // the arithmetic of dequantize_f64_ri, with the row and column terms formed once
      const double t1 = e.cc * (double)(int32_t)y[j] + e.rs * ri;
      const double l0 = e.l0a + e.l0b * rl;
      double v = t1 + l0 * colterm;
      if (e.col_a) v = v * (double)ca + (double)cb;
      if (e.relu && v < 0.0) v = 0.0;
      if (c_ok && row < p.rows) reinterpret_cast<float*>(e.out)[(int64_t)row * e.ld_out + c] = (float)v;
    }
  } else {
    const int qbits = e.rq_nbits;
    const uint32_t qmax = qbits >= 32 ? 0xffffffffu : ((1u << qbits) - 1u);
    const float qmaxf = (float)qmax;
    // A LEFT operand has zeros in the words between the last data word of a row and its
    // leading dimension; the workgroup of the last column group writes them for its rows.
    const int data_words = (p.cols + 31) >> 5;
    const int pad_words = (int)e.ld_out - data_words;
    if (pad_words > 0 && cg == p.n_cg - 1) {
      const int rows_here = min(16, p.rows - out_row0);
      for (int idx = (int)threadIdx.x; idx < qbits * rows_here * pad_words; idx += (int)blockDim.x) {
        const int w = idx % pad_words;
        const int rj = (idx / pad_words) % rows_here;
        const int pl = idx / (pad_words * rows_here);
        reinterpret_cast<uint32_t*>(e.out)[(int64_t)pl * e.ps_out + (int64_t)(out_row0 + rj) * e.ld_out +
                                          data_words + w] = 0u;
      }
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const bool ok = c_ok && (out_row0 + j) < p.rows;
      y[j] = ok ? requantize_i32(y[j], min(c, p.cols - 1), e, qmax, qmaxf) : 0u;
    }
    if (!MULTI && qbits == S && p.ksplit == 1) {
      uint32_t ow[S];
#pragma unroll
      for (int i = 0; i < S; ++i) ow[i] = 0u;
      pack_rows_fast<0, S>(y, ow);
      const int sj = lane >> 2;
      const int sk = lane & 3;
      const int srow_out = tr * 16 + sj;
      const int sword = cg * 2 + sk;
      bool mine = sk < 2;
      mine = mine && srow_out < p.rows && sword < ((p.cols + 31) >> 5);
      if (mine) {
        uint32_t* dst = reinterpret_cast<uint32_t*>(e.out) + (int64_t)srow_out * e.ld_out + sword;
#pragma unroll
        for (int i = 0; i < S; ++i) dst[(int64_t)i * e.ps_out] = ow[i];
      }
      return;
    }
    // lane 4*j + k will store word k (k = 0, 1) of row j of the column group
    const int sj = lane >> 2;
    const int sk = lane & 3;
    bool mine = (sj & km) == wave && sk < 2;
    const int srow_out = tr * 16 + sj;
    const int sword = cg * 2 + sk;
    mine = mine && srow_out < p.rows && sword < ((p.cols + 31) >> 5);
    uint32_t* dst = reinterpret_cast<uint32_t*>(e.out) + (mine ? (int64_t)srow_out * e.ld_out + sword : 0);

    for (int pg = 0; pg < qbits; pg += 8) {
      uint32_t ow[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) ow[i] = 0u;
      gather_rows<0>(y, ow, pg, km, wave);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (mine && pg + i < qbits) dst[(int64_t)(pg + i) * e.ps_out] = ow[i];
    }
  }
}

template <int S, bool MULTI, int TW, int KS>
qgtc_status launch_one(const AggParams& p, hipStream_t stream) {
  const unsigned grid = xcd_deal_grid(p.nblocks, p.chunk_shift);
  const size_t lds = p.ksplit > 1 ? (size_t)p.ksplit * 16 * 64 * sizeof(uint32_t) : 0;
  if constexpr (S >= kPack16MinPlanes && !MULTI) {
    if (p.skip_words && p.pack16) {
      hipLaunchKernelGGL((aggregate_kernel<S, MULTI, TW, KS, true, true>), dim3(grid), dim3(64 * p.ksplit), lds, stream, p);
      return launch_status();
    }
  }
  if constexpr (S >= kSkipMinPlanes) {
    if (p.skip_words) {
      hipLaunchKernelGGL((aggregate_kernel<S, MULTI, TW, KS, true>), dim3(grid), dim3(64 * p.ksplit), lds, stream, p);
      return launch_status();
    }
  }
  hipLaunchKernelGGL((aggregate_kernel<S, MULTI, TW, KS, false>), dim3(grid), dim3(64 * p.ksplit), lds, stream, p);
  return launch_status();
}

template <int S, bool MULTI>
qgtc_status launch(const AggParams& p, hipStream_t stream) {
  switch (p.tile_words * 8 + p.kslices) {
    case 4 * 8 + 1: return launch_one<S, MULTI, 4, 1>(p, stream);
    case 4 * 8 + 2: return launch_one<S, MULTI, 4, 2>(p, stream);
    case 4 * 8 + 4: return launch_one<S, MULTI, 4, 4>(p, stream);
    case 2 * 8 + 1: return launch_one<S, MULTI, 2, 1>(p, stream);
    case 2 * 8 + 2: return launch_one<S, MULTI, 2, 2>(p, stream);
    case 1 * 8 + 1: return launch_one<S, MULTI, 1, 1>(p, stream);
    default: return QGTC_ERR_UNSUPPORTED;
  }
}

qgtc_status dispatch(const AggParams& p, hipStream_t stream) {
  switch (p.s) {
    case 1: return launch<1, false>(p, stream);
    case 2: return launch<2, false>(p, stream);
    case 3: return launch<3, false>(p, stream);
    case 4: return launch<4, false>(p, stream);
    case 5: return launch<5, false>(p, stream);
    case 6: return launch<6, false>(p, stream);
    case 7: return launch<7, false>(p, stream);
    case 8: return launch<8, false>(p, stream);
    default: return launch<8, true>(p, stream);
  }
}

}  // namespace
}  // namespace qgtc

using namespace qgtc;

extern "C" qgtc_status qgtc_aggregate(const qgtc_bits* A, const qgtc_tile_map* map, const qgtc_bits* X,
                                      const qgtc_epilogue* ep, void* out, int64_t ld_out, void* stream) {
  if (!A || !X || !ep) return QGTC_ERR_NULL;
  AggParams p{};
  qgtc_status st = agg_fill_params(A, map, X, &p);
  if (st != QGTC_OK) return st;
  if (!out) return (A->rows == 0 || X->cols == 0) ? QGTC_OK : QGTC_ERR_NULL;   // an empty result needs no buffer
  const bool square = A->block_rows > 0 || A->rows == A->cols;
  st = make_epilogue(ep, out, ld_out, A->rows, X->cols, QGTC_LEFT, square, &p.ep);
  if (st != QGTC_OK) return st;
  st = check_tuning(ep->tuning);
  if (st != QGTC_OK) return st;
  if (A->rows == 0 || X->cols == 0) return QGTC_OK;

  p.kslices = agg_kslices(X->cols, p.tile_words);
  p.n_cg = cdiv(X->cols, 64);
  p.nblocks = (uint32_t)p.n_cg * (uint32_t)p.n_tile_rows;
  // few waves: let the four waves of a workgroup split each tile list
  // (fewer than the wave slots of the device: CUs x 4 SIMDs x waves per SIMD)
  const unsigned slots = (unsigned)(device_compute_units() * 4 * agg_waves_per_simd(X->nbits > 8 ? 8 : X->nbits));
  p.ksplit = p.nblocks >= slots ? 1 : 4;
  // Each XCD takes runs of `chunk` consecutive workgroups, run k going to XCD
  // k % 8.  A run covers all column groups of a few neighbouring tile rows, which
  // read the same word rows of X from the XCD's L2 (with few tiles per row these
  // are the diagonal tiles); dealing short runs round-robin spreads the rows of
  // one subgraph over all XCDs, so a subgraph that holds far more tiles than the
  // others (the hubs of a power-law graph) does not leave seven XCDs idle.
  agg_set_dealing(&p, p.n_cg, ep->tuning ? ep->tuning->agg_xcd_run : 0);
  p.skip_words = agg_skip_words(p.s > 8 ? 8 : p.s, ep->tuning ? ep->tuning->zero_words : 0, map != nullptr);
  p.pack16 = agg_pack16(p.skip_words, p.s, p.n_tile_cols, p.tile_words);

  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  ProfScope prof(QGTC_KERNEL_AGGREGATE, s);
  return dispatch(p, s);
}
