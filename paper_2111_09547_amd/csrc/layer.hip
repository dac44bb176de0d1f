// One quantized GNN layer in a single kernel (Algorithm 1 of the paper with the
// inter-layer fusion of Section 4.5 taken one step further): neighbour
// aggregation on the vector ALUs, requantization, node update on the int8 matrix
// cores and the output epilogue, with the aggregated tile never leaving the CU.
//
// A workgroup owns one 16-row tile of A.
//   1. Aggregation: as in aggregate.hip (lane <-> feature column, AND + popcount
//      with the adjacency word broadcast by DPP, zero tiles jumped through the
//      tile list).  The workgroup's waves stand side by side over the 64-column
//      groups of X (a wave walks several groups when there are more groups than
//      waves) and, for short grids, split the tile list between them.
//   2. Each wave requantizes its 16 x 64 results to codes of at most 8 bits and
//      writes them as bytes into the Y tile in LDS, row-major: this is already
//      the operand order of the matrix instruction (16 consecutive K positions
//      per lane), so the popcount side hands over to the matrix cores without
//      a transposition.
//   3. Update: v_mfma_i32_16x16x64_i8 over the Y tile and the weights, which a
//      small kernel has put into operand order as bytes beforehand.  8-bit codes
//      are split into 7 bits + top bit because the instruction is signed.  The
//      16-column output tiles (and chunks of K) are dealt to the waves; results
//      are added into the Z tile in LDS.
//   4. Epilogue: lane <-> output column, 16 rows per lane: int32, dequantized
//      fp32, or requantized codes whose 8 x 16 bit matrix is transposed in
//      registers into the 16-bit halves of the packed words of the next layer's X
//      (32 nodes per word, so a 16-row tile owns half a word).
#include "qgtc_internal.h"

#include <cmath>

namespace qgtc {
namespace {

#include "agg_core.inc"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

struct LayerParams {
  AggParams a;            // aggregation operands; a.ep: requantization of its result
  EpiParams up;           // epilogue of the update
  const uint8_t* wb;      // weights as bytes in operand order: [part][tile][k step][lane][16]
  int64_t wb_part;        // bytes between the two parts (7 low bits / top bit)
  int32_t h;              // output columns
  int32_t n_nt_w;         // 16-column output tiles that come from W
  int32_t n_nt;           // ... plus the all-ones tile that yields the row sums of Y
  int32_t n_ks;           // 64-wide steps along the contraction dimension
  int32_t n_kc, ks_per;   // chunks of steps dealt to different waves, steps per chunk
  int32_t ys;             // bytes per row of the Y tile
  int32_t zs;             // words per row of the Z tile
  int32_t cgw;            // waves side by side over the column groups
  int32_t n_pass;         // column groups per wave
  int32_t split_y, split_w;
  int32_t want_rowsum;
  int32_t yb_off, z_off;  // LDS offsets in words
};

// Weights: packed planes -> bytes in the operand order of the matrix instruction.
// Thread (tile nt, step ks, lane l) writes the 16 bytes of column 16 nt + l % 16,
// K positions 64 ks + 16 (l / 16) .. + 15.
__global__ __launch_bounds__(256) void weight_bytes_kernel(const uint32_t* W, int64_t ldw, int64_t psw,
                                                           int t, int kwords, int cols, int n_nt_w,
                                                           int n_ks, int split_w, uint8_t* wb,
                                                           int64_t wb_part) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int lane = idx & 63;
  const int ks = (idx >> 6) % n_ks;
  const int nt = (idx >> 6) / n_ks;
  if (nt >= n_nt_w) return;
  const int col = nt * 16 + (lane & 15);
  const int k0 = ks * 64 + (lane >> 4) * 16;
  const int kw = k0 >> 5;
  const int sh = k0 & 31;
  uint32_t f[8];
#pragma unroll
  for (int pl = 0; pl < 8; ++pl) {
    f[pl] = 0u;
    if (pl < t && col < cols && kw < kwords)
      f[pl] = (W[(int64_t)pl * psw + (int64_t)kw * ldw + col] >> sh) & 0xffffu;
  }
  uint32_t d[4];
  planes_to_bytes(f, t, d);
  v4u lo = {d[0], d[1], d[2], d[3]};
  uint8_t* dst = wb + (int64_t)idx * 16;
  if (split_w) {
    v4u hi = (lo >> 7) & 0x01010101u;
    lo = lo & 0x7f7f7f7fu;
    *reinterpret_cast<v4u*>(dst + wb_part) = hi;
  }
  *reinterpret_cast<v4u*>(dst) = lo;
}

// Parameters that only the phases after the tile loop need are read from the
// kernel-argument segment through a pointer the compiler cannot see through, at
// the point of use: loaded at kernel entry (where the compiler puts every argument
// load) they would sit in ~200 SGPRs across the tile loop and be spilled.
typedef const __attribute__((address_space(4))) LayerParams* LateParams;
#define QGTC_LATE(ptr) asm volatile("" : "+s"(ptr))

// PK: the jumping form with two rows per accumulator register (agg_core.inc): 64 instead of
// 128 accumulator registers at 8 planes, four waves per SIMD instead of three.
template <int S, int TW, int KS, bool SKIP, bool PK = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(PK ? kPack16Waves : agg_waves_per_simd(S)))) void layer_kernel(const LayerParams p) {
  extern __shared__ uint32_t lds[];
  __builtin_amdgcn_s_setprio(3);
  const AggParams& a = p.a;
  int tr, n;                                         // tile row of this workgroup, its tile count
  if (!agg_pick_tile_row(a, &tr, &n)) return;        // whole workgroup leaves together
  LateParams kp = (LateParams)__builtin_amdgcn_kernarg_segment_ptr();

  const int nw = (int)(blockDim.x >> 6);
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int lane = threadIdx.x & 63;
  const int wcg = wave % p.cgw;                      // position over the column groups
  const int kpart = wave / p.cgw;                    // share of the tile list
  uint32_t* part = lds;                              // [wave][16][64] partial sums (K split)
  uint8_t* yb = reinterpret_cast<uint8_t*>(lds + p.yb_off);
  uint32_t* z = lds + p.z_off;

  for (int i = threadIdx.x; i < 16 * p.zs; i += (int)blockDim.x) z[i] = 0u;

  const int out_row0 = tr * 16;
  const __amdgpu_buffer_rsrc_t ra = agg_row_tile_rsrc(a, tr);
  constexpr int CW = 64 / KS;                        // columns per wave (K slices: see agg_core.inc)
  n = __builtin_amdgcn_readfirstlane(n);
  // (a list that holds every tile of the row is not read: one dependent load less before the first tile)
  const int32_t* ci = (a.col_idx && n < a.n_tile_cols) ? a.col_idx + (int64_t)tr * a.n_tile_cols : nullptr;
  uint32_t kw_base = 0u;
  if (a.block_rows > 0) kw_base = (uint32_t)(out_row0 / a.block_rows) * (uint32_t)(a.block_rows >> 5);
  const uint32_t kw_max = (uint32_t)(a.x_kwords - 1);
  __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)a.X, 0, (int)a.x_bytes, 0x00020000);
  const int km = a.ksplit - 1;                       // ksplit is 1, 2 or 4
  const bool self_term = a.ep.self_term != 0;

  // B operands of the first matrix instruction of this wave, fetched while the Y tile
  // is still being finished
  const int ln = lane & 15;                          // row of Y / column of W inside a tile
  const int g = lane >> 4;                           // K sub-block, and row group of the result
  v4u b7_first, bb_first;                            // set in the last pass
  // Short form of phase 3 (one K step, at most four output tiles per wave - every layer of up to
  // 64 input columns): the operands of all the wave's tiles are requested at once
  v4u bq7[4], bqb[4];
  // (not below three planes: those kernels need fewer registers than this form, and a wave per
  // SIMD more is worth more to them)
  const bool short3 = S >= 3 && a.n_cg == 1 && p.n_nt_w <= 4 * nw;      // one column group: one pass below

  // ---- 1 + 2: aggregate, requantize, bytes into the Y tile ---------------------
  for (int pass = 0; pass < p.n_pass; ++pass) {
    const int cg = pass * p.cgw + wcg;               // wave-uniform
    const bool cg_ok = cg < a.n_cg;
    const int c = cg * 64 + (lane & (CW - 1));
    const bool c_ok = cg_ok && c < a.cols && (KS == 1 || lane < CW);   // slice 0 hands the results on
    const uint32_t col4 = (uint32_t)min(c, a.cols - 1) * 4u;
    uint32_t va_off, xoff;
    agg_lane_offsets<TW, KS>(a, lane, col4, &va_off, &xoff);

    constexpr int AR = PK ? 8 : 16;                  // accumulator rows (two tile rows per register when PK)
    uint32_t acc[AR][S];
    zero_acc<S, AR>(acc);
    // The tile loop runs at the lowest issue priority, everything around it (short chains
    // of dependent loads, LDS traffic and matrix instructions) above it: those sections
    // have few instructions, and the sooner they are through, the sooner the wave's slot
    // takes the next tile row.
    __builtin_amdgcn_s_setprio(0);
    if (cg_ok)
      agg_loop_uniform<S, TW, KS, false, SKIP, AR, true>(acc, a, ra, va_off, rx, xoff, ci, n, kpart, a.ksplit, kw_base, kw_max, 0);
    __builtin_amdgcn_s_setprio(3);
    // GIN self term: the 16 bits (row0 % 32 ..) of word row (row0 / 32) of every plane of X
    // are this lane's codes of the 16 rows, bit-transposed; requested here, used behind the
    // shift-and-add, so that their way through the memory system is not waited for (the
    // words are left unset without a self term: set to zero on that path, the two paths would
    // meet in a copy that waits for the loads)
    uint32_t f[8];
    if (self_term) {
      const uint32_t srow = min((uint32_t)(out_row0 >> 5), kw_max);
      const uint32_t voff = srow * a.ldx4 + col4;
#pragma unroll
      for (int i = 0; i < S; ++i) f[i] = __builtin_amdgcn_raw_buffer_load_b32(rx, voff, (uint32_t)i * a.psx4, 0);
    }
    uint32_t y[16];
    agg_shift_add<S>(acc, y);
#pragma unroll
    for (int j = 0; j < 16; ++j) y[j] = agg_slice_sum<KS>(y[j]);

    // (the same for the wave-uniform row tests below: computed up front they are kept as
    // sixteen SGPR pairs across the loop and spilled)
    // (the sums take part in the same statement: whatever is fetched through k2 below is
    // requested behind the shift-and-add, when the accumulators' registers are free)
    LateParams k2 = kp;
    asm volatile("" : "+s"(k2), "+v"(y[0]), "+v"(y[1]), "+v"(y[2]), "+v"(y[3]), "+v"(y[4]), "+v"(y[5]), "+v"(y[6]),
                 "+v"(y[7]), "+v"(y[8]), "+v"(y[9]), "+v"(y[10]), "+v"(y[11]), "+v"(y[12]), "+v"(y[13]),
                 "+v"(y[14]), "+v"(y[15]));
    int km2 = km, kpart2 = kpart, rows_left = a.rows - out_row0;
    asm volatile("" : "+s"(km2), "+s"(kpart2), "+s"(rows_left));
    if (pass == p.n_pass - 1) {
      // unit `wave` is output tile `wave`, first chunk of K (see phase 3); a wave
      // without such a unit fetches tile 0 and does not use it
      const int nt0 = wave < k2->n_nt_w ? wave : 0;
      const uint8_t* src = k2->wb + ((int64_t)(nt0 * k2->n_ks) * 64 + lane) * 16;
      b7_first = *reinterpret_cast<const v4u*>(src);
      bb_first = *reinterpret_cast<const v4u*>(src + (k2->split_w ? k2->wb_part : 0));
    }

    // K split: wave (wcg, kpart) finishes the rows j with j % ksplit == kpart
    if (a.ksplit > 1) {
      if (pass > 0) __syncthreads();                 // the sums of the previous pass have been read
#pragma unroll
      for (int j = 0; j < 16; ++j) part[(wave * 16 + j) * 64 + lane] = y[j];
      __syncthreads();
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        if ((j & km2) != kpart2) continue;           // wave-uniform
        uint32_t v = 0u;
        for (int kp2 = 0; kp2 < a.ksplit; ++kp2) v += part[((kp2 * p.cgw + wcg) * 16 + j) * 64 + lane];
        y[j] = v;
      }
    }

    if (self_term) {
      const int bit0 = out_row0 & 31;
#pragma unroll
      for (int i = 0; i < 8; ++i) f[i] = i < S ? f[i] >> bit0 : 0u;
      uint32_t lo0 = (f[0] & 0xffu) | ((f[1] & 0xffu) << 8) | ((f[2] & 0xffu) << 16) | (f[3] << 24);
      uint32_t hi0 = (f[4] & 0xffu) | ((f[5] & 0xffu) << 8) | ((f[6] & 0xffu) << 16) | (f[7] << 24);
      uint32_t lo1 = ((f[0] >> 8) & 0xffu) | (f[1] & 0xff00u) | ((f[2] & 0xff00u) << 8) | ((f[3] & 0xff00u) << 16);
      uint32_t hi1 = ((f[4] >> 8) & 0xffu) | (f[5] & 0xff00u) | ((f[6] & 0xff00u) << 8) | ((f[7] & 0xff00u) << 16);
      transpose_bits_8x8(lo0, hi0);                  // byte j: code of row j (rows 0..7)
      transpose_bits_8x8(lo1, hi1);                  // rows 8..15
      const uint32_t sw[4] = {lo0, hi0, lo1, hi1};
#pragma unroll
      for (int j = 0; j < 16; ++j) y[j] += (sw[j >> 2] >> (8 * (j & 3))) & 0xffu;
    }

    {
      const int32_t relu_floor = k2->a.ep.relu ? 0 : (int32_t)0x80000000;
      const int32_t rq_lo = k2->a.ep.rq_lo;
      const float rq_inv = k2->a.ep.rq_inv_scale;
      const float qmaxf = (float)((1u << k2->a.ep.rq_nbits) - 1u);   // at most 8 bits here
      const int ys = k2->ys;
      // with the usual range [0, hi) the integer part of the rule is max(c, 0), with or without ReLU
      const bool from_zero = rq_lo == 0;                              // wave-uniform
      uint8_t* yrow = yb + cg * 64 + lane;
      if (from_zero && a.ksplit == 1) {
        // the common case on its own: no test per row, one form of the rule
        if (cg_ok) {
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const uint32_t q = requantize_code_relu0(y[j], rq_inv, qmaxf);
            yrow[j * ys] = (uint8_t)((c_ok && j < rows_left) ? q : 0u);   // zeros from the lanes past the last column
          }
        }
      } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          if ((j & km2) != kpart2) continue;
          uint32_t q = from_zero ? requantize_code_relu0(y[j], rq_inv, qmaxf)
                                 : requantize_code_small(y[j], relu_floor, rq_lo, rq_inv, qmaxf);
          q = (c_ok && j < rows_left) ? q : 0u;
          if (cg_ok) yrow[j * ys] = (uint8_t)q;
        }
      }
    }
  }
  if (short3) {
    // (the first tile's operands are on their way since the end of the tile loop; the others
    // are requested behind the pass loop: inside it, the compiler keeps their 24 registers
    // allocated across the tile loop and spills them)
    LateParams k2 = kp;
    QGTC_LATE(k2);
    bq7[0] = b7_first;
    bqb[0] = bb_first;
#pragma unroll
    for (int q = 1; q < 4; ++q) {
      const int nt = wave + q * nw;                  // wave-uniform
      if (nt < k2->n_nt_w) {
        const uint8_t* src = k2->wb + ((int64_t)nt * 64 + lane) * 16;
        bq7[q] = *reinterpret_cast<const v4u*>(src);
        bqb[q] = *reinterpret_cast<const v4u*>(src + (k2->split_w ? k2->wb_part : 0));
      }
    }
  }
  __syncthreads();

  // ---- 3: Z += Y tile x W on the matrix cores -----------------------------------
  // A unit is an output tile (16 columns) times a chunk of K steps; unit u goes to
  // wave u % nw, units u < n_nt cover the first chunk.
  {
    LateParams k3 = kp;
    QGTC_LATE(k3);
    const int n_nt = k3->n_nt, n_nt_w = k3->n_nt_w, n_ks = k3->n_ks, ks_per = k3->ks_per;
    const int ys = k3->ys, zs = p.zs;
    const bool split_y = k3->split_y != 0, split_w = k3->split_w != 0;
    const uint8_t* wb = k3->wb;
    const int64_t wb_part = k3->wb_part;
    const int n_units = n_nt * k3->n_kc;
    if (short3) {
      // the Y tile is one operand (16 rows x 64 bytes); every tile of the wave is one to four
      // independent matrix instructions on it, and each element of Z has one writer
      const v4u av = *reinterpret_cast<const v4u*>(yb + ln * ys + g * 16);
      v4u a7 = av, ab = {0u, 0u, 0u, 0u};
      if (split_y) {
        a7 = av & 0x7f7f7f7fu;
        ab = (av >> 7) & 0x01010101u;
      }
      const v4i zero = {0, 0, 0, 0};
#pragma unroll
      for (int q = 0; q < 5; ++q) {                  // (a fifth tile can only be the one that sums the rows)
        const int nt = wave + q * nw;
        if (nt >= n_nt) break;                       // wave-uniform
        v4u b7 = bq7[q < 4 ? q : 0];
        const bool ones = nt >= n_nt_w;              // the tile whose column 0 sums the rows of Y
        if (ones) {
          const uint32_t one = ln == 0 ? 0x01010101u : 0u;
          b7 = (v4u){one, one, one, one};
        }
        v4i acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8((v4i)a7, (v4i)b7, zero, 0, 0, 0);
        v4i acc7 = zero, acc14 = zero;
        if (split_y) acc7 = __builtin_amdgcn_mfma_i32_16x16x64_i8((v4i)ab, (v4i)b7, acc7, 0, 0, 0);
        if (split_w && !ones) {
          acc7 = __builtin_amdgcn_mfma_i32_16x16x64_i8((v4i)a7, (v4i)bqb[q < 4 ? q : 0], acc7, 0, 0, 0);
          if (split_y) acc14 = __builtin_amdgcn_mfma_i32_16x16x64_i8((v4i)ab, (v4i)bqb[q < 4 ? q : 0], acc14, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
          z[(4 * g + r) * zs + nt * 16 + ln] = (uint32_t)acc1[r] + ((uint32_t)acc7[r] << 7) + ((uint32_t)acc14[r] << 14);
      }
    } else {
    // The wave's (unit, K step) pairs one after the other; the weights of the next pair are
    // requested before the matrix instructions of the current one, into the other of two
    // operand buffers (the loop body is written out twice, so no buffer is ever copied).
    auto load_b = [&](int u, int ks, v4u& b7, v4u& bb) {
      const int nt = u % n_nt;
      if (nt >= n_nt_w) {                            // the tile whose column 0 sums the rows of Y (bb is not read)
        const uint32_t one = ln == 0 ? 0x01010101u : 0u;
        b7 = (v4u){one, one, one, one};
      } else {
        const uint8_t* src = wb + ((int64_t)(nt * n_ks + ks) * 64 + lane) * 16;
        b7 = *reinterpret_cast<const v4u*>(src);
        if (split_w) bb = *reinterpret_cast<const v4u*>(src + wb_part);   // read only when split_w
      }
    };
    int u = wave;
    int ks = (u / n_nt) * ks_per;
    v4u b7a = b7_first, bba = bb_first;              // fetched early for unit `wave` when it is a tile of W, step 0
    v4u b7b = {0u, 0u, 0u, 0u}, bbb = {0u, 0u, 0u, 0u};
    if (u < n_units && !(u < n_nt_w && ks == 0)) load_b(u, ks, b7a, bba);
    v4i acc1 = {0, 0, 0, 0}, acc7 = {0, 0, 0, 0}, acc14 = {0, 0, 0, 0};
    // one pair with the operands (b7, bb), the next pair's into (nb7, nbb); false after the last
    auto pair = [&](const v4u& b7, const v4u& bb, v4u& nb7, v4u& nbb) -> bool {
      const int nt = u % n_nt;
      const int ks1 = min((u / n_nt) * ks_per + ks_per, n_ks);
      const bool ones = nt >= n_nt_w;
      int nu = u, nks = ks + 1;
      if (nks >= ks1) { nu = u + nw; nks = (nu / n_nt) * ks_per; }
      if (nu < n_units) load_b(nu, nks, nb7, nbb);
      const v4u av = *reinterpret_cast<const v4u*>(yb + ln * ys + ks * 64 + g * 16);
      v4u a7 = av, ab = {0u, 0u, 0u, 0u};
      if (split_y) {
        a7 = av & 0x7f7f7f7fu;
        ab = (av >> 7) & 0x01010101u;
      }
      acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8((v4i)a7, (v4i)b7, acc1, 0, 0, 0);
      if (split_y) acc7 = __builtin_amdgcn_mfma_i32_16x16x64_i8((v4i)ab, (v4i)b7, acc7, 0, 0, 0);
      if (split_w && !ones) {
        acc7 = __builtin_amdgcn_mfma_i32_16x16x64_i8((v4i)a7, (v4i)bb, acc7, 0, 0, 0);
        if (split_y) acc14 = __builtin_amdgcn_mfma_i32_16x16x64_i8((v4i)ab, (v4i)bb, acc14, 0, 0, 0);
      }
      if (nu != u) {
        // the unit is complete; element r of the result: row 4 g + r, column ln of the tile
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t v = (uint32_t)acc1[r] + ((uint32_t)acc7[r] << 7) + ((uint32_t)acc14[r] << 14);
          atomicAdd(&z[(4 * g + r) * zs + nt * 16 + ln], v);
        }
        acc1 = (v4i){0, 0, 0, 0};
        acc7 = (v4i){0, 0, 0, 0};
        acc14 = (v4i){0, 0, 0, 0};
      }
      u = nu;
      ks = nks;
      return u < n_units;
    };
    if (u < n_units) {
      while (true) {
        if (!pair(b7a, bba, b7b, bbb)) break;
        if (!pair(b7b, bbb, b7a, bba)) break;
      }
    }
    }
  }
  __syncthreads();

  // ---- 4: epilogue, lane <-> output column ---------------------------------------
  LateParams k4 = kp;
  QGTC_LATE(k4);
  const int n_out = k4->h;
  const int zs = p.zs;
  const int mode = k4->up.mode;
  int valid_rows = a.rows - out_row0;
  asm volatile("" : "+s"(valid_rows));
  for (int hb = wave * 64; hb < n_out; hb += nw * 64) {
    const int h = hb + lane;
    const bool h_ok = h < n_out;
    const int hc = h_ok ? h : n_out - 1;
    uint32_t zz[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) zz[j] = z[j * zs + hc];

    if (mode == QGTC_OUT_I32) {
      const int relu = k4->up.relu;
      int32_t* out = reinterpret_cast<int32_t*>(k4->up.out) + (int64_t)out_row0 * k4->up.ld_out + h;
      const int64_t ld_out = k4->up.ld_out;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        int32_t o = (int32_t)zz[j];
        if (relu && o < 0) o = 0;
        if (h_ok && j < valid_rows) out[j * ld_out] = o;
      }
    } else if (mode == QGTC_OUT_F32) {
      EpiParams e;
      e.relu = k4->up.relu;
      e.cc = k4->up.cc; e.rs = k4->up.rs; e.l0a = k4->up.l0a; e.l0b = k4->up.l0b;
      e.ck = k4->up.ck; e.cs = k4->up.cs;
      e.row_i = k4->up.row_i; e.row_l = k4->up.row_l; e.col_i = k4->up.col_i;
      e.col_a = k4->up.col_a; e.col_b = k4->up.col_b;
      float* out = reinterpret_cast<float*>(k4->up.out);
      const int64_t ld_out = k4->up.ld_out;
      const int want_rowsum = k4->want_rowsum;
      const int sum_col = k4->n_nt_w * 16;
      // The per-row vectors (degree-like sums) of the 16 rows: one load per wave, lane j holds
      // row j, and a lane's row loop reads them back lane by lane - instead of 16 loads of
      // one address each, waited for one after the other.
      const int rj = out_row0 + min(lane & 15, valid_rows - 1);
      int32_t ri_lane = 0, rl_lane = 0;
      if (want_rowsum) ri_lane = (int32_t)z[(lane & 15) * zs + sum_col];
      else if (e.row_i) ri_lane = e.row_i[rj];
      if (e.row_l) rl_lane = e.row_l[rj];
      const double colterm = e.ck + e.cs * (e.col_i ? (double)e.col_i[hc] : 0.0);
      const float ca = e.col_a ? e.col_a[hc] : 1.0f;
      const float cb = (e.col_a && e.col_b) ? e.col_b[hc] : 0.0f;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int row = out_row0 + j;
        const int32_t rij = __builtin_amdgcn_readlane(ri_lane, j);
        const double ri = want_rowsum ? (double)(uint32_t)rij : (double)rij;   // a sum of codes, or the caller's int32
        const double rl = (double)__builtin_amdgcn_readlane(rl_lane, j);
        // the arithmetic of dequantize_f64_ri, with the row and column terms formed once
        const double t1 = e.cc * (double)(int32_t)zz[j] + e.rs * ri;
        const double l0 = e.l0a + e.l0b * rl;
        double v = t1 + l0 * colterm;
        if (e.col_a) v = v * (double)ca + (double)cb;
        if (e.relu && v < 0.0) v = 0.0;
        if (h_ok && j < valid_rows) out[(int64_t)row * ld_out + h] = (float)v;
      }
    } else {
      const int relu = k4->up.relu;
      const int32_t rq_lo = k4->up.rq_lo;
      const float rq_inv = k4->up.rq_inv_scale;
      const int qbits = k4->up.rq_nbits;             // at most 8 here
      const uint32_t qmax = (1u << qbits) - 1u;
      const float qmaxf = (float)qmax;
      uint32_t b[4] = {0u, 0u, 0u, 0u};
      const float* col_a = k4->up.col_a;             // folded batch normalization, or NULL
      if (col_a) {
        const float* col_b = k4->up.col_b;
        const float ca = col_a[hc];
        const float cb = col_b ? col_b[hc] : 0.0f;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          uint32_t q = requantize_affine(zz[j], ca, cb, relu, rq_lo, rq_inv, qmax, qmaxf);
          q = (h_ok && j < valid_rows) ? q : 0u;
          b[j >> 2] |= q << (8 * (j & 3));
        }
      } else if (rq_lo == 0) {                       // wave-uniform; max(c, 0) with or without ReLU
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          uint32_t q = requantize_code_relu0(zz[j], rq_inv, qmaxf);
          q = (h_ok && j < valid_rows) ? q : 0u;
          b[j >> 2] |= q << (8 * (j & 3));
        }
      } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          uint32_t q = requantize_code_small(zz[j], relu ? 0 : (int32_t)0x80000000, rq_lo, rq_inv, qmaxf);
          q = (h_ok && j < valid_rows) ? q : 0u;
          b[j >> 2] |= q << (8 * (j & 3));
        }
      }
      transpose_bits_8x8(b[0], b[1]);                // byte i: bit i of the codes of rows 0..7
      transpose_bits_8x8(b[2], b[3]);                // rows 8..15
      // RIGHT layout of the next layer's X: 32 consecutive rows per word; this tile
      // owns the lower or the upper 16 bits.  The last tile of a matrix whose row
      // count leaves the upper half without a tile writes the whole word.
      const bool upper = (out_row0 & 16) != 0;
      const bool whole = !upper && valid_rows <= 16;
      const int64_t ps4 = k4->up.ps_out * 4;
      uint8_t* dst = reinterpret_cast<uint8_t*>(k4->up.out) +
                     (((int64_t)(out_row0 >> 5) * k4->up.ld_out + hc) << 2) + (upper ? 2 : 0);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t w0 = (b[i >> 2] >> (8 * (i & 3))) & 0xffu;
        const uint32_t w1 = (b[2 + (i >> 2)] >> (8 * (i & 3))) & 0xffu;
        const uint32_t word = w0 | (w1 << 8);
        if (i < qbits && h_ok) {
          uint8_t* d = dst + i * ps4;
          if (whole) *reinterpret_cast<uint32_t*>(d) = word;
          else *reinterpret_cast<uint16_t*>(d) = (uint16_t)word;
        }
      }
    }
  }
}

template <int S, bool SKIP, bool PK = false>
qgtc_status launch_form(const LayerParams& p, unsigned nw, size_t lds_bytes, hipStream_t stream) {
  const unsigned grid = xcd_deal_grid(p.a.nblocks, p.a.chunk_shift);
  const dim3 g(grid), b(64 * nw);
  switch (p.a.tile_words * 8 + p.a.kslices) {
    case 4 * 8 + 1: hipLaunchKernelGGL((layer_kernel<S, 4, 1, SKIP, PK>), g, b, lds_bytes, stream, p); break;
    case 4 * 8 + 2: hipLaunchKernelGGL((layer_kernel<S, 4, 2, SKIP, PK>), g, b, lds_bytes, stream, p); break;
    case 4 * 8 + 4: hipLaunchKernelGGL((layer_kernel<S, 4, 4, SKIP, PK>), g, b, lds_bytes, stream, p); break;
    case 2 * 8 + 1: hipLaunchKernelGGL((layer_kernel<S, 2, 1, SKIP, PK>), g, b, lds_bytes, stream, p); break;
    case 2 * 8 + 2: hipLaunchKernelGGL((layer_kernel<S, 2, 2, SKIP, PK>), g, b, lds_bytes, stream, p); break;
    case 1 * 8 + 1: hipLaunchKernelGGL((layer_kernel<S, 1, 1, SKIP, PK>), g, b, lds_bytes, stream, p); break;
    default: return QGTC_ERR_UNSUPPORTED;
  }
  return launch_status();
}

template <int S>
qgtc_status launch(const LayerParams& p, unsigned nw, size_t lds_bytes, hipStream_t stream) {
  if constexpr (S >= kPack16MinPlanes) {
    if (p.a.skip_words && p.a.pack16) return launch_form<S, true, true>(p, nw, lds_bytes, stream);
  }
  if constexpr (S >= kSkipMinPlanes) {
    if (p.a.skip_words) return launch_form<S, true>(p, nw, lds_bytes, stream);
  }
  return launch_form<S, false>(p, nw, lds_bytes, stream);
}

}  // namespace

size_t layer_fused_workspace_bytes(int32_t in_cols, int32_t out_cols) {
  // two parts of ceil(out/16) x ceil(in/64) operand blocks of 1 KiB
  return (size_t)2 * (size_t)cdiv(out_cols, 16) * (size_t)cdiv(in_cols, 64) * 1024;
}

qgtc_status layer_fused(const qgtc_bits* A, const qgtc_tile_map* map, const qgtc_bits* X,
                        const qgtc_bits* W, const qgtc_epilogue* agg_ep, const qgtc_epilogue* upd_ep,
                        void* workspace, size_t workspace_bytes, void* out, int64_t ld_out,
                        hipStream_t stream, bool* done) {
  *done = false;
  if (!A || !X || !W || !agg_ep || !upd_ep || !workspace || !out) return QGTC_OK;
  const qgtc_tuning* tn = upd_ep->tuning;
  if (tn && tn->layer_path == 1 && W->layout != QGTC_RIGHT_BYTES) return QGTC_OK;
  // what the kernel covers; everything else takes the two-kernel path
  if (!plan_fused_applies(X->cols, W->cols, X->nbits, W->nbits)) return QGTC_OK;
  if (agg_ep->rq_nbits < 1 || agg_ep->rq_nbits > 8) return QGTC_OK;
  if (upd_ep->mode == QGTC_OUT_BITS && upd_ep->rq_nbits > 8) return QGTC_OK;
  if (A->rows < 1) return QGTC_OK;
  const bool w_bytes = W->layout == QGTC_RIGHT_BYTES;
  if (!w_bytes && workspace_bytes < layer_fused_workspace_bytes(X->cols, W->cols)) return QGTC_OK;
  if (!(agg_ep->rq_inv_scale > 0.0f) || !(agg_ep->rq_inv_scale < INFINITY)) return QGTC_OK;

  LayerParams p{};
  if (agg_fill_params(A, map, X, &p.a) != QGTC_OK) return QGTC_OK;
  if (check_bits(W, w_bytes ? QGTC_RIGHT_BYTES : QGTC_RIGHT) != QGTC_OK || W->rows != X->cols) return QGTC_OK;
  const bool square = A->block_rows > 0 || A->rows == A->cols;
  if (agg_ep->self_term && !square) return QGTC_OK;
  if (make_epilogue(upd_ep, out, ld_out, A->rows, W->cols, QGTC_RIGHT, false, &p.up) != QGTC_OK)
    return QGTC_OK;

  EpiParams& ea = p.a.ep;
  ea = EpiParams{};
  ea.mode = QGTC_OUT_BITS;
  ea.relu = agg_ep->relu ? 1 : 0;
  ea.self_term = agg_ep->self_term ? 1 : 0;
  ea.rq_nbits = agg_ep->rq_nbits;
  ea.rq_lo = agg_ep->rq_lo;
  ea.rq_inv_scale = agg_ep->rq_inv_scale;

  AggParams& a = p.a;
  a.kslices = agg_kslices(X->cols, a.tile_words);
  a.n_cg = cdiv(X->cols, 64);
  a.nblocks = (uint32_t)a.n_tile_rows;
  // waves side by side over the column groups, and waves that split each tile list
  a.skip_words = agg_skip_words(a.s, tn ? tn->zero_words : 0, map != nullptr);
  a.pack16 = agg_pack16(a.skip_words, a.s, a.n_tile_cols, a.tile_words);
  int cgw = 1, ksplit = 1;
  plan_layer_shape(a.n_tile_rows, X->cols, X->nbits, a.skip_words != 0, &cgw, &ksplit);
  p.cgw = cgw;
  p.n_pass = cdiv(a.n_cg, p.cgw);
  a.ksplit = ksplit;
  if (tn && tn->layer_ksplit > 0) {
    a.ksplit = tn->layer_ksplit;
    while (p.cgw * a.ksplit > 4 && a.ksplit > 1) a.ksplit >>= 1;
  }
  const unsigned nw = (unsigned)(p.cgw * a.ksplit);
  {
    // one round of waves at most: all of them are resident from the start
    const int per_simd = (a.skip_words && a.pack16) ? kPack16Waves : agg_waves_per_simd(a.s);
    const int64_t slots = (int64_t)device_compute_units() * 4 * per_simd;
    a.even_progress = (int64_t)a.n_tile_rows * nw <= slots ? 1 : 0;
    if (tn && tn->even_progress) a.even_progress = tn->even_progress == 2 ? 1 : 0;   // the caller knows what runs beside it
  }
  agg_set_dealing(&a, 1, tn ? tn->agg_xcd_run : 0);

  p.h = W->cols;
  p.n_nt_w = cdiv(W->cols, 16);
  p.want_rowsum = upd_ep->mode == QGTC_OUT_F32 && upd_ep->row_i == nullptr && upd_ep->rs != 0.0;
  p.n_nt = p.n_nt_w + (p.want_rowsum ? 1 : 0);
  p.n_ks = a.n_cg;
  p.n_kc = (int)nw / p.n_nt;
  if (p.n_kc < 1) p.n_kc = 1;
  if (p.n_kc > p.n_ks) p.n_kc = p.n_ks;
  p.ks_per = cdiv(p.n_ks, p.n_kc);
  p.n_kc = cdiv(p.n_ks, p.ks_per);
  p.ys = p.n_ks * 64 + 16;
  p.zs = p.n_nt * 16;
  p.split_y = agg_ep->rq_nbits == 8;
  p.split_w = W->nbits == 8;
  p.yb_off = a.ksplit > 1 ? (int)nw * 16 * 64 : 0;
  p.z_off = p.yb_off + 4 * p.ys;
  const size_t lds_bytes = (size_t)(p.z_off + 16 * p.zs) * 4;
  if (lds_bytes > 64 * 1024) return QGTC_OK;

  ProfScope prof(QGTC_KERNEL_LAYER, stream);
  if (w_bytes) {
    p.wb = reinterpret_cast<const uint8_t*>(W->data);
    p.wb_part = W->plane_stride_words * 4;
  } else {
    uint8_t* wb = reinterpret_cast<uint8_t*>(workspace);
    p.wb = wb;
    p.wb_part = (int64_t)p.n_nt_w * p.n_ks * 1024;
    const int prep_threads = p.n_nt_w * p.n_ks * 64;
    hipLaunchKernelGGL(weight_bytes_kernel, dim3((unsigned)cdiv(prep_threads, 256)), dim3(256), 0, stream,
                       W->data, W->ld_words, W->plane_stride_words, W->nbits, cdiv(W->rows, 32), W->cols,
                       p.n_nt_w, p.n_ks, p.split_w, wb, p.wb_part);
    qgtc_status st = launch_status();
    if (st != QGTC_OK) return st;
  }
  *done = true;
  switch (X->nbits) {
    case 1: return launch<1>(p, nw, lds_bytes, stream);
    case 2: return launch<2>(p, nw, lds_bytes, stream);
    case 3: return launch<3>(p, nw, lds_bytes, stream);
    case 4: return launch<4>(p, nw, lds_bytes, stream);
    case 5: return launch<5>(p, nw, lds_bytes, stream);
    case 6: return launch<6>(p, nw, lds_bytes, stream);
    case 7: return launch<7>(p, nw, lds_bytes, stream);
    default: return launch<8>(p, nw, lds_bytes, stream);
  }
}

}  // namespace qgtc
