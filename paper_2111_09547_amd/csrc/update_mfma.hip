// Node update C = Y.W on the matrix cores, for operands of at most 8 bits.
//
// Algorithm 1 of the paper composes the s-bit x t-bit product out of s*t 1-bit
// products because its hardware primitive is the 1-bit Tensor-Core tile.
// CDNA4 has no 1-bit matrix instruction but it has an int8 one
// (v_mfma_i32_16x16x64_i8); for the dense, short-K update it covers up to 8 x 8
// bit planes per multiply-accumulate, so here the planes are put back together
// into bytes in registers and multiplied as integers.  The result is the same
// integer modulo 2^32, bit for bit; inputs (packed planes) and outputs (int32,
// fp32 or packed planes) are exactly those of the popcount kernel.
//
// The instruction is signed, codes of 8 bits are not: an 8-bit code c is taken as
// c' = c - 128 (one XOR with 0x80 per byte), and with K' the staged length of K
//   sum_k y_k w_k = sum_k y'_k w'_k + 128 sum_k y'_k + 128 sum_k w'_k + 16384 K'
//                 = sum_k y'_k w'_k + 128 (sum_k y'_k + sum_k w_k)
// (only Y with 8 bits: sum_k y'_k w_k + 128 sum_k w_k; only W: sum_k y_k w'_k + 128 sum_k y_k).
// The column sums of W are taken once per workgroup while W is staged, the row sums of
// Y by one more matrix instruction against an all-ones operand.  All of it modulo 2^32.
//
// Work split: a workgroup of four waves puts the byte form of its slice of W (up to
// 64 output columns) into LDS once; each wave then walks over groups of 32 rows (two
// 16-row tiles), with the loads of its next item in flight while it works on the
// current one.  The kernel is bound by reading Y from HBM, so the loads decide the
// lane mapping.  The instruction contracts over 64 K positions, 16 per lane: lane
// (row or column = lane % 16, block g = lane / 16) supplies 16 bytes.  Which 64
// positions of K a step covers, and in which order, is free as long as both operands
// agree, so a lane of the Y side owns LW consecutive 16-bit pieces of its row per
// "super-step":
//   LW = 1: half a word   (K up to 64: the whole contraction is one step)
//   LW = 2: one word      (rows of up to 32 bytes)
//   LW = 8: four words    (one 16-byte load per plane and lane; a wave reads the 16
//                          rows x 64 bytes of a tile and plane as 1 KiB in one piece)
// and runs LW steps on what it has loaded.
// Planes -> bytes.  The 8 planes of one 32-bit word are an 8 x 32 bit matrix; three
// rounds of masked swaps between the plane registers transpose its four 8 x 8 blocks at
// once and leave 8 words whose 32 bytes are the 32 codes, code of K position 8 b + r in
// byte b of word r.  Words 0..3 feed one step, words 4..7 the next; W is put into LDS
// through the same transposition, so the pairing of K positions is consistent without
// ever un-permuting.  Y as bytes (QGTC_LEFT_BYTES) needs no re-assembly (LW 16-byte loads
// per row), and W is then staged in natural K order.
// The 16x16 result tile has column lane % 16 and rows 4*(lane / 16) + r in register r.
#include "qgtc_internal.h"

#include <type_traits>

namespace qgtc {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int kRowsPerGroup = 32;
constexpr int kPad = 16;   // bytes of padding per LDS row of W
constexpr uint32_t kOutOfRange = 0x80000000u;   // buffer offset past any operand: the load returns 0

// One masked swap between two plane registers: the bits of x at positions p + SH and the
// bits of y at positions p trade places, for every p in mask M.
template <int SH, uint32_t M>
__device__ __forceinline__ void swap_bits(uint32_t& x, uint32_t& y) {
  const uint32_t nx = (x & ~(M << SH)) | ((y & M) << SH);
  const uint32_t ny = (y & ~M) | ((x >> SH) & M);
  x = nx;
  y = ny;
}

// a[p] = 32 K positions of plane p  ->  a[r] = the codes of K positions r, 8 + r, 16 + r,
// 24 + r in its bytes 0..3 (bit p of a code = its bit in plane p).
__device__ __forceinline__ void planes_word_to_codes(uint32_t (&a)[8]) {
#pragma unroll
  for (int p = 0; p < 4; ++p) swap_bits<4, 0x0f0f0f0fu>(a[p], a[p + 4]);
#pragma unroll
  for (int p = 0; p < 8; p += 4) {
    swap_bits<2, 0x33333333u>(a[p], a[p + 2]);
    swap_bits<2, 0x33333333u>(a[p + 1], a[p + 3]);
  }
#pragma unroll
  for (int p = 0; p < 8; p += 2) swap_bits<1, 0x55555555u>(a[p], a[p + 1]);
}

// SPLIT_Y / SPLIT_W: the operand has 8 planes and is taken as code - 128 (see the top);
// NTC: 16-column tiles per workgroup (1 or 4); LW: see above (1, 2 or 8).
template <bool SPLIT_Y, bool SPLIT_W, int NTC, int LW>
__global__ __launch_bounds__(256) void update_mfma_kernel(const UpdParams p) {
  extern __shared__ uint32_t wl_words[];            // W bytes: [part][col][kpad + kPad]
  constexpr int CC = 16 * NTC;                      // columns per workgroup
  constexpr int WPL = LW >= 2 ? LW / 2 : 1;         // words a lane loads per plane and super-step
  constexpr int SSW = 2 * LW;                       // words of K per super-step
  uint8_t* wl = reinterpret_cast<uint8_t*>(wl_words);

  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int lane = threadIdx.x & 63;
  const int ln = lane & 15;                         // row / column inside a tile
  const int g = lane >> 4;                          // K block, and row group of the result
  const int c0 = blockIdx.y * CC;

  const int n_ss = (p.kwords + SSW - 1) / SSW;
  const int kpad = n_ss * SSW * 32;                 // K positions per column in LDS, one byte each
  const int wstride = kpad + kPad;
  int32_t* colsum = reinterpret_cast<int32_t*>(wl + CC * wstride);   // [CC], sum of the codes of a column

  // ---- stage W[.][c0 .. c0+CC) in LDS as bytes ------------------------------------
  // one thread turns one word (32 K positions) of one column, all planes, into 32 bytes
  if (SPLIT_Y) {
    for (int i = threadIdx.x; i < CC; i += 256) colsum[i] = 0;
    __syncthreads();
  }
  for (int idx = threadIdx.x; idx < CC * (kpad >> 5); idx += 256) {
    const int cl = idx % CC;
    const int kw = idx / CC;
    uint32_t wv[8];
#pragma unroll
    for (int pl = 0; pl < 8; ++pl) {
      wv[pl] = 0u;
      if (pl < p.t && kw < p.kwords && c0 + cl < p.cols)
        wv[pl] = p.W[(int64_t)pl * p.psw + (int64_t)kw * p.ldw + c0 + cl];
    }
    uint32_t d[8];
    if (p.y_bytes) {                                // natural order: byte k <-> K position 32 kw + k
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        uint32_t v = 0u;
#pragma unroll
        for (int pl = 0; pl < 8; ++pl) v |= spread4((wv[pl] >> (4 * q)) & 0xfu) << pl;
        d[q] = v;
      }
    } else {                                        // the order planes_word_to_codes gives Y
      planes_word_to_codes(wv);
#pragma unroll
      for (int q = 0; q < 8; ++q) d[q] = wv[q];
    }
    if (SPLIT_Y) {
      uint32_t sum = 0u;
#pragma unroll
      for (int q = 0; q < 8; ++q) sum = __builtin_amdgcn_sad_u8(d[q], 0u, sum);
      if (sum != 0u) atomicAdd(&colsum[cl], (int32_t)sum);
    }
    uint8_t* dst = wl + cl * wstride + kw * 32;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      v4u lo = {d[4 * h], d[4 * h + 1], d[4 * h + 2], d[4 * h + 3]};
      if (SPLIT_W) lo = lo ^ 0x80808080u;           // codes - 128, padding included
      *reinterpret_cast<v4u*>(dst + 16 * h) = lo;
    }
  }
  __syncthreads();

  const int n_groups = (p.rows + kRowsPerGroup - 1) / kRowsPerGroup;
  const EpiParams& e = p.ep;
  const int qbits = e.rq_nbits;
  const uint32_t qmax = qbits >= 32 ? 0xffffffffu : ((1u << qbits) - 1u);
  const float qmaxf = (float)qmax;
  // Y through buffer loads: what lies outside (rows past the last, words past the end of a
  // row) gets an offset beyond the buffer and reads as zero, with no branch around the load
  const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc((void*)p.Y, 0, (int)p.y_span_bytes, 0x00020000);
  const uint32_t ldy4 = (uint32_t)p.ldy * 4u, psy4 = (uint32_t)p.psy * 4u;

  // This lane's part of tile mt (16 rows) of row group rg for super-step ss, all loads issued
  // together.  planes: word k of plane pl at [pl * WPL + k]; bytes: dword c of step j at [4 * j + c]
  static_assert(4 * LW <= 8 * WPL, "the byte form fits into the registers of the plane form");
  auto load_tile = [&](int rg, int ss, int mt, uint32_t (&raw)[8 * WPL]) {
    const int row = rg * kRowsPerGroup + mt * 16 + ln;
    if (p.y_bytes) {
#pragma unroll
      for (int j = 0; j < LW; ++j) {
        const uint32_t kb = (uint32_t)((ss * LW + j) * 64 + g * 16);
        const uint32_t off = (row < p.rows && kb < ldy4) ? (uint32_t)row * ldy4 + kb : kOutOfRange;
        const v4u v = __builtin_amdgcn_raw_buffer_load_b128(ry, off, 0, 0);
        raw[4 * j] = v.x; raw[4 * j + 1] = v.y; raw[4 * j + 2] = v.z; raw[4 * j + 3] = v.w;
      }
    } else {
      // words up to the leading dimension are data or zero padding; beyond it the next row begins
      const int w0 = LW == 1 ? ss * 2 + (g >> 1) : ss * SSW + g * WPL;
      const uint32_t off = (row < p.rows && w0 < p.ldy) ? (uint32_t)row * ldy4 + (uint32_t)w0 * 4u : kOutOfRange;
      static_assert(WPL == 4 || WPL == 1, "one word or four per lane");
#pragma unroll
      for (int pl = 0; pl < 8; ++pl) {
        if (WPL == 4) {                             // the host picks LW = 8 only for 16-byte aligned rows
          v4u v = {0u, 0u, 0u, 0u};
          if (pl < p.s) v = __builtin_amdgcn_raw_buffer_load_b128(ry, off, (uint32_t)pl * psy4, 0);
          raw[pl * WPL] = v.x; raw[pl * WPL + 1] = v.y; raw[pl * WPL + 2] = v.z; raw[pl * WPL + WPL - 1] = v.w;
        } else {
          raw[pl] = 0u;
          if (pl < p.s) raw[pl] = __builtin_amdgcn_raw_buffer_load_b32(ry, off, (uint32_t)pl * psy4, 0);
        }
      }
    }
  };

  v4i acc[2][NTC], rsum[2];                          // products; row sums of Y (8-bit W only)

  // LW steps on the matrix cores for one tile: two per loaded word (one for LW = 1).  A
  // step's 16 bytes of W sit at kb in its column's LDS row, for both forms of Y.
  auto compute_tile = [&](const uint32_t (&raw)[8 * WPL], int ss, auto mt_c) {
    constexpr int mt = decltype(mt_c)::value;
#pragma unroll
    for (int k = 0; k < WPL; ++k) {
      uint32_t codes[8];                            // the word's 32 codes
      if (!p.y_bytes) {
#pragma unroll
        for (int pl = 0; pl < 8; ++pl) codes[pl] = raw[pl * WPL + k];
        planes_word_to_codes(codes);
      }
#pragma unroll
      for (int h = 0; h < (LW == 1 ? 1 : 2); ++h) {
        const int j = 2 * k + h;
        const int kb = p.y_bytes ? (ss * LW + j) * 64 + g * 16
                                 : (LW == 1 ? ss * 64 + g * 16 : ss * SSW * 32 + g * 16 * LW + j * 16);
        uint32_t d[4];
        if (p.y_bytes) {
          d[0] = raw[4 * j]; d[1] = raw[4 * j + 1]; d[2] = raw[4 * j + 2]; d[3] = raw[4 * j + 3];
        } else {
          // words 0..3 or 4..7 of the codes; LW = 1: the half of the word this lane owns
          // (chosen with a lane mask: a select between two array elements would become an
          // indexed access to an array in scratch memory)
          const uint32_t hi = LW == 1 ? 0u - (uint32_t)(g & 1) : (h != 0 ? 0xffffffffu : 0u);
#pragma unroll
          for (int i = 0; i < 4; ++i) d[i] = (codes[4 + i] & hi) | (codes[i] & ~hi);
        }
        if (SPLIT_Y) {                              // codes - 128
#pragma unroll
          for (int i = 0; i < 4; ++i) d[i] ^= 0x80808080u;
        }
        const v4i av = {(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
        if (SPLIT_W) {
          const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
          rsum[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, ones, rsum[mt], 0, 0, 0);
        }
#pragma unroll
        for (int nt = 0; nt < NTC; ++nt) {
          const v4i bv = *reinterpret_cast<const v4i*>(wl + (nt * 16 + ln) * wstride + kb);
          acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, bv, acc[mt][nt], 0, 0, 0);
        }
      }
    }
  };

  // Items (row group, super-step) of this wave, one after the other, each as two tiles;
  // while one tile is on the matrix cores the loads of the next one are in flight.
  const int rg_step = (int)gridDim.x * 4;
  int rg = blockIdx.x * 4 + wave, ss = 0;
  if (rg >= n_groups) return;                       // whole wave; no barrier follows
  uint32_t buf0[8 * WPL], buf1[8 * WPL];
  load_tile(rg, 0, 0, buf0);
  while (true) {
    load_tile(rg, ss, 1, buf1);
    const int row0 = rg * kRowsPerGroup;
    if (ss == 0) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        rsum[mt] = (v4i){0, 0, 0, 0};
#pragma unroll
        for (int nt = 0; nt < NTC; ++nt) acc[mt][nt] = (v4i){0, 0, 0, 0};
      }
    }
    compute_tile(buf0, ss, std::integral_constant<int, 0>{});
    int nrg = rg, nss = ss + 1;
    if (nss == n_ss) { nss = 0; nrg = rg + rg_step; }
    const bool more = nrg < n_groups;               // wave-uniform
    if (more) load_tile(nrg, nss, 0, buf0);
    compute_tile(buf1, ss, std::integral_constant<int, 1>{});

    if (ss == n_ss - 1) {
    // ---- epilogue: element (mt, nt, r) is row row0 + 16 mt + 4 g + r, column c0 + 16 nt + ln ----
#pragma unroll
    for (int nt = 0; nt < NTC; ++nt) {
      const int col = c0 + nt * 16 + ln;
      const bool col_ok = col < p.cols;
      uint32_t z[2][4];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          uint32_t corr = 0u;                       // see the top of the file
          if (SPLIT_W) corr += (uint32_t)rsum[mt][r];
          if (SPLIT_Y) corr += (uint32_t)colsum[nt * 16 + ln];
          z[mt][r] = (uint32_t)acc[mt][nt][r] + (corr << 7);
        }
      if (e.mode == QGTC_OUT_I32) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int row = row0 + mt * 16 + g * 4 + r;
            int32_t o = (int32_t)z[mt][r];
            if (e.relu && o < 0) o = 0;
            if (col_ok && row < p.rows) reinterpret_cast<int32_t*>(e.out)[(int64_t)row * e.ld_out + col] = o;
          }
      } else if (e.mode == QGTC_OUT_F32) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int row = row0 + mt * 16 + g * 4 + r;
            if (col_ok && row < p.rows)
              reinterpret_cast<float*>(e.out)[(int64_t)row * e.ld_out + col] =
                  dequantize_f64(z[mt][r], row, col, e);
          }
      } else {
        // packed planes along the rows (next layer's X): this lane owns bits
        // 16 mt + 4 g + r of the word; the four row groups are OR-ed across lanes.
        // The lane's 8 codes as an 8 x 8 bit matrix, transposed: byte i = bit i of the codes
        // of rows r = 0..3 of tile 0 (low nibble) and of tile 1 (high nibble).
        uint32_t qlo = 0u, qhi = 0u;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int ra = row0 + g * 4 + r, rb = ra + 16;
          const int cc = min(col, p.cols - 1);
          qlo |= ((col_ok && ra < p.rows) ? requantize_i32(z[0][r], cc, e, qmax, qmaxf) : 0u) << (8 * r);
          qhi |= ((col_ok && rb < p.rows) ? requantize_i32(z[1][r], cc, e, qmax, qmaxf) : 0u) << (8 * r);
        }
        transpose_bits_8x8(qlo, qhi);
        uint32_t part[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint32_t byte = ((i < 4 ? qlo : qhi) >> (8 * (i & 3))) & 0xffu;
          part[i] = ((byte & 0xfu) | ((byte & 0xf0u) << 12)) << (4 * g);
        }
        uint32_t* dst = reinterpret_cast<uint32_t*>(e.out) + (int64_t)(row0 >> 5) * e.ld_out + (col_ok ? col : 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          uint32_t w = part[i];
          w |= (uint32_t)__shfl_xor((int)w, 16, 64);
          w |= (uint32_t)__shfl_xor((int)w, 32, 64);
          if (i < qbits && g == 0 && col_ok) dst[(int64_t)i * e.ps_out] = w;
        }
      }
    }
    }   // last super-step of the row group

    if (!more) break;
    rg = nrg;
    ss = nss;
  }
}

int pick_lw(const UpdParams& p) {
  if (p.y_bytes) return p.ldy * 4 <= 64 ? 1 : (p.ldy * 4 <= 128 ? 2 : 8);
  // four words per lane and plane are one 16-byte load: rows, planes and base at multiples of 16 bytes
  const bool vec = (p.ldy & 3) == 0 && (p.psy & 3) == 0 && ((uintptr_t)p.Y & 15u) == 0;
  return p.kwords <= 2 ? 1 : ((p.kwords <= 8 || !vec) ? 2 : 8);
}

size_t lds_bytes(const UpdParams& p, int ntc, int lw) {
  const int ssw = 2 * lw;
  const int kpad = cdiv(p.kwords, ssw) * ssw * 32;
  return (size_t)16 * ntc * (size_t)(kpad + kPad) + (size_t)16 * ntc * sizeof(int32_t);
}

int pick_ntc(const UpdParams& p) {
  const int lw = pick_lw(p);
  int ntc = p.cols > 16 ? 4 : 1;
  if (ntc == 4 && lds_bytes(p, 4, lw) > 60 * 1024) ntc = 1;
  if (lds_bytes(p, ntc, lw) > 60 * 1024) return 0;
  return ntc;
}

template <bool SY, bool SW, int NTC, int LW>
qgtc_status launch(const UpdParams& p, hipStream_t stream) {
  const int n_groups = cdiv(p.rows, kRowsPerGroup);
  const unsigned col_blocks = (unsigned)cdiv(p.cols, 16 * NTC);
  const size_t lds = lds_bytes(p, NTC, LW);
  // Every workgroup converts its slice of W first, and a wave keeps the next item's loads
  // in flight while it works on the current one: the grid is what the device holds at
  // once (by registers, asked from the runtime once per kernel, and by LDS), each
  // workgroup walking over many row groups.
  static int by_regs = 0;                           // workgroups per CU that the registers allow
  if (by_regs == 0) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, update_mfma_kernel<SY, SW, NTC, LW>, 256, 0) != hipSuccess ||
        n < 1)
      n = 1;
    by_regs = n > 3 ? 3 : n;
  }
  int per_cu = by_regs;
  const int by_lds = (int)((size_t)(160 * 1024) / (lds + 256));
  if (by_lds < per_cu) per_cu = by_lds < 1 ? 1 : by_lds;
  unsigned row_blocks = (unsigned)cdiv(n_groups, 4);
  unsigned cap = (unsigned)(device_compute_units() * per_cu) / col_blocks;
  if (cap < 1u) cap = 1u;
  if (row_blocks > cap) row_blocks = cap;
  dim3 grid(row_blocks, col_blocks);
  hipLaunchKernelGGL((update_mfma_kernel<SY, SW, NTC, LW>), grid, dim3(256), lds, stream, p);
  return launch_status();
}

template <bool SY, bool SW, int NTC>
qgtc_status dispatch_lw(const UpdParams& p, hipStream_t stream) {
  switch (pick_lw(p)) {
    case 1: return launch<SY, SW, NTC, 1>(p, stream);
    case 2: return launch<SY, SW, NTC, 2>(p, stream);
    default: return launch<SY, SW, NTC, 8>(p, stream);
  }
}

template <bool SY, bool SW>
qgtc_status dispatch_n(const UpdParams& p, hipStream_t stream) {
  switch (pick_ntc(p)) {
    case 4: return dispatch_lw<SY, SW, 4>(p, stream);
    case 1: return dispatch_lw<SY, SW, 1>(p, stream);
    default: return QGTC_ERR_UNSUPPORTED;
  }
}

}  // namespace

bool update_mfma_eligible(const UpdParams& p) {
  if (p.s < 1 || p.s > 8 || p.t < 1 || p.t > 8) return false;
  if (p.ep.mode == QGTC_OUT_BITS && p.ep.rq_nbits > 8) return false;
  // Y is read through 32-bit buffer offsets, with 2^31 standing for "outside"
  if (p.y_span_bytes >= ((int64_t)1 << 31)) return false;
  return pick_ntc(p) != 0;
}

qgtc_status update_mfma_launch(const UpdParams& p, hipStream_t stream) {
  if (p.s == 8) return p.t == 8 ? dispatch_n<true, true>(p, stream) : dispatch_n<true, false>(p, stream);
  return p.t == 8 ? dispatch_n<false, true>(p, stream) : dispatch_n<false, false>(p, stream);
}

}  // namespace qgtc
