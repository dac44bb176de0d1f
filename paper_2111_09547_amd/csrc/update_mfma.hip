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
// The instruction is signed, codes of 8 bits are not: an 8-bit code c is split
// into c7 = c & 127 and its top bit b7, and
//   y.w = y7.w7 + 128 (b7y.w7 + y7.b7w) + 16384 b7y.b7w
// is taken with up to four instructions into three accumulators.
//
// Work split: a wave owns 32 rows (two 16-row tiles) and up to 64 output columns
// (four 16-column tiles); a workgroup of four waves shares the byte form of its
// slice of W in LDS.  Operand bytes of a lane: row (or column) lane % 16, the 16
// consecutive K positions 64*step + 16*(lane / 16) .. +15; both operands use the
// same mapping, so the pairing inside the instruction is consistent.  The 16x16
// result tile has column lane % 16 and rows 4*(lane / 16) + r in register r.
#include "qgtc_internal.h"

namespace qgtc {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kRowsPerWave = 32;
constexpr int kPad = 16;   // bytes of padding per LDS row of W

__device__ __forceinline__ v4i as_v4i(const uint32_t (&d)[4]) {
  v4i v = {(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
  return v;
}

// SPLIT_Y / SPLIT_W: the operand has 8 planes and is split into 7 bits + top bit;
// NTC: 16-column tiles per wave (1, 2 or 4).
template <bool SPLIT_Y, bool SPLIT_W, int NTC>
__global__ __launch_bounds__(256) void update_mfma_kernel(const UpdParams p) {
  extern __shared__ uint32_t wl_words[];            // W bytes: [part][col][kpad + kPad]
  constexpr int CC = 16 * NTC;                      // columns per workgroup
  uint8_t* wl = reinterpret_cast<uint8_t*>(wl_words);

  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int lane = threadIdx.x & 63;
  const int ln = lane & 15;                         // row / column inside a tile
  const int g = lane >> 4;                          // K sub-block, and row group of the result
  const int c0 = blockIdx.y * CC;
  const int row0 = (blockIdx.x * 4 + wave) * kRowsPerWave;

  const int k_steps = (p.kwords + 1) >> 1;          // 64 bits of K per step
  const int kpad = k_steps * 64;
  const int wstride = kpad + kPad;                  // bytes per column in LDS
  const int part_bytes = CC * wstride;

  // ---- stage W[.][c0 .. c0+CC) in LDS as bytes, K contiguous per column ----------
  // one thread handles 4 consecutive K positions of one column
  for (int idx = threadIdx.x; idx < CC * (kpad >> 2); idx += 256) {
    const int cl = idx % CC;
    const int kq = idx / CC;                        // K quad: positions 4*kq .. 4*kq+3
    const int kw = kq >> 3;
    const int sh = (kq & 7) * 4;
    uint32_t v = 0u;
    if (kw < p.kwords && c0 + cl < p.cols) {
      for (int pl = 0; pl < p.t; ++pl) {
        const uint32_t word = p.W[(int64_t)pl * p.psw + (int64_t)kw * p.ldw + c0 + cl];
        v |= spread4((word >> sh) & 0xfu) << pl;
      }
    }
    uint32_t* dst = reinterpret_cast<uint32_t*>(wl + cl * wstride + kq * 4);
    if (SPLIT_W) {
      dst[0] = v & 0x7f7f7f7fu;
      *reinterpret_cast<uint32_t*>(wl + part_bytes + cl * wstride + kq * 4) = (v >> 7) & 0x01010101u;
    } else {
      dst[0] = v;
    }
  }
  __syncthreads();
  if (row0 >= p.rows) return;                       // whole wave; no barrier follows

  v4i acc1[2][NTC], acc7[2][NTC], acc14[2][NTC];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < NTC; ++nt) {
      acc1[mt][nt] = (v4i){0, 0, 0, 0};
      acc7[mt][nt] = (v4i){0, 0, 0, 0};
      acc14[mt][nt] = (v4i){0, 0, 0, 0};
    }

  for (int ks = 0; ks < k_steps; ++ks) {
    // B operands of this step: 16 bytes per lane and column tile
    v4i b7[NTC], bb[NTC];
#pragma unroll
    for (int nt = 0; nt < NTC; ++nt) {
      const uint8_t* src = wl + (nt * 16 + ln) * wstride + ks * 64 + g * 16;
      b7[nt] = *reinterpret_cast<const v4i*>(src);
      if (SPLIT_W) bb[nt] = *reinterpret_cast<const v4i*>(src + part_bytes);
    }
    const int dw = ks * 2 + (g >> 1);               // word of Y holding this lane's 16 bits
    const int sh = (g & 1) * 16;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      const int row = row0 + mt * 16 + ln;
      uint32_t d[4] = {0u, 0u, 0u, 0u};
      if (p.y_bytes) {
        // codes as bytes: the lane's 16 K positions are 16 consecutive bytes of its row
        const int kb = ks * 64 + g * 16;
        if (row < p.rows && kb < p.ldy * 4) {
          const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint8_t*>(p.Y) +
                                                          (int64_t)row * p.ldy * 4 + kb);
          d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
        }
      } else {
        uint32_t f[8];
#pragma unroll
        for (int pl = 0; pl < 8; ++pl) {
          f[pl] = 0u;
          if (pl < p.s && row < p.rows && dw < p.kwords)
            f[pl] = (p.Y[(int64_t)pl * p.psy + (int64_t)row * p.ldy + dw] >> sh) & 0xffffu;
        }
        planes_to_bytes(f, p.s, d);
      }
      v4i a7, ab;
      if (SPLIT_Y) {
        uint32_t lo[4], hi[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) { lo[q] = d[q] & 0x7f7f7f7fu; hi[q] = (d[q] >> 7) & 0x01010101u; }
        a7 = as_v4i(lo);
        ab = as_v4i(hi);
      } else {
        a7 = as_v4i(d);
      }
#pragma unroll
      for (int nt = 0; nt < NTC; ++nt) {
        acc1[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a7, b7[nt], acc1[mt][nt], 0, 0, 0);
        if (SPLIT_Y) acc7[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ab, b7[nt], acc7[mt][nt], 0, 0, 0);
        if (SPLIT_W) acc7[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a7, bb[nt], acc7[mt][nt], 0, 0, 0);
        if (SPLIT_Y && SPLIT_W)
          acc14[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ab, bb[nt], acc14[mt][nt], 0, 0, 0);
      }
    }
  }

  // ---- epilogue: element (mt, nt, r) is row row0 + 16 mt + 4 g + r, column c0 + 16 nt + ln ----
  const EpiParams& e = p.ep;
  const int qbits = e.rq_nbits;
  const uint32_t qmax = qbits >= 32 ? 0xffffffffu : ((1u << qbits) - 1u);
  const float qmaxf = (float)qmax;
#pragma unroll
  for (int nt = 0; nt < NTC; ++nt) {
    const int col = c0 + nt * 16 + ln;
    const bool col_ok = col < p.cols;
    uint32_t z[2][4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        uint32_t v = (uint32_t)acc1[mt][nt][r];
        if (SPLIT_Y || SPLIT_W) v += (uint32_t)acc7[mt][nt][r] << 7;
        if (SPLIT_Y && SPLIT_W) v += (uint32_t)acc14[mt][nt][r] << 14;
        z[mt][r] = v;
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
      // 16 mt + 4 g + r of the word; the four row groups are OR-ed across lanes
      uint32_t part[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) part[i] = 0u;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = row0 + mt * 16 + g * 4 + r;
          const uint32_t q = (col_ok && row < p.rows) ? requantize_i32(z[mt][r], min(col, p.cols - 1), e, qmax, qmaxf) : 0u;
          const int bit = mt * 16 + g * 4 + r;
#pragma unroll
          for (int i = 0; i < 8; ++i) part[i] |= ((q >> i) & 1u) << bit;
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
}

template <bool SY, bool SW, int NTC>
qgtc_status launch(const UpdParams& p, hipStream_t stream) {
  const int k_steps = (p.kwords + 1) / 2;
  const int parts = SW ? 2 : 1;
  const size_t lds = (size_t)parts * 16 * NTC * (size_t)(k_steps * 64 + kPad);
  dim3 grid((unsigned)cdiv(p.rows, 4 * kRowsPerWave), (unsigned)cdiv(p.cols, 16 * NTC));
  hipLaunchKernelGGL((update_mfma_kernel<SY, SW, NTC>), grid, dim3(256), lds, stream, p);
  return launch_status();
}

int pick_ntc(const UpdParams& p) {
  const int k_steps = (p.kwords + 1) / 2;
  const int parts = p.t == 8 ? 2 : 1;
  int ntc = p.cols > 32 ? 4 : (p.cols > 16 ? 2 : 1);
  while (ntc > 1 && (size_t)parts * 16 * ntc * (size_t)(k_steps * 64 + kPad) > 60 * 1024) ntc >>= 1;
  if ((size_t)parts * 16 * ntc * (size_t)(k_steps * 64 + kPad) > 60 * 1024) return 0;
  return ntc;
}

template <bool SY, bool SW>
qgtc_status dispatch_n(const UpdParams& p, hipStream_t stream) {
  switch (pick_ntc(p)) {
    case 4: return launch<SY, SW, 4>(p, stream);
    case 2: return launch<SY, SW, 2>(p, stream);
    case 1: return launch<SY, SW, 1>(p, stream);
    default: return QGTC_ERR_UNSUPPORTED;
  }
}

}  // namespace

bool update_mfma_eligible(const UpdParams& p) {
  if (p.s < 1 || p.s > 8 || p.t < 1 || p.t > 8) return false;
  if (p.ep.mode == QGTC_OUT_BITS && p.ep.rq_nbits > 8) return false;
  return pick_ntc(p) != 0;
}

qgtc_status update_mfma_launch(const UpdParams& p, hipStream_t stream) {
  if (p.s == 8) return p.t == 8 ? dispatch_n<true, true>(p, stream) : dispatch_n<true, false>(p, stream);
  return p.t == 8 ? dispatch_n<false, true>(p, stream) : dispatch_n<false, false>(p, stream);
}

}  // namespace qgtc
