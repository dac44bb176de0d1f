// Quantize + bit-decompose + pack ("Tensor.to_bit"), decode ("Tensor.to_val")
// and the value sums of packed operands.  Eq. (2) and the 3D-stacked bit
// compression of Section 4.2 of the paper, for gfx950.  All of these are
// streaming kernels bound by HBM bandwidth.
#include "qgtc_internal.h"

namespace qgtc {
namespace {

struct PackParams {
  const void* src;
  int64_t ld_src;
  int32_t rows, cols;
  int32_t nbits;
  uint32_t* dst;
  int64_t ld, ps;       // words
  float lo, inv;        // Eq. (2), fp32 sources only
  uint32_t qmax;
  float qmaxf;
};

template <int SRC> struct src_type { using type = uint32_t; };
template <> struct src_type<QGTC_SRC_F32> { using type = float; };
template <> struct src_type<QGTC_SRC_U8> { using type = uint8_t; };

// Raw element (the load) and its code (Eq. (2) or masking) are kept apart so
// that many loads can be in flight before the first conversion.
template <int SRC>
__device__ __forceinline__ typename src_type<SRC>::type fetch_raw(const PackParams& p, int64_t idx) {
  return reinterpret_cast<const typename src_type<SRC>::type*>(p.src)[idx];
}

template <int SRC>
__device__ __forceinline__ uint32_t to_code(const PackParams& p, typename src_type<SRC>::type v) {
  if constexpr (SRC == QGTC_SRC_F32) {
    return quantize_f32(v, p.lo, p.inv, p.qmax, p.qmaxf);
  } else {
    return (uint32_t)v & p.qmax;
  }
}

template <int SRC>
__device__ __forceinline__ uint32_t fetch(const PackParams& p, int64_t idx) {
  return to_code<SRC>(p, fetch_raw<SRC>(p, idx));
}

// RIGHT layout: 32 consecutive ROWS of one column share a word.
// thread <-> (column c, word row w); the 32 loads of a thread are each
// coalesced across the threads of the wave (consecutive columns).
template <int SRC>
__global__ __launch_bounds__(256) void pack_right_kernel(const PackParams p) {
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int w_row = blockIdx.y * 4 + (threadIdx.x >> 6);
  const int n_wr = (p.rows + 31) >> 5;
  if (c >= p.cols || w_row >= n_wr) return;
  // all 32 loads of the word are issued before the first one is used
  typename src_type<SRC>::type raw[32];
#pragma unroll
  for (int b = 0; b < 32; ++b) {
    const int r = min(w_row * 32 + b, p.rows - 1);      // clamped: no branch around the load
    raw[b] = fetch_raw<SRC>(p, (int64_t)r * p.ld_src + c);
  }
  uint32_t q[32];
#pragma unroll
  for (int b = 0; b < 32; ++b) q[b] = (w_row * 32 + b < p.rows) ? to_code<SRC>(p, raw[b]) : 0u;
  // 8 planes at a time: the codes of 8 rows are an 8 x 8 bit matrix (a byte per row)
  // whose transpose has a byte per plane; four of them make the 32 rows of a word
  for (int p0 = 0; p0 < p.nbits; p0 += 8) {
    uint32_t L[4], H[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint32_t lo = 0u, hi = 0u;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        lo |= ((q[8 * g + k] >> p0) & 0xffu) << (8 * k);
        hi |= ((q[8 * g + 4 + k] >> p0) & 0xffu) << (8 * k);
      }
      transpose_bits_8x8(lo, hi);
      L[g] = lo;
      H[g] = hi;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int sh = 8 * (i & 3);
      uint32_t w = 0u;
#pragma unroll
      for (int g = 0; g < 4; ++g) w |= (((i < 4 ? L[g] : H[g]) >> sh) & 0xffu) << (8 * g);
      if (p0 + i < p.nbits) p.dst[(int64_t)(p0 + i) * p.ps + (int64_t)w_row * p.ld + c] = w;
    }
  }
}

// LEFT layout: 32 consecutive COLUMNS of one row share a word.
// One wave per row; lane <-> column inside a 64-column chunk, so the loads are
// coalesced and a ballot over the lanes yields two finished words.  The words
// of 32 chunks are gathered lane by lane and stored 256 bytes at a time.
// Every word up to ld (the zero padding included) is written.
template <int SRC>
__global__ __launch_bounds__(256) void pack_left_kernel(const PackParams p) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= p.rows) return;                       // whole wave
  const int n_words = (int)p.ld;
  for (int pl = 0; pl < p.nbits; ++pl) {
    uint32_t* drow = p.dst + (int64_t)pl * p.ps + (int64_t)r * p.ld;
    for (int w0 = 0; w0 < n_words; w0 += 64) {   // 64 words = 2048 columns per pass
      uint32_t mine = 0u;
      const int n_chunks = min(32, (n_words - w0 + 1) >> 1);
      for (int ch = 0; ch < n_chunks; ++ch) {
        const int c = (w0 + 2 * ch) * 32 + lane;
        uint32_t bit = 0u;
        if (c < p.cols) bit = (fetch<SRC>(p, (int64_t)r * p.ld_src + c) >> pl) & 1u;
        const unsigned long long m = __builtin_amdgcn_ballot_w64(bit != 0u);
        if (lane == 2 * ch) mine = (uint32_t)m;
        if (lane == 2 * ch + 1) mine = (uint32_t)(m >> 32);
      }
      if (w0 + lane < n_words) drow[w0 + lane] = mine;
    }
  }
}

// Fast path for a 0/1 byte matrix into one plane (the adjacency): every lane
// loads 16 consecutive bytes, squeezes them into 16 bits, neighbouring lanes
// merge their halves with a DPP shift, and the even lanes store finished words.
// Needs cols and ld_src multiples of 16 and a 16-byte aligned source.
__device__ __forceinline__ uint32_t squeeze4(uint32_t d) {
  uint32_t t = d & 0x01010101u;     // bit 0 of each byte
  t |= t >> 7;                      // bytes 0,1 -> bits 0,1 ; bytes 2,3 -> bits 16,17
  t |= t >> 14;                     // -> bits 0..3
  return t & 0xfu;
}

// A unit is 1024 columns of one row (64 lanes x 16 bytes); a wave takes UNITS units, all
// of their loads in flight together.  Measured on 64 MiB to 1 GiB of input with 1, 2, 4
// and 8 units per wave and grids capped at 2048 to 8192 workgroups or not at all: two units
// and one wave per pair of units is the fastest or level everywhere (5.0 - 5.7 TB/s of
// read + written bytes from 128 MiB on).
constexpr int kU8Units = 2;

template <int UNITS>
__global__ __launch_bounds__(256) void pack_left_u8_kernel(const PackParams p) {
  const int lane = threadIdx.x & 63;
  const int n_words = (int)p.ld;
  const int n_pass = (n_words + 31) >> 5;          // units per row
  const int64_t n_units = (int64_t)p.rows * n_pass;
  const int64_t wave_id = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
  const int64_t step = (int64_t)gridDim.x * 4 * UNITS;
  // (row, unit within the row) of the wave's first unit and of the stride: one division
  // each per wave, then additions only
  int64_t r0 = wave_id * UNITS / n_pass;
  int q0 = (int)(wave_id * UNITS % n_pass);
  const int64_t step_r = step / n_pass;
  const int step_q = (int)(step % n_pass);
  const uint8_t* src = reinterpret_cast<const uint8_t*>(p.src);
  for (int64_t u0 = wave_id * UNITS; u0 < n_units; u0 += step) {
    uint4 v[UNITS];
    int64_t r = r0;
    int q = q0;
#pragma unroll
    for (int k = 0; k < UNITS; ++k) {
      const int c = q * 1024 + lane * 16;
      v[k] = make_uint4(0u, 0u, 0u, 0u);
      if (r < p.rows && c < p.cols) v[k] = *reinterpret_cast<const uint4*>(src + r * p.ld_src + c);
      if (++q == n_pass) { q = 0; ++r; }
    }
    r = r0;
    q = q0;
#pragma unroll
    for (int k = 0; k < UNITS; ++k) {
      const int w = q * 32 + (lane >> 1);
      const uint32_t h = squeeze4(v[k].x) | (squeeze4(v[k].y) << 4) | (squeeze4(v[k].z) << 8) |
                         (squeeze4(v[k].w) << 12);
      // odd lane's half moves down to the even lane (wave shift left by one lane)
      const uint32_t up = (uint32_t)__shfl_down((int)h, 1, 64);
      if ((lane & 1) == 0 && r < p.rows && w < n_words) p.dst[r * p.ld + w] = h | (up << 16);
      if (++q == n_pass) { q = 0; ++r; }
    }
    r0 += step_r;
    q0 += step_q;
    if (q0 >= n_pass) { q0 -= n_pass; ++r0; }
  }
}

// RIGHT_BYTES: thread (tile nt, step ks, lane l) writes the 16 codes of column
// 16 nt + l % 16, rows 64 ks + 16 (l / 16) .. + 15, as bytes (see qgtc.h).
template <int SRC>
__global__ __launch_bounds__(256) void pack_bytes_kernel(const PackParams p, int n_nt, int n_ks) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int lane = idx & 63;
  const int ks = (idx >> 6) % n_ks;
  const int nt = (idx >> 6) / n_ks;
  if (nt >= n_nt) return;
  const int col = nt * 16 + (lane & 15);
  const int k0 = ks * 64 + (lane >> 4) * 16;
  typename src_type<SRC>::type raw[16];
#pragma unroll
  for (int b = 0; b < 16; ++b) {
    const bool ok = col < p.cols && k0 + b < p.rows;
    raw[b] = fetch_raw<SRC>(p, ok ? (int64_t)(k0 + b) * p.ld_src + col : 0);
  }
  uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int b = 0; b < 16; ++b) {
    const bool ok = col < p.cols && k0 + b < p.rows;
    const uint32_t code = ok ? to_code<SRC>(p, raw[b]) : 0u;
    d[b >> 2] |= code << (8 * (b & 3));
  }
  uint4* dst = reinterpret_cast<uint4*>(reinterpret_cast<uint8_t*>(p.dst) + (int64_t)idx * 16);
  if (p.nbits == 8) {
    dst[p.ps / 4] = make_uint4((d[0] >> 7) & 0x01010101u, (d[1] >> 7) & 0x01010101u,
                               (d[2] >> 7) & 0x01010101u, (d[3] >> 7) & 0x01010101u);
    dst[0] = make_uint4(d[0] & 0x7f7f7f7fu, d[1] & 0x7f7f7f7fu, d[2] & 0x7f7f7f7fu, d[3] & 0x7f7f7f7fu);
  } else {
    dst[0] = make_uint4(d[0], d[1], d[2], d[3]);
  }
}

// LEFT_BYTES: one code per byte, row-major; a thread writes 4 consecutive bytes.
template <int SRC>
__global__ __launch_bounds__(256) void pack_left_bytes_kernel(const PackParams p) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;   // dword index
  const int64_t r = idx / p.ld;
  const int w = (int)(idx % p.ld);
  if (r >= p.rows) return;
  typename src_type<SRC>::type raw[4];
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const int c = w * 4 + b;
    raw[b] = fetch_raw<SRC>(p, c < p.cols ? r * p.ld_src + c : 0);
  }
  uint32_t v = 0u;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const int c = w * 4 + b;
    v |= (c < p.cols ? to_code<SRC>(p, raw[b]) : 0u) << (8 * b);
  }
  p.dst[idx] = v;
}

struct UnpackParams {
  const uint32_t* src;
  int64_t ld, ps;
  int32_t rows, cols, nbits, layout;
  uint32_t* dst;
  int64_t ld_dst;
};

__global__ __launch_bounds__(256) void unpack_kernel(const UnpackParams p) {
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int r = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (c >= p.cols || r >= p.rows) return;
  uint32_t v = 0u;
  if (p.layout == QGTC_LEFT_BYTES) {
    p.dst[(int64_t)r * p.ld_dst + c] = reinterpret_cast<const uint8_t*>(p.src)[(int64_t)r * p.ld * 4 + c];
    return;
  }
  if (p.layout == QGTC_RIGHT_BYTES) {
    const uint8_t* bytes = reinterpret_cast<const uint8_t*>(p.src);
    const int64_t off = (int64_t)(c >> 4) * p.ld * 4 + (int64_t)(r >> 6) * 1024 +
                        ((c & 15) + 16 * ((r & 63) >> 4)) * 16 + (r & 15);
    v = bytes[off];
    if (p.nbits == 8) v |= (uint32_t)bytes[p.ps * 4 + off] << 7;
    p.dst[(int64_t)r * p.ld_dst + c] = v;
    return;
  }
  for (int i = 0; i < p.nbits; ++i) {
    uint32_t word, bit;
    if (p.layout == QGTC_LEFT) {
      word = p.src[(int64_t)i * p.ps + (int64_t)r * p.ld + (c >> 5)];
      bit = c & 31;
    } else {
      word = p.src[(int64_t)i * p.ps + (int64_t)(r >> 5) * p.ld + c];
      bit = r & 31;
    }
    v |= ((word >> bit) & 1u) << i;
  }
  p.dst[(int64_t)r * p.ld_dst + c] = v;
}

// sum_p 2^p popcount(row r of plane p): one wave per row, lanes stride over words.
__global__ __launch_bounds__(256) void row_sums_kernel(const UnpackParams p, int32_t* out) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= p.rows) return;
  const int n_words = (p.cols + 31) >> 5;
  uint32_t acc = 0u;
  for (int i = 0; i < p.nbits; ++i) {
    const uint32_t* row = p.src + (int64_t)i * p.ps + (int64_t)r * p.ld;
    uint32_t cnt = 0u;
    for (int w = lane; w < n_words; w += 64) cnt += __builtin_popcount(row[w]);
    acc += cnt << i;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if (lane == 0) out[r] = (int32_t)acc;
}

// Same for short rows (a few words): one thread per row.
__global__ __launch_bounds__(256) void row_sums_short_kernel(const UnpackParams p, int32_t* out) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= p.rows) return;
  const int n_words = (p.cols + 31) >> 5;
  uint32_t acc = 0u;
  for (int i = 0; i < p.nbits; ++i) {
    const uint32_t* row = p.src + (int64_t)i * p.ps + (int64_t)r * p.ld;
    uint32_t cnt = 0u;
    for (int w = 0; w < n_words; ++w) cnt += __builtin_popcount(row[w]);
    acc += cnt << i;
  }
  out[r] = (int32_t)acc;
}

// sum_p 2^p popcount(column c of plane p): thread per column.
__global__ __launch_bounds__(256) void col_sums_kernel(const UnpackParams p, int32_t* out) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= p.cols) return;
  if (p.layout == QGTC_RIGHT_BYTES) {
    // bytes of column c: 16 at a time (one 16-byte load), both parts; rows past the
    // last one are stored as zeros
    const uint8_t* bytes = reinterpret_cast<const uint8_t*>(p.src);
    uint32_t sum = 0u, top = 0u;
#pragma unroll 4
    for (int r0 = 0; r0 < p.rows; r0 += 16) {
      const int64_t off = (int64_t)(c >> 4) * p.ld * 4 + (int64_t)(r0 >> 6) * 1024 +
                          ((c & 15) + 16 * ((r0 & 63) >> 4)) * 16;
      const uint4 v = *reinterpret_cast<const uint4*>(bytes + off);
      sum = __builtin_amdgcn_sad_u8(v.x, 0u, sum);
      sum = __builtin_amdgcn_sad_u8(v.y, 0u, sum);
      sum = __builtin_amdgcn_sad_u8(v.z, 0u, sum);
      sum = __builtin_amdgcn_sad_u8(v.w, 0u, sum);
      if (p.nbits == 8) {
        const uint4 h = *reinterpret_cast<const uint4*>(bytes + p.ps * 4 + off);
        top = __builtin_amdgcn_sad_u8(h.x, 0u, top);
        top = __builtin_amdgcn_sad_u8(h.y, 0u, top);
        top = __builtin_amdgcn_sad_u8(h.z, 0u, top);
        top = __builtin_amdgcn_sad_u8(h.w, 0u, top);
      }
    }
    sum += top << 7;
    out[c] = (int32_t)sum;
    return;
  }
  const int n_wr = (p.rows + 31) >> 5;
  uint32_t acc = 0u;
  for (int i = 0; i < p.nbits; ++i) {
    uint32_t cnt = 0u;
    for (int w = 0; w < n_wr; ++w) cnt += __builtin_popcount(p.src[(int64_t)i * p.ps + (int64_t)w * p.ld + c]);
    acc += cnt << i;
  }
  out[c] = (int32_t)acc;
}

template <int SRC>
qgtc_status launch_pack(const PackParams& p, int layout, hipStream_t s) {
  if (layout == QGTC_LEFT_BYTES) {
    hipLaunchKernelGGL((pack_left_bytes_kernel<SRC>), dim3((unsigned)cdiv((int64_t)p.rows * p.ld, 256)), dim3(256),
                       0, s, p);
  } else if (layout == QGTC_RIGHT_BYTES) {
    const int n_nt = cdiv(p.cols, 16), n_ks = cdiv(p.rows, 64);
    hipLaunchKernelGGL((pack_bytes_kernel<SRC>), dim3((unsigned)cdiv((int64_t)n_nt * n_ks * 64, 256)), dim3(256),
                       0, s, p, n_nt, n_ks);
  } else if (layout == QGTC_RIGHT) {
    dim3 grid((unsigned)cdiv(p.cols, 64), (unsigned)cdiv(cdiv(p.rows, 32), 4));
    hipLaunchKernelGGL((pack_right_kernel<SRC>), grid, dim3(256), 0, s, p);
  } else if (SRC == QGTC_SRC_U8 && p.nbits == 1 && (p.cols & 15) == 0 && (p.ld_src & 15) == 0 &&
             ((uintptr_t)p.src & 15u) == 0) {
    const int64_t units = (int64_t)p.rows * cdiv(p.ld, 32);
    const int64_t blocks = cdiv(units, 4 * kU8Units);        // beyond 2^24 workgroups the waves loop
    hipLaunchKernelGGL(pack_left_u8_kernel<kU8Units>, dim3((unsigned)(blocks < (1 << 24) ? blocks : (1 << 24))),
                       dim3(256), 0, s, p);
  } else {
    hipLaunchKernelGGL((pack_left_kernel<SRC>), dim3((unsigned)cdiv(p.rows, 4)), dim3(256), 0, s, p);
  }
  return launch_status();
}

UnpackParams unpack_params(const qgtc_bits* m) {
  UnpackParams p{};
  p.src = m->data;
  p.ld = m->ld_words;
  p.ps = m->plane_stride_words;
  p.rows = m->rows;
  p.cols = m->cols;
  p.nbits = m->nbits;
  p.layout = m->layout;
  return p;
}

}  // namespace
}  // namespace qgtc

using namespace qgtc;

extern "C" qgtc_status qgtc_pack_bits(const void* src, int32_t src_dtype, int32_t rows, int32_t cols,
                                      int64_t ld_src, const qgtc_quant* q, const qgtc_bits* dst,
                                      void* stream) {
  if (!src || !dst) return QGTC_ERR_NULL;
  qgtc_status st = check_bits(dst, dst->layout);
  if (st != QGTC_OK) return st;
  if (rows != dst->rows || cols != dst->cols || ld_src < cols) return QGTC_ERR_SHAPE;
  if (src_dtype != QGTC_SRC_F32 && src_dtype != QGTC_SRC_U8 && src_dtype != QGTC_SRC_I32)
    return QGTC_ERR_UNSUPPORTED;
  if (src_dtype == QGTC_SRC_F32) {
    if (!q) return QGTC_ERR_NULL;
    if (q->nbits != dst->nbits) return QGTC_ERR_BITWIDTH;
    if (!(q->hi > q->lo)) return QGTC_ERR_SHAPE;
  }
  if (dst->layout == QGTC_RIGHT && dst->ld_words < cols) return QGTC_ERR_SHAPE;
  if (rows == 0 || cols == 0) return QGTC_OK;

  PackParams p{};
  p.src = src;
  p.ld_src = ld_src;
  p.rows = rows;
  p.cols = cols;
  p.nbits = dst->nbits;
  p.dst = dst->data;
  p.ld = dst->ld_words;
  p.ps = dst->plane_stride_words;
  p.qmax = dst->nbits >= 32 ? 0xffffffffu : ((1u << dst->nbits) - 1u);
  p.qmaxf = (float)p.qmax;
  if (src_dtype == QGTC_SRC_F32) {
    p.lo = (float)q->lo;
    p.inv = (float)((double)(1ull << q->nbits) / (q->hi - q->lo));
  }
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  ProfScope prof(QGTC_KERNEL_PACK, s);
  switch (src_dtype) {
    case QGTC_SRC_F32: return launch_pack<QGTC_SRC_F32>(p, dst->layout, s);
    case QGTC_SRC_U8: return launch_pack<QGTC_SRC_U8>(p, dst->layout, s);
    default: return launch_pack<QGTC_SRC_I32>(p, dst->layout, s);
  }
}

extern "C" qgtc_status qgtc_unpack_bits(const qgtc_bits* src, uint32_t* dst, int64_t ld_dst, void* stream) {
  if (!src || !dst) return QGTC_ERR_NULL;
  qgtc_status st = check_bits(src, src->layout);
  if (st != QGTC_OK) return st;
  if (ld_dst < src->cols) return QGTC_ERR_SHAPE;
  if (src->rows == 0 || src->cols == 0) return QGTC_OK;
  UnpackParams p = unpack_params(src);
  p.dst = dst;
  p.ld_dst = ld_dst;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  ProfScope prof(QGTC_KERNEL_PACK, s);
  dim3 grid((unsigned)cdiv(p.cols, 64), (unsigned)cdiv(p.rows, 4));
  hipLaunchKernelGGL(unpack_kernel, grid, dim3(256), 0, s, p);
  return launch_status();
}

extern "C" qgtc_status qgtc_row_sums(const qgtc_bits* m, int32_t* out, void* stream) {
  if (!m || !out) return QGTC_ERR_NULL;
  qgtc_status st = check_bits(m, QGTC_LEFT);
  if (st != QGTC_OK) return st;
  if (m->rows == 0) return QGTC_OK;
  UnpackParams p = unpack_params(m);
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  ProfScope prof(QGTC_KERNEL_SUMS, s);
  if (p.cols <= 256)
    hipLaunchKernelGGL(row_sums_short_kernel, dim3((unsigned)cdiv(p.rows, 256)), dim3(256), 0, s, p, out);
  else
    hipLaunchKernelGGL(row_sums_kernel, dim3((unsigned)cdiv(p.rows, 4)), dim3(256), 0, s, p, out);
  return launch_status();
}

extern "C" qgtc_status qgtc_col_sums(const qgtc_bits* m, int32_t* out, void* stream) {
  if (!m || !out) return QGTC_ERR_NULL;
  qgtc_status st = check_bits(m, m->layout == QGTC_RIGHT_BYTES ? QGTC_RIGHT_BYTES : QGTC_RIGHT);
  if (st != QGTC_OK) return st;
  if (m->cols == 0) return QGTC_OK;
  UnpackParams p = unpack_params(m);
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  ProfScope prof(QGTC_KERNEL_SUMS, s);
  hipLaunchKernelGGL(col_sums_kernel, dim3((unsigned)cdiv(p.cols, 256)), dim3(256), 0, s, p, out);
  return launch_status();
}
