// Bandwidth-optimized subgraph packing (Section 4.6 of the paper), host side: the
// adjacency and the node features of a batch are quantized and packed into bit
// planes on the CPU, side by side in ONE buffer, so that a single transfer of
// low-bit data crosses the PCIe link instead of dense fp32 matrices in several
// transfers.  Same layouts, same Eq. (2) arithmetic (fp32, separately rounded
// operations) as the device packing in pack.hip, so both give the same words.
// Plain C++; nothing here touches the GPU.
#include "qgtc_internal.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

namespace qgtc {
namespace {

struct HostPack {
  const void* src;
  int src_dtype;
  int64_t ld_src;
  int32_t rows, cols, nbits;
  uint32_t* dst;
  int64_t ld, ps;
  float lo, inv;
  uint32_t qmax;
  float qmaxf;
};

inline uint32_t host_code(const HostPack& p, int64_t idx) {
  if (p.src_dtype == QGTC_SRC_F32) {
    const float x = reinterpret_cast<const float*>(p.src)[idx];
    const float d = x - p.lo;                       // Eq. (2), as quantize_f32 on the device
    const float t = std::floor(d * p.inv);
    if (!(t > 0.0f)) return 0u;
    if (t >= p.qmaxf) return p.qmax;
    return (uint32_t)t;
  }
  if (p.src_dtype == QGTC_SRC_U8) return (uint32_t)reinterpret_cast<const uint8_t*>(p.src)[idx] & p.qmax;
  return reinterpret_cast<const uint32_t*>(p.src)[idx] & p.qmax;
}

// The adjacency: one bit from each of 32 bytes.  Eight bytes at a time: the lowest bit
// of byte k goes to bit k of the top byte of (x & 0x01..01) * 0x0102040810204080.
void pack_left_rows_u8_1bit(const HostPack& p, int r0, int r1) {
  const uint8_t* src = reinterpret_cast<const uint8_t*>(p.src);
  for (int r = r0; r < r1; ++r) {
    const uint8_t* row = src + (int64_t)r * p.ld_src;
    uint32_t* out = p.dst + (int64_t)r * p.ld;
    const int full = p.cols / 32;
    for (int w = 0; w < full; ++w) {
      uint32_t word = 0u;
      for (int k = 0; k < 4; ++k) {
        uint64_t x;
        std::memcpy(&x, row + w * 32 + k * 8, 8);
        word |= (uint32_t)(((x & 0x0101010101010101ull) * 0x0102040810204080ull) >> 56) << (8 * k);
      }
      out[w] = word;
    }
    for (int64_t w = full; w < p.ld; ++w) {
      uint32_t word = 0u;
      for (int b = 0; b < 32 && w * 32 + b < p.cols; ++b) word |= (uint32_t)(row[w * 32 + b] & 1u) << b;
      out[w] = word;
    }
  }
}

// LEFT: rows [r0, r1); bit b of word w of a row <-> column 32 w + b; all ld words written.
void pack_left_rows(const HostPack& p, int r0, int r1) {
  if (p.src_dtype == QGTC_SRC_U8 && p.nbits == 1) {
    pack_left_rows_u8_1bit(p, r0, r1);
    return;
  }
  std::vector<uint32_t> codes(32);
  for (int r = r0; r < r1; ++r) {
    for (int64_t w = 0; w < p.ld; ++w) {
      const int c0 = (int)(w * 32);
      const int n = std::max(0, std::min(32, p.cols - c0));
      for (int b = 0; b < n; ++b) codes[b] = host_code(p, (int64_t)r * p.ld_src + c0 + b);
      for (int pl = 0; pl < p.nbits; ++pl) {
        uint32_t word = 0u;
        for (int b = 0; b < n; ++b) word |= ((codes[b] >> pl) & 1u) << b;
        p.dst[(int64_t)pl * p.ps + (int64_t)r * p.ld + w] = word;
      }
    }
  }
}

// RIGHT: word rows [w0, w1); bit b of word (kw, c) <-> row 32 kw + b.
void pack_right_words(const HostPack& p, int w0, int w1) {
  std::vector<uint32_t> words((size_t)p.nbits * p.cols);
  std::vector<uint32_t> codes((size_t)p.cols);
  for (int kw = w0; kw < w1; ++kw) {
    std::fill(words.begin(), words.end(), 0u);
    const int n = std::min(32, p.rows - kw * 32);
    for (int b = 0; b < n; ++b) {                   // walk the source row by row (contiguous)
      const int64_t base = (int64_t)(kw * 32 + b) * p.ld_src;
      for (int c = 0; c < p.cols; ++c) codes[c] = host_code(p, base + c);
      for (int pl = 0; pl < p.nbits; ++pl) {        // plain loops over the columns: vectorizable
        uint32_t* wp = words.data() + (size_t)pl * p.cols;
        for (int c = 0; c < p.cols; ++c) wp[c] |= ((codes[c] >> pl) & 1u) << b;
      }
    }
    for (int pl = 0; pl < p.nbits; ++pl)
      std::copy(words.begin() + (size_t)pl * p.cols, words.begin() + (size_t)(pl + 1) * p.cols,
                p.dst + (int64_t)pl * p.ps + (int64_t)kw * p.ld);
  }
}

template <typename F>
void run_parallel(int n_items, int threads, F fn) {
  threads = std::max(1, std::min(threads, n_items));
  if (threads == 1) {
    fn(0, n_items);
    return;
  }
  std::vector<std::thread> pool;
  const int per = (n_items + threads - 1) / threads;
  for (int t = 0; t < threads; ++t) {
    const int a = t * per, b = std::min(n_items, a + per);
    if (a >= b) continue;
    try {
      pool.emplace_back(fn, a, b);
    } catch (...) {                                  // no more threads to be had: do the range here
      fn(a, b);
    }
  }
  for (auto& th : pool) th.join();
}

}  // namespace
}  // namespace qgtc

using namespace qgtc;

extern "C" qgtc_status qgtc_pack_bits_host(const void* src, int32_t src_dtype, int32_t rows, int32_t cols,
                                           int64_t ld_src, const qgtc_quant* q, const qgtc_bits* dst,
                                           int32_t threads) {
  if (!src || !dst) return QGTC_ERR_NULL;
  if (dst->layout != QGTC_LEFT && dst->layout != QGTC_RIGHT) return QGTC_ERR_UNSUPPORTED;
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
  if (threads < 0) return QGTC_ERR_SHAPE;
  if (rows == 0 || cols == 0) return QGTC_OK;

  HostPack p{};
  p.src = src;
  p.src_dtype = src_dtype;
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
  if (threads == 0) threads = (int)std::max(1u, std::thread::hardware_concurrency());
  if (dst->layout == QGTC_LEFT)
    run_parallel(rows, threads, [&p](int a, int b) { pack_left_rows(p, a, b); });
  else
    run_parallel(cdiv(rows, 32), threads, [&p](int a, int b) { pack_right_words(p, a, b); });
  return QGTC_OK;
}

extern "C" size_t qgtc_compound_layout(const size_t* bytes, int32_t n, size_t* offsets) {
  if (n < 0 || (n > 0 && (!bytes || !offsets))) return 0;
  size_t total = 0;
  for (int i = 0; i < n; ++i) {
    offsets[i] = total;
    total += (bytes[i] + 255) / 256 * 256;
  }
  return total;
}
