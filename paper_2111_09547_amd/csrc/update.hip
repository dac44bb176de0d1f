// Node update C = Y.W on packed bit planes (second half of Algorithm 1 of the
// paper: every plane of Y against every plane of W, shifted by the sum of the
// plane indices and added up), written for gfx950.
//
// The contraction dimension D is short here (a few 32-bit words) and the row
// count N is large, so the roles are the reverse of the aggregation kernel:
//   lane <-> row (node): the lane keeps the packed words of its own row of Y in
//   VGPRs; the words of W for the output column in flight are the same for all
//   lanes: the workgroup stages its slice of W in LDS once (W is a few KiB) and
//   every lane reads the same LDS address (a broadcast, free of bank
//   conflicts), so a (plane, plane, word) triple is one v_and_b32 plus one
//   v_bcnt_u32_b32.
// Plane pairs with the same index sum share an accumulator ("bit level" in
// Algorithm 1), so the shift-and-add costs s + t - 1 operations per output.
// A wave covers 64 rows and a run of output columns; the column range is split
// over the grid when there are few rows.
#include "qgtc_internal.h"

namespace qgtc {
namespace {

#include "popc_blocks.inc"

// B = planes handled per chunk (both operands), KC = words of K kept in registers.
template <int B, int KC>
__global__ __launch_bounds__(256) void update_kernel(const UpdParams p) {
  extern __shared__ uint32_t wl[];                  // [hc][n_wc*B][n_kc*KC], zero padded
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int lane = threadIdx.x & 63;
  const int rw = blockIdx.x * 4 + wave;             // 64-row group of this wave
  const int row0 = rw * 64;
  const int row = row0 + lane;
  const bool row_ok = row < p.rows;
  const uint32_t* yrow = p.Y + (int64_t)(row_ok ? row : 0) * p.ldy;

  const int h_begin = blockIdx.y * p.hc;
  const int h_end = min(h_begin + p.hc, p.cols);

  const int n_yc = (p.s + B - 1) / B;               // plane chunks of Y
  const int n_wc = (p.t + B - 1) / B;               // plane chunks of W
  const int n_kc = (p.kwords + KC - 1) / KC;        // word chunks of K

  // stage W[.][.][h_begin .. h_end) in LDS, column-major per output column
  const int wp = n_wc * B, wk = n_kc * KC;
  for (int idx = threadIdx.x; idx < p.hc * wp * wk; idx += 256) {
    const int hl = idx % p.hc;
    const int kw = (idx / p.hc) % wk;
    const int pl = idx / (p.hc * wk);
    uint32_t v = 0u;
    if (pl < p.t && kw < p.kwords && h_begin + hl < h_end)
      v = p.W[(int64_t)pl * p.psw + (int64_t)kw * p.ldw + h_begin + hl];
    wl[(hl * wp + pl) * wk + kw] = v;
  }
  __syncthreads();
  if (rw >= p.n_row_waves) return;                  // whole wave leaves (no barrier follows)
  const bool hoist = n_yc == 1 && n_kc == 1;        // Y words loaded once per wave

  uint32_t y[B][KC];
  auto load_y = [&](int ic, int kc) {
#pragma unroll
    for (int i = 0; i < B; ++i)
#pragma unroll
      for (int k = 0; k < KC; ++k) {
        const int pl = ic * B + i;
        const int kw = kc * KC + k;
        y[i][k] = (row_ok && pl < p.s && kw < p.kwords) ? yrow[(int64_t)pl * p.psy + kw] : 0u;
      }
  };
  if (hoist) load_y(0, 0);

  const EpiParams& e = p.ep;
  const int qbits = e.rq_nbits;
  const uint32_t qmax = qbits >= 32 ? 0xffffffffu : ((1u << qbits) - 1u);
  const float qmaxf = (float)qmax;
  // low-bit output with at most B planes: ballot words are gathered in lanes
  const bool fast_bits = e.mode == QGTC_OUT_BITS && qbits <= B;
  uint32_t ow_lo[B], ow_hi[B];
#pragma unroll
  for (int i = 0; i < B; ++i) { ow_lo[i] = 0u; ow_hi[i] = 0u; }

  for (int h = h_begin; h < h_end; ++h) {
    const uint32_t* wcol = wl + (h - h_begin) * wp * wk;
    uint32_t z = 0u;
    for (int ic = 0; ic < n_yc; ++ic) {
      for (int kc = 0; kc < n_kc; ++kc) {
        if (!hoist) load_y(ic, kc);
        for (int jc = 0; jc < n_wc; ++jc) {
          const int shift0 = (ic + jc) * B;
          if (shift0 >= 32) continue;               // vanishes modulo 2^32
          uint32_t diag[2 * B - 1];
#pragma unroll
          for (int d = 0; d < 2 * B - 1; ++d) diag[d] = 0u;
#pragma unroll
          for (int jj = 0; jj < B; ++jj) {
#pragma unroll
            for (int k = 0; k < KC; ++k) {
              // same LDS address in every lane: a broadcast read
              const uint32_t w = wcol[((jc * B + jj) * n_kc + kc) * KC + k];
#pragma unroll
              for (int i = 0; i < B; ++i) diag[i + jj] += __builtin_popcount(w & y[i][k]);
            }
          }
          uint32_t v = 0u;
#pragma unroll
          for (int d = 0; d < 2 * B - 1; ++d) v += diag[d] << d;
          z += v << shift0;
        }
      }
    }

    // ---- epilogue for entry (row, h) ----------------------------------------
    if (e.mode == QGTC_OUT_I32) {
      int32_t o = (int32_t)z;
      if (e.relu && o < 0) o = 0;
      if (row_ok) reinterpret_cast<int32_t*>(e.out)[(int64_t)row * e.ld_out + h] = o;
    } else if (e.mode == QGTC_OUT_F32) {
      if (row_ok) reinterpret_cast<float*>(e.out)[(int64_t)row * e.ld_out + h] = dequantize_f64(z, row, h, e);
    } else {
      // RIGHT layout for the next aggregation: 32 consecutive rows per word, so a
      // ballot over the lanes is two finished words of column h.
      const uint32_t q = row_ok ? requantize_i32(z, h, e, qmax, qmaxf) : 0u;
      if (fast_bits) {
        // keep them in lane (h - h_begin) until the whole column run is done
        uint32_t lo[B], hi[B];
#pragma unroll
        for (int i = 0; i < B; ++i) {
          const unsigned long long m = __builtin_amdgcn_ballot_w64(((q >> i) & 1u) != 0u);
          lo[i] = (uint32_t)m;
          hi[i] = (uint32_t)(m >> 32);
        }
        lane_pack_m0<B>::run(lo, hi, ow_lo, ow_hi, (h - h_begin) & 63);
        if (((h - h_begin) & 63) == 63 || h + 1 == h_end) {
          // flush: lane l holds the words of column h0 + l
          const int h0 = h - ((h - h_begin) & 63);
          const int hh = h0 + lane;
          const int wr0 = row0 >> 5;
          const int n_wr = (p.rows + 31) >> 5;
          if (hh <= h) {
            uint32_t* dst = reinterpret_cast<uint32_t*>(e.out) + (int64_t)wr0 * e.ld_out + hh;
#pragma unroll
            for (int i = 0; i < B; ++i) {
              if (i < qbits) {
                dst[(int64_t)i * e.ps_out] = ow_lo[i];
                if (wr0 + 1 < n_wr) dst[(int64_t)i * e.ps_out + e.ld_out] = ow_hi[i];
              }
            }
          }
        }
      } else {
        const int wr = (row0 >> 5) + (lane & 1);
        const bool st = lane < 2 && wr < ((p.rows + 31) >> 5);
        uint32_t* dst = reinterpret_cast<uint32_t*>(e.out) + (st ? (int64_t)wr * e.ld_out + h : 0);
        for (int i = 0; i < qbits; ++i) {
          const unsigned long long m = __builtin_amdgcn_ballot_w64(((q >> i) & 1u) != 0u);
          const uint32_t word = (lane & 1) ? (uint32_t)(m >> 32) : (uint32_t)m;
          if (st) dst[(int64_t)i * e.ps_out] = word;
        }
      }
    }
  }
}

template <int B, int KC>
qgtc_status launch(const UpdParams& p, int hsplit, hipStream_t stream) {
  dim3 grid((unsigned)cdiv(p.n_row_waves, 4), (unsigned)hsplit);
  const size_t lds = (size_t)p.hc * (size_t)(cdiv(p.t, B) * B) * (size_t)(cdiv(p.kwords, KC) * KC) * 4;
  if (lds > 64 * 1024) return QGTC_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((update_kernel<B, KC>), grid, dim3(256), lds, stream, p);
  return launch_status();
}

template <int B>
qgtc_status dispatch_k(const UpdParams& p, int hsplit, hipStream_t stream) {
  if (p.kwords <= 1) return launch<B, 1>(p, hsplit, stream);
  if (p.kwords <= 2) return launch<B, 2>(p, hsplit, stream);
  if (p.kwords <= 4 || B > 4) return launch<B, 4>(p, hsplit, stream);
  return launch<B, 8>(p, hsplit, stream);
}

}  // namespace
}  // namespace qgtc

using namespace qgtc;

extern "C" qgtc_status qgtc_update(const qgtc_bits* Y, const qgtc_bits* W, const qgtc_epilogue* ep,
                                   void* out, int64_t ld_out, void* stream) {
  if (!Y || !W || !ep) return QGTC_ERR_NULL;
  if (!out && !(Y->rows == 0 || W->cols == 0)) return QGTC_ERR_NULL;   // an empty result needs no buffer
  const bool y_bytes = Y->layout == QGTC_LEFT_BYTES;
  qgtc_status st = check_bits(Y, y_bytes ? QGTC_LEFT_BYTES : QGTC_LEFT);
  if (st != QGTC_OK) return st;
  st = check_bits(W, QGTC_RIGHT);
  if (st != QGTC_OK) return st;
  if (Y->cols != W->rows) return QGTC_ERR_SHAPE;
  if (Y->block_rows != 0) return QGTC_ERR_LAYOUT;

  UpdParams p{};
  p.Y = Y->data;
  p.y_bytes = y_bytes ? 1 : 0;
  p.ldy = Y->ld_words;
  p.psy = Y->plane_stride_words;
  p.y_span_bytes = span_words(Y) * 4;
  p.rows = Y->rows;
  p.s = Y->nbits;
  p.kwords = cdiv(Y->cols, 32);
  p.W = W->data;
  p.ldw = W->ld_words;
  p.psw = W->plane_stride_words;
  p.t = W->nbits;
  p.cols = W->cols;
  if (Y->rows == 0 || W->cols == 0) return QGTC_OK;
  st = make_epilogue(ep, out, ld_out, Y->rows, W->cols, QGTC_RIGHT, false, &p.ep);
  if (st != QGTC_OK) return st;
  st = check_tuning(ep->tuning);
  if (st != QGTC_OK) return st;

  p.n_row_waves = cdiv(Y->rows, 64);
  // enough waves to fill 256 CUs x 4 SIMDs a few times over
  int hsplit = cdiv(4096, p.n_row_waves);
  if (hsplit > W->cols) hsplit = W->cols;
  if (hsplit < 1) hsplit = 1;
  p.hc = cdiv(W->cols, hsplit);
  // keep the staged slice of W below 32 KiB (planes and words padded to 8)
  const int64_t per_col = (int64_t)((W->nbits + 7) / 8 * 8) * ((p.kwords + 7) / 8 * 8) * 4;
  if (per_col > 32 * 1024) return QGTC_ERR_UNSUPPORTED;
  while ((int64_t)p.hc * per_col > 32 * 1024) p.hc = (p.hc + 1) / 2;
  hsplit = cdiv(W->cols, p.hc);

  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  ProfScope prof(QGTC_KERNEL_UPDATE, s);
  // popcount kernel or int8 matrix cores: the caller's choice, else the selector's rule
  int path = ep->tuning ? ep->tuning->update_path : 0;
  if (path == 0) path = plan_update_path(Y->nbits, W->nbits);
  if (y_bytes) return update_mfma_eligible(p) ? update_mfma_launch(p, s) : QGTC_ERR_UNSUPPORTED;
  if (path == 2 && update_mfma_eligible(p)) return update_mfma_launch(p, s);
  const int b = Y->nbits > W->nbits ? Y->nbits : W->nbits;
  switch (b) {
    case 1: return dispatch_k<1>(p, hsplit, s);
    case 2: return dispatch_k<2>(p, hsplit, s);
    case 3: return dispatch_k<3>(p, hsplit, s);
    case 4: return dispatch_k<4>(p, hsplit, s);
    case 5: return dispatch_k<5>(p, hsplit, s);
    case 6: return dispatch_k<6>(p, hsplit, s);
    case 7: return dispatch_k<7>(p, hsplit, s);
    default: return dispatch_k<8>(p, hsplit, s);
  }
}
