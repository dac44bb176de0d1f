// Shared host/device helpers of the library (not part of the public ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qgtc.h"
#include "qgtc_bench.h"

namespace qgtc {

constexpr int kWave = 64;

// ---- host side -------------------------------------------------------------
inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// Common checks on a packed-planes descriptor.
qgtc_status check_bits(const qgtc_bits* b, int want_layout);
// Stricter checks for an adjacency operand (1 bit, LEFT, 128-bit row padding).
qgtc_status check_adjacency(const qgtc_bits* A);
// Number of 32-bit words spanned by the descriptor (last addressed word + 1).
int64_t span_words(const qgtc_bits* b);

// Compute units of the current device (asked from the runtime once per device and kept);
// 256 on MI355X, which the launch shapes are tuned for.
int device_compute_units();

// Status of the launch that was just issued.
inline qgtc_status launch_status() {
  return hipGetLastError() == hipSuccess ? QGTC_OK : QGTC_ERR_HIP;
}

// Brackets the launches of one entry point with HIP events while profiling is on.
class ProfScope {
 public:
  ProfScope(int kind, hipStream_t stream);
  ~ProfScope();

 private:
  int slot_;
  hipStream_t stream_;
};

// Chunked dealing of workgroups to the XCDs: runs of 2^shift consecutive logical
// ids share an XCD, run k lands on XCD k % 8.  Grid size for nblocks logical ids:
inline unsigned xcd_deal_grid(unsigned nblocks, int shift) {
  const unsigned runs = (nblocks + (1u << shift) - 1u) >> shift;
  return ((runs + 7u) / 8u * 8u) << shift;
}

// Epilogue parameters as the kernels take them (device-visible copy).
struct EpiParams {
  int32_t mode, relu, self_term, rq_nbits;
  int32_t rq_lo;
  float rq_inv_scale;
  double cc, rs, l0a, l0b, ck, cs;
  const int32_t* row_i;
  const int32_t* row_l;
  const int32_t* col_i;
  const float* col_a;  // per-column affine in front of the activation (NULL: none)
  const float* col_b;
  void* out;           // int32_t* / float* / planes base (uint32_t*)
  int64_t ld_out;      // elements (I32/F32) or words (BITS)
  int64_t ps_out;      // BITS: plane stride in words
};

qgtc_status make_epilogue(const qgtc_epilogue* ep, void* out, int64_t ld_out,
                          int rows, int cols, int bits_layout, bool allow_self,
                          EpiParams* p);

// Arguments of the update kernels (popcount and int8-MFMA variants).
struct UpdParams {
  const uint32_t* Y;
  int32_t y_bytes;        // Y holds codes as bytes, row-major (ldy words per row)
  int64_t ldy, psy;       // words between rows / planes of Y
  int64_t y_span_bytes;   // bytes from the first to the last addressed word of Y
  int32_t rows;           // rows of Y (= output rows)
  int32_t s;              // planes of Y
  int32_t kwords;         // 32-bit words along the contraction dimension
  const uint32_t* W;
  int64_t ldw, psw;       // words between word rows / planes of W
  int32_t t;              // planes of W
  int32_t cols;           // columns of W (= output columns)
  int32_t hc;             // output columns per wave
  int32_t n_row_waves;
  EpiParams ep;
};


// Fused layer (layer.hip): aggregation, requantization and update in one kernel,
// the intermediate staying in LDS.  *done is false when the shapes or bit widths
// do not fit; nothing has been launched then.
qgtc_status layer_fused(const qgtc_bits* A, const qgtc_tile_map* map, const qgtc_bits* X,
                        const qgtc_bits* W, const qgtc_epilogue* agg_ep, const qgtc_epilogue* upd_ep,
                        void* workspace, size_t workspace_bytes, void* out, int64_t ld_out,
                        hipStream_t stream, bool* done);
size_t layer_fused_workspace_bytes(int32_t in_cols, int32_t out_cols);
// The selector's rules (plan.hip), shared by qgtc_plan_layer and the entry points.
bool plan_fused_applies(int in_cols, int out_cols, int s, int t);
int plan_update_path(int s, int t);                 // 1 popcount, 2 matrix cores
void plan_layer_shape(int n_tile_rows, int in_cols, int s, bool jumping, int* cgw, int* ksplit);
// Range check of a caller's tuning (NULL is fine).
qgtc_status check_tuning(const qgtc_tuning* t);

// int8 matrix-core variant of the update for s, t <= 8 (update_mfma.hip).
bool update_mfma_eligible(const UpdParams& p);
qgtc_status update_mfma_launch(const UpdParams& p, hipStream_t stream);

// ---- device side -------------------------------------------------------------
#if defined(__HIPCC__)

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).
// Logical id of hardware workgroup `bid` under xcd_deal_grid(); ids >= nblocks
// are to be dropped.
__device__ __forceinline__ unsigned xcd_deal(unsigned bid, int shift) {
  const unsigned slot = bid >> 3;                    // position inside the XCD's queue
  const unsigned run = ((slot >> shift) << 3) | (bid & 7u);
  return (run << shift) | (slot & ((1u << shift) - 1u));
}

// Eq. (2) with the clamp; see qgtc_quant in qgtc.h.
__device__ __forceinline__ uint32_t quantize_f32(float x, float lo, float inv,
                                                 uint32_t qmax, float qmaxf) {
  const float d = x - lo;
  const float t = floorf(d * inv);
  if (!(t > 0.0f)) return 0u;
  if (t >= qmaxf) return qmax;
  return (uint32_t)t;
}

// Requantization of a 32-bit accumulator; see QGTC_OUT_BITS in qgtc.h.
__device__ __forceinline__ uint32_t requantize_code(uint32_t c_u32, int relu, int32_t rq_lo,
                                                    float rq_inv_scale, uint32_t qmax, float qmaxf) {
  int32_t c = (int32_t)c_u32;
  if (relu && c < 0) c = 0;
  // max(c - rq_lo, 0) as an exact 64-bit difference: it is below 2^32, and when
  // c > rq_lo the wrapped 32-bit subtraction is that difference
  const uint32_t du = c > rq_lo ? (uint32_t)c - (uint32_t)rq_lo : 0u;
  const float f = (float)du;                      // round to nearest even
  const float t = floorf(f * rq_inv_scale);
  if (t >= qmaxf) return qmax;
  return (uint32_t)t;
}

// requantize_code for codes of at most 24 bits: relu_floor is 0 with ReLU, INT32_MIN
// without; 2^bits - 1 is exact in fp32, so the clamp can be taken on the float (t is never
// negative or NaN: the difference is >= 0, the scale finite and > 0), and the conversion to
// an integer truncates, which is the floor of a non-negative value.
__device__ __forceinline__ uint32_t requantize_code_small(uint32_t c_u32, int32_t relu_floor, int32_t rq_lo,
                                                          float rq_inv_scale, float qmaxf) {
  const int32_t c = max((int32_t)c_u32, relu_floor);
  const uint32_t du = (uint32_t)max(c, rq_lo) - (uint32_t)rq_lo;
  return (uint32_t)fminf((float)du * rq_inv_scale, qmaxf);
}

// The same for a range that starts at 0, [0, hi): max(c, 0) is the whole integer part,
// with or without ReLU.
__device__ __forceinline__ uint32_t requantize_code_relu0(uint32_t c_u32, float rq_inv_scale, float qmaxf) {
  return (uint32_t)fminf((float)(uint32_t)max((int32_t)c_u32, 0) * rq_inv_scale, qmaxf);
}

// The same behind a per-column affine map (a folded batch normalization); see
// col_scale in qgtc.h.  Two separately rounded fp32 operations, then Eq. (2).
__device__ __forceinline__ uint32_t requantize_affine(uint32_t c_u32, float a, float b, int relu,
                                                      int32_t rq_lo, float rq_inv_scale,
                                                      uint32_t qmax, float qmaxf) {
  float v = (float)(int32_t)c_u32 * a;
  v = v + b;
  if (relu && !(v > 0.0f)) v = 0.0f;
  return quantize_f32(v, (float)rq_lo, rq_inv_scale, qmax, qmaxf);
}

__device__ __forceinline__ uint32_t requantize_i32(uint32_t c_u32, int col, const EpiParams& e,
                                                   uint32_t qmax, float qmaxf) {
  if (e.col_a)
    return requantize_affine(c_u32, e.col_a[col], e.col_b ? e.col_b[col] : 0.0f, e.relu, e.rq_lo,
                             e.rq_inv_scale, qmax, qmaxf);
  return requantize_code(c_u32, e.relu, e.rq_lo, e.rq_inv_scale, qmax, qmaxf);
}

// fp32 output of the dequantizing epilogue; see QGTC_OUT_F32 in qgtc.h.
// ri: the entry of row_i for this row (0 when there is none).
__device__ __forceinline__ float dequantize_f64_ri(uint32_t c_u32, double ri, int row, int col,
                                                   const EpiParams& e) {
  const double c = (double)(int32_t)c_u32;
  const double rl = e.row_l ? (double)e.row_l[row] : 0.0;
  const double ci = e.col_i ? (double)e.col_i[col] : 0.0;
  const double t1 = e.cc * c + e.rs * ri;
  const double l0 = e.l0a + e.l0b * rl;
  const double t2 = l0 * (e.ck + e.cs * ci);
  double v = t1 + t2;
  if (e.col_a) v = v * (double)e.col_a[col] + (e.col_b ? (double)e.col_b[col] : 0.0);
  if (e.relu && v < 0.0) v = 0.0;
  return (float)v;
}

__device__ __forceinline__ float dequantize_f64(uint32_t c_u32, int row, int col,
                                                const EpiParams& e) {
  return dequantize_f64_ri(c_u32, e.row_i ? (double)e.row_i[row] : 0.0, row, col, e);
}

// 4 bits -> bit 0 of each of 4 bytes: the four shifted copies of x do not overlap.
__device__ __forceinline__ uint32_t spread4(uint32_t x4) {
  return __umul24(x4, 0x204081u) & 0x01010101u;
}

// 16-bit fields of up to 8 planes -> 16 bytes (as 4 dwords), byte j = sum_p bit_j(plane p) << p.
// Planes past the operand's bit width are passed as zeros.
__device__ __forceinline__ void planes_to_bytes(const uint32_t (&f)[8], int nplanes, uint32_t (&d)[4]) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    uint32_t v = 0u;
#pragma unroll
    for (int pl = 0; pl < 8; ++pl)
      if (pl < nplanes) v |= spread4((f[pl] >> (4 * q)) & 0xfu) << pl;   // wave-uniform test
    d[q] = v;
  }
}

// Transpose of an 8 x 8 bit matrix held as 8 bytes (byte r of hi:lo = row r, bit c
// of it = column c): afterwards byte c holds column c, bit r of it = row r.
// Three rounds of swapping ever larger off-diagonal blocks.
__device__ __forceinline__ void transpose_bits_8x8(uint32_t& lo, uint32_t& hi) {
  uint32_t t;
  t = (lo ^ (lo >> 7)) & 0x00AA00AAu;  lo = lo ^ t ^ (t << 7);
  t = (hi ^ (hi >> 7)) & 0x00AA00AAu;  hi = hi ^ t ^ (t << 7);
  t = (lo ^ (lo >> 14)) & 0x0000CCCCu; lo = lo ^ t ^ (t << 14);
  t = (hi ^ (hi >> 14)) & 0x0000CCCCu; hi = hi ^ t ^ (t << 14);
  t = (lo ^ ((lo >> 28) | (hi << 4))) & 0xF0F0F0F0u;
  lo = lo ^ t ^ (t << 28);
  hi = hi ^ (t >> 4);
}

#endif  // __HIPCC__

}  // namespace qgtc
