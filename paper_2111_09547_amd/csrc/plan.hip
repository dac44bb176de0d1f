// Host-only parts of the C ABI: the selector (which tile width, kernels and launch shape
// a layer takes) and the scalar algebra around a stack of layers.  Nothing here touches
// the GPU.
#include "qgtc_internal.h"

#include <cmath>

namespace qgtc {

// Relative cost of one adjacency bit column by tile width, measured on the fused layer
// kernel: 64-bit tiles cost what 128-bit tiles cost per bit, 32-bit tiles 1.0 - 1.4 times
// as much (one word step per tile leaves less to overlap the tile fetch with).
static const double kTileCost[3] = {1.3, 1.0, 1.0};   // 32, 64, 128 bits
static const int kTileBits[3] = {32, 64, 128};
static const double kJumpTileSteps = 5.8;             // cost of a tile in word steps, zero-word jumping form

// Sustained rates the time estimates use (MI355X, measured): the aggregation at 0.70 of
// the vector-ALU AND + popcount ceiling (0.45 with 16 or fewer columns, where the lanes
// split K), the streaming kernels at 4.3 TB/s, 10 us per launch that does not overlap.
static const double kPopcountRate = 0.70 * 1.258e15;
static const double kPopcountRateNarrow = 0.45 * 1.258e15;
static const double kStreamRate = 4.3e12;
static const double kLaunchUs = 10.0;

bool plan_fused_applies(int in_cols, int out_cols, int s, int t) {
  return s >= 1 && s <= 8 && t >= 1 && t <= 8 && in_cols >= 1 && in_cols <= 1024 && out_cols >= 1 &&
         out_cols <= 256;
}

int plan_update_path(int s, int t) {
  // int8 matrix cores whenever both operands fit in bytes: on MI355X they are ahead of the
  // popcount kernel at every bit width from 1 x 1 upwards once the launch is long enough to
  // measure, and level with it below (both at the launch floor)
  return (s >= 1 && s <= 8 && t >= 1 && t <= 8) ? 2 : 1;
}

// Wave slots of the device for the aggregation loop: waves per SIMD by the planes a lane
// accumulates (the register budget), four in the jumping form from five planes on, where
// two rows share an accumulator register.
static int64_t plan_wave_slots(int s, bool jumping) {
  const int planes = s > 8 ? 8 : s;
  const int per_simd = planes >= 5 ? (jumping ? 4 : 3) : (planes >= 3 ? 4 : 5);
  return (int64_t)device_compute_units() * 4 * per_simd;
}

void plan_layer_shape(int n_tile_rows, int in_cols, int s, bool jumping, int* cgw, int* ksplit) {
  const int n_cg = cdiv(in_cols, 64);
  int w = n_cg <= 4 ? n_cg : (n_cg % 3 == 0 ? 3 : 4);
  const int64_t slots = plan_wave_slots(s, jumping);
  // Jumping form: when the tile rows alone fit the wave slots, no more waves side by side than
  // still fit them, and more passes per wave instead - the launch then is one round of
  // resident waves that move through their lists abreast (qgtc_tuning.even_progress), which
  // measures ahead of two rounds of half the work (config 4's 128-column layer: 212 against
  // 220 us for the five layers).
  if (jumping && n_tile_rows <= slots) {
    while (w > 1 && ((int64_t)n_tile_rows * w > slots || n_cg % w != 0)) --w;
  }
  // Waves that split each tile list: as many as it takes to fill the wave slots of the
  // device when there are few tile rows; with two column groups, workgroups of four
  // waves measured faster than pairs, so the lists are split in two there as well.
  int k = 1;
  while ((int64_t)n_tile_rows * w * k < slots && w * k * 2 <= 4) k *= 2;
  // (not in the form that jumps over zero words: its waves are bound by latency, and the
  // exchange of partial sums only adds to it - 252 against 263 us on config 4's five layers)
  if (w == 2 && k == 1 && !jumping) k = 2;
  *cgw = w;
  *ksplit = k;
}

}  // namespace qgtc

using namespace qgtc;

extern "C" qgtc_status qgtc_plan_layer(const qgtc_plan_in* in, qgtc_plan_out* out) {
  if (!in || !out) return QGTC_ERR_NULL;
  if (in->rows < 0 || in->in_cols < 1 || in->out_cols < 1 || in->n_tile_rows < 0 || in->a_cols < 0 ||
      in->subgraphs < 0 || in->nnz_row_words < 0)
    return QGTC_ERR_SHAPE;
  if (in->s < 1 || in->s > 32 || in->t < 1 || in->t > 32) return QGTC_ERR_BITWIDTH;
  for (int k = 0; k < 3; ++k)
    if (in->nnz_tiles[k] < 0) return QGTC_ERR_SHAPE;

  // tile width: least executed work; without statistics every 128-bit tile counts
  int best = 2;
  double work[3];
  const bool known = in->nnz_tiles[0] > 0 || in->nnz_tiles[1] > 0 || in->nnz_tiles[2] > 0;
  for (int k = 0; k < 3; ++k)
    work[k] = known ? (double)in->nnz_tiles[k] * kTileBits[k] * kTileCost[k]
                    : (double)in->n_tile_rows * (double)cdiv(in->a_cols, 128) * 128.0 * (k == 2 ? 1.0 : 2.0);
  for (int k = 1; k >= 0; --k)
    if (work[k] < 0.98 * work[best]) best = k;
  out->fused = plan_fused_applies(in->in_cols, in->out_cols, in->s, in->t) ? 1 : 0;
  out->update_path = plan_update_path(in->s, in->t);
  // zero-word jumping: pays while fewer than 70 % of the (row, word) pairs of the kept tiles
  // hold a bit (measured: a present row costs about two issue slots more in that form), 60 %
  // from five planes on, where half of the present rows cost a third instruction per plane
  // (two rows per accumulator register)
  auto sparse_at = [&](int k) {
    const double pairs = 16.0 * (double)in->nnz_tiles[k] * (kTileBits[k] / 32);
    return (double)in->nnz_row_words < (in->s >= 5 ? 0.6 : 0.7) * pairs;
  };
  out->zero_words = 0;
  if (in->nnz_row_words > 0 && known) {
    out->zero_words = (in->s >= 3 && sparse_at(best)) ? 2 : 1;
    if (out->zero_words == 2) {
      // The jumping form visits the same non-zero (row, word) pairs at every tile width;
      // what differs is the word steps it tests (tiles x words per tile) and the tiles it
      // fetches, one of which costs about as much as kJumpTileSteps word steps (fitted to
      // config 5, where 64-bit tiles measure 2 - 4 % ahead of both other widths from 3 to
      // 8 bits; config 4 keeps its 128-bit tiles).  The wider tile stays unless a narrower
      // one wins by 2 %; any width at least as wide as the visit-all choice is still sparse.
      int bj = 2;
      auto steps = [&](int k) { return (double)in->nnz_tiles[k] * (kTileBits[k] / 32 + kJumpTileSteps); };
      for (int k = 1; k >= 0; --k)
        if (steps(k) < 0.98 * steps(bj)) bj = k;
      if (sparse_at(bj)) best = bj;
    }
  }
  out->tile_kbits = kTileBits[best];
  const double tiles = known ? (double)in->nnz_tiles[best] : (double)in->n_tile_rows * cdiv(in->a_cols, 128);
  // without the statistic the library jumps whenever it gets a tile map and 3 planes or more
  const bool jumping = out->zero_words == 2 || (out->zero_words == 0 && in->s >= 3);
  int cgw = 1, ksplit = 1;
  plan_layer_shape(in->n_tile_rows, in->in_cols, in->s, jumping, &cgw, &ksplit);
  out->ksplit = ksplit;
  // A launch of at most one wave per wave slot has all its waves resident from the start:
  // the tile loop then gives the waves that are behind the higher issue priority
  // (qgtc_tuning.even_progress).  Independent runs: a fused launch of more than one and at
  // most two rounds of the wave slots leaves the device part empty while it drains; two
  // runs of whole subgraphs on two streams overlap one run's drain with the other's work.
  // Runs of at least eight subgraphs, so that the XCD dealing inside a run still has one
  // subgraph per XCD.
  const int64_t slots = plan_wave_slots(in->s, jumping);
  const int64_t waves = (int64_t)in->n_tile_rows * cgw * ksplit;
  out->even_progress = waves <= slots ? 2 : 1;
  out->reserved = 0;
  out->runs = 1;
  if (out->fused && in->subgraphs >= 16 && in->subgraphs % 2 == 0 && waves > slots && waves <= 2 * slots)
    out->runs = 2;

  // rough times of the two orders of the products
  const double bits = 16.0 * kTileBits[best] * kTileCost[best] * tiles;   // adjacency bits visited, weighted
  auto agg_us = [&](int cols) {
    const double ops = 2.0 * bits * cols * in->s;
    return ops / (cols <= 16 ? kPopcountRateNarrow : kPopcountRate) * 1e6 + kLaunchUs;
  };
  auto upd_us = [&](double bytes_per_row) {
    const double bytes = (double)in->rows * (bytes_per_row + in->out_cols * (double)in->s / 8.0);
    const double mfma = 2.0 * in->rows * (double)in->in_cols * in->out_cols / 2.0e15;   // int8, well below the peak
    const double popc = 2.0 * in->rows * (double)in->in_cols * in->out_cols * in->s * in->t / (0.2 * 1.258e15);
    const double compute = out->update_path == 2 ? mfma : popc;
    const double stream = bytes / kStreamRate;
    return (compute > stream ? compute : stream) * 1e6 + kLaunchUs;
  };
  const double y_bytes = (double)in->in_cols * in->s / 8.0;
  out->est_us_aggregate_first = out->fused ? agg_us(in->in_cols) : agg_us(in->in_cols) + upd_us(y_bytes);
  // update first: the features as bytes (at most 8 bits) or planes into the update, then the
  // aggregation on out_cols columns
  out->est_us_update_first = upd_us(in->s <= 8 && in->t <= 8 ? (double)in->in_cols : y_bytes) + agg_us(in->out_cols);
  return QGTC_OK;
}

extern "C" float qgtc_quant_inv_scale(double lo, double hi, int32_t nbits) {
  if (nbits < 1 || nbits > 32 || !(hi > lo)) return 0.0f;
  return (float)(std::ldexp(1.0, nbits) / (hi - lo));
}

extern "C" qgtc_status qgtc_layer_epilogues(const qgtc_layer_spec* sp, qgtc_epilogue* first_ep,
                                            qgtc_epilogue* second_ep, double* z_scale,
                                            double* next_x_scale) {
  if (!sp || !first_ep || !second_ep) return QGTC_ERR_NULL;
  if (sp->s < 1 || sp->s > 32 || sp->t < 1 || sp->t > 32) return QGTC_ERR_BITWIDTH;
  if (sp->in_cols < 1 || (sp->order != 0 && sp->order != 1)) return QGTC_ERR_SHAPE;
  if (!(sp->agg_hi > 0.0) || !(sp->w_hi > sp->w_lo) || !(sp->x_scale > 0.0)) return QGTC_ERR_SHAPE;
  if (!sp->last && !(sp->out_hi > 0.0)) return QGTC_ERR_SHAPE;
  if (sp->order == 1 && sp->batchnorm) return QGTC_ERR_UNSUPPORTED;

  const double inv_first = (double)qgtc_quant_inv_scale(0.0, sp->agg_hi, sp->s);
  const double sw = (sp->w_hi - sp->w_lo) / std::ldexp(1.0, sp->t);
  // real value of one unit of the second product's accumulator (codes read as pure scales)
  const double zs = sp->order == 0 ? (sp->x_scale / inv_first) * sw : (sp->x_scale * sw) / inv_first;

  auto scalars_only = [](qgtc_epilogue* e) {
    e->mode = QGTC_OUT_I32; e->relu = 0; e->self_term = 0; e->rq_nbits = 0; e->rq_lo = 0; e->rq_inv_scale = 0.0f;
    e->cc = e->rs = e->l0a = e->l0b = e->ck = e->cs = 0.0;
  };
  scalars_only(first_ep);
  scalars_only(second_ep);
  first_ep->mode = QGTC_OUT_BITS;
  first_ep->rq_nbits = sp->s;
  first_ep->rq_inv_scale = (float)inv_first;
  // the GIN self term belongs to the aggregation, whichever product that is
  (sp->order == 0 ? first_ep : second_ep)->self_term = sp->self_term ? 1 : 0;

  double next = 0.0;
  if (!sp->last) {
    const double inv_out = (double)qgtc_quant_inv_scale(0.0, sp->out_hi, sp->s);
    second_ep->mode = QGTC_OUT_BITS;
    second_ep->relu = 1;
    second_ep->rq_nbits = sp->s;
    second_ep->rq_inv_scale = (float)inv_out;
    next = sp->batchnorm ? 1.0 / inv_out : zs / inv_out;
  } else {
    second_ep->mode = QGTC_OUT_F32;
    if (sp->order == 0) {
      // left operand l0[i] + sl * Yq, l0[i] = x_lo * (deg[i] + self); right operand w_lo + sw * Wq
      const double sl = sp->x_scale / inv_first;
      second_ep->cc = sl * sw;
      second_ep->rs = sl * sp->w_lo;
      second_ep->l0a = sp->self_term ? sp->x_lo : 0.0;
      second_ep->l0b = sp->x_lo;
      second_ep->ck = sp->w_lo * (double)sp->in_cols;
      second_ep->cs = sw;
    } else {
      second_ep->cc = zs;                            // every code a pure scale
    }
  }
  if (z_scale) *z_scale = zs;
  if (next_x_scale) *next_x_scale = next;
  return QGTC_OK;
}

extern "C" qgtc_status qgtc_fold_batchnorm(const double* gamma, const double* beta, const double* mean,
                                           const double* var, double eps, double value_scale, int32_t n,
                                           float* col_scale, float* col_shift) {
  if (n < 0) return QGTC_ERR_SHAPE;
  if (n == 0) return QGTC_OK;
  if (!gamma || !beta || !mean || !var || !col_scale || !col_shift) return QGTC_ERR_NULL;
  for (int32_t j = 0; j < n; ++j) {
    if (!(var[j] + eps > 0.0)) return QGTC_ERR_SHAPE;
    const double a = gamma[j] / std::sqrt(var[j] + eps);
    col_scale[j] = (float)(a * value_scale);
    col_shift[j] = (float)(beta[j] - a * mean[j]);
  }
  return QGTC_OK;
}
