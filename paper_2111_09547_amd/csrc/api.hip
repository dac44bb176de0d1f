// Host-side parts of the C ABI: argument checks, descriptors, the one-layer
// driver and the optional event-based kernel timing.
#include <cstring>
#include <mutex>
#include <vector>

#include "qgtc_internal.h"

#include <cmath>

namespace qgtc {

int64_t span_words(const qgtc_bits* b) {
  if (b->rows == 0 || b->cols == 0 || b->nbits == 0) return 0;
  if (b->layout == QGTC_RIGHT_BYTES) return (int64_t)(b->nbits == 8 ? 2 : 1) * b->plane_stride_words;
  if (b->layout == QGTC_LEFT_BYTES) return (int64_t)(b->rows - 1) * b->ld_words + cdiv(b->cols, 4);
  if (b->layout == QGTC_LEFT)
    return (int64_t)(b->nbits - 1) * b->plane_stride_words + (int64_t)(b->rows - 1) * b->ld_words +
           cdiv(b->cols, 32);
  return (int64_t)(b->nbits - 1) * b->plane_stride_words + (int64_t)(cdiv(b->rows, 32) - 1) * b->ld_words +
         b->cols;
}

qgtc_status check_bits(const qgtc_bits* b, int want_layout) {
  if (!b) return QGTC_ERR_NULL;
  if (b->layout != QGTC_LEFT && b->layout != QGTC_RIGHT && b->layout != QGTC_RIGHT_BYTES &&
      b->layout != QGTC_LEFT_BYTES)
    return QGTC_ERR_LAYOUT;
  if (b->layout != want_layout) return QGTC_ERR_LAYOUT;
  if (b->nbits < 1 || b->nbits > 32) return QGTC_ERR_BITWIDTH;
  if (b->rows < 0 || b->cols < 0) return QGTC_ERR_SHAPE;
  if (b->rows > 0 && b->cols > 0 && !b->data) return QGTC_ERR_NULL;
  if (((uintptr_t)b->data & 3u) != 0) return QGTC_ERR_ALIGN;
  if (b->layout == QGTC_LEFT_BYTES) {
    if (b->nbits > 8) return QGTC_ERR_BITWIDTH;
    if (((uintptr_t)b->data & 15u) != 0 || (b->ld_words & 3) != 0) return QGTC_ERR_ALIGN;
    if (b->ld_words * 4 < b->cols) return QGTC_ERR_SHAPE;
    if (b->block_rows != 0) return QGTC_ERR_LAYOUT;
  } else if (b->layout == QGTC_RIGHT_BYTES) {
    if (b->nbits > 8) return QGTC_ERR_BITWIDTH;
    if (((uintptr_t)b->data & 15u) != 0) return QGTC_ERR_ALIGN;
    if (b->ld_words != 256 * (int64_t)cdiv(b->rows, 64)) return QGTC_ERR_SHAPE;
    if (b->plane_stride_words < (int64_t)cdiv(b->cols, 16) * b->ld_words) return QGTC_ERR_SHAPE;
    if (b->block_rows != 0) return QGTC_ERR_LAYOUT;
  } else if (b->layout == QGTC_LEFT) {
    if (b->ld_words < cdiv(b->cols, 32)) return QGTC_ERR_SHAPE;
    if (b->nbits > 1 && b->plane_stride_words < (int64_t)b->rows * b->ld_words) return QGTC_ERR_SHAPE;
  } else {
    if (b->ld_words < b->cols) return QGTC_ERR_SHAPE;
    if (b->nbits > 1 && b->plane_stride_words < (int64_t)cdiv(b->rows, 32) * b->ld_words)
      return QGTC_ERR_SHAPE;
    if (b->block_rows != 0) return QGTC_ERR_LAYOUT;
  }
  return QGTC_OK;
}

qgtc_status check_adjacency(const qgtc_bits* A) {
  qgtc_status st = check_bits(A, QGTC_LEFT);
  if (st != QGTC_OK) return st;
  if (A->nbits != 1) return QGTC_ERR_BITWIDTH;
  if (A->cols < 1) return QGTC_ERR_SHAPE;
  if ((A->ld_words & 3) != 0 || ((uintptr_t)A->data & 15u) != 0) return QGTC_ERR_ALIGN;
  if (A->ld_words < 4 * (int64_t)cdiv(A->cols, 128)) return QGTC_ERR_SHAPE;
  if (A->block_rows < 0) return QGTC_ERR_SHAPE;
  if (A->block_rows > 0) {
    if ((A->block_rows & 31) != 0) return QGTC_ERR_ALIGN;
    if (A->cols != A->block_rows) return QGTC_ERR_SHAPE;
  }
  return QGTC_OK;
}

qgtc_status make_epilogue(const qgtc_epilogue* ep, void* out, int64_t ld_out, int rows, int cols,
                          int bits_layout, bool allow_self, EpiParams* p) {
  if (!ep || !out) return QGTC_ERR_NULL;
  if (ep->mode != QGTC_OUT_I32 && ep->mode != QGTC_OUT_F32 && ep->mode != QGTC_OUT_BITS)
    return QGTC_ERR_UNSUPPORTED;
  if (ep->self_term && !allow_self) return QGTC_ERR_SHAPE;
  p->mode = ep->mode;
  p->relu = ep->relu ? 1 : 0;
  p->self_term = ep->self_term ? 1 : 0;
  p->rq_nbits = ep->rq_nbits;
  p->rq_lo = ep->rq_lo;
  p->rq_inv_scale = ep->rq_inv_scale;
  p->cc = ep->cc; p->rs = ep->rs; p->l0a = ep->l0a; p->l0b = ep->l0b; p->ck = ep->ck; p->cs = ep->cs;
  p->row_i = ep->row_i;
  p->row_l = ep->row_l;
  p->col_i = ep->col_i;
  if (ep->col_shift && !ep->col_scale) return QGTC_ERR_NULL;
  if (ep->col_scale && ep->mode == QGTC_OUT_I32) return QGTC_ERR_UNSUPPORTED;
  p->col_a = ep->col_scale;
  p->col_b = ep->col_shift;
  if (ep->mode == QGTC_OUT_BITS) {
    const qgtc_bits* d = reinterpret_cast<const qgtc_bits*>(out);
    qgtc_status st = check_bits(d, bits_layout);
    if (st != QGTC_OK) return st;
    if (d->rows != rows || d->cols != cols) return QGTC_ERR_SHAPE;
    if (ep->rq_nbits < 1 || ep->rq_nbits > 32 || d->nbits != ep->rq_nbits) return QGTC_ERR_BITWIDTH;
    if (d->block_rows != 0) return QGTC_ERR_LAYOUT;
    if (!(ep->rq_inv_scale > 0.0f) || !(ep->rq_inv_scale < INFINITY)) return QGTC_ERR_SHAPE;   // finite, positive
    p->out = d->data;
    p->ld_out = d->ld_words;
    p->ps_out = d->plane_stride_words;
  } else {
    if (ld_out < cols) return QGTC_ERR_SHAPE;
    if (((uintptr_t)out & 3u) != 0) return QGTC_ERR_ALIGN;
    p->out = out;
    p->ld_out = ld_out;
    p->ps_out = 0;
  }
  return QGTC_OK;
}

// ---- device facts --------------------------------------------------------------------
namespace {
std::mutex g_device_mutex;
int g_device_cus[64] = {};
}
int device_compute_units() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  std::lock_guard<std::mutex> lock(g_device_mutex);
  if (g_device_cus[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    g_device_cus[dev] = n;
  }
  return g_device_cus[dev];
}

}  // namespace qgtc

extern "C" qgtc_status qgtc_device_info(qgtc_device* out) {
  if (!out) return QGTC_ERR_NULL;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    (void)hipGetLastError();
    return QGTC_ERR_HIP;
  }
  out->compute_units = prop.multiProcessorCount;
  out->xcds = prop.multiProcessorCount / 32;
  out->is_gfx950 = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : 0;
  out->xcds_assumed = 8;
  return out->is_gfx950 ? QGTC_OK : QGTC_ERR_UNSUPPORTED;
}

namespace qgtc {

qgtc_status check_tuning(const qgtc_tuning* t) {
  if (!t) return QGTC_OK;
  if (t->update_path < 0 || t->update_path > 2) return QGTC_ERR_UNSUPPORTED;
  if (t->layer_path < 0 || t->layer_path > 1) return QGTC_ERR_UNSUPPORTED;
  if (t->layer_ksplit != 0 && t->layer_ksplit != 1 && t->layer_ksplit != 2 && t->layer_ksplit != 4)
    return QGTC_ERR_UNSUPPORTED;
  if (t->agg_xcd_run > 4096) return QGTC_ERR_UNSUPPORTED;
  if (t->zero_words < 0 || t->zero_words > 2) return QGTC_ERR_UNSUPPORTED;
  if (t->even_progress < 0 || t->even_progress > 2) return QGTC_ERR_UNSUPPORTED;
  return QGTC_OK;
}

// ---- event-based kernel timing ------------------------------------------------
namespace {
struct Span {
  int kind;
  hipEvent_t start, stop;
};
std::mutex g_prof_mutex;
bool g_prof_on = false;
std::vector<Span> g_spans;       // recorded since the last reset
std::vector<hipEvent_t> g_pool;  // events ready for reuse

hipEvent_t take_event() {
  if (!g_pool.empty()) {
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

ProfScope::ProfScope(int kind, hipStream_t stream) : slot_(-1), stream_(stream) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  if (!g_prof_on) return;
  Span s{kind, take_event(), take_event()};
  if (!s.start || !s.stop) return;
  (void)hipEventRecord(s.start, stream);
  g_spans.push_back(s);
  slot_ = (int)g_spans.size() - 1;
}

ProfScope::~ProfScope() {
  if (slot_ < 0) return;
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  if (slot_ < (int)g_spans.size()) (void)hipEventRecord(g_spans[slot_].stop, stream_);
}

}  // namespace qgtc

using namespace qgtc;

extern "C" const char* qgtc_status_string(qgtc_status s) {
  switch (s) {
    case QGTC_OK: return "ok";
    case QGTC_ERR_NULL: return "null pointer";
    case QGTC_ERR_SHAPE: return "shape mismatch";
    case QGTC_ERR_BITWIDTH: return "bit width out of range";
    case QGTC_ERR_ALIGN: return "misaligned pointer or leading dimension";
    case QGTC_ERR_LAYOUT: return "wrong packed layout";
    case QGTC_ERR_WORKSPACE: return "workspace too small";
    case QGTC_ERR_UNSUPPORTED: return "unsupported request";
    case QGTC_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

extern "C" int32_t qgtc_version(void) { return 200; }

extern "C" size_t qgtc_describe(qgtc_bits* d, int32_t rows, int32_t cols, int32_t nbits, int32_t layout,
                                int32_t block_rows) {
  if (!d || rows < 0 || cols < 0 || nbits < 1 || nbits > 32) return 0;
  if (layout != QGTC_LEFT && layout != QGTC_RIGHT && layout != QGTC_RIGHT_BYTES && layout != QGTC_LEFT_BYTES)
    return 0;
  if (block_rows < 0 || (layout != QGTC_LEFT && block_rows != 0)) return 0;
  if ((layout == QGTC_RIGHT_BYTES || layout == QGTC_LEFT_BYTES) && nbits > 8) return 0;
  d->nbits = nbits;
  d->rows = rows;
  d->cols = cols;
  d->layout = layout;
  d->block_rows = block_rows;
  d->reserved = 0;
  if (layout == QGTC_LEFT_BYTES) {
    d->ld_words = 4 * (int64_t)cdiv(cols, 16);
    d->plane_stride_words = (int64_t)rows * d->ld_words;
    return (size_t)d->plane_stride_words;
  }
  if (layout == QGTC_RIGHT_BYTES) {
    d->ld_words = 256 * (int64_t)cdiv(rows, 64);
    d->plane_stride_words = (int64_t)cdiv(cols, 16) * d->ld_words;
    return (size_t)(d->plane_stride_words * (nbits == 8 ? 2 : 1));
  }
  if (layout == QGTC_LEFT) {
    d->ld_words = 4 * (int64_t)cdiv(cols, 128);
    d->plane_stride_words = (int64_t)rows * d->ld_words;
  } else {
    d->ld_words = cols;
    d->plane_stride_words = (int64_t)cdiv(rows, 32) * d->ld_words;
  }
  return (size_t)(d->plane_stride_words * nbits);
}

namespace {
// Two-kernel path: bytes of the packed planes of Y (rounded up to 16) ...
size_t layer_y_bytes(int32_t rows, int32_t cols, int32_t nbits) {
  return ((size_t)rows * (size_t)cdiv(cols, 32) * (size_t)nbits * 4 + 15) / 16 * 16;
}
}  // namespace

extern "C" size_t qgtc_layer_workspace_bytes(int32_t rows, int32_t in_cols, int32_t out_cols,
                                             int32_t nbits) {
  if (rows < 0 || in_cols < 0 || out_cols < 0 || nbits < 1 || nbits > 32) return 0;
  // ... plus one int32 per row for the row sums of Y; the fused kernel keeps only
  // the weights in operand order there
  const size_t two = layer_y_bytes(rows, in_cols, nbits) + (size_t)rows * 4 + 16;
  const size_t fused = layer_fused_workspace_bytes(in_cols, out_cols);
  return two > fused ? two : fused;
}

extern "C" qgtc_status qgtc_layer(const qgtc_bits* A, const qgtc_tile_map* map, const qgtc_bits* X,
                                  const qgtc_bits* W, const qgtc_epilogue* agg_ep,
                                  const qgtc_epilogue* upd_ep, void* workspace, size_t workspace_bytes,
                                  void* out, int64_t ld_out, void* stream) {
  if (!A || !X || !W || !agg_ep || !upd_ep || !workspace || !out) return QGTC_ERR_NULL;
  if (agg_ep->mode != QGTC_OUT_BITS) return QGTC_ERR_UNSUPPORTED;
  if (agg_ep->col_scale || agg_ep->col_shift) return QGTC_ERR_UNSUPPORTED;   // the affine map belongs to upd_ep
  if (((uintptr_t)workspace & 15u) != 0) return QGTC_ERR_ALIGN;
  if (agg_ep->rq_nbits < 1 || agg_ep->rq_nbits > 32) return QGTC_ERR_BITWIDTH;
  if (workspace_bytes < qgtc_layer_workspace_bytes(A->rows, X->cols, W->cols, agg_ep->rq_nbits))
    return QGTC_ERR_WORKSPACE;
  // the requantized aggregation result, packed as the left operand of the update
  qgtc_bits Y{};
  Y.data = reinterpret_cast<uint32_t*>(workspace);
  Y.nbits = agg_ep->rq_nbits;
  Y.rows = A->rows;
  Y.cols = X->cols;
  Y.layout = QGTC_LEFT;
  Y.block_rows = 0;
  Y.ld_words = cdiv(X->cols, 32);
  Y.plane_stride_words = (int64_t)A->rows * Y.ld_words;
  // validate everything before anything is launched
  qgtc_status st = check_adjacency(A);
  if (st != QGTC_OK) return st;
  st = check_bits(X, QGTC_RIGHT);
  if (st != QGTC_OK) return st;
  st = check_bits(W, W->layout == QGTC_RIGHT_BYTES ? QGTC_RIGHT_BYTES : QGTC_RIGHT);
  if (st != QGTC_OK) return st;
  if (W->rows != X->cols) return QGTC_ERR_SHAPE;
  st = check_tuning(upd_ep->tuning);
  if (st != QGTC_OK) return st;
  EpiParams probe;
  st = make_epilogue(upd_ep, out, ld_out, A->rows, W->cols, QGTC_RIGHT, false, &probe);
  if (st != QGTC_OK) return st;

  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  bool done = false;
  st = layer_fused(A, map, X, W, agg_ep, upd_ep, workspace, workspace_bytes, out, ld_out, s, &done);
  if (st != QGTC_OK || done) return st;
  if (W->layout == QGTC_RIGHT_BYTES) return QGTC_ERR_UNSUPPORTED;   // only the fused kernel reads bytes

  qgtc_epilogue agg = *agg_ep;                       // the call's tuning is upd_ep's
  agg.tuning = upd_ep->tuning;
  st = qgtc_aggregate(A, map, X, &agg, &Y, 0, stream);
  if (st != QGTC_OK) return st;
  qgtc_epilogue upd = *upd_ep;
  if (upd.mode == QGTC_OUT_F32 && upd.row_i == nullptr && upd.rs != 0.0) {
    // the row sums of Y only exist now
    int32_t* sums = reinterpret_cast<int32_t*>(reinterpret_cast<uint8_t*>(workspace) +
                                               layer_y_bytes(A->rows, X->cols, agg_ep->rq_nbits));
    st = qgtc_row_sums(&Y, sums, stream);
    if (st != QGTC_OK) return st;
    upd.row_i = sums;
  }
  return qgtc_update(&Y, W, &upd, out, ld_out, stream);
}

// ---- qgtc_layer for callers that cannot allocate -----------------------------------
// The workspace of qgtc_layer (weights in operand order for the fused kernel; packed
// planes of Y and their row sums for the two-kernel path) in device memory that comes
// with the code object instead of from the caller.  Every GPU the library runs on holds
// its own copy of the array, at its own address, until the process ends.
static __device__ __align__(256) unsigned char scratch[QGTC_LAYER_STATIC_MAX_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` per device, set on first use

// Device address of the current device's copy of `scratch` (the array's name is a
// host-side handle only, never an address to hand to a kernel).
qgtc_status scratch_address(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return QGTC_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return QGTC_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return QGTC_OK;
}
}  // namespace

extern "C" qgtc_status qgtc_layer_static(const qgtc_bits* A, const qgtc_tile_map* map, const qgtc_bits* X,
                                         const qgtc_bits* W, const qgtc_epilogue* agg_ep,
                                         const qgtc_epilogue* upd_ep, void* out, int64_t ld_out,
                                         void* stream) {
  if (!A || !X || !W || !agg_ep || !upd_ep || !out) return QGTC_ERR_NULL;
  if (agg_ep->rq_nbits < 1 || agg_ep->rq_nbits > 32) return QGTC_ERR_BITWIDTH;
  const size_t need = qgtc_layer_workspace_bytes(A->rows, X->cols, W->cols, agg_ep->rq_nbits);
  if (need == 0 || need > (size_t)QGTC_LAYER_STATIC_MAX_BYTES) return QGTC_ERR_WORKSPACE;
  void* ws = nullptr;
  qgtc_status st = scratch_address(&ws);
  if (st != QGTC_OK) return st;
  // every word of the workspace that a kernel of the layer reads has been written by an
  // earlier kernel of the same call, so nothing needs clearing between calls
  return qgtc_layer(A, map, X, W, agg_ep, upd_ep, ws, (size_t)QGTC_LAYER_STATIC_MAX_BYTES, out, ld_out,
                    stream);
}

extern "C" qgtc_status qgtc_prof_enable(int32_t on) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  g_prof_on = on != 0;
  return QGTC_OK;
}

extern "C" qgtc_status qgtc_prof_reset(void) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  for (Span& s : g_spans) {
    (void)hipEventSynchronize(s.stop);
    g_pool.push_back(s.start);
    g_pool.push_back(s.stop);
  }
  g_spans.clear();
  return QGTC_OK;
}

extern "C" qgtc_status qgtc_prof_read(int32_t kind, double* total_ms, int64_t* launches) {
  if (!total_ms || !launches) return QGTC_ERR_NULL;
  if (kind < 0 || kind >= QGTC_KERNEL_KINDS) return QGTC_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  double ms = 0.0;
  int64_t n = 0;
  for (Span& s : g_spans) {
    if (s.kind != kind) continue;
    if (hipEventSynchronize(s.stop) != hipSuccess) return QGTC_ERR_HIP;
    float t = 0.f;
    if (hipEventElapsedTime(&t, s.start, s.stop) != hipSuccess) return QGTC_ERR_HIP;
    ms += t;
    ++n;
  }
  *total_ms = ms;
  *launches = n;
  return QGTC_OK;
}
