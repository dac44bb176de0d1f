/*
 * qgtc_bench.h - measurement aids of libqgtc.so, apart from the product's C ABI
 * (qgtc.h): event-based per-kernel timing and a register-only probe of the vector
 * ALUs' AND + popcount rate.  bench.py and the sweeps use them; a product caller
 * needs none of them.
 */
#ifndef QGTC_BENCH_H
#define QGTC_BENCH_H

#include "qgtc.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---------------------------------------------------------------------------
 * Optional per-kernel timing.  While enabled, every kernel launch is bracketed
 * by HIP events recorded on the launch stream (the events are created on first
 * use and kept in a pool: the only host-side allocation of the library).
 * qgtc_prof_read synchronizes with the recorded events and returns, for one
 * kernel kind, the summed duration in milliseconds and the number of launches
 * since the last reset.  Thread-safe; off by default.
 * ------------------------------------------------------------------------- */
enum {
  QGTC_KERNEL_PACK = 0,
  QGTC_KERNEL_TILE_MAP = 1,
  QGTC_KERNEL_AGGREGATE = 2,
  QGTC_KERNEL_UPDATE = 3,
  QGTC_KERNEL_SUMS = 4,
  QGTC_KERNEL_LAYER = 5, /* fused layer kernel (with its weight re-ordering) */
  QGTC_KERNEL_KINDS = 6
};
qgtc_status qgtc_prof_enable(int32_t on);
qgtc_status qgtc_prof_reset(void);
qgtc_status qgtc_prof_read(int32_t kind, double* total_ms, int64_t* launches);

/* Runs the AND + popcount inner block of the aggregation (Section 3.1, Eq. (7):
 * 16 rows x 8 planes = 256 vector instructions = 64 lanes x 32 x 128 one-bit
 * multiply-accumulates per wave and call) 4 * iters times per wave on registers
 * only, in `workgroups` workgroups of `waves_per_workgroup` (1..4) waves.  Timing
 * the launch gives the attainable AND + popcount rate of the device as it is
 * clocked at that moment.  sink: one device word, practically never written. */
qgtc_status qgtc_probe_popcount(int32_t workgroups, int32_t waves_per_workgroup,
                                int32_t iters, uint32_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QGTC_BENCH_H */
