// Register-only probe of the AND + popcount rate of the vector ALUs: the inner
// block of the aggregation kernel (v_and_b32 with DPP broadcast + v_bcnt_u32_b32,
// 16 rows x 8 planes) in a loop without any memory traffic.  It gives the
// measured ceiling that the aggregation is priced against beside the nominal one
// (256 CUs x 64 lanes per clock x 2.4 GHz).
#include "qgtc_internal.h"

namespace qgtc {
namespace {

#include "popc_blocks.inc"

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void popcount_probe_kernel(int iters, uint32_t* sink) {
  uint32_t acc[16][8];
#pragma unroll
  for (int j = 0; j < 16; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[j][i] = 0u;
  uint32_t x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = threadIdx.x * 0x9e3779b9u + i;
  uint32_t a = threadIdx.x ^ 0x5bd1e995u;
  for (int k = 0; k < iters; ++k) {
    popc_rows<8>::run(a, x, acc);
    popc_rows<8>::run(a, x, acc);
    popc_rows<8>::run(a, x, acc);
    popc_rows<8>::run(a, x, acc);
  }
  uint32_t v = 0u;
#pragma unroll
  for (int j = 0; j < 16; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) v += acc[j][i];
  if (v == 0x12345678u) sink[0] = v;               // keeps the loop alive; practically never true
}

}  // namespace
}  // namespace qgtc

using namespace qgtc;

extern "C" qgtc_status qgtc_probe_popcount(int32_t workgroups, int32_t waves_per_workgroup, int32_t iters,
                                           uint32_t* sink, void* stream) {
  if (!sink) return QGTC_ERR_NULL;
  if (workgroups < 1 || waves_per_workgroup < 1 || waves_per_workgroup > 4 || iters < 1) return QGTC_ERR_SHAPE;
  hipLaunchKernelGGL(popcount_probe_kernel, dim3((unsigned)workgroups), dim3(64 * waves_per_workgroup), 0,
                     reinterpret_cast<hipStream_t>(stream), iters, sink);
  return launch_status();
}
