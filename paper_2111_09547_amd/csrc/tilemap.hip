// Zero-tile map of a packed adjacency (zero-tile jumping, Section 4.3 of the
// paper).  The paper ORs the words of each 8x128 tile inside the product kernel
// and skips the tile when the result is zero; the adjacency is the same for all
// layers, so here the test runs once and leaves, per row of tiles, the list of
// tile columns that hold an edge.  HBM-bound: A is read once for the map and
// once for the degrees.
#include "qgtc_internal.h"

namespace qgtc {
namespace {

struct MapParams {
  const uint32_t* A;
  int64_t lda;
  int32_t rows;
  int32_t n_words;        // data words per row, ceil(cols/32)
  int32_t tile_rows, tile_words;
  int32_t n_tile_rows, n_tile_cols;
  int32_t* row_cnt;
  int32_t* col_idx;
  int32_t* nnz;
  int32_t* deg;
};

// One wave per tile row.  lane <-> tile column inside a group of 64; the OR over
// the tile's words decides, a ballot and a prefix count over the lanes compact
// the surviving tile columns in ascending order.
__global__ __launch_bounds__(256) void tile_list_kernel(const MapParams p) {
  const int lane = threadIdx.x & 63;
  const int tr = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tr >= p.n_tile_rows) return;               // whole wave
  const int r0 = tr * p.tile_rows;
  const int r1 = min(r0 + p.tile_rows, p.rows);
  int32_t* list = p.col_idx + (int64_t)tr * p.n_tile_cols;
  int count = 0;
  for (int tc0 = 0; tc0 < p.n_tile_cols; tc0 += 64) {
    const int tc = tc0 + lane;
    uint32_t any = 0u;
    if (tc < p.n_tile_cols) {
      const int w0 = tc * p.tile_words;
      const int w1 = min(w0 + p.tile_words, p.n_words);
      for (int r = r0; r < r1; ++r) {
        const uint32_t* row = p.A + (int64_t)r * p.lda;
        for (int w = w0; w < w1; ++w) any |= row[w];
      }
    }
    const unsigned long long m = __builtin_amdgcn_ballot_w64(any != 0u);
    const int before = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    if (any != 0u) list[count + before] = tc;
    count += __builtin_popcountll(m);
  }
  if (lane == 0) p.row_cnt[tr] = count;
}

// The shape the aggregation kernel uses (16 rows x 32/64/128 bits): one wave per
// tile row, lane <-> (row = lane % 16, one of four consecutive 128-bit columns =
// lane / 16).  Rows are padded to 128 bits, so every row is read once with 16-byte
// loads whatever the tile width, the loads of four iterations (16 columns of a row)
// issued before the first ballot; a 128-bit column holds 4 / TW tiles, and a ballot per
// tile over the wave tells which of them hold a bit.  The same pass counts the degrees.
template <int TW>
__global__ __launch_bounds__(256) void tile_list16_kernel(const MapParams p) {
  constexpr int SUB = 4 / TW;                    // tiles per 128-bit column
  const int lane = threadIdx.x & 63;
  const int tr = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tr >= p.n_tile_rows) return;               // whole wave
  const int r = tr * 16 + (lane & 15);
  const int g = lane >> 4;
  const bool r_ok = r < p.rows;
  const uint32_t* row = p.A + (int64_t)(r_ok ? r : 0) * p.lda;
  int32_t* list = p.col_idx + (int64_t)tr * p.n_tile_cols;
  const int n128 = (p.n_words + 3) >> 2;
  int count = 0;
  int deg = 0;
  for (int tc0 = 0; tc0 < n128; tc0 += 16) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int tc = tc0 + 4 * u + g;
      v[u] = make_uint4(0u, 0u, 0u, 0u);
      if (r_ok && tc < n128) v[u] = *reinterpret_cast<const uint4*>(row + 4 * tc);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      deg += __builtin_popcount(v[u].x) + __builtin_popcount(v[u].y) + __builtin_popcount(v[u].z) +
             __builtin_popcount(v[u].w);
      uint32_t any[SUB];
      if constexpr (TW == 4) {
        any[0] = v[u].x | v[u].y | v[u].z | v[u].w;
      } else if constexpr (TW == 2) {
        any[0] = v[u].x | v[u].y;
        any[1] = v[u].z | v[u].w;
      } else {
        any[0] = v[u].x; any[1] = v[u].y; any[2] = v[u].z; any[3] = v[u].w;
      }
      unsigned long long m[SUB];
#pragma unroll
      for (int c = 0; c < SUB; ++c) m[c] = __builtin_amdgcn_ballot_w64(any[c] != 0u);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
#pragma unroll
        for (int c = 0; c < SUB; ++c) {
          const int tile = (tc0 + 4 * u + k) * SUB + c;
          // wave-uniform; the bound keeps a destination whose row padding was not
          // zeroed (a contract violation) from writing past the list
          if (((m[c] >> (16 * k)) & 0xffffull) != 0ull && tile < p.n_tile_cols) {
            if (lane == 0) list[count] = tile;
            ++count;
          }
        }
      }
    }
  }
  deg += __shfl_xor(deg, 16, 64);
  deg += __shfl_xor(deg, 32, 64);
  if (lane < 16 && r_ok) p.deg[r] = deg;
  if (lane == 0) p.row_cnt[tr] = count;
}

// Total number of non-zero tiles, and the length of the runs of tile rows that the
// product kernels deal to one XCD: one workgroup.
//
// Tile rows next to each other read the same word rows of X (inside a subgraph
// all of them do), so the longer the run of tile rows that stays on one XCD, the
// fewer L2s fetch the same rows of X from HBM.  Runs go round-robin to the 8
// XCDs, and the XCD with the most work ends the kernel: the longest run is
// chosen whose heaviest XCD carries at most 2 % more than the mean, a tile row
// counted as its non-zero tiles plus one (the fixed part of a tile row costs
// about one tile).  nnz[1] = log2 of that run, 3..6 (8..64 tile rows).
__global__ __launch_bounds__(256) void tile_total_kernel(const MapParams p) {
  __shared__ unsigned long long load[4 * 8];     // [candidate: run of 8 << c tile rows][XCD]
  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  if (t < 32) load[t] = 0ull;
  // Thread t sees tile rows t, t + 256, ...: their runs of 8, 16 and 32 tile rows land
  // on one XCD each, (t >> 3) & 7, (t >> 4) & 7 and (t >> 5) & 7 (256 is a multiple of
  // 8 runs of 32), their runs of 64 alternate between two XCDs, wave and wave + 4.
  unsigned long long even = 0ull, odd = 0ull;
#pragma unroll 4
  for (int i = t; i < p.n_tile_rows; i += 512) {     // several independent loads in flight
    const int j = i + 256;
    const int ce = p.row_cnt[i];
    const int co = j < p.n_tile_rows ? p.row_cnt[j] + 1 : 0;
    even += (unsigned long long)(ce + 1);
    odd += (unsigned long long)co;
  }
  __syncthreads();
  auto group_sum = [&](unsigned long long v, int width) {   // sum over aligned groups of `width` lanes
    for (int off = 1; off < width; off <<= 1) {
      const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)v, off, 64);
      const unsigned hi = (unsigned)__shfl_xor((int)(unsigned)(v >> 32), off, 64);
      v += ((unsigned long long)hi << 32) | lo;
    }
    return v;
  };
  const unsigned long long all = even + odd;
  const unsigned long long s8 = group_sum(all, 8), s16 = group_sum(all, 16), s32 = group_sum(all, 32);
  const unsigned long long e64 = group_sum(even, 64), o64 = group_sum(odd, 64);
  if ((lane & 7) == 0) atomicAdd(&load[0 * 8 + ((t >> 3) & 7)], s8);
  if ((lane & 15) == 0) atomicAdd(&load[1 * 8 + ((t >> 4) & 7)], s16);
  if ((lane & 31) == 0) atomicAdd(&load[2 * 8 + ((t >> 5) & 7)], s32);
  if (lane == 0) {
    atomicAdd(&load[3 * 8 + wave], e64);
    atomicAdd(&load[3 * 8 + wave + 4], o64);
  }
  __syncthreads();
  if (t == 0) {
    unsigned long long total = 0ull;
    for (int x = 0; x < 8; ++x) total += load[x];
    int best = 3;
    for (int c = 3; c >= 1; --c) {
      unsigned long long mx = 0ull;
      for (int x = 0; x < 8; ++x) mx = load[c * 8 + x] > mx ? load[c * 8 + x] : mx;
      if (mx * 8ull * 50ull <= total * 51ull) { best = 3 + c; break; }
    }
    p.nnz[0] = (int)(total - (unsigned long long)p.n_tile_rows);
    p.nnz[1] = best;
  }
}

// deg[r] = popcount of row r: one wave per row.
__global__ __launch_bounds__(256) void degree_kernel(const MapParams p) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= p.rows) return;
  const uint32_t* row = p.A + (int64_t)r * p.lda;
  int cnt = 0;
  for (int w = lane; w < p.n_words; w += 64) cnt += __builtin_popcount(row[w]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, 64);
  if (lane == 0) p.deg[r] = cnt;
}

// Non-zero tiles at 16 x 32, 16 x 64 and 16 x 128 in one pass: a wave per row of tiles,
// lane <-> (row = lane % 16, one of four consecutive 128-bit groups = lane / 16).  A ballot
// per word of the group tells, for each of the four groups, whether any of the 16 rows has
// a bit there; the three counts follow from the four answers.
__global__ __launch_bounds__(256) void tile_stats_kernel(const MapParams p, int32_t* counts) {
  __shared__ int part[3];
  __shared__ unsigned long long part_rw;
  const int lane = threadIdx.x & 63;
  if (threadIdx.x < 3) part[threadIdx.x] = 0;
  if (threadIdx.x == 3) part_rw = 0ull;
  __syncthreads();
  unsigned long long rw = 0ull;                   // (row, 32-bit word) pairs that hold a bit
  const int n128 = (p.n_words + 3) >> 2;          // rows are padded to 128 bits with zeros
  const int g = lane >> 4;
  int c32 = 0, c64 = 0, c128 = 0;
  // a wave walks over rows of tiles with the stride of the grid: few, long-lived waves, and
  // three atomic additions per workgroup at the end
  for (int tr = blockIdx.x * 4 + (threadIdx.x >> 6); tr < p.n_tile_rows; tr += (int)gridDim.x * 4) {
    const int r = tr * 16 + (lane & 15);
    const bool r_ok = r < p.rows;
    const uint32_t* row = p.A + (int64_t)(r_ok ? r : 0) * p.lda;
    for (int t0 = 0; t0 < n128; t0 += 16) {
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {               // 16 groups of a row in flight together
        const int tc = t0 + 4 * u + g;
        v[u] = make_uint4(0u, 0u, 0u, 0u);
        if (r_ok && tc < n128) v[u] = *reinterpret_cast<const uint4*>(row + 4 * tc);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const unsigned long long mx = __builtin_amdgcn_ballot_w64(v[u].x != 0u);
        const unsigned long long my = __builtin_amdgcn_ballot_w64(v[u].y != 0u);
        const unsigned long long mz = __builtin_amdgcn_ballot_w64(v[u].z != 0u);
        const unsigned long long mw = __builtin_amdgcn_ballot_w64(v[u].w != 0u);
        rw += (unsigned long long)(__builtin_popcountll(mx) + __builtin_popcountll(my) +
                                   __builtin_popcountll(mz) + __builtin_popcountll(mw));
#pragma unroll
        for (int k = 0; k < 4; ++k) {             // wave-uniform arithmetic
          const int bx = ((mx >> (16 * k)) & 0xffffull) != 0ull, by = ((my >> (16 * k)) & 0xffffull) != 0ull;
          const int bz = ((mz >> (16 * k)) & 0xffffull) != 0ull, bw = ((mw >> (16 * k)) & 0xffffull) != 0ull;
          c32 += bx + by + bz + bw;
          c64 += (bx | by) + (bz | bw);
          c128 += bx | by | bz | bw;
        }
      }
    }
  }
  if (lane == 0) {
    atomicAdd(&part[0], c32);
    atomicAdd(&part[1], c64);
    atomicAdd(&part[2], c128);
    atomicAdd(&part_rw, rw);
  }
  __syncthreads();
  if (threadIdx.x < 3 && part[threadIdx.x] != 0) atomicAdd(&counts[threadIdx.x], part[threadIdx.x]);
  if (threadIdx.x == 3 && part_rw != 0ull)
    atomicAdd(reinterpret_cast<unsigned long long*>(counts + 4), part_rw);    // counts[4], counts[5]: one 64-bit number
}

// Start values of the counters (a kernel, so that the call can be recorded into a HIP graph).
__global__ void tile_stats_init_kernel(int32_t* counts, int32_t n_tile_rows) {
  if (threadIdx.x < 8) counts[threadIdx.x] = threadIdx.x == 3 ? n_tile_rows : 0;
}

bool tile_shape_ok(int tile_rows, int tile_kbits) {
  const bool r = tile_rows == 8 || tile_rows == 16 || tile_rows == 32 || tile_rows == 64;
  const bool k = tile_kbits == 32 || tile_kbits == 64 || tile_kbits == 128 || tile_kbits == 256 ||
                 tile_kbits == 512;
  return r && k;
}

size_t align16(size_t v) { return (v + 15) & ~(size_t)15; }

}  // namespace
}  // namespace qgtc

using namespace qgtc;

extern "C" size_t qgtc_tile_map_bytes(int32_t rows, int32_t kbits, int32_t tile_rows, int32_t tile_kbits) {
  if (rows < 0 || kbits < 0 || !tile_shape_ok(tile_rows, tile_kbits)) return 0;
  const size_t ntr = (size_t)cdiv(rows, tile_rows), ntc = (size_t)cdiv(kbits, tile_kbits);
  return align16(ntr * 4) + align16(ntr * ntc * 4) + 16 + align16((size_t)rows * 4) + 16;
}

extern "C" qgtc_status qgtc_tile_map_carve(qgtc_tile_map* map, void* buffer, int32_t rows, int32_t kbits,
                                           int32_t tile_rows, int32_t tile_kbits) {
  if (!map || !buffer) return QGTC_ERR_NULL;
  if (rows < 0 || kbits < 0) return QGTC_ERR_SHAPE;
  if (!tile_shape_ok(tile_rows, tile_kbits)) return QGTC_ERR_UNSUPPORTED;
  if (((uintptr_t)buffer & 15u) != 0) return QGTC_ERR_ALIGN;
  const size_t ntr = (size_t)cdiv(rows, tile_rows), ntc = (size_t)cdiv(kbits, tile_kbits);
  char* b = reinterpret_cast<char*>(buffer);
  map->tile_rows = tile_rows;
  map->tile_kbits = tile_kbits;
  map->n_tile_rows = (int32_t)ntr;
  map->n_tile_cols = (int32_t)ntc;
  map->row_cnt = reinterpret_cast<int32_t*>(b);
  b += align16(ntr * 4);
  map->col_idx = reinterpret_cast<int32_t*>(b);
  b += align16(ntr * ntc * 4);
  map->nnz_tiles = reinterpret_cast<int32_t*>(b);
  b += 16;
  map->deg = reinterpret_cast<int32_t*>(b);
  return QGTC_OK;
}

extern "C" qgtc_status qgtc_build_tile_map(const qgtc_bits* A, const qgtc_tile_map* map, void* stream) {
  if (!A || !map) return QGTC_ERR_NULL;
  qgtc_status st = check_adjacency(A);
  if (st != QGTC_OK) return st;
  if (!map->row_cnt || !map->col_idx || !map->nnz_tiles || !map->deg) return QGTC_ERR_NULL;
  if (!tile_shape_ok(map->tile_rows, map->tile_kbits)) return QGTC_ERR_UNSUPPORTED;
  if (map->n_tile_rows != cdiv(A->rows, map->tile_rows) || map->n_tile_cols != cdiv(A->cols, map->tile_kbits))
    return QGTC_ERR_SHAPE;

  MapParams p{};
  p.A = A->data;
  p.lda = A->ld_words;
  p.rows = A->rows;
  p.n_words = cdiv(A->cols, 32);
  p.tile_rows = map->tile_rows;
  p.tile_words = map->tile_kbits / 32;
  p.n_tile_rows = map->n_tile_rows;
  p.n_tile_cols = map->n_tile_cols;
  p.row_cnt = map->row_cnt;
  p.col_idx = map->col_idx;
  p.nnz = map->nnz_tiles;
  p.deg = map->deg;

  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  ProfScope prof(QGTC_KERNEL_TILE_MAP, s);
  const bool fused = p.tile_rows == 16 && p.tile_words <= 4;
  if (p.n_tile_rows > 0 && p.n_tile_cols > 0) {
    if (fused && p.tile_words == 4)
      hipLaunchKernelGGL(tile_list16_kernel<4>, dim3((unsigned)cdiv(p.n_tile_rows, 4)), dim3(256), 0, s, p);
    else if (fused && p.tile_words == 2)
      hipLaunchKernelGGL(tile_list16_kernel<2>, dim3((unsigned)cdiv(p.n_tile_rows, 4)), dim3(256), 0, s, p);
    else if (fused)
      hipLaunchKernelGGL(tile_list16_kernel<1>, dim3((unsigned)cdiv(p.n_tile_rows, 4)), dim3(256), 0, s, p);
    else
      hipLaunchKernelGGL(tile_list_kernel, dim3((unsigned)cdiv(p.n_tile_rows, 4)), dim3(256), 0, s, p);
    if (launch_status() != QGTC_OK) return QGTC_ERR_HIP;
  }
  hipLaunchKernelGGL(tile_total_kernel, dim3(1), dim3(256), 0, s, p);
  if (launch_status() != QGTC_OK) return QGTC_ERR_HIP;
  if (p.rows > 0 && !(fused && p.n_tile_rows > 0 && p.n_tile_cols > 0)) {
    hipLaunchKernelGGL(degree_kernel, dim3((unsigned)cdiv(p.rows, 4)), dim3(256), 0, s, p);
    if (launch_status() != QGTC_OK) return QGTC_ERR_HIP;
  }
  return QGTC_OK;
}

extern "C" qgtc_status qgtc_tile_stats(const qgtc_bits* A, int32_t* counts, void* stream) {
  if (!A || !counts) return QGTC_ERR_NULL;
  qgtc_status st = check_adjacency(A);
  if (st != QGTC_OK) return st;
  if (((uintptr_t)counts & 7u) != 0) return QGTC_ERR_ALIGN;
  MapParams p{};
  p.A = A->data;
  p.lda = A->ld_words;
  p.rows = A->rows;
  p.n_words = cdiv(A->cols, 32);
  p.n_tile_rows = cdiv(A->rows, 16);
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  ProfScope prof(QGTC_KERNEL_TILE_MAP, s);
  hipLaunchKernelGGL(tile_stats_init_kernel, dim3(1), dim3(64), 0, s, counts, p.n_tile_rows);
  if (launch_status() != QGTC_OK) return QGTC_ERR_HIP;
  if (p.n_tile_rows > 0) {
    const int blocks = cdiv(p.n_tile_rows, 4);
    const int cap = device_compute_units() * 8;
    hipLaunchKernelGGL(tile_stats_kernel, dim3((unsigned)(blocks < cap ? blocks : cap)), dim3(256), 0, s, p, counts);
    if (launch_status() != QGTC_OK) return QGTC_ERR_HIP;
  }
  return QGTC_OK;
}
