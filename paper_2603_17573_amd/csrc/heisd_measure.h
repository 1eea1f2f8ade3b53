// Reference kernels for the measurements the design rests on (not part of the method): how fast this
// chip reads HBM with the access patterns the weight-streaming GEMMs use, with nothing else in the
// kernel - the ceiling any of those GEMMs can reach - and what an empty launch costs.
#pragma once
#include "heisd_common.h"

namespace heisd {

constexpr int kMeasureThreads = 512;    // 8 waves per workgroup, like the GEMM kernels

typedef unsigned int mu32x4 __attribute__((ext_vector_type(4)));

// Pattern 0: every wave reads one contiguous span, U loads of 16 bytes per lane (U KB per wave) in flight.
template <int U>
__global__ __launch_bounds__(kMeasureThreads) void measure_read_contiguous(const mu32x4 *p, size_t n_vec, unsigned *sink) {
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * (kMeasureThreads / 64) + (threadIdx.x >> 6);
  const size_t nw = (size_t)gridDim.x * (kMeasureThreads / 64);
  const size_t per = n_vec / nw / (64 * U) * (64 * U);           // vectors per wave, whole rounds only
  const mu32x4 *q = p + wave * per + lane;
  unsigned acc = 0;
  for (size_t i = 0; i < per; i += (size_t)64 * U) {
    mu32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = q[i + (size_t)u * 64];
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x12345678u) sink[0] = acc;                           // keeps the loads alive; practically never taken
}

// Pattern 1: the fragment-ordered weight copy as the <= 8-row GEMMs walk it: a workgroup owns the 16-row
// tiles wg, wg + grid, ...; wave w owns a contiguous eighth of a tile's k-steps (1 KB each) and keeps
// U of them in flight.  tile_bytes = bytes of one tile (k-steps * 1 KB).
template <int U>
__global__ __launch_bounds__(kMeasureThreads) void measure_read_tiles(const mu32x4 *p, int n_tiles, int ksteps, unsigned *sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ksw = (ksteps + 7) / 8, s0 = wave * ksw, s1 = min(ksteps, s0 + ksw);
  unsigned acc = 0;
  for (int t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const mu32x4 *q = p + ((size_t)t * ksteps) * 64 + lane;
    for (int s = s0; s < s1; s += U) {
      mu32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = q[(size_t)min(s + u, s1 - 1) * 64];
#pragma unroll
      for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
  }
  if (acc == 0x12345678u) sink[0] = acc;
}

__global__ __launch_bounds__(kMeasureThreads) void measure_empty() {}

}  // namespace heisd
