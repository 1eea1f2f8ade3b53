// The verify-skip decision (paper Sec. 4.1, Alg. 1): features of the final layer, their cosine
// similarity over pairs of trajectory points, the offline stage's minimum acceptable similarity and
// its point distance, and the per-episode decision that produces the skip mask the verify step
// consumes.  Small fp32 kernels: one wavefront per pair of feature vectors.
#pragma once
#include "heisd_common.h"

namespace heisd {

// feat[b][:] = RMSNorm(x[m][:]; gain, eps) for row m = b * rows_per_ep + row[b] (the last row of the
// episode when `row` is null): the LM head's input of that row.  One workgroup per episode.
__global__ __launch_bounds__(256) void export_features(const float *x, const int32_t *row, int rows_per_ep, int d,
                                                      const float *gain, float eps, float *feat) {
  __shared__ float part[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int r = row ? row[b] : rows_per_ep - 1;
  r = max(0, min(r, rows_per_ep - 1));
  const float *src = x + ((size_t)b * rows_per_ep + r) * d;
  float ss = 0.f;
  for (int c = tid * 4; c < d; c += 256 * 4) {
    const float4 v = *reinterpret_cast<const float4 *>(src + c);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = wave_sum(ss);
  if (lane == 0) part[wave] = ss;
  __syncthreads();
  const float inv = rsqrtf((part[0] + part[1] + part[2] + part[3]) / (float)d + eps);
  for (int c = tid * 4; c < d; c += 256 * 4) {
    const float4 v = *reinterpret_cast<const float4 *>(src + c);
    const float4 g = *reinterpret_cast<const float4 *>(gain + c);
    *reinterpret_cast<float4 *>(feat + (size_t)b * d + c) = make_float4(v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w);
  }
}

// Cosine similarity of two d-vectors by one wavefront; 0 if either is all zero.
__device__ __forceinline__ float wave_cosine(const float *a, const float *b, int d, int lane) {
  float ab = 0.f, aa = 0.f, bb = 0.f;
  for (int c = lane * 4; c < d; c += kWave * 4) {
    const float4 u = *reinterpret_cast<const float4 *>(a + c);
    const float4 v = *reinterpret_cast<const float4 *>(b + c);
    ab += u.x * v.x + u.y * v.y + u.z * v.z + u.w * v.w;
    aa += u.x * u.x + u.y * u.y + u.z * u.z + u.w * u.w;
    bb += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ab = wave_sum(ab);
  aa = wave_sum(aa);
  bb = wave_sum(bb);
  return (aa == 0.f || bb == 0.f) ? 0.f : ab / (sqrtf(aa) * sqrtf(bb));
}

// Floats as unsigned integers of the same order.
__device__ __forceinline__ uint32_t ordered_bits(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_bits(uint32_t o) {
  return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}

__global__ void skip_key_init(unsigned long long *key) { *key = ~0ull; }

// S[i][j] = cosine(a[i], b[j]), one wavefront per pair.  With `key` given (offline stage of Alg. 1;
// a and b are then the same n trajectory points): every pair i < j whose similarity exceeds T offers
// (similarity, i, j - i) to a 64-bit minimum, so that the smallest similarity above T wins and, among
// equals, the pair found first by the algorithm's loops (i ascending, then distance ascending).
__global__ __launch_bounds__(256) void pair_similarity(const float *a, const float *b, int n, int m, int d, float *S,
                                                      float T, unsigned long long *key) {
  const int lane = threadIdx.x & 63;
  const long long pair = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (pair >= (long long)n * m) return;
  const int i = (int)(pair / m), j = (int)(pair % m);
  if (!S && key && i >= j) return;          // offline stage without the matrix: only pairs i < j count
  const float s = wave_cosine(a + (size_t)i * d, b + (size_t)j * d, d, lane);
  if (lane != 0) return;
  if (S) S[(size_t)i * m + j] = s;
  if (key && i < j && s > T)
    atomicMin(key, ((unsigned long long)ordered_bits(s) << 32) | ((unsigned long long)i << 16) | (unsigned long long)(j - i));
}

__global__ void skip_key_decode(const unsigned long long *key, float *min_s, int32_t *o_dist) {
  const unsigned long long k = *key;
  if (k == ~0ull) {
    *min_s = INFINITY;          // nothing above the boundary: never skip
    *o_dist = 0;
  } else {
    *min_s = from_ordered_bits((uint32_t)(k >> 32));
    *o_dist = (int32_t)(k & 0xFFFFull);
  }
}

// skip[b] = dist[b] <= O_dist and cosine(feat_prev[b], feat_last[b]) >= min_S.  One wavefront per episode.
__global__ __launch_bounds__(64) void skip_decide(const float *feat_prev, const float *feat_last, const int32_t *dist,
                                                  int d, const float *min_s, const int32_t *o_dist, uint8_t *skip,
                                                  float *S_out) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const float s = wave_cosine(feat_prev + (size_t)b * d, feat_last + (size_t)b * d, d, lane);
  if (lane != 0) return;
  if (S_out) S_out[b] = s;
  skip[b] = (dist[b] <= *o_dist && s >= *min_s) ? 1 : 0;
}

}  // namespace heisd
