// The retrieval branch's nearest-neighbour search (paper App. C: C.1 database construction, C.2 performance): cosine Top-K of a query embedding
// over the database of L2-normalised embeddings, as an exact brute-force scan.  The database is read
// once per group of up to four queries (2.4 GB at the paper's size: an HBM stream), the scores go to
// a small buffer, and the K best per query are selected in two rounds.
#pragma once
#include "heisd_common.h"

namespace heisd {

constexpr int kScanThreads = 512;      // 8 wavefronts per workgroup
constexpr int kTopChunk = 2048;        // scores per workgroup in the first selection round
constexpr int kTopMaxK = 64;

// scores[q][i] = <db[i], queries[q]>, q < NQ.  A wavefront takes two database rows per iteration (the
// query slices it reads from LDS serve both); lane l covers elements 256 t + 4 l .. + 3 of a row, one
// 8-byte load each, so a wavefront's loads are 512 contiguous bytes.
template <int NQ>
__global__ __launch_bounds__(kScanThreads) void retrieve_scores(const uint16_t *db, long long N, int d, const float *queries,
                                                               float *scores, long long ld_scores) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float *qs = reinterpret_cast<float *>(smem);          // [NQ][d]
  const int tid = threadIdx.x, lane = tid & 63;
  for (int i = tid * 4; i < NQ * d; i += kScanThreads * 4)
    *reinterpret_cast<float4 *>(qs + i) = *reinterpret_cast<const float4 *>(queries + i);
  __syncthreads();
  const long long waves = (long long)gridDim.x * (kScanThreads / 64);
  const long long gw = (long long)blockIdx.x * (kScanThreads / 64) + (tid >> 6);
  const int steps = (d + 255) / 256;
  for (long long pr = gw; 2 * pr < N; pr += waves) {
    const long long r0 = 2 * pr, r1 = min(2 * pr + 1, N - 1);       // an odd tail computes its last row twice
    const uint16_t *p0 = db + r0 * d, *p1 = db + r1 * d;
    float acc0[NQ], acc1[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) acc0[q] = acc1[q] = 0.f;
#pragma unroll 4
    for (int t = 0; t < steps; ++t) {
      const int c = t * 256 + lane * 4;
      if (c < d) {
        const uint2 a = *reinterpret_cast<const uint2 *>(p0 + c);
        const uint2 b = *reinterpret_cast<const uint2 *>(p1 + c);
        const float a0 = __uint_as_float(a.x << 16), a1 = __uint_as_float(a.x & 0xFFFF0000u);
        const float a2 = __uint_as_float(a.y << 16), a3 = __uint_as_float(a.y & 0xFFFF0000u);
        const float b0 = __uint_as_float(b.x << 16), b1 = __uint_as_float(b.x & 0xFFFF0000u);
        const float b2 = __uint_as_float(b.y << 16), b3 = __uint_as_float(b.y & 0xFFFF0000u);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
          const float4 w = *reinterpret_cast<const float4 *>(qs + q * d + c);
          acc0[q] = fmaf(a0, w.x, fmaf(a1, w.y, fmaf(a2, w.z, fmaf(a3, w.w, acc0[q]))));
          acc1[q] = fmaf(b0, w.x, fmaf(b1, w.y, fmaf(b2, w.z, fmaf(b3, w.w, acc1[q]))));
        }
      }
    }
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const float s0 = wave_sum(acc0[q]), s1 = wave_sum(acc1[q]);
      if (lane == 0) {
        scores[q * ld_scores + r0] = s0;
        scores[q * ld_scores + r1] = s1;
      }
    }
  }
}

// (value, index) order of the search: higher value first, equal values by lower index; NaN last.
__device__ __forceinline__ bool top_before(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

// The K best of `n` (value, index) pairs (in LDS or in global memory), by K rounds of a workgroup-wide arg-max; the
// winner of a round is taken out.  Results to out_val/out_idx [K] (index -1, value -inf when fewer
// than K pairs exist).  All 256 threads call this.
__device__ __forceinline__ void top_select(float *val, const int *idx, int n, int K, float *out_val, int *out_idx,
                                           float *red_v, int *red_i, int *red_p) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int k = 0; k < K; ++k) {
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF, bp = -1;
    for (int p = tid; p < n; p += 256) {
      const float v = val[p];
      const int i = idx ? idx[p] : p;
      if (i >= 0 && (top_before(v, i, bv, bi) || (bp < 0 && v == -INFINITY))) { bv = v; bi = i; bp = p; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(bv, o, kWave);
      const int oi = __shfl_xor(bi, o, kWave), op = __shfl_xor(bp, o, kWave);
      if (op >= 0 && (bp < 0 || top_before(ov, oi, bv, bi))) { bv = ov; bi = oi; bp = op; }
    }
    if (lane == 0) { red_v[wave] = bv; red_i[wave] = bi; red_p[wave] = bp; }
    __syncthreads();
    if (tid == 0) {
      for (int w = 1; w < 4; ++w)
        if (red_p[w] >= 0 && (red_p[0] < 0 || top_before(red_v[w], red_i[w], red_v[0], red_i[0]))) {
          red_v[0] = red_v[w]; red_i[0] = red_i[w]; red_p[0] = red_p[w];
        }
      if (red_p[0] >= 0) {
        out_val[k] = red_v[0];
        out_idx[k] = red_i[0];
        val[red_p[0]] = -INFINITY;
        // taken out: an index of -1 can never be chosen again
        if (idx) const_cast<int *>(idx)[red_p[0]] = -1;
      } else {
        out_val[k] = -INFINITY;
        out_idx[k] = -1;
      }
    }
    __syncthreads();
  }
}

// First round: one workgroup per chunk of kTopChunk scores of one query.
__global__ __launch_bounds__(256) void retrieve_top_chunks(const float *scores, long long ld_scores, long long N, int K,
                                                          float *cand_val, int *cand_idx, int n_chunks) {
  __shared__ float val[kTopChunk];
  __shared__ int idx[kTopChunk];
  __shared__ float red_v[4];
  __shared__ int red_i[4], red_p[4];
  const int chunk = blockIdx.x, q = blockIdx.y, tid = threadIdx.x;
  const long long base = (long long)chunk * kTopChunk;
  const int n = (int)min((long long)kTopChunk, N - base);
  for (int p = tid; p < n; p += 256) {
    float v = scores[q * ld_scores + base + p];
    if (v != v) v = -INFINITY;
    val[p] = v;
    idx[p] = (int)(base + p);
  }
  __syncthreads();
  top_select(val, idx, n, K, cand_val + ((size_t)q * n_chunks + chunk) * K, cand_idx + ((size_t)q * n_chunks + chunk) * K,
             red_v, red_i, red_p);
}

// Second round: one workgroup per query over the chunk winners; also fetches the winners' payload rows.
__global__ __launch_bounds__(256) void retrieve_top_merge(float *cand_val, int *cand_idx, int n_cand, int K, float *top_val,
                                                         int *top_idx, const int32_t *payload, int payload_len,
                                                         int32_t *top_payload) {
  __shared__ float red_v[4];
  __shared__ int red_i[4], red_p[4];
  const int q = blockIdx.x, tid = threadIdx.x;
  top_select(cand_val + (size_t)q * n_cand, cand_idx + (size_t)q * n_cand, n_cand, K, top_val + (size_t)q * K,
             top_idx + (size_t)q * K, red_v, red_i, red_p);
  if (payload && top_payload) {
    __threadfence_block();
    __syncthreads();
    for (int e = tid; e < K * payload_len; e += 256) {
      const int i = top_idx[(size_t)q * K + e / payload_len];
      top_payload[(size_t)q * K * payload_len + e] = i >= 0 ? payload[(size_t)i * payload_len + e % payload_len] : -1;
    }
  }
}

}  // namespace heisd
