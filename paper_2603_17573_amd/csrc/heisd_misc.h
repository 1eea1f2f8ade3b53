// Small kernels around the decoder: embedding gather, greedy choice over the action bins
// and the sequence-wise relaxed acceptance scan.
#pragma once
#include "heisd_common.h"

namespace heisd {

// x[m][:] = E[clamp(id[m])][:]  (token embeddings e_t of Eq. 2-2), bf16 -> fp32.
__global__ __launch_bounds__(256) void embed_rows(const int32_t *ids, const uint16_t *emb, int vocab,
                                                 int d, float *x) {
  const int m = blockIdx.x;
  int id = ids[m];
  id = max(0, min(id, vocab - 1));
  const uint16_t *src = emb + (size_t)id * d;
  for (int k = threadIdx.x * 8; k < d; k += 256 * 8) {
    const uint4 v = *reinterpret_cast<const uint4 *>(src + k);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float4 lo4, hi4;
    lo4.x = __uint_as_float(w[0] << 16); lo4.y = __uint_as_float(w[0] & 0xFFFF0000u);
    lo4.z = __uint_as_float(w[1] << 16); lo4.w = __uint_as_float(w[1] & 0xFFFF0000u);
    hi4.x = __uint_as_float(w[2] << 16); hi4.y = __uint_as_float(w[2] & 0xFFFF0000u);
    hi4.z = __uint_as_float(w[3] << 16); hi4.w = __uint_as_float(w[3] & 0xFFFF0000u);
    *reinterpret_cast<float4 *>(x + (size_t)m * d + k) = lo4;
    *reinterpret_cast<float4 *>(x + (size_t)m * d + k + 4) = hi4;
  }
}

struct AcceptArgs {
  const float *logits;        // [batch][K][n_bins] (read; rows of skipped episodes are set to NaN)
  float *logits_rw;           // same buffer, writable
  const int32_t *draft;       // [batch][K] vocabulary ids
  const int32_t *first_pred;  // [batch]
  const uint8_t *skip;        // [batch] or nullptr
  int32_t *accepted_len;      // [batch]
  int32_t *next_token;        // [batch]
  int32_t *target_bins;       // [batch][K+1]
  int K, n_bins, bin_base;
  int tok_threshold, seq_budget, n_groups, mode;
  int group_sizes[8];
  unsigned exact_mask;
};

// One workgroup per episode.  Greedy bin per position (Eq. 2-1: argmax; lowest index on
// ties, NaN never wins), then the acceptance rule of Sec. 4.2 walked group by group.
// Integer work: bit-exact by construction.
__global__ __launch_bounds__(256) void argmax_accept(AcceptArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = a.K;
  int32_t *tb = a.target_bins + (size_t)b * (K + 1);
  if (a.skip && a.skip[b]) {
    for (int i = tid; i < K * a.n_bins; i += 256) a.logits_rw[(size_t)b * K * a.n_bins + i] = __uint_as_float(0x7FC00000u);
    for (int j = tid; j <= K; j += 256) tb[j] = -1;
    if (tid == 0) {
      a.accepted_len[b] = K;   // an unverified draft is executed as is
      a.next_token[b] = -1;
    }
    return;
  }
  if (tid == 0) tb[0] = a.first_pred[b];
  // one wave per row: lanes stride over the bins, butterfly arg-max (lowest index wins ties)
  for (int j = wave; j < K; j += 4) {
    const float *row = a.logits + ((size_t)b * K + j) * a.n_bins;
    float best = -INFINITY;
    int bi = 0x7FFFFFFF;
    for (int t = lane; t < a.n_bins; t += kWave) {
      float v = row[t];
      if (v != v) v = -INFINITY;
      if (v > best || (v == best && t < bi)) { best = v; bi = t; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(best, o, kWave);
      const int oi = __shfl_xor(bi, o, kWave);
      if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
    }
    if (lane == 0) tb[j + 1] = (bi == 0x7FFFFFFF) ? 0 : bi;
  }
  __threadfence_block();
  __syncthreads();          // thread 0 reads the rows' bins back from tb below
  if (tid != 0) return;
  // ---- acceptance: leading run of accepted groups ----
  const int32_t *dr = a.draft + (size_t)b * K;
  int n = 0;
  if (a.mode == 0) {
    int j = 0, g = 0;
    while (j < K) {
      const int gi = g % a.n_groups;
      const int e = min(j + a.group_sizes[gi], K);
      const bool exact = (a.exact_mask >> gi) & 1u;
      bool ok = true;
      long long sum = 0;
      for (int i = j; i < e; ++i) {
        const int dbin = dr[i] - a.bin_base;
        const long long bias = (dbin >= 0 && dbin < a.n_bins) ? (long long)abs(dbin - tb[i]) : 0x7FFFFFFFLL;
        if (exact) ok = ok && (bias == 0);
        else ok = ok && (bias <= a.tok_threshold);
        sum += bias;
      }
      if (!exact) ok = ok && (sum <= a.seq_budget);
      if (!ok) break;
      n = e;
      j = e;
      ++g;
    }
  } else {
    int j = 0, g = 0;
    long long run = 0;
    bool stop = false;
    while (j < K && !stop) {
      const int gi = g % a.n_groups;
      const int e = min(j + a.group_sizes[gi], K);
      const bool exact = (a.exact_mask >> gi) & 1u;
      for (int i = j; i < e; ++i) {
        const int dbin = dr[i] - a.bin_base;
        const long long bias = (dbin >= 0 && dbin < a.n_bins) ? (long long)abs(dbin - tb[i]) : 0x7FFFFFFFLL;
        run += bias;
        if ((exact && bias != 0) || bias > a.tok_threshold || run > a.seq_budget) { stop = true; break; }
        n = i + 1;
      }
      j = e;
      ++g;
    }
  }
  a.accepted_len[b] = n;
  a.next_token[b] = a.bin_base + tb[n];
}

}  // namespace heisd
