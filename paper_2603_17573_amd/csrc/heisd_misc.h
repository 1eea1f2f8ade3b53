// Small kernels around the decoder: embedding gather, greedy choice over the action bins
// and the sequence-wise relaxed acceptance scan.
#pragma once
#include "heisd_common.h"
#include "heisd_fast.h"

namespace heisd {

// x[m][:] = E[clamp(id[m])][:]  (token embeddings e_t of Eq. 2-2), bf16 -> fp32.
// With `rows` (fp32 [M][d]) a row whose id is negative is copied from there instead.
__global__ __launch_bounds__(256) void embed_rows(const int32_t *ids, const uint16_t *emb, int vocab,
                                                 int d, float *x, const float *rows = nullptr) {
  const int m = blockIdx.x;
  int id = ids[m];
  if (rows && id < 0) {                               // uniform over the workgroup
    for (int k = threadIdx.x * 4; k < d; k += 256 * 4)
      *reinterpret_cast<float4 *>(x + (size_t)m * d + k) = *reinterpret_cast<const float4 *>(rows + (size_t)m * d + k);
    return;
  }
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
  const int32_t *prefix_len;  // [batch]: an episode whose K new rows do not fit its cache was left unverified
  int cap;
  unsigned *err;              // device error word (kErrOverflow is raised for such an episode)
};

// Episode b, by one workgroup of NT threads (all of them call this; it holds a workgroup barrier).
// Greedy bin per position (Eq. 2-1: argmax; lowest index on ties, NaN never wins), then the
// acceptance rule of Sec. 4.2 walked group by group.  Integer work: bit-exact by construction.
template <int NT>
__device__ __forceinline__ void accept_episode(const AcceptArgs &a, int b, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  const int K = a.K;
  int32_t *tb = a.target_bins + (size_t)b * (K + 1);
  const bool overflow = episode_overflows(a.prefix_len, b, K, a.cap);
  if (overflow || (a.skip && a.skip[b])) {
    for (int i = tid; i < K * a.n_bins; i += NT) a.logits_rw[(size_t)b * K * a.n_bins + i] = __uint_as_float(0x7FC00000u);
    for (int j = tid; j <= K; j += NT) tb[j] = -1;
    if (tid == 0) {
      a.accepted_len[b] = overflow ? -1 : K;   // an unverified draft is executed as is; no room in the cache: an error
      a.next_token[b] = -1;
      if (overflow) atomicOr(a.err, kErrOverflow);
    }
    return;
  }
  if (tid == 0) tb[0] = a.first_pred[b];
  // one wave per row: lanes stride over the bins, butterfly arg-max (lowest index wins ties)
  for (int j = wave; j < K; j += NT / 64) {
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

// One workgroup per episode.
__global__ __launch_bounds__(256) void argmax_accept(AcceptArgs a) { accept_episode<256>(a, blockIdx.x, threadIdx.x); }

// The LM-head slice of the <= 8-row kernels with the greedy bins and the acceptance scan in the same
// launch: the workgroup that finishes its logit tiles last (a wrapping device-scope counter tells it)
// judges every episode (K4/K5 in one launch with the GEMM).  The logits are written with device-scope stores and each workgroup waits for
// its own before it counts itself, so the last one reads complete rows.
__global__ __launch_bounds__(kFastThreads) void fast_lmhead_accept_kernel(FastGemm g, AcceptArgs a, int batch,
                                                                          unsigned *done_counter) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int s_last;
  Frag16 A;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  fast_issue16(A, g, blockIdx.x, gridDim.x, 0, wave, lane & 15, lane >> 4);
  fast_gemm_phase(g, blockIdx.x, gridDim.x, smem, A, true);
  __builtin_amdgcn_s_waitcnt(0);                       // this wave's logit stores have reached memory
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned old = atomicInc(done_counter, gridDim.x - 1);      // wraps to 0 with the last arrival: no reset
    s_last = old == gridDim.x - 1 ? 1 : 0;
  }
  __syncthreads();
  if (!s_last) return;
  for (int b = 0; b < batch; ++b) accept_episode<kFastThreads>(a, b, threadIdx.x);
}

// Greedy bin after the LAST of the n new rows of every episode (Eq. 2-1: the target's own next token),
// and optionally that row's logits.  One wave per episode.
// An episode whose n new rows did not fit its cache was left out by the attention kernels: its
// prediction is -1, its logits NaN, and the error word is raised.
__global__ __launch_bounds__(64) void last_row_argmax(const float *logits, int n, int n_bins, int32_t *pred,
                                                      float *last_logits, const int32_t *prefix_len, int cap,
                                                      unsigned *err) {
  const int b = blockIdx.x, lane = threadIdx.x;
  if (episode_overflows(prefix_len, b, n, cap)) {
    if (last_logits)
      for (int t = lane; t < n_bins; t += kWave) last_logits[(size_t)b * n_bins + t] = __uint_as_float(0x7FC00000u);
    if (lane == 0) {
      pred[b] = -1;
      atomicOr(err, kErrOverflow);
    }
    return;
  }
  const float *row = logits + ((size_t)b * n + (n - 1)) * n_bins;
  float best = -INFINITY;
  int bi = 0x7FFFFFFF;
  for (int t = lane; t < n_bins; t += kWave) {
    float v = row[t];
    if (last_logits) last_logits[(size_t)b * n_bins + t] = v;
    if (v != v) v = -INFINITY;
    if (v > best || (v == best && t < bi)) { best = v; bi = t; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, kWave);
    const int oi = __shfl_xor(bi, o, kWave);
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
  }
  if (lane == 0) pred[b] = (bi == 0x7FFFFFFF) ? 0 : bi;
}

// ---- tree verification (Sec. 4.2: a sequence-wise draft tree, every chain checked from the root) ----

constexpr int kTreeMax = 256;    // tree tokens per episode (four 64-bit words of visibility bits)

// depth[b][t]: tokens between the prefix and token t; anc[b][t][4]: bit u set iff token u is t or one
// of its ancestors.  A token whose chain does not reach the prefix through parent indices in [-1, own
// index) is padding: depth 0, sees only itself.  One thread per token; the walk ends because the index
// strictly decreases.
__global__ __launch_bounds__(kTreeMax) void tree_setup(const int32_t *parent, int T, int32_t *depth,
                                                      unsigned long long *anc) {
  const int b = blockIdx.x, t = threadIdx.x;
  if (t >= T) return;
  const int32_t *par = parent + (size_t)b * T;
  unsigned long long w[4] = {0, 0, 0, 0};
  auto set_bit = [&](int u) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] |= ((u >> 6) == i) ? (1ull << (u & 63)) : 0ull;
  };
  int dep = 0, cur = t;
  bool ok = true;
  for (;;) {
    const int p = par[cur];
    if (p == -1) break;
    if (p < 0 || p >= cur) { ok = false; break; }
    set_bit(p);
    ++dep;
    cur = p;
  }
  if (!ok) {
    dep = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = 0;
  }
  set_bit(t);
  depth[(size_t)b * T + t] = dep;
#pragma unroll
  for (int i = 0; i < 4; ++i) anc[((size_t)b * T + t) * 4 + i] = w[i];
}

struct TreeAcceptArgs {
  const float *logits;        // [batch][T][n_bins]
  float *logits_rw;
  const int32_t *tokens;      // [batch][T] vocabulary ids
  const int32_t *parent;      // [batch][T]
  const int32_t *first_pred;  // [batch]
  const uint8_t *skip;        // [batch] or nullptr
  int32_t *accepted_len;      // [batch]
  int32_t *next_token;        // [batch]
  int32_t *path;              // [batch][T]
  int32_t *target_bins;       // [batch][T+1]
  int T, n_bins, bin_base;
  int tok_threshold, seq_budget, n_groups, mode;
  int group_sizes[8];
  unsigned exact_mask;
  const int32_t *prefix_len;  // as in AcceptArgs
  int cap;
  unsigned *err;
};

// One workgroup per episode, thread t for tree token t.  Greedy bin after every tree token, then the
// chain selection level by level (all tokens of one depth at once; a parent is one level up): each
// token extends the state of its parent - the running max and sum of the sequence it is in, and
// whether everything before that sequence was accepted - so that for every point where a chain may
// stop (the end of a sequence, or a leaf) it is known whether the chain is accepted up to there.  The
// deepest such point wins, among equals the lowest token index.  Integer work: bit-exact by
// construction.
__global__ __launch_bounds__(256) void tree_accept(TreeAcceptArgs a) {
  __shared__ int32_t s_par[kTreeMax], s_pred[kTreeMax], s_depth[kTreeMax], s_gmax[kTreeMax], s_child[kTreeMax];
  __shared__ long long s_gsum[kTreeMax];
  __shared__ unsigned char s_valid[kTreeMax], s_alive[kTreeMax], s_end[kTreeMax];
  __shared__ unsigned char s_gi[kTreeMax], s_first[kTreeMax], s_last[kTreeMax];    // by depth
  __shared__ int s_maxd;
  __shared__ unsigned s_best;                                                      // (n << 16) | (0xFFFF - t)
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int T = a.T;
  int32_t *tb = a.target_bins + (size_t)b * (T + 1);
  int32_t *path = a.path + (size_t)b * T;
  const int32_t *par = a.parent + (size_t)b * T;
  const bool overflow = episode_overflows(a.prefix_len, b, T, a.cap);
  const bool skipped = overflow || (a.skip && a.skip[b]);
  if (tid < T) {
    s_par[tid] = par[tid];
    s_child[tid] = 0x7FFFFFFF;       // lowest-index child
  }
  if (tid == 0) {
    s_maxd = 0;
    s_best = 0;
    // the sequence pattern by depth
    int dpt = 0, g = 0;
    while (dpt < T) {
      const int gi = g % a.n_groups, size = a.group_sizes[gi];
      for (int i = 0; i < size && dpt < T; ++i, ++dpt) {
        s_gi[dpt] = (unsigned char)gi;
        s_first[dpt] = i == 0;
        s_last[dpt] = i == size - 1;
      }
      ++g;
    }
  }
  __syncthreads();
  // which tokens are in the tree, and how deep: walk up (the index strictly decreases)
  int my_depth = 0;
  bool my_valid = false;
  if (tid < T) {
    int cur = tid, dep = 0;
    bool ok = true;
    for (;;) {
      const int p = s_par[cur];
      if (p == -1) break;
      if (p < 0 || p >= cur) { ok = false; break; }
      ++dep;
      cur = p;
    }
    my_valid = ok;
    my_depth = ok ? dep : 0;
    s_valid[tid] = ok;
    s_depth[tid] = my_depth;
    if (ok) {
      atomicMax(&s_maxd, dep);
      if (s_par[tid] >= 0) atomicMin(&s_child[s_par[tid]], tid);
    }
  }
  if (skipped) {
    for (int i = tid; i < T * a.n_bins; i += 256) a.logits_rw[(size_t)b * T * a.n_bins + i] = __uint_as_float(0x7FC00000u);
    for (int j = tid; j <= T; j += 256) tb[j] = -1;
    for (int j = tid; j < T; j += 256) path[j] = -1;
    __syncthreads();
    if (tid == 0) {
      // an unverified draft is executed as is: the first chain
      int n = 0;
      if (s_valid[0] && s_par[0] == -1) {
        int cur = 0;
        for (;;) {
          path[n++] = cur;
          const int c = s_child[cur];
          if (c == 0x7FFFFFFF) break;
          cur = c;
        }
      }
      a.accepted_len[b] = overflow ? -1 : n;
      a.next_token[b] = -1;
      if (overflow) {
        for (int j = 0; j < n; ++j) path[j] = -1;
        atomicOr(a.err, kErrOverflow);
      }
    }
    return;
  }
  // greedy bin after every token: one wave per row, lowest index wins ties, NaN never wins.  A wave takes
  // kRows rows at a time and requests a slice of all of them before it compares anything: one row at a time
  // is one memory round trip per row (76 rows: 19 per wave, 38 of the kernel's 48 us).
  constexpr int kRows = 8;
  for (int j0 = wave * kRows; j0 < T; j0 += 4 * kRows) {
    float best[kRows];
    int bi[kRows];
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      best[u] = -INFINITY;
      bi[u] = 0x7FFFFFFF;
    }
    for (int t = lane; t < a.n_bins; t += kWave) {
      float v[kRows];
#pragma unroll
      for (int u = 0; u < kRows; ++u)
        v[u] = a.logits[((size_t)b * T + min(j0 + u, T - 1)) * a.n_bins + t];
#pragma unroll
      for (int u = 0; u < kRows; ++u) {
        float x = v[u];
        if (x != x) x = -INFINITY;
        if (x > best[u] || (x == best[u] && t < bi[u])) { best[u] = x; bi[u] = t; }
      }
    }
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best[u], o, kWave);
        const int oi = __shfl_xor(bi[u], o, kWave);
        if (ov > best[u] || (ov == best[u] && oi < bi[u])) { best[u] = ov; bi[u] = oi; }
      }
      if (lane == 0 && j0 + u < T) s_pred[j0 + u] = (bi[u] == 0x7FFFFFFF) ? 0 : bi[u];
    }
  }
  __syncthreads();
  const int fp = a.first_pred[b];
  if (tid < T) {
    tb[tid + 1] = my_valid ? s_pred[tid] : -1;
    path[tid] = -1;
  }
  if (tid == 0) tb[0] = fp;
  // this token's own bias
  long long bias = 0;
  bool exact = false, leaf = false;
  int p = -1;
  if (tid < T && my_valid) {
    p = s_par[tid];
    const int dbin = a.tokens[(size_t)b * T + tid] - a.bin_base;
    const int target = p < 0 ? fp : s_pred[p];
    bias = (dbin >= 0 && dbin < a.n_bins) ? (long long)abs(dbin - target) : 0x7FFFFFFFLL;
    exact = (a.exact_mask >> s_gi[my_depth]) & 1u;
    leaf = s_child[tid] == 0x7FFFFFFF;
  }
  const int maxd = s_maxd;
  for (int lvl = 0; lvl <= maxd; ++lvl) {           // uniform trip count
    if (tid < T && my_valid && my_depth == lvl) {
      unsigned cand = 0;
      if (a.mode == 0) {
        const bool first = s_first[lvl];
        // everything before this token's sequence accepted?
        const bool alive = first ? (p < 0 || s_end[p]) : s_alive[p];
        const long long gsum = (first ? 0 : s_gsum[p]) + bias;
        const long long gmax = first ? bias : (bias > s_gmax[p] ? bias : (long long)s_gmax[p]);
        s_alive[tid] = alive;
        s_gsum[tid] = gsum;
        s_gmax[tid] = (int32_t)gmax;
        const bool pass = exact ? gmax == 0 : (gmax <= a.tok_threshold && gsum <= a.seq_budget);
        const bool stop_ok = alive && pass && (s_last[lvl] || leaf);
        s_end[tid] = stop_ok;
        if (stop_ok) cand = ((unsigned)(lvl + 1) << 16) | (unsigned)(0xFFFF - tid);
      } else {
        const long long run = (p < 0 ? 0 : s_gsum[p]) + bias;
        const bool alive = (p < 0 || s_alive[p]) && !(exact && bias != 0) && bias <= a.tok_threshold &&
                           run <= a.seq_budget;
        s_gsum[tid] = run;
        s_alive[tid] = alive;
        if (alive) cand = ((unsigned)(lvl + 1) << 16) | (unsigned)(0xFFFF - tid);
      }
      if (cand) atomicMax(&s_best, cand);
    }
    __syncthreads();
  }
  if (tid != 0) return;
  const unsigned best = s_best;
  const int best_n = (int)(best >> 16), best_t = best ? 0xFFFF - (int)(best & 0xFFFFu) : -1;
  a.accepted_len[b] = best_n;
  a.next_token[b] = a.bin_base + (best_t < 0 ? fp : s_pred[best_t]);
  for (int cur = best_t, j = best_n - 1; j >= 0; --j) {
    path[j] = cur;
    cur = s_par[cur];
  }
}

struct TreeCompactArgs {
  uint16_t *k_cache, *v_cache;   // bf16 [L][batch][H][cap][HD]
  const int32_t *prefix_len;     // [batch]
  const uint8_t *skip;           // [batch] or nullptr
  const int32_t *accepted_len;   // [batch]
  const int32_t *path;           // [batch][T]
  int T, H, cap, HD, batch;
};

// After the selection: the key/value rows of the n accepted tokens (written at prefix_len + token
// index by the attention kernel) move to rows prefix_len .. prefix_len + n - 1.  One workgroup per
// (head, episode, layer).  path[j] >= j and strictly increasing, so a chunk of rows is read whole,
// then written: a source row is never overwritten before it is read.
__global__ __launch_bounds__(256) void tree_compact(TreeCompactArgs a) {
  const int h = blockIdx.x, b = blockIdx.y, l = blockIdx.z, tid = threadIdx.x;
  if (episode_sits_out(a.skip, a.prefix_len, b, a.T, a.cap)) return;
  const int n = max(0, min(a.accepted_len[b], a.T));
  int P = a.prefix_len[b];
  P = max(0, min(P, a.cap - a.T));
  const int LPR = a.HD / 8, rows_per_pass = 256 / LPR;
  const size_t base = (((size_t)l * a.batch + b) * a.H + h) * (size_t)a.cap * a.HD;
  uint16_t *kc = a.k_cache + base, *vc = a.v_cache + base;
  const int32_t *path = a.path + (size_t)b * a.T;
  const int li = tid % LPR, rj = tid / LPR;
  for (int j0 = 0; j0 < n; j0 += rows_per_pass) {      // n is the same for the whole workgroup
    const int j = j0 + rj;
    uint4 kk = make_uint4(0, 0, 0, 0), vv = kk;
    int src = -1;
    if (j < n) {
      src = path[j];
      if (src != j && src >= 0 && src < a.T) {
        kk = *reinterpret_cast<const uint4 *>(kc + (size_t)(P + src) * a.HD + li * 8);
        vv = *reinterpret_cast<const uint4 *>(vc + (size_t)(P + src) * a.HD + li * 8);
      } else {
        src = -1;
      }
    }
    __syncthreads();
    if (src >= 0) {
      *reinterpret_cast<uint4 *>(kc + (size_t)(P + j) * a.HD + li * 8) = kk;
      *reinterpret_cast<uint4 *>(vc + (size_t)(P + j) * a.HD + li * 8) = vv;
    }
    __syncthreads();
  }
}

}  // namespace heisd
