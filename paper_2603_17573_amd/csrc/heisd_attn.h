// Verify attention with fused RoPE and KV-append (paper Sec. 2.2: the target scores all K
// drafts in one pass; App. A.2: causal attention over visual, text and earlier action
// tokens).  One workgroup per (episode, head).
//
//   1. rotate this head's new keys (rotate-half, absolute position prefix_len + j), round
//      keys and values to bf16 and append them to the episode's cache rows; the rotated keys
//      are also kept in fp32 (in place, in the projection scratch) so that the block attends
//      to its own rows at full precision and only the prefix is read as bf16;
//   2. per block of 8 queries: scores of every visible key into LDS (each key row is read
//      once, 16 bytes per lane, and dotted with all 8 queries; partial dots are summed with
//      wavefront shuffles), softmax per query with wavefront reductions, then one pass over
//      the value rows accumulating all 8 outputs.
// Skipped episodes (verify-skip, Sec. 4.1) touch neither the cache nor the scores.
//
// Tree verification (Sec. 4.2: chains of a sequence-wise draft tree are checked in one pass):
// with `depth` and `anc` given, new row j sits at position prefix_len + depth[j] and sees, among
// the new rows, exactly those whose bit is set in its 256-bit ancestor mask (itself included).
// Its key and value still go to cache row prefix_len + j.
#pragma once
#include "heisd_common.h"

namespace heisd {

constexpr int kAttnQB = 8;  // queries per block
constexpr int kAttnU = 6;   // cache rows a value stream requests at once

__device__ __forceinline__ void attn_unpack8(const uint4 v, float (&f)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(w[i] << 16);
    f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}

struct AttnArgs {
  float *qkv;                // [M][3*d] fp32: q | k | v of the new rows, not yet rotated; k is rotated in place
  uint16_t *k_cache;         // this layer: bf16 [batch][H][cap][HD]
  uint16_t *v_cache;
  const int32_t *prefix_len; // [batch]
  const uint8_t *skip;       // [batch] or nullptr
  const float2 *rope;        // [cap][HD/2] (cos, sin) of position * theta_i
  float *out;                // [M][d] fp32 rows, or nullptr
  uint16_t *o_planes;        // or: records [d/16][CTS][16][16] bf16 (head rows 0-7, tail rows 8-15 of each
  int CTS;                   //     column tile of 8 activation rows), the B-operand format of the GEMMs
  int single;                // records hold ONE bf16 per value: 16 activation rows per column tile (see BatGemm::single)
  int K, H, cap, d;
  float scale;               // 1/sqrt(HD)
  const int32_t *depth;              // tree mode: [batch][K] tokens between the prefix and row j; else nullptr
  const unsigned long long *anc;     // tree mode: [batch][K][4] visibility bits over the K new rows
};

// waves: 4 or 8 (workgroups of 256 or 512 threads)
inline size_t attn_lds_bytes(int hd, int cap, int waves) {
  return sizeof(float) * ((size_t)kAttnQB * hd + (size_t)kAttnQB * cap + kAttnQB + (size_t)waves * kAttnQB * hd) +
         kAttnQB * 4 * sizeof(unsigned long long);   // tree mode: visibility bits of the block's queries
}

// Attention output element (row m, column col).
__device__ __forceinline__ void attn_store(const AttnArgs &a, int m, int col, float v) {
  if (a.out) a.out[(size_t)m * a.d + col] = v;
  if (a.o_planes) {
    uint32_t hi, lo;
    split_bf16(v, hi, lo);
    if (a.single) {
      a.o_planes[((size_t)(col >> 4) * a.CTS + (m >> 4)) * 256 + (m & 15) * 16 + (col & 15)] = (uint16_t)hi;
      return;
    }
    uint16_t *rec = a.o_planes + ((size_t)(col >> 4) * a.CTS + (m >> 3)) * 256 + (m & 7) * 16 + (col & 15);
    rec[0] = (uint16_t)hi;
    rec[128] = (uint16_t)lo;
  }
}

// RoPE on the new keys of (episode b, head h), in place in fp32, and the append of keys and values
// (bf16) to the episode's cache rows P .. P+K-1.
template <int HD, bool TREE>
__device__ __forceinline__ void attn_append_rows(const AttnArgs &a, int b, int h, int P, int tid, int nthreads,
                                                 int jb, int je) {
  constexpr int HALF = HD / 2;
  const int K = a.K, d = a.d, row0 = b * K;
  uint16_t *kc = a.k_cache + ((size_t)(b * a.H + h) * a.cap) * HD;
  uint16_t *vc = a.v_cache + ((size_t)(b * a.H + h) * a.cap) * HD;
  for (int idx = tid + jb * HALF; idx < je * HALF; idx += nthreads) {
    const int j = idx / HALF, i = idx - j * HALF;
    float *src = a.qkv + (size_t)(row0 + j) * 3 * d + h * HD;
    const float2 cs = a.rope[(size_t)(P + (TREE ? a.depth[row0 + j] : j)) * HALF + i];
    const float k1 = src[d + i], k2 = src[d + i + HALF];
    const float kr1 = k1 * cs.x - k2 * cs.y, kr2 = k2 * cs.x + k1 * cs.y;
    src[d + i] = kr1;
    src[d + i + HALF] = kr2;
    uint16_t *kr = kc + (size_t)(P + j) * HD;
    kr[i] = (uint16_t)f32_to_bf16_bits(kr1);
    kr[i + HALF] = (uint16_t)f32_to_bf16_bits(kr2);
    uint16_t *vr = vc + (size_t)(P + j) * HD;
    vr[i] = (uint16_t)f32_to_bf16_bits(src[2 * d + i]);
    vr[i + HALF] = (uint16_t)f32_to_bf16_bits(src[2 * d + i + HALF]);
  }
}

// The append alone, one workgroup per (head, episode, 8 new rows): first half of a step whose attention
// runs with one workgroup per block of 8 queries (attn_verify with SPLIT).
template <int HD, bool TREE>
__global__ __launch_bounds__(256) void attn_append(AttnArgs a) {
  const int h = blockIdx.x, b = blockIdx.y;
  if (episode_sits_out(a.skip, a.prefix_len, b, a.K, a.cap)) return;
  int P = a.prefix_len[b];
  P = max(0, min(P, a.cap - a.K));
  const int jb = (int)blockIdx.z * kAttnQB;
  attn_append_rows<HD, TREE>(a, b, h, P, threadIdx.x, 256, jb, min(a.K, jb + kAttnQB));
}

// THREADS: 256 or 512.  With few (episode, head) pairs - fewer workgroups than would fill the
// compute units twice - the larger workgroup hides more latency (M = 56: 31 -> 26 us per layer);
// with many pairs the smaller one is faster (M = 448: 131 against 167 us).
// TREE: tree mode compiled in (the linear kernel carries none of its registers).
// A workgroup serves one block of at most 8 queries of one (head, episode): blockIdx.z names the block.
// SPLIT = false: the episode has a single block and the workgroup also rotates and appends the new keys
// and values; SPLIT = true: several blocks per episode, the append ran as attn_append before.  With many
// queries per episode and few episodes the blocks are what fills the chip (76 tree tokens, one episode:
// 225 us per layer with one workgroup per head, 64 us with one per block).
template <int HD, int THREADS, bool TREE, bool SPLIT>
// The 256-thread single-block variant is held to 128 registers (four waves per SIMD: 108 -> 98 us per layer
// at 64 episodes); the same limit on the per-block variant measured slower (long prefixes: 72 -> 86 us).
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu((THREADS == 256 && !SPLIT) ? 4 : 2))) void attn_verify(AttnArgs a) {
  constexpr int kAttnThreads = THREADS, kAttnWaves = THREADS / 64;
  constexpr int HALF = HD / 2;
  constexpr int LPK = HD / 8;              // lanes that share one key row (16 bytes each)
  constexpr int G = kAttnThreads / LPK;    // key rows in flight per pass
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float *qs = reinterpret_cast<float *>(smem);        // [QB][HD]
  float *sc = qs + kAttnQB * HD;                       // [QB][cap]
  float *inv_l = sc + (size_t)kAttnQB * a.cap;         // [QB]
  float *ored = inv_l + kAttnQB;                       // [waves][QB][HD]
  unsigned long long *amask = reinterpret_cast<unsigned long long *>(ored + (size_t)kAttnWaves * kAttnQB * HD);   // [QB][4]

  const int h = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = a.K, d = a.d, cap = a.cap;
  const int row0 = b * K;
  const int jb = SPLIT ? (int)blockIdx.z * kAttnQB : 0, je = SPLIT ? min(K, jb + kAttnQB) : K;   // this workgroup's queries
  if (episode_sits_out(a.skip, a.prefix_len, b, K, cap)) {
    for (int idx = tid; idx < (je - jb) * HD; idx += kAttnThreads)
      attn_store(a, row0 + jb + idx / HD, h * HD + (idx % HD), 0.f);
    return;
  }
  int P = a.prefix_len[b];
  P = max(0, min(P, cap - K));  // never index past the cache, whatever the caller passed
  uint16_t *kc = a.k_cache + ((size_t)(b * a.H + h) * cap) * HD;
  uint16_t *vc = a.v_cache + ((size_t)(b * a.H + h) * cap) * HD;

  if (!SPLIT) {
    attn_append_rows<HD, TREE>(a, b, h, P, tid, kAttnThreads, 0, K);
    __syncthreads();  // the rotated fp32 keys are read back below by other waves of this workgroup
  }

  const int li = tid % LPK;   // which 8 channels of a row this lane covers
  const int g = tid / LPK;    // which key stream this lane belongs to
  {                       // one block of at most 8 queries per workgroup
    const int j0 = jb;
    const int nq = min(kAttnQB, K - j0);
    const int nkeys = P + j0 + nq;  // keys visible to the last query of the block
    for (int idx = tid; idx < kAttnQB * HALF; idx += kAttnThreads) {
      const int j = idx / HALF, i = idx - j * HALF;
      float r1 = 0.f, r2 = 0.f;
      if (j < nq) {
        const float *src = a.qkv + (size_t)(row0 + j0 + j) * 3 * d + h * HD;
        const float2 cs = a.rope[(size_t)(P + (TREE ? a.depth[row0 + j0 + j] : j0 + j)) * HALF + i];
        const float q1 = src[i], q2 = src[i + HALF];
        r1 = (q1 * cs.x - q2 * cs.y) * a.scale;
        r2 = (q2 * cs.x + q1 * cs.y) * a.scale;
      }
      qs[j * HD + i] = r1;
      qs[j * HD + i + HALF] = r2;
    }
    if (TREE && tid < kAttnQB * 4)
      amask[tid] = (tid >> 2) < nq ? a.anc[(size_t)(row0 + j0 + (tid >> 2)) * 4 + (tid & 3)] : 0ull;
    __syncthreads();
    float qf[kAttnQB][8];
#pragma unroll
    for (int j = 0; j < kAttnQB; ++j)
#pragma unroll
      for (int i = 0; i < 8; ++i) qf[j][i] = qs[j * HD + li * 8 + i];

    // is new row r - P visible to query j0 + li?  (tree mode: the bits were put in LDS with the queries)
    auto sees_new = [&](int r) __attribute__((always_inline)) {
      if (!TREE) return r <= P + j0 + li;
      const int t = r - P;
      return li < kAttnQB && ((amask[li * 4 + (t >> 6)] >> (t & 63)) & 1ull) != 0;
    };

    // ---- pass 1: scores ----
    auto score_key = [&](const float (&kf)[8], int r, bool vis) __attribute__((always_inline)) {
      float s[kAttnQB];
#pragma unroll
      for (int j = 0; j < kAttnQB; ++j) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) t = fmaf(qf[j][i], kf[i], t);
        s[j] = t;
      }
#pragma unroll
      for (int off = LPK / 2; off > 0; off >>= 1)
#pragma unroll
        for (int j = 0; j < kAttnQB; ++j) s[j] += __shfl_xor(s[j], off, kWave);
      float mine = s[0];
#pragma unroll
      for (int j = 1; j < kAttnQB; ++j) mine = (li == j) ? s[j] : mine;
      if (li < kAttnQB) sc[(size_t)li * cap + r] = vis ? mine : -INFINITY;
    };
    // prefix rows (bf16, from the cache) on the matrix cores: a tile of 16 keys is the A operand of
    // v_mfma_f32_16x16x32_bf16 straight from the cache (lane l: key l%16, 8 consecutive channels), the
    // block's queries are the B operand, each fp32 query as a bf16 head (columns 0-7) and a bf16 tail
    // (columns 8-15), kept in registers for the whole pass; lane l then holds the scores of keys
    // 4*(l/16)..+3 against column l%16, and head and tail columns are added with one exchange.  (With
    // plain FMAs every key cost 64 of them plus a 32-step butterfly over the 16 lanes that share a row.)
    {
      constexpr int KS = HD / 32;
      const int lr = lane & 15, lg = lane >> 4;
      typedef unsigned int attn_u32x4 __attribute__((ext_vector_type(4)));
      attn_u32x4 qb[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float x0 = qs[(lr & 7) * HD + ks * 32 + lg * 8 + 2 * i], x1 = qs[(lr & 7) * HD + ks * 32 + lg * 8 + 2 * i + 1];
          uint32_t h0, l0, h1, l1;
          split_bf16(x0, h0, l0);
          split_bf16(x1, h1, l1);
          w[i] = lr < 8 ? (h0 | (h1 << 16)) : (l0 | (l1 << 16));
        }
        qb[ks] = attn_u32x4{w[0], w[1], w[2], w[3]};
      }
      constexpr int TU = 2;                           // tiles a wave requests before it uses the first
      const int n_tiles = (P + 15) / 16;
      for (int t0 = wave; t0 < n_tiles; t0 += kAttnWaves * TU) {
        attn_u32x4 kf[TU][KS];
#pragma unroll
        for (int u = 0; u < TU; ++u) {
          const int r = min((t0 + u * kAttnWaves) * 16 + lr, P - 1);      // rows past the prefix repeat its last row
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            kf[u][ks] = *reinterpret_cast<const attn_u32x4 *>(kc + (size_t)r * HD + ks * 32 + lg * 8);
        }
#pragma unroll
        for (int u = 0; u < TU; ++u) {
          const int t = t0 + u * kAttnWaves;
          if (t < n_tiles) {                          // uniform over the wave
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
              acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[u][ks]), __builtin_bit_cast(bf16x8, qb[ks]),
                                                            acc, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float v = acc[i] + __shfl_xor(acc[i], 8, kWave);     // head column + tail column
              const int r = t * 16 + lg * 4 + i;
              if (lr < kAttnQB && r < P) sc[(size_t)lr * cap + r] = v;
            }
          }
        }
      }
    }
    // the block's own rows (fp32, rotated in place above)
    for (int r = P + g; r < nkeys; r += G) {
      const float *kp = a.qkv + (size_t)(row0 + r - P) * 3 * d + d + h * HD + li * 8;
      const float4 k0 = *reinterpret_cast<const float4 *>(kp), k1 = *reinterpret_cast<const float4 *>(kp + 4);
      const float kf[8] = {k0.x, k0.y, k0.z, k0.w, k1.x, k1.y, k1.z, k1.w};
      score_key(kf, r, sees_new(r));
    }
    __syncthreads();

    // ---- softmax per query: one wave per row, lanes stride over the keys ----
    for (int j = wave; j < nq; j += kAttnWaves) {
      float *row = sc + (size_t)j * cap;
      float mx = -INFINITY;
      for (int r = lane; r < nkeys; r += kWave) mx = fmaxf(mx, row[r]);
      mx = wave_max(mx);
      float sum = 0.f;
      for (int r = lane; r < nkeys; r += kWave) {
        const float p = expf(row[r] - mx);
        row[r] = p;
        sum += p;
      }
      sum = wave_sum(sum);
      if (lane == 0) inv_l[j] = 1.0f / sum;
    }
    __syncthreads();

    // ---- pass 2: weighted sum of the value rows ----
    float o[kAttnQB][8];
#pragma unroll
    for (int j = 0; j < kAttnQB; ++j)
#pragma unroll
      for (int i = 0; i < 8; ++i) o[j][i] = 0.f;
    auto add_value = [&](const float (&vf)[8], int r) __attribute__((always_inline)) {
#pragma unroll
      for (int j = 0; j < kAttnQB; ++j) {
        const float p = (j < nq) ? sc[(size_t)j * cap + r] : 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[j][i] = fmaf(p, vf[i], o[j][i]);
      }
    };
    for (int r0 = g; r0 < P; r0 += G * kAttnU) {
      uint4 vv[kAttnU];
#pragma unroll
      for (int u = 0; u < kAttnU; ++u) {
        const int r = r0 + u * G;
        vv[u] = r < P ? *reinterpret_cast<const uint4 *>(vc + (size_t)r * HD + li * 8) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < kAttnU; ++u) {
        const int r = r0 + u * G;
        if (r < P) {
          float vf[8];
          attn_unpack8(vv[u], vf);
          add_value(vf, r);
        }
      }
    }
    for (int r = P + g; r < nkeys; r += G) {
      const float *vp = a.qkv + (size_t)(row0 + r - P) * 3 * d + 2 * d + h * HD + li * 8;
      const float4 v0 = *reinterpret_cast<const float4 *>(vp), v1 = *reinterpret_cast<const float4 *>(vp + 4);
      const float vf[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
      add_value(vf, r);
    }
#pragma unroll
    for (int off = LPK; off < kWave; off <<= 1)
#pragma unroll
      for (int j = 0; j < kAttnQB; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) o[j][i] += __shfl_xor(o[j][i], off, kWave);
    if (lane < LPK) {
#pragma unroll
      for (int j = 0; j < kAttnQB; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) ored[(size_t)(wave * kAttnQB + j) * HD + lane * 8 + i] = o[j][i];
    }
    __syncthreads();
    for (int idx = tid; idx < nq * HD; idx += kAttnThreads) {
      const int j = idx / HD, c = idx - j * HD;
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < kAttnWaves; ++w) t += ored[(size_t)(w * kAttnQB + j) * HD + c];
      attn_store(a, row0 + j0 + j, h * HD + c, t * inv_l[j]);
    }
    __syncthreads();
  }
}

}  // namespace heisd
