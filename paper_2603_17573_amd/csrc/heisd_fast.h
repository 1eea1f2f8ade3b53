// Fast path of the verify forward for M = batch*K <= 8 rows (the headline case: one episode,
// K = 7 drafts; paper Sec. 2.2 "parallel verification" of one action slice).
//
// Activations travel between phases as two bf16 "planes" of 16 rows: rows 0-7 hold the bf16
// heads of the (up to) 8 activation rows, rows 8-15 the bf16 tails (x ~= head + tail).  A
// plane row is exactly one column of the MFMA B operand, so a consumer lane loads its B
// fragment with one 16-byte read and no conversion; the producer's epilogue does the split
// once per element.  RMSNorm is folded in: the planes hold x*g, the producer also emits the
// per-tile partial sums of squares, and the consumer multiplies its accumulators by 1/rms.
//
// A GEMM phase gives every workgroup a list of 16-row weight tiles over the whole reduction;
// its 8 waves split each 4096-wide k-chunk (16 k-steps of 32 per wave), keep the chunk's B
// fragments in registers, stream the weight tiles through two 16-tile register buffers, and are
// reduced through LDS in a fixed order.  The same phase bodies serve one-launch-per-phase and
// the persistent whole-step kernel.
#pragma once
#include "heisd_common.h"

namespace heisd {

constexpr int kFastThreads = 512;
constexpr int kFastWaves = 8;
constexpr int kKS = 16;                    // k-steps (of 32) per wave per chunk
constexpr int kChunkK = kFastWaves * kKS * 32;  // 4096
constexpr int kMaxT = 6;                   // weight tiles a workgroup accumulates at once

enum { FEPI_STORE = 0, FEPI_RESID_NORM = 1, FEPI_SWIGLU = 2 };

struct FastGemm {
  const uint16_t *w[3];   // weight segments, bf16 row-major [rows][Kd]
  int seg_tiles;          // n-tiles per segment
  int n_units;            // n-tiles, or (gate, up) pairs for FEPI_SWIGLU
  int Kd;
  const uint16_t *b;      // activation planes [16][Kd] bf16 (rows 0-7 heads, 8-15 tails)
  const float *ssq;       // [8][n_ssq] partial sums of squares of the un-normalised rows, or nullptr
  int n_ssq;
  float eps;
  int M;                  // valid rows (<= 8)
  // outputs
  float *out;             // FEPI_STORE: [M][ldo];  FEPI_RESID_NORM: residual stream x [M][ldo], updated in place
  int ldo;
  const float *next_gain; // FEPI_RESID_NORM: gain of the norm that consumes x next
  uint16_t *o_planes;     // FEPI_RESID_NORM / FEPI_SWIGLU: planes [16][ldo]
  float *ssq_out;         // FEPI_RESID_NORM: [8][n_units]
};

struct ABuf {
  uint4 v[kKS];
};

// Which weight tile is list entry `e` of workgroup `wg` (of `nwg`)?  Units are dealt round-robin.
template <int EPI>
__device__ __forceinline__ bool fast_tile(const FastGemm &g, int wg, int nwg, int e, const uint16_t *&wbase,
                                          int &wrow0, int &unit) {
  if (EPI == FEPI_SWIGLU) {
    unit = wg + (e >> 1) * nwg;
    wbase = (e & 1) ? g.w[1] : g.w[0];
    wrow0 = unit * 16;
    return unit < g.n_units;
  }
  unit = wg + e * nwg;
  const int u = unit < g.n_units ? unit : 0;
  const int seg = u / g.seg_tiles;
  wbase = seg == 0 ? g.w[0] : (seg == 1 ? g.w[1] : g.w[2]);
  wrow0 = (u - seg * g.seg_tiles) * 16;
  return unit < g.n_units;
}

// Request the weight fragments of tile entry e, k-chunk c for this wave.
template <int EPI>
__device__ __forceinline__ void fast_issue(ABuf &A, const FastGemm &g, int wg, int nwg, int e, int c, int wave,
                                           int lr, int lg) {
  const uint16_t *wbase;
  int wrow0, unit;
  const bool ok = fast_tile<EPI>(g, wg, nwg, e, wbase, wrow0, unit);
  const int k0 = c * kChunkK + wave * (kKS * 32) + lg * 8;
  const uint16_t *p = wbase + (size_t)(wrow0 + lr) * g.Kd + k0;
#pragma unroll
  for (int s = 0; s < kKS; ++s)
    A.v[s] = (ok && k0 + s * 32 + 8 <= g.Kd) ? *reinterpret_cast<const uint4 *>(p + s * 32) : make_uint4(0, 0, 0, 0);
}

// B fragments of k-chunk c for this wave: lane (lr, lg) reads plane row lr at its k offset.
__device__ __forceinline__ void fast_load_b(ABuf &Bf, const FastGemm &g, int c, int wave, int lr, int lg) {
  const int k0 = c * kChunkK + wave * (kKS * 32) + lg * 8;
  const uint16_t *p = g.b + (size_t)lr * g.Kd + k0;
#pragma unroll
  for (int s = 0; s < kKS; ++s)
    Bf.v[s] = (k0 + s * 32 + 8 <= g.Kd) ? *reinterpret_cast<const uint4 *>(p + s * 32) : make_uint4(0, 0, 0, 0);
}

__device__ __forceinline__ void fast_mma(f32x4 &acc, const ABuf &A, const ABuf &Bf) {
#pragma unroll
  for (int s = 0; s < kKS; ++s)
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A.v[s]), __builtin_bit_cast(bf16x8, Bf.v[s]),
                                                  acc, 0, 0, 0);
}

// LDS needed by a phase: reduction buffer + scales.
constexpr size_t kFastLds = (size_t)kFastWaves * kMaxT * 64 * 16 + 16 * sizeof(float);

// One GEMM phase for workgroup `wg` of `nwg`.  MAXC = number of k-chunks the shape needs.
// `A0` may already hold the fragments of (entry 0, chunk 0) when `pre` is true (requested by the
// caller before it waited for this phase's inputs).
template <int EPI, int MAXC>
__device__ __forceinline__ void fast_gemm_phase(const FastGemm &g, int wg, int nwg, unsigned char *smem, ABuf &A0,
                                                ABuf &A1, bool pre) {
  constexpr int MAXE = (MAXC == 1) ? kMaxT : 2;  // tile entries per pass
  float *red = reinterpret_cast<float *>(smem);
  float *scale_s = reinterpret_cast<float *>(smem + (size_t)kFastWaves * kMaxT * 64 * 16);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int unit_tiles = (EPI == FEPI_SWIGLU) ? 2 : 1;
  // entries this workgroup owns
  const int my_units = g.n_units > wg ? (g.n_units - wg + nwg - 1) / nwg : 0;
  const int my_entries = my_units * unit_tiles;

  // 1/rms of each row from the producer's partial sums (fixed order: lanes stride, butterfly sum)
  if (g.ssq) {
    float t = 0.f;
    for (int p = lane; p < g.n_ssq; p += kWave) t += g.ssq[(size_t)wave * g.n_ssq + p];
    t = wave_sum(t);
    if (lane == 0) scale_s[wave] = rsqrtf(t / (float)g.Kd + g.eps);
  } else if (lane == 0) {
    scale_s[wave] = 1.0f;
  }

  for (int e0 = 0; e0 < my_entries; e0 += MAXE) {
    f32x4 acc[MAXE];
#pragma unroll
    for (int t = 0; t < MAXE; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    ABuf Bf;
    if (!(pre && e0 == 0)) fast_issue<EPI>(A0, g, wg, nwg, e0, 0, wave, lr, lg);
    // flattened (entry, chunk) groups, ping-pong between A0 and A1
#pragma unroll
    for (int t = 0; t < MAXE; ++t) {
#pragma unroll
      for (int c = 0; c < MAXC; ++c) {
        const int gi = t * MAXC + c;          // static group index
        ABuf &cur = (gi & 1) ? A1 : A0;
        ABuf &nxt = (gi & 1) ? A0 : A1;
        // request the next group
        const int nt = (c + 1 < MAXC) ? t : t + 1, nc = (c + 1 < MAXC) ? c + 1 : 0;
        if (nt < MAXE && e0 + nt < my_entries) fast_issue<EPI>(nxt, g, wg, nwg, e0 + nt, nc, wave, lr, lg);
        if (e0 + t < my_entries) {
          if (t == 0 || MAXC > 1) fast_load_b(Bf, g, c, wave, lr, lg);
          fast_mma(acc[t], cur, Bf);
        }
      }
    }
    // ---- fixed-order reduction over the waves and the epilogue ----
    __syncthreads();
#pragma unroll
    for (int t = 0; t < MAXE; ++t)
      *reinterpret_cast<f32x4 *>(red + ((size_t)(wave * kMaxT + t) * 64 + lane) * 4) = acc[t];
    __syncthreads();
    const int n_out_units = (min(MAXE, my_entries - e0) + unit_tiles - 1) / unit_tiles;
    for (int o = tid; o < n_out_units * 128; o += kFastThreads) {
      const int i = o & 15, jm = (o >> 4) & 7, un = o >> 7;
      const int t = un * unit_tiles;
      const int l_hi = (i >> 2) * 16 + jm, r = i & 3;
      float s0 = 0.f, s1 = 0.f;
#pragma unroll
      for (int w = 0; w < kFastWaves; ++w) {
        const float *p = red + ((size_t)(w * kMaxT + t) * 64) * 4;
        s0 += p[l_hi * 4 + r] + p[(l_hi + 8) * 4 + r];
        if (EPI == FEPI_SWIGLU) {
          const float *q = p + 64 * 4;
          s1 += q[l_hi * 4 + r] + q[(l_hi + 8) * 4 + r];
        }
      }
      const uint16_t *wbase;
      int wrow0, unit;
      fast_tile<EPI>(g, wg, nwg, e0 + t, wbase, wrow0, unit);
      const int col = unit * 16 + i;
      const float sc = scale_s[jm];
      if (EPI == FEPI_STORE) {
        if (jm < g.M) g.out[(size_t)jm * g.ldo + col] = s0 * sc;
      } else if (EPI == FEPI_SWIGLU) {
        const float gt = s0 * sc, up = s1 * sc;
        const float a = (jm < g.M) ? gt / (1.0f + expf(-gt)) * up : 0.f;
        uint32_t hi, lo;
        split_bf16(a, hi, lo);
        g.o_planes[(size_t)jm * g.ldo + col] = (uint16_t)hi;
        g.o_planes[(size_t)(jm + 8) * g.ldo + col] = (uint16_t)lo;
      } else {
        float xn = 0.f;
        if (jm < g.M) {
          xn = g.out[(size_t)jm * g.ldo + col] + s0 * sc;
          g.out[(size_t)jm * g.ldo + col] = xn;
        }
        uint32_t hi, lo;
        split_bf16(xn * g.next_gain[col], hi, lo);
        g.o_planes[(size_t)jm * g.ldo + col] = (uint16_t)hi;
        g.o_planes[(size_t)(jm + 8) * g.ldo + col] = (uint16_t)lo;
        float q = xn * xn;                 // sum over the tile's 16 columns: lanes i = 0..15 are adjacent
        q += __shfl_xor(q, 8, kWave);
        q += __shfl_xor(q, 4, kWave);
        q += __shfl_xor(q, 2, kWave);
        q += __shfl_xor(q, 1, kWave);
        if (i == 0) g.ssq_out[(size_t)jm * g.n_units + unit] = q;
      }
    }
    __syncthreads();
  }
}

// ---- verify attention, one (episode, head) unit per workgroup pass ---------------------------

struct FastAttn {
  float *qkv;                // [M][3*d] fp32 q | k | v of the new rows; k is rotated in place
  uint16_t *k_cache;         // this layer: bf16 [batch][H][cap][HD]
  uint16_t *v_cache;
  const int32_t *prefix_len; // [batch]
  const uint8_t *skip;       // [batch] or nullptr
  const float2 *rope;        // [cap][HD/2]
  uint16_t *o_planes;        // [16][d]: attention output as head/tail planes
  int K, H, cap, d, batch;
  float scale;
};

constexpr int kAttnR = 10;   // key rows a stream keeps in flight

inline size_t fast_attn_lds(int hd, int cap) {
  return sizeof(float) * ((size_t)8 * hd + (size_t)8 * cap + 8 + (size_t)kFastWaves * 8 * hd);
}

__device__ __forceinline__ void unpack8(const uint4 v, float (&f)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(w[i] << 16);
    f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}

// K <= 8 queries of episode b, head h.  512 threads: 512/(HD/8) key streams, each keeping kAttnR
// rows in flight; scores in LDS; softmax one wave per query; second pass over the values.
template <int HD>
__device__ __forceinline__ void fast_attn_unit(const FastAttn &a, int b, int h, unsigned char *smem) {
  constexpr int HALF = HD / 2;
  constexpr int LPK = HD / 8;
  constexpr int G = kFastThreads / LPK;
  float *qs = reinterpret_cast<float *>(smem);   // [8][HD]
  float *sc = qs + 8 * HD;                        // [8][cap]
  float *inv_l = sc + (size_t)8 * a.cap;          // [8]
  float *ored = inv_l + 8;                        // [waves][8][HD]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = a.K, d = a.d, cap = a.cap;
  const int row0 = b * K;
  if (a.skip && a.skip[b]) {
    for (int idx = tid; idx < K * HD; idx += kFastThreads) {
      const size_t o = (size_t)(row0 + idx / HD) * d + h * HD + (idx % HD);
      a.o_planes[o] = 0;
      a.o_planes[o + (size_t)8 * d] = 0;
    }
    return;
  }
  int P = a.prefix_len[b];
  P = max(0, min(P, cap - K));
  const uint16_t *kc = a.k_cache + ((size_t)(b * a.H + h) * cap) * HD;
  const uint16_t *vc = a.v_cache + ((size_t)(b * a.H + h) * cap) * HD;
  uint16_t *kcw = a.k_cache + ((size_t)(b * a.H + h) * cap) * HD;
  uint16_t *vcw = a.v_cache + ((size_t)(b * a.H + h) * cap) * HD;
  const int li = tid % LPK, g = tid / LPK;

  // rotate q (scaled) into LDS; rotate k in place, append k and v to the cache
  for (int idx = tid; idx < 8 * HALF; idx += kFastThreads) {
    const int j = idx / HALF, i = idx - j * HALF;
    float r1 = 0.f, r2 = 0.f;
    if (j < K) {
      float *src = a.qkv + (size_t)(row0 + j) * 3 * d + h * HD;
      const float2 cs = a.rope[(size_t)(P + j) * HALF + i];
      const float q1 = src[i], q2 = src[i + HALF];
      r1 = (q1 * cs.x - q2 * cs.y) * a.scale;
      r2 = (q2 * cs.x + q1 * cs.y) * a.scale;
      const float k1 = src[d + i], k2 = src[d + i + HALF];
      const float kr1 = k1 * cs.x - k2 * cs.y, kr2 = k2 * cs.x + k1 * cs.y;
      src[d + i] = kr1;
      src[d + i + HALF] = kr2;
      uint16_t *kr = kcw + (size_t)(P + j) * HD;
      kr[i] = (uint16_t)f32_to_bf16_bits(kr1);
      kr[i + HALF] = (uint16_t)f32_to_bf16_bits(kr2);
      uint16_t *vr = vcw + (size_t)(P + j) * HD;
      vr[i] = (uint16_t)f32_to_bf16_bits(src[2 * d + i]);
      vr[i + HALF] = (uint16_t)f32_to_bf16_bits(src[2 * d + i + HALF]);
    }
    qs[j * HD + i] = r1;
    qs[j * HD + i + HALF] = r2;
  }
  __syncthreads();
  float qf[8][8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) qf[j][i] = qs[j * HD + li * 8 + i];

  auto score_row = [&](const float (&kf)[8], int r) {
    float s[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float t = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) t = fmaf(qf[j][i], kf[i], t);
      s[j] = t;
    }
#pragma unroll
    for (int off = LPK / 2; off > 0; off >>= 1)
#pragma unroll
      for (int j = 0; j < 8; ++j) s[j] += __shfl_xor(s[j], off, kWave);
    float mine = s[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) mine = (li == j) ? s[j] : mine;
    if (li < 8) sc[(size_t)li * cap + r] = (r <= P + li) ? mine : -INFINITY;
  };

  // ---- pass 1: prefix keys (bf16 cache), kAttnR rows in flight per stream ----
  for (int r0 = 0; r0 < P; r0 += G * kAttnR) {
    uint4 kk[kAttnR];
#pragma unroll
    for (int u = 0; u < kAttnR; ++u) {
      const int r = r0 + u * G + g;
      kk[u] = (r < P) ? *reinterpret_cast<const uint4 *>(kc + (size_t)r * HD + li * 8) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < kAttnR; ++u) {
      const int r = r0 + u * G + g;
      if (r < P) {
        float kf[8];
        unpack8(kk[u], kf);
        score_row(kf, r);
      }
    }
  }
  // the block's own keys at fp32
  if (g < K) {
    const float *kp = a.qkv + (size_t)(row0 + g) * 3 * d + d + h * HD + li * 8;
    const float4 k0 = *reinterpret_cast<const float4 *>(kp), k1 = *reinterpret_cast<const float4 *>(kp + 4);
    const float kf[8] = {k0.x, k0.y, k0.z, k0.w, k1.x, k1.y, k1.z, k1.w};
    score_row(kf, P + g);
  }
  __syncthreads();
  const int nkeys = P + K;
  // ---- softmax: wave j owns query j ----
  if (wave < K) {
    float *row = sc + (size_t)wave * cap;
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
    if (lane == 0) inv_l[wave] = 1.0f / sum;
  }
  __syncthreads();
  // ---- pass 2: values ----
  float o[8][8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) o[j][i] = 0.f;
  auto add_row = [&](const float (&vf)[8], int r) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float p = (j < K) ? sc[(size_t)j * cap + r] : 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) o[j][i] = fmaf(p, vf[i], o[j][i]);
    }
  };
  for (int r0 = 0; r0 < P; r0 += G * kAttnR) {
    uint4 vv[kAttnR];
#pragma unroll
    for (int u = 0; u < kAttnR; ++u) {
      const int r = r0 + u * G + g;
      vv[u] = (r < P) ? *reinterpret_cast<const uint4 *>(vc + (size_t)r * HD + li * 8) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < kAttnR; ++u) {
      const int r = r0 + u * G + g;
      if (r < P) {
        float vf[8];
        unpack8(vv[u], vf);
        add_row(vf, r);
      }
    }
  }
  if (g < K) {
    const float *vp = a.qkv + (size_t)(row0 + g) * 3 * d + 2 * d + h * HD + li * 8;
    const float4 v0 = *reinterpret_cast<const float4 *>(vp), v1 = *reinterpret_cast<const float4 *>(vp + 4);
    const float vf[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
    add_row(vf, P + g);
  }
#pragma unroll
  for (int off = LPK; off < kWave; off <<= 1)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 8; ++i) o[j][i] += __shfl_xor(o[j][i], off, kWave);
  if (lane < LPK) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 8; ++i) ored[(size_t)(wave * 8 + j) * HD + lane * 8 + i] = o[j][i];
  }
  __syncthreads();
  for (int idx = tid; idx < K * HD; idx += kFastThreads) {
    const int j = idx / HD, c = idx - j * HD;
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kFastWaves; ++w) t += ored[(size_t)(w * 8 + j) * HD + c];
    uint32_t hi, lo;
    split_bf16(t * inv_l[j], hi, lo);
    const size_t oo = (size_t)(row0 + j) * d + h * HD + c;
    a.o_planes[oo] = (uint16_t)hi;
    a.o_planes[oo + (size_t)8 * d] = (uint16_t)lo;
  }
  __syncthreads();
}

template <int HD>
__global__ __launch_bounds__(kFastThreads) void fast_attn_kernel(FastAttn a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  fast_attn_unit<HD>(a, blockIdx.y, blockIdx.x, smem);
}

// ---- one launch per phase ---------------------------------------------------------------

template <int EPI, int MAXC>
__global__ __launch_bounds__(kFastThreads) void fast_gemm_kernel(FastGemm g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  ABuf A0, A1;
  fast_gemm_phase<EPI, MAXC>(g, blockIdx.x, gridDim.x, smem, A0, A1, false);
}

// x[m] = E[id[m]] (fp32), planes = x * gain split into heads and tails, partial sums of squares
// per 16-column tile.  One workgroup per 16-column tile, 128 threads: thread (i, m).
__global__ __launch_bounds__(128) void fast_embed(const int32_t *ids, const uint16_t *emb, int vocab, int d, int M,
                                                 const float *gain, float *x, uint16_t *planes, float *ssq_out) {
  const int tile = blockIdx.x, i = threadIdx.x & 15, m = threadIdx.x >> 4;
  const int col = tile * 16 + i;
  float v = 0.f;
  if (m < M) {
    int id = ids[m];
    id = max(0, min(id, vocab - 1));
    v = bf16_bits_to_f32(emb[(size_t)id * d + col]);
    x[(size_t)m * d + col] = v;
  }
  uint32_t hi, lo;
  split_bf16(v * gain[col], hi, lo);
  planes[(size_t)m * d + col] = (uint16_t)hi;
  planes[(size_t)(m + 8) * d + col] = (uint16_t)lo;
  float q = v * v;
  q += __shfl_xor(q, 8, kWave);
  q += __shfl_xor(q, 4, kWave);
  q += __shfl_xor(q, 2, kWave);
  q += __shfl_xor(q, 1, kWave);
  if (i == 0) ssq_out[(size_t)m * (d / 16) + tile] = q;
}

}  // namespace heisd
