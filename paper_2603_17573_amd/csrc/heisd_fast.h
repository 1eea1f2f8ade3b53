// Fast path of the verify forward for M = batch*K <= 8 rows (the headline case: one episode,
// K = 7 drafts; paper Sec. 2.2 "parallel verification" of one action slice), as phase bodies
// that run either one launch per phase or inside one persistent whole-step kernel.
//
// Data exchanged between workgroups
// ---------------------------------
// Activations travel between phases as "plane records": for every 16-column tile one 512-byte
// record [16 rows][16 cols] of bf16, rows 0-7 = bf16 heads of the (up to) 8 activation rows,
// rows 8-15 = bf16 tails (x ~= head + tail, ~16 mantissa bits).  A record row is a piece of one
// column of the MFMA B operand, so a consumer lane loads its B fragment with one 16-byte read
// and no conversion; the producer's epilogue splits each element once.  RMSNorm is folded in:
// the records hold x*g, the producer also emits per-tile partial sums of squares, the consumer
// multiplies its accumulators by 1/rms.  q/k/v travel as fp32 records [tile][8][16].
//
// Every record is written by exactly one workgroup and covers whole 128-byte cache lines, lives
// at an address used once per launch (per-layer buffers), and is written with device-scope
// (write-through) stores.  A consumer on another XCD therefore finds the line neither stale in
// its own L2 nor dirty in the producer's, and reads it with ordinary cached loads after the
// grid barrier - no L2 write-back or invalidate is ever issued inside the step.
//
// GEMM phases
// -----------
// A workgroup (8 waves) owns a list of 16-row weight tiles over the whole reduction; wave w owns
// a contiguous share of the k-steps.  Weight tiles go straight from HBM into the MFMA A-operand
// register layout (lane l: 16 bytes at W[n0 + l%16][k + 8*(l/16)]); the waves are reduced through
// LDS in a fixed order.  For Kd <= 4096 a wave keeps its 16 B fragments in registers and streams
// tiles through two 16-fragment buffers; for longer reductions (the down projection) A and B
// fragments stream together through a ring of three 8-step buffers.  Each phase can be told that
// its first buffers were requested earlier and is handed a callback that requests the next
// phase's first tiles before it starts its own epilogue, so HBM stays busy across grid barriers.
#pragma once
#include "heisd_common.h"

namespace heisd {

constexpr int kFastThreads = 512;
constexpr int kFastWaves = 8;
constexpr int kKS = 16;      // k-steps (of 32) per register buffer, resident-B phases
constexpr int kKS2 = 8;      // k-steps per ring slot, streaming phases
constexpr int kMaxT = 6;     // weight tiles a workgroup accumulates at once (resident-B phases)
constexpr int kSsqStride = 32;  // floats per partial-sum record (8 used): one 128-byte line

enum { FEPI_STORE_REC = 0, FEPI_RESID_NORM = 1, FEPI_SWIGLU = 2, FEPI_STORE_ROWS = 3 };

// ---- device-scope (write-through) stores for data other workgroups will read -----------------
__device__ __forceinline__ void st_dev(uint32_t *p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev2(float *p, float a, float b) {
  const unsigned long long q = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct FastGemm {
  const uint16_t *w[3];   // weight segments, bf16 row-major [rows][Kd]
  int seg_tiles;          // n-tiles per segment
  int n_units;            // n-tiles, or (gate, up) pairs for FEPI_SWIGLU
  int Kd;
  const uint16_t *b;      // activation plane records [Kd/16][16][16] bf16
  const float *ssq;       // [n_ssq][kSsqStride] partial sums of squares of the raw rows, or nullptr
  int n_ssq;
  float eps;
  int M;                  // valid rows (<= 8)
  // outputs
  float *out;             // STORE_REC: fp32 records [unit][8][16]; STORE_ROWS: [M][ldo] rows;
                          // RESID_NORM: residual stream x [8][ldo] (read and written by its owner only)
  int ldo;
  const float *next_gain; // RESID_NORM: gain of the norm that consumes x next
  uint16_t *o_planes;     // RESID_NORM / SWIGLU: plane records [unit][16][16]
  float *ssq_out;         // RESID_NORM: [n_units][kSsqStride]
};

struct Frag16 {
  uint4 v[kKS];
};
struct Frag8 {
  uint4 a[kKS2];
  uint4 b[kKS2];
};

// k-steps per wave (wave w owns steps [w*ksw, w*ksw + fast_steps(w)))
__device__ __forceinline__ int fast_ksw(int Kd) { return ((Kd + 31) / 32 + kFastWaves - 1) / kFastWaves; }
__device__ __forceinline__ int fast_steps(int Kd, int wave) {
  const int total = (Kd + 31) / 32, ksw = fast_ksw(Kd);
  return max(0, min(ksw, total - wave * ksw));
}

// Which weight tile is list entry `e` of workgroup `wg` (of `nwg`)?  Units are dealt round-robin,
// so unit u always belongs to workgroup u % nwg.
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

template <int EPI>
__device__ __forceinline__ int fast_my_entries(const FastGemm &g, int wg, int nwg) {
  const int my_units = g.n_units > wg ? (g.n_units - wg + nwg - 1) / nwg : 0;
  return my_units * (EPI == FEPI_SWIGLU ? 2 : 1);
}

// Address of the B fragment of k-step `ks` for lane (lr, lg): record ks*2 + lg/2, row lr, half lg&1.
__device__ __forceinline__ const uint4 *fast_b_ptr(const uint16_t *planes, int ks, int lr, int lg) {
  return reinterpret_cast<const uint4 *>(planes + ((size_t)(ks * 2 + (lg >> 1)) * 256 + lr * 16 + (lg & 1) * 8));
}

// ---- resident-B phases (Kd <= 4096: at most kKS steps per wave) --------------------------------

template <int EPI>
__device__ __forceinline__ void fast_issue16(Frag16 &A, const FastGemm &g, int wg, int nwg, int e, int wave, int lr,
                                             int lg) {
  const uint16_t *wbase;
  int wrow0, unit;
  const bool ok = fast_tile<EPI>(g, wg, nwg, e, wbase, wrow0, unit);
  const int ks0 = wave * fast_ksw(g.Kd), ns = ok ? fast_steps(g.Kd, wave) : 0;
  const uint16_t *p = wbase + (size_t)(wrow0 + lr) * g.Kd + ks0 * 32 + lg * 8;
#pragma unroll
  for (int s = 0; s < kKS; ++s)
    A.v[s] = (s < ns && (ks0 + s) * 32 + lg * 8 + 8 <= g.Kd) ? *reinterpret_cast<const uint4 *>(p + s * 32)
                                                              : make_uint4(0, 0, 0, 0);
}

__device__ __forceinline__ void fast_load_b16(Frag16 &Bf, const FastGemm &g, int wave, int lr, int lg) {
  const int ks0 = wave * fast_ksw(g.Kd), ns = fast_steps(g.Kd, wave);
#pragma unroll
  for (int s = 0; s < kKS; ++s)
    Bf.v[s] = (s < ns && (ks0 + s) * 32 + lg * 8 + 8 <= g.Kd) ? *fast_b_ptr(g.b, ks0 + s, lr, lg) : make_uint4(0, 0, 0, 0);
}

__device__ __forceinline__ void fast_mma16(f32x4 &acc, const Frag16 &A, const Frag16 &Bf) {
#pragma unroll
  for (int s = 0; s < kKS; ++s)
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A.v[s]), __builtin_bit_cast(bf16x8, Bf.v[s]),
                                                  acc, 0, 0, 0);
}

// LDS of a GEMM phase: reduction buffer [waves][kMaxT][64 lanes][4] + 8 scales.
constexpr size_t kFastRedBytes = (size_t)kFastWaves * kMaxT * 64 * 16;
constexpr size_t kFastLds = kFastRedBytes + 16 * sizeof(float);

// 1/rms of each row from the producer's partial sums (fixed order: lanes stride, butterfly sum);
// wave w computes row w.  Must be followed by a __syncthreads before scale_s is read.
__device__ __forceinline__ void fast_row_scales(const FastGemm &g, float *scale_s, int wave, int lane) {
  if (g.ssq) {
    float t = 0.f;
    for (int p = lane; p < g.n_ssq; p += kWave) t += g.ssq[(size_t)p * kSsqStride + wave];
    t = wave_sum(t);
    if (lane == 0) scale_s[wave] = rsqrtf(t / (float)g.Kd + g.eps);
  } else if (lane == 0) {
    scale_s[wave] = 1.0f;
  }
}

// Reduction over the waves (fixed order) and epilogue of `n_tiles` accumulated tile entries
// starting at list entry e0.  acc tiles were stored to `red` by the caller.
template <int EPI>
__device__ __forceinline__ void fast_epilogue(const FastGemm &g, int wg, int nwg, int e0, int n_tiles, const float *red,
                                              const float *scale_s) {
  constexpr int UT = (EPI == FEPI_SWIGLU) ? 2 : 1;
  const int tid = threadIdx.x;
  const int n_units_out = (n_tiles + UT - 1) / UT;
  for (int o = tid; o < n_units_out * 64; o += kFastThreads) {
    const int c2 = o & 7, jm = (o >> 3) & 7, un = o >> 6;
    const int t = un * UT;
    const int i = 2 * c2;                       // this thread covers columns i, i+1 of the tile
    const int l_hi = (i >> 2) * 16 + jm, r = i & 3;
    float s0 = 0.f, s1 = 0.f, u0 = 0.f, u1 = 0.f;
#pragma unroll
    for (int w = 0; w < kFastWaves; ++w) {
      const float *p = red + ((size_t)(w * kMaxT + t) * 64) * 4;
      const float2 a = *reinterpret_cast<const float2 *>(p + l_hi * 4 + r);
      const float2 b = *reinterpret_cast<const float2 *>(p + (l_hi + 8) * 4 + r);
      s0 += a.x + b.x;
      s1 += a.y + b.y;
      if (EPI == FEPI_SWIGLU) {
        const float2 c = *reinterpret_cast<const float2 *>(p + 256 + l_hi * 4 + r);
        const float2 d = *reinterpret_cast<const float2 *>(p + 256 + (l_hi + 8) * 4 + r);
        u0 += c.x + d.x;
        u1 += c.y + d.y;
      }
    }
    const uint16_t *wbase;
    int wrow0, unit;
    fast_tile<EPI>(g, wg, nwg, e0 + t, wbase, wrow0, unit);
    const float sc = scale_s[jm];
    const bool live = jm < g.M;
    if (EPI == FEPI_STORE_REC) {
      st_dev2(g.out + (size_t)unit * 128 + jm * 16 + i, live ? s0 * sc : 0.f, live ? s1 * sc : 0.f);
    } else if (EPI == FEPI_STORE_ROWS) {
      if (live) st_dev2(g.out + (size_t)jm * g.ldo + unit * 16 + i, s0 * sc, s1 * sc);
    } else {
      float a0, a1;
      if (EPI == FEPI_SWIGLU) {
        const float g0 = s0 * sc, g1 = s1 * sc;
        a0 = live ? g0 / (1.0f + expf(-g0)) * (u0 * sc) : 0.f;
        a1 = live ? g1 / (1.0f + expf(-g1)) * (u1 * sc) : 0.f;
      } else {
        a0 = 0.f;
        a1 = 0.f;
        float *xp = g.out + (size_t)jm * g.ldo + unit * 16 + i;
        if (live) {
          const float2 xo = *reinterpret_cast<const float2 *>(xp);
          a0 = xo.x + s0 * sc;
          a1 = xo.y + s1 * sc;
          *reinterpret_cast<float2 *>(xp) = make_float2(a0, a1);
        }
        float q = a0 * a0 + a1 * a1;       // sum over the tile's 16 columns: 8 adjacent lanes
        q += __shfl_xor(q, 4, kWave);
        q += __shfl_xor(q, 2, kWave);
        q += __shfl_xor(q, 1, kWave);
        if (c2 == 0) st_dev(g.ssq_out + (size_t)unit * kSsqStride + jm, q);
        const float2 gn = *reinterpret_cast<const float2 *>(g.next_gain + unit * 16 + i);
        a0 *= gn.x;
        a1 *= gn.y;
      }
      uint32_t h0, l0, h1, l1;
      split_bf16(a0, h0, l0);
      split_bf16(a1, h1, l1);
      uint32_t *rec = reinterpret_cast<uint32_t *>(g.o_planes + (size_t)unit * 256);
      st_dev(rec + (jm * 16 + i) / 2, h0 | (h1 << 16));
      st_dev(rec + ((jm + 8) * 16 + i) / 2, l0 | (l1 << 16));
    }
  }
}

// One resident-B GEMM phase for workgroup `wg` of `nwg`.  NPRE leading tile entries (0, 1 or 2)
// were already requested by the caller into buf0 / buf1.  `next()` is called once after the last
// weight tile has been consumed (buffers free), before the reduction and the epilogue.
template <int EPI, int NPRE, typename Next>
__device__ __forceinline__ void fast_gemm_phase(const FastGemm &g, int wg, int nwg, unsigned char *smem, Frag16 &buf0,
                                                Frag16 &buf1, Next next) {
  float *red = reinterpret_cast<float *>(smem);
  float *scale_s = reinterpret_cast<float *>(smem + kFastRedBytes);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int my_entries = fast_my_entries<EPI>(g, wg, nwg);
  fast_row_scales(g, scale_s, wave, lane);
  if (my_entries == 0) {
    next();
    __syncthreads();
    return;
  }
  Frag16 Bf;
  fast_load_b16(Bf, g, wave, lr, lg);
  for (int e0 = 0; e0 < my_entries; e0 += kMaxT) {
    f32x4 acc[kMaxT];
#pragma unroll
    for (int t = 0; t < kMaxT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    const bool first = (e0 == 0);
    if (!(first && NPRE >= 1)) fast_issue16<EPI>(buf0, g, wg, nwg, e0, wave, lr, lg);
    if (!(first && NPRE >= 2) && e0 + 1 < my_entries) fast_issue16<EPI>(buf1, g, wg, nwg, e0 + 1, wave, lr, lg);
#pragma unroll
    for (int t = 0; t < kMaxT; ++t) {
      Frag16 &cur = (t & 1) ? buf1 : buf0;
      if (e0 + t < my_entries) fast_mma16(acc[t], cur, Bf);
      if (t + 2 < kMaxT && e0 + t + 2 < my_entries) fast_issue16<EPI>(cur, g, wg, nwg, e0 + t + 2, wave, lr, lg);
    }
    if (e0 + kMaxT >= my_entries) next();
    __syncthreads();
#pragma unroll
    for (int t = 0; t < kMaxT; ++t)
      *reinterpret_cast<f32x4 *>(red + ((size_t)(wave * kMaxT + t) * 64 + lane) * 4) = acc[t];
    __syncthreads();
    fast_epilogue<EPI>(g, wg, nwg, e0, min(kMaxT, my_entries - e0), red, scale_s);
    __syncthreads();
  }
}

// ---- streaming phases (long reductions: A and B fragments stream together) -------------------------

template <int EPI>
__device__ __forceinline__ void fast_issue8(Frag8 &F, const FastGemm &g, const uint16_t *wrow, bool ok, int ks0, int ns,
                                            int grp, int lr, int lg) {
  // group `grp` of this wave: steps ks0 + grp*8 .. +7, limited to ns steps in total
#pragma unroll
  for (int s = 0; s < kKS2; ++s) {
    const int sl = grp * kKS2 + s;
    const bool v = ok && sl < ns && (ks0 + sl) * 32 + lg * 8 + 8 <= g.Kd;
    F.a[s] = v ? *reinterpret_cast<const uint4 *>(wrow + (size_t)(ks0 + sl) * 32) : make_uint4(0, 0, 0, 0);
  }
}
__device__ __forceinline__ void fast_issue8_b(Frag8 &F, const FastGemm &g, int ks0, int ns, int grp, int lr, int lg) {
#pragma unroll
  for (int s = 0; s < kKS2; ++s) {
    const int sl = grp * kKS2 + s;
    const bool v = sl < ns && (ks0 + sl) * 32 + lg * 8 + 8 <= g.Kd;
    F.b[s] = v ? *fast_b_ptr(g.b, ks0 + sl, lr, lg) : make_uint4(0, 0, 0, 0);
  }
}
__device__ __forceinline__ void fast_mma8(f32x4 &acc, const Frag8 &F) {
#pragma unroll
  for (int s = 0; s < kKS2; ++s)
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, F.a[s]), __builtin_bit_cast(bf16x8, F.b[s]),
                                                  acc, 0, 0, 0);
}

// Request the weight halves of the first two ring slots of a streaming phase (entry 0); used by a
// preceding phase before the grid barrier.  The B halves are loaded by the phase itself.
template <int EPI>
__device__ __forceinline__ void fast_stream_prefetch(const FastGemm &g, int wg, int nwg, Frag8 &r0, Frag8 &r1) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lr = lane & 15, lg = lane >> 4;
  const uint16_t *wbase;
  int wrow0, unit;
  const bool ok = fast_tile<EPI>(g, wg, nwg, 0, wbase, wrow0, unit);
  const int ks0 = wave * fast_ksw(g.Kd), ns = fast_steps(g.Kd, wave);
  const uint16_t *wrow = wbase + (size_t)(wrow0 + lr) * g.Kd + lg * 8;
  fast_issue8<EPI>(r0, g, wrow, ok, ks0, ns, 0, lr, lg);
  fast_issue8<EPI>(r1, g, wrow, ok, ks0, ns, 1, lr, lg);
}

// One streaming GEMM phase: one tile entry per pass, ring of three (A, B) slots of 8 k-steps.
// PRE: the weight halves of slots r0, r1 for (entry 0, groups 0 and 1) were requested by the caller.
template <int EPI, bool PRE, typename Next>
__device__ __forceinline__ void fast_gemm_stream_phase(const FastGemm &g, int wg, int nwg, unsigned char *smem, Frag8 &r0,
                                                       Frag8 &r1, Frag8 &r2, Next next) {
  float *red = reinterpret_cast<float *>(smem);
  float *scale_s = reinterpret_cast<float *>(smem + kFastRedBytes);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int my_entries = fast_my_entries<EPI>(g, wg, nwg);
  fast_row_scales(g, scale_s, wave, lane);
  if (my_entries == 0) {
    next();
    __syncthreads();
    return;
  }
  const int ks0 = wave * fast_ksw(g.Kd), ns = fast_steps(g.Kd, wave);
  const int ngrp = (fast_ksw(g.Kd) + kKS2 - 1) / kKS2;     // same for every wave (tail groups are empty)
  for (int e = 0; e < my_entries; ++e) {
    const uint16_t *wbase;
    int wrow0, unit;
    const bool ok = fast_tile<EPI>(g, wg, nwg, e, wbase, wrow0, unit);
    const uint16_t *wrow = wbase + (size_t)(wrow0 + lr) * g.Kd + lg * 8;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    if (!(PRE && e == 0)) {
      fast_issue8<EPI>(r0, g, wrow, ok, ks0, ns, 0, lr, lg);
      fast_issue8<EPI>(r1, g, wrow, ok, ks0, ns, 1, lr, lg);
    }
    fast_issue8_b(r0, g, ks0, ns, 0, lr, lg);
    fast_issue8_b(r1, g, ks0, ns, 1, lr, lg);
    for (int gi = 0; gi < ngrp; gi += 3) {
      fast_issue8<EPI>(r2, g, wrow, ok, ks0, ns, gi + 2, lr, lg);
      fast_issue8_b(r2, g, ks0, ns, gi + 2, lr, lg);
      fast_mma8(acc, r0);
      fast_issue8<EPI>(r0, g, wrow, ok, ks0, ns, gi + 3, lr, lg);
      fast_issue8_b(r0, g, ks0, ns, gi + 3, lr, lg);
      fast_mma8(acc, r1);
      fast_issue8<EPI>(r1, g, wrow, ok, ks0, ns, gi + 4, lr, lg);
      fast_issue8_b(r1, g, ks0, ns, gi + 4, lr, lg);
      fast_mma8(acc, r2);
    }
    if (e + 1 == my_entries) next();
    __syncthreads();
    *reinterpret_cast<f32x4 *>(red + ((size_t)(wave * kMaxT) * 64 + lane) * 4) = acc;
    __syncthreads();
    fast_epilogue<EPI>(g, wg, nwg, e, 1, red, scale_s);
    __syncthreads();
  }
}

// ---- embedding: x = E[id] (fp32, owner-private), plane records of x*gain, partial sums of squares ----
// One 16-column tile per call; the first 64 threads of the workgroup work: thread (c2, m).
__device__ __forceinline__ void fast_embed_tile(const int32_t *ids, const uint16_t *emb, int vocab, int d, int M, int tile,
                                                const float *gain, float *x, uint16_t *planes, float *ssq_out) {
  const int tid = threadIdx.x;
  if (tid >= 64) return;
  const int c2 = tid & 7, m = tid >> 3;
  const int col = tile * 16 + 2 * c2;
  float v0 = 0.f, v1 = 0.f;
  if (m < M) {
    int id = ids[m];
    id = max(0, min(id, vocab - 1));
    const uint32_t pr = *reinterpret_cast<const uint32_t *>(emb + (size_t)id * d + col);
    v0 = __uint_as_float(pr << 16);
    v1 = __uint_as_float(pr & 0xFFFF0000u);
    *reinterpret_cast<float2 *>(x + (size_t)m * d + col) = make_float2(v0, v1);
  }
  float q = v0 * v0 + v1 * v1;
  q += __shfl_xor(q, 4, kWave);
  q += __shfl_xor(q, 2, kWave);
  q += __shfl_xor(q, 1, kWave);
  if (c2 == 0) st_dev(ssq_out + (size_t)tile * kSsqStride + m, q);
  const float2 gn = *reinterpret_cast<const float2 *>(gain + col);
  uint32_t h0, l0, h1, l1;
  split_bf16(v0 * gn.x, h0, l0);
  split_bf16(v1 * gn.y, h1, l1);
  uint32_t *rec = reinterpret_cast<uint32_t *>(planes + (size_t)tile * 256);
  st_dev(rec + (m * 16 + 2 * c2) / 2, h0 | (h1 << 16));
  st_dev(rec + ((m + 8) * 16 + 2 * c2) / 2, l0 | (l1 << 16));
}

// ---- verify attention, one (episode, head) unit ---------------------------------------------

struct FastAttn {
  const float *qkv;          // fp32 records [3*d/16][8][16]: q tiles, then k tiles, then v tiles (not rotated)
  uint16_t *k_cache;         // this layer: bf16 [batch][H][cap][HD]
  uint16_t *v_cache;
  const int32_t *prefix_len; // [batch]
  const uint8_t *skip;       // [batch] or nullptr
  const float2 *rope;        // [cap][HD/2]
  uint16_t *o_planes;        // plane records [d/16][16][16]: attention output
  int K, H, cap, d, batch;
  float scale;
};

constexpr int kAttnR = 12;   // prefix rows a key stream requests at once

inline size_t fast_attn_lds(int hd, int cap) {
  return sizeof(float) * ((size_t)8 * hd * 3 + (size_t)8 * cap + 8 + (size_t)kFastWaves * 8 * hd);
}

__device__ __forceinline__ void unpack8(const uint4 v, float (&f)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(w[i] << 16);
    f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}

struct AttnPre {
  uint4 k[kAttnR];
  uint4 v[kAttnR];
};

// Request the first kAttnR prefix key and value rows of this lane's stream (no dependence on the
// current step's activations: may be called before the grid barrier that publishes q/k/v).
template <int HD>
__device__ __forceinline__ void fast_attn_prefetch(const FastAttn &a, int b, int h, AttnPre &pre) {
  constexpr int LPK = HD / 8, G = kFastThreads / LPK;
  const int tid = threadIdx.x, li = tid % LPK, g = tid / LPK;
  int P = a.prefix_len[b];
  P = max(0, min(P, a.cap - a.K));
  const bool skip = a.skip && a.skip[b];
  const uint16_t *kc = a.k_cache + ((size_t)(b * a.H + h) * a.cap) * HD;
  const uint16_t *vc = a.v_cache + ((size_t)(b * a.H + h) * a.cap) * HD;
#pragma unroll
  for (int u = 0; u < kAttnR; ++u) {
    const int r = u * G + g;
    const bool ok = !skip && r < P;
    pre.k[u] = ok ? *reinterpret_cast<const uint4 *>(kc + (size_t)r * HD + li * 8) : make_uint4(0, 0, 0, 0);
    pre.v[u] = ok ? *reinterpret_cast<const uint4 *>(vc + (size_t)r * HD + li * 8) : make_uint4(0, 0, 0, 0);
  }
}

// K <= 8 queries of episode b, head h.  512 threads = 512/(HD/8) key streams; `pre` holds the
// first kAttnR rows of each stream.  Scores in LDS; softmax one wave per query; the block's own
// keys and values stay in fp32 (LDS), only the stored cache rows are rounded to bf16.
template <int HD>
__device__ __forceinline__ void fast_attn_unit(const FastAttn &a, int b, int h, unsigned char *smem, const AttnPre &pre) {
  constexpr int HALF = HD / 2;
  constexpr int LPK = HD / 8;
  constexpr int G = kFastThreads / LPK;
  constexpr int TPH = HD / 16;                      // 16-column tiles per head
  float *qs = reinterpret_cast<float *>(smem);     // [8][HD] rotated, scaled queries
  float *kb = qs + 8 * HD;                          // [8][HD] rotated keys of the block
  float *vb = kb + 8 * HD;                          // [8][HD] values of the block
  float *sc = vb + 8 * HD;                          // [8][cap]
  float *inv_l = sc + (size_t)8 * a.cap;            // [8]
  float *ored = inv_l + 8;                          // [waves][8][HD]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = a.K, d = a.d, cap = a.cap;
  const int row0 = b * K;
  const int li = tid % LPK, g = tid / LPK;
  if (a.skip && a.skip[b]) {
    for (int idx = tid; idx < K * HALF; idx += kFastThreads) {       // zero this head's slice of the records
      const int j = idx / HALF, c = (idx - j * HALF) * 2;
      uint32_t *rec = reinterpret_cast<uint32_t *>(a.o_planes + (size_t)(h * TPH + c / 16) * 256);
      st_dev(rec + ((row0 + j) * 16 + (c & 15)) / 2, 0u);
      st_dev(rec + ((row0 + j + 8) * 16 + (c & 15)) / 2, 0u);
    }
    return;
  }
  int P = a.prefix_len[b];
  P = max(0, min(P, cap - K));
  uint16_t *kc = a.k_cache + ((size_t)(b * a.H + h) * cap) * HD;
  uint16_t *vc = a.v_cache + ((size_t)(b * a.H + h) * cap) * HD;
  const int n_t = d / 16;

  // rotate q (scaled) and k into LDS, copy v; append k and v (bf16) to the cache
  for (int idx = tid; idx < 8 * HALF; idx += kFastThreads) {
    const int j = idx / HALF, i = idx - j * HALF;
    float r1 = 0.f, r2 = 0.f, kr1 = 0.f, kr2 = 0.f, v1 = 0.f, v2 = 0.f;
    if (j < K) {
      const int m = row0 + j;
      const float *qa = a.qkv + (size_t)(h * TPH + i / 16) * 128 + m * 16 + (i & 15);
      const float *qb = a.qkv + (size_t)(h * TPH + (i + HALF) / 16) * 128 + m * 16 + ((i + HALF) & 15);
      const size_t ko = (size_t)n_t * 128, vo = (size_t)2 * n_t * 128;
      const float2 cs = a.rope[(size_t)(P + j) * HALF + i];
      const float q1 = qa[0], q2 = qb[0], k1 = qa[ko], k2 = qb[ko];
      v1 = qa[vo];
      v2 = qb[vo];
      r1 = (q1 * cs.x - q2 * cs.y) * a.scale;
      r2 = (q2 * cs.x + q1 * cs.y) * a.scale;
      kr1 = k1 * cs.x - k2 * cs.y;
      kr2 = k2 * cs.x + k1 * cs.y;
      uint16_t *kr = kc + (size_t)(P + j) * HD;
      kr[i] = (uint16_t)f32_to_bf16_bits(kr1);
      kr[i + HALF] = (uint16_t)f32_to_bf16_bits(kr2);
      uint16_t *vr = vc + (size_t)(P + j) * HD;
      vr[i] = (uint16_t)f32_to_bf16_bits(v1);
      vr[i + HALF] = (uint16_t)f32_to_bf16_bits(v2);
    }
    qs[j * HD + i] = r1;
    qs[j * HD + i + HALF] = r2;
    kb[j * HD + i] = kr1;
    kb[j * HD + i + HALF] = kr2;
    vb[j * HD + i] = v1;
    vb[j * HD + i + HALF] = v2;
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

  // ---- pass 1: prefix keys ----
#pragma unroll
  for (int u = 0; u < kAttnR; ++u) {
    const int r = u * G + g;
    if (r < P) {
      float kf[8];
      unpack8(pre.k[u], kf);
      score_row(kf, r);
    }
  }
  for (int r0 = G * kAttnR; r0 < P; r0 += G * kAttnR) {
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
  if (g < K) {   // the block's own keys at fp32
    float kf[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) kf[i] = kb[g * HD + li * 8 + i];
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
#pragma unroll
  for (int u = 0; u < kAttnR; ++u) {
    const int r = u * G + g;
    if (r < P) {
      float vf[8];
      unpack8(pre.v[u], vf);
      add_row(vf, r);
    }
  }
  for (int r0 = G * kAttnR; r0 < P; r0 += G * kAttnR) {
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
    float vf[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) vf[i] = vb[g * HD + li * 8 + i];
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
  for (int idx = tid; idx < K * HALF; idx += kFastThreads) {      // two adjacent channels per thread
    const int j = idx / HALF, c = (idx - j * HALF) * 2;
    float t0 = 0.f, t1 = 0.f;
#pragma unroll
    for (int w = 0; w < kFastWaves; ++w) {
      t0 += ored[(size_t)(w * 8 + j) * HD + c];
      t1 += ored[(size_t)(w * 8 + j) * HD + c + 1];
    }
    uint32_t h0, l0, h1, l1;
    split_bf16(t0 * inv_l[j], h0, l0);
    split_bf16(t1 * inv_l[j], h1, l1);
    uint32_t *rec = reinterpret_cast<uint32_t *>(a.o_planes + (size_t)(h * TPH + c / 16) * 256);
    st_dev(rec + ((row0 + j) * 16 + (c & 15)) / 2, h0 | (h1 << 16));
    st_dev(rec + ((row0 + j + 8) * 16 + (c & 15)) / 2, l0 | (l1 << 16));
  }
  __syncthreads();
}

// ---- one launch per phase ---------------------------------------------------------------------

struct NoNext {
  __device__ __forceinline__ void operator()() const {}
};

template <int EPI>
__global__ __launch_bounds__(kFastThreads) void fast_gemm_kernel(FastGemm g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  Frag16 b0, b1;
  fast_gemm_phase<EPI, 0>(g, blockIdx.x, gridDim.x, smem, b0, b1, NoNext());
}

template <int EPI>
__global__ __launch_bounds__(kFastThreads) void fast_gemm_stream_kernel(FastGemm g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  Frag8 r0, r1, r2;
  fast_gemm_stream_phase<EPI, false>(g, blockIdx.x, gridDim.x, smem, r0, r1, r2, NoNext());
}

template <int HD>
__global__ __launch_bounds__(kFastThreads) void fast_attn_kernel(FastAttn a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  AttnPre pre;
  fast_attn_prefetch<HD>(a, blockIdx.y, blockIdx.x, pre);
  fast_attn_unit<HD>(a, blockIdx.y, blockIdx.x, smem, pre);
}

__global__ __launch_bounds__(64) void fast_embed_kernel(const int32_t *ids, const uint16_t *emb, int vocab, int d, int M,
                                                       const float *gain, float *x, uint16_t *planes, float *ssq_out) {
  fast_embed_tile(ids, emb, vocab, d, M, blockIdx.x, gain, x, planes, ssq_out);
}

}  // namespace heisd
