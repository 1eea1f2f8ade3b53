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
// register layout (lane l: 16 bytes = W[n0 + l%16][k + 8*(l/16) .. +8), read from a copy of the
// weights stored in exactly that order); the waves are reduced through
// LDS in a fixed order.  A wave keeps one ring of 16 weight fragments: a fragment's registers are
// refilled with the same k-step of the next tile right after the MFMA that consumed it, so 16
// loads (16 KB) per wave are always in flight.  For Kd <= 4096 the wave's 16 B fragments stay in
// registers; for longer reductions (the down projection) B fragments stream through a second
// ring.  A phase can be told that the ring already holds its first tile (the persistent kernel
// requests it while it waits at the grid barrier), so HBM stays busy across barriers.
#pragma once
#include "heisd_common.h"

namespace heisd {

constexpr int kFastThreads = 512;
constexpr int kFastWaves = 8;
constexpr int kKS = 16;      // k-steps (of 32) per register buffer, resident-B phases
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
  int epi;                // FEPI_*: how tiles map to units and what the epilogue does
  const uint16_t *w[3];   // weight segments, bf16, in the packed fragment order of fast_pack_weights
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
  int xcd_heads;          // STORE_REC with seg_tiles == workgroups == 256 and 8 tiles per head (the QKV projection at
                          // d_model 4096, head_dim 128): tiles are dealt so that the eight tiles of head h run on
                          // workgroups of XCD h % 8, where that head's attention units run (see fast_xcd_tile)
};

// Workgroup w of 256 (XCD w % 8, since workgroup ids are dealt to the 8 XCDs round-robin) takes, in each segment,
// tile 8 * head + c with head = w % 8 + 8 * (w / 64) and c = (w / 8) % 8: a head's q, k and v rows are then produced
// on the XCD that consumes them, and the attention unit's first loads hit that XCD's L2.
__host__ __device__ __forceinline__ int fast_xcd_tile(int w) { return 8 * ((w & 7) + 8 * (w >> 6)) + ((w >> 3) & 7); }

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
struct Frag16 {
  u32x4 v[kKS];
};

typedef const u32x4 __attribute__((address_space(1))) *gptr_u4;   // global address space: no flat loads
__device__ __forceinline__ u32x4 ld_g(const void *p) {
  return *reinterpret_cast<gptr_u4>(reinterpret_cast<uintptr_t>(p));
}

// k-steps per wave (wave w owns steps [w*ksw, w*ksw + fast_steps(w)))
__device__ __forceinline__ int fast_ksw(int Kd) { return ((Kd + 31) / 32 + kFastWaves - 1) / kFastWaves; }
__device__ __forceinline__ int fast_steps(int Kd, int wave) {
  const int total = (Kd + 31) / 32, ksw = fast_ksw(Kd);
  return max(0, min(ksw, total - wave * ksw));
}

// Which weight tile is list entry `e` of workgroup `wg` (of `nwg`)?  Units are dealt round-robin,
// so unit u always belongs to workgroup u % nwg.
// (The three segment pointers are read unconditionally and then selected by value: a descriptor that
// lives in a local variable stays in registers that way, whereas a load through a selected address
// would force it onto the stack.)
__device__ __forceinline__ bool fast_tile(const FastGemm &g, int wg, int nwg, int e, const uint16_t *&wbase,
                                          int &wrow0, int &unit) {
  const uint16_t *const w0 = g.w[0], *const w1 = g.w[1], *const w2 = g.w[2];
  if (g.epi == FEPI_SWIGLU) {
    unit = wg + (e >> 1) * nwg;
    wbase = (e & 1) ? w1 : w0;
    wrow0 = unit * 16;
    return unit < g.n_units;
  }
  unit = wg + e * nwg;
  if (g.xcd_heads && nwg == 256) unit = fast_xcd_tile(wg) + e * nwg;
  const int u = unit < g.n_units ? unit : 0;
  const int seg = u / g.seg_tiles;
  wbase = seg == 0 ? w0 : (seg == 1 ? w1 : w2);
  wrow0 = (u - seg * g.seg_tiles) * 16;
  return unit < g.n_units;
}

__device__ __forceinline__ int fast_my_entries(const FastGemm &g, int wg, int nwg) {
  const int my_units = g.n_units > wg ? (g.n_units - wg + nwg - 1) / nwg : 0;
  return my_units * (g.epi == FEPI_SWIGLU ? 2 : 1);
}

// All fragment loads are unconditional: instead of predicating lanes, an out-of-range k-step reads
// a clamped (valid) weight address and is paired with an all-zero B record.  The plane buffers end
// with zero records for that purpose.
__host__ __device__ __forceinline__ int fast_plane_records(int Kd) { return 2 * ((Kd + 31) / 32) + 2; }

// Weights are read from a copy made once at init, laid out the way the MFMA consumes them:
// [16-row tile][k-step of 32][lane][8 bf16], lane l holding W[16*tile + l%16][32*ks + 8*(l/16) .. +8)
// (k past Kd is stored as zero).  A fragment load is then 1 KB of consecutive bytes and a wave's
// walk along k is one sequential stream, instead of 64-byte pieces of 16 rows that lie a whole
// matrix row apart: measured 4 % of the step at M = 7 (mostly the down projection, whose rows are
// 22 KB long) and 18 % at M = 56.
__host__ __device__ __forceinline__ size_t fast_packed_elems(int rows, int Kd) {
  return (size_t)(rows / 16) * (size_t)((Kd + 31) / 32) * 512;
}
// This lane's piece of k-step 0 of the tile that starts at row wrow0 (a multiple of 16).
__device__ __forceinline__ const uint16_t *fast_wfrag(const uint16_t *wbase, int wrow0, int Kd, int lane) {
  return wbase + ((size_t)(wrow0 >> 4) * (size_t)((Kd + 31) / 32) * 64 + lane) * 8;
}
// Weight fragment of k-step `ks` (clamped into the matrix).
__device__ __forceinline__ u32x4 fast_ld_a(const uint16_t *wfrag, int Kd, int ks) {
  const int total = (Kd + 31) / 32;
  return ld_g(wfrag + (size_t)min(ks, total - 1) * 512);
}
// The copy: one thread per 16-byte piece of dst.
__global__ __launch_bounds__(256) void fast_pack_weights(const uint16_t *src, int rows, int Kd, uint16_t *dst) {
  const int KS = (Kd + 31) / 32;
  const size_t n = (size_t)(rows / 16) * KS * 64;
  for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < n; idx += (size_t)gridDim.x * 256) {
    const int lane = (int)(idx & 63);
    const size_t q = idx >> 6;
    const int ks = (int)(q % KS);
    const size_t tile = q / KS;
    const int k = ks * 32 + (lane >> 4) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (k + 8 <= Kd) v = *reinterpret_cast<const uint4 *>(src + (tile * 16 + (lane & 15)) * (size_t)Kd + k);
    *reinterpret_cast<uint4 *>(dst + idx * 8) = v;
  }
}
// B fragment of step `s` of a wave that owns `ns` steps from ks0 (the zero records if s >= ns):
// record ks*2 + lg/2, row lr, half lg&1.
__device__ __forceinline__ u32x4 fast_ld_b(const uint16_t *planes, int Kd, int ks0, int s, int ns, int lr, int lg) {
  const int total = (Kd + 31) / 32;
  const int ks = (s < ns) ? ks0 + s : total;
  return ld_g(planes + ((size_t)(ks * 2 + (lg >> 1)) * 256 + lr * 16 + (lg & 1) * 8));
}

__device__ __forceinline__ f32x4 fast_mfma(const u32x4 a, const u32x4 b, const f32x4 acc) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}

// Fill the ring with the first kKS weight fragments of tile entry e (this wave's k-steps 0..15).
__device__ __forceinline__ void fast_issue16(Frag16 &A, const FastGemm &g, int wg, int nwg, int e, int wave, int lr,
                                             int lg) {
  const uint16_t *wbase;
  int wrow0, unit;
  if (!fast_tile(g, wg, nwg, e, wbase, wrow0, unit)) return;   // uniform: the ring stays unused
  const int ks0 = wave * fast_ksw(g.Kd);
  const uint16_t *wf = fast_wfrag(wbase, wrow0, g.Kd, lg * 16 + lr);
#pragma unroll
  for (int s = 0; s < kKS; ++s) A.v[s] = fast_ld_a(wf, g.Kd, ks0 + s);
}

// LDS of a GEMM phase: reduction buffer [waves][kMaxT][64 lanes][4] + 8 scales.
constexpr size_t kFastRedBytes = (size_t)kFastWaves * kMaxT * 64 * 16;
constexpr size_t kFastLds = kFastRedBytes + 16 * sizeof(float);

// 1/rms of each row from the producer's partial sums (fixed order: lanes stride, butterfly sum);
// wave w computes row w.  In two halves: the partial sums are REQUESTED first thing in a phase,
// ahead of the activation and weight fragments, and only summed after the first pass of matrix
// products - a loop that waits for each partial sum in turn costs one memory round trip per 64 tiles
// before the first weight is even requested (four round trips, about 3 us, at d_model = 4096).
struct SsqPre {
  float v[4];
};
__device__ __forceinline__ SsqPre fast_row_scales_issue(const FastGemm &g, int wave, int lane) {
  SsqPre s;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int p = lane + u * kWave;
    s.v[u] = (g.ssq && p < g.n_ssq) ? g.ssq[(size_t)p * kSsqStride + wave] : 0.f;
  }
  return s;
}
// Must be followed by a workgroup barrier before scale_s is read.
__device__ __forceinline__ void fast_row_scales_finish(const FastGemm &g, const SsqPre &s, float *scale_s, int wave,
                                                       int lane) {
  if (g.ssq) {
    float t = ((s.v[0] + s.v[1]) + s.v[2]) + s.v[3];
    for (int p = lane + 4 * kWave; p < g.n_ssq; p += kWave) t += g.ssq[(size_t)p * kSsqStride + wave];   // d_model > 4096 only
    t = wave_sum(t);
    if (lane == 0) scale_s[wave] = rsqrtf(t / (float)g.Kd + g.eps);
  } else if (lane == 0) {
    scale_s[wave] = 1.0f;
  }
}

// Reduction over the waves (fixed order) and epilogue of `n_tiles` accumulated tile entries
// starting at list entry e0.  acc tiles were stored to `red` by the caller.
struct EpiPre {           // FEPI_RESID_NORM: this thread's residual and gain pair, requested before the reduction loop
  float2 xo, gn;
};
// What thread `tid` will need in the epilogue of a pass over tile entries e0.. (its output is
// element (jm, 2*c2..2*c2+1) of entry e0 + tid/64).
__device__ __forceinline__ EpiPre fast_epilogue_preload(const FastGemm &g, int wg, int nwg, int e0, int n_tiles, int tid) {
  EpiPre p;
  p.xo = make_float2(0.f, 0.f);
  p.gn = make_float2(0.f, 0.f);
  const int un = tid >> 6, jm = (tid >> 3) & 7, i = 2 * (tid & 7);
  if (g.epi == FEPI_RESID_NORM && un < n_tiles) {
    const uint16_t *wbase;
    int wrow0, unit;
    fast_tile(g, wg, nwg, e0 + un, wbase, wrow0, unit);
    if (jm < g.M) p.xo = *reinterpret_cast<const float2 *>(g.out + (size_t)jm * g.ldo + unit * 16 + i);
    p.gn = *reinterpret_cast<const float2 *>(g.next_gain + unit * 16 + i);
  }
  return p;
}

__device__ __forceinline__ void fast_epilogue(const FastGemm &g, int wg, int nwg, int e0, int n_tiles, const float *red,
                                              const float *scale_s, const EpiPre &pre, int tid) {
  const int EPI = g.epi;
  const int UT = (EPI == FEPI_SWIGLU) ? 2 : 1;
  const int n_units_out = (n_tiles + UT - 1) / UT;
  if (tid < n_units_out * 64) {                 // n_units_out <= kMaxT < 8: one output pair per thread
    const int o = tid;
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
    fast_tile(g, wg, nwg, e0 + t, wbase, wrow0, unit);
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
          a0 = pre.xo.x + s0 * sc;
          a1 = pre.xo.y + s1 * sc;
          *reinterpret_cast<float2 *>(xp) = make_float2(a0, a1);
        }
        float q = a0 * a0 + a1 * a1;       // sum over the tile's 16 columns: 8 adjacent lanes
        q = sum8(q);
        if (c2 == 0) st_dev(g.ssq_out + (size_t)unit * kSsqStride + jm, q);
        a0 *= pre.gn.x;
        a1 *= pre.gn.y;
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

// One resident-B GEMM phase (Kd <= 4096: at most kKS steps per wave) for workgroup `wg` of `nwg`.
// The ring A holds the weight fragments of the tile being multiplied; as soon as a fragment has
// been consumed its registers are refilled with the same step of the next tile, so kKS loads per
// wave are always in flight.  `pre`: the ring already holds tile entry 0 (requested by the caller
// before it waited for this phase's inputs).  On return the ring is free.
__device__ __forceinline__ void fast_gemm_phase(const FastGemm &g, int wg, int nwg, unsigned char *smem, Frag16 &A,
                                                bool pre) {
  float *red = reinterpret_cast<float *>(smem);
  float *scale_s = reinterpret_cast<float *>(smem + kFastRedBytes);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 15, lg = lane >> 4;
  const int my_entries = fast_my_entries(g, wg, nwg);
  if (my_entries == 0) {
    lds_barrier();
    return;
  }
  const SsqPre sp = fast_row_scales_issue(g, wave, lane);
  const int ks0 = wave * fast_ksw(g.Kd), ns = fast_steps(g.Kd, wave);
  Frag16 Bf;
#pragma unroll
  for (int s = 0; s < kKS; ++s) Bf.v[s] = fast_ld_b(g.b, g.Kd, ks0, s, ns, lr, lg);
  for (int e0 = 0; e0 < my_entries; e0 += kMaxT) {
    f32x4 acc[kMaxT];
#pragma unroll
    for (int t = 0; t < kMaxT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    const EpiPre ep = fast_epilogue_preload(g, wg, nwg, e0, min(kMaxT, my_entries - e0), tid);
    if (!(pre && e0 == 0)) fast_issue16(A, g, wg, nwg, e0, wave, lr, lg);
#pragma unroll
    for (int t = 0; t < kMaxT; ++t) {
      if (e0 + t < my_entries) {
        if (t + 1 < kMaxT && e0 + t + 1 < my_entries) {
          const uint16_t *wbase;
          int wrow0, unit;
          fast_tile(g, wg, nwg, e0 + t + 1, wbase, wrow0, unit);
          const uint16_t *wf = fast_wfrag(wbase, wrow0, g.Kd, lane);
#pragma unroll
          for (int s = 0; s < kKS; ++s) {
            acc[t] = fast_mfma(A.v[s], Bf.v[s], acc[t]);
            A.v[s] = fast_ld_a(wf, g.Kd, ks0 + s);
          }
        } else {
#pragma unroll
          for (int s = 0; s < kKS; ++s) acc[t] = fast_mfma(A.v[s], Bf.v[s], acc[t]);
        }
      }
    }
    lds_barrier();
    if (e0 == 0) fast_row_scales_finish(g, sp, scale_s, wave, lane);
#pragma unroll
    for (int t = 0; t < kMaxT; ++t)
      *reinterpret_cast<f32x4 *>(red + ((size_t)(wave * kMaxT + t) * 64 + lane) * 4) = acc[t];
    lds_barrier();
    fast_epilogue(g, wg, nwg, e0, min(kMaxT, my_entries - e0), red, scale_s, ep, tid);
    lds_barrier();
  }
}

// One streaming GEMM phase (long reductions, e.g. the down projection): one tile entry per pass;
// weight and activation fragments stream together through two rings of kKS steps.  `pre`: ring A
// already holds steps 0..kKS-1 of tile entry 0.
__device__ __forceinline__ void fast_gemm_stream_phase(const FastGemm &g, int wg, int nwg, unsigned char *smem, Frag16 &A,
                                                       bool pre) {
  float *red = reinterpret_cast<float *>(smem);
  float *scale_s = reinterpret_cast<float *>(smem + kFastRedBytes);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 15, lg = lane >> 4;
  const int my_entries = fast_my_entries(g, wg, nwg);
  if (my_entries == 0) {
    lds_barrier();
    return;
  }
  const SsqPre sp = fast_row_scales_issue(g, wave, lane);
  const int ksw = fast_ksw(g.Kd), ks0 = wave * ksw, ns = fast_steps(g.Kd, wave);
  // Steps past this wave's share are multiplied with zero records; their weight fragment is read
  // from the wave's own last step (a line it has just fetched), not from the next wave's share.
  const int ks_last = ks0 + max(ns, 1) - 1;
  for (int e = 0; e < my_entries; ++e) {
    const uint16_t *wbase;
    int wrow0, unit;
    fast_tile(g, wg, nwg, e, wbase, wrow0, unit);     // e < my_entries: always a valid tile
    const uint16_t *wf = fast_wfrag(wbase, wrow0, g.Kd, lane);
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    Frag16 Bs;
    const EpiPre ep = fast_epilogue_preload(g, wg, nwg, e, 1, tid);
    if (!(pre && e == 0)) {
#pragma unroll
      for (int s = 0; s < kKS; ++s) A.v[s] = fast_ld_a(wf, g.Kd, min(ks0 + s, ks_last));
    }
#pragma unroll
    for (int s = 0; s < kKS; ++s) Bs.v[s] = fast_ld_b(g.b, g.Kd, ks0, s, ns, lr, lg);
    for (int base = 0; base < ksw; base += kKS) {
      if (base + kKS < ksw) {        // uniform: more steps follow, refill while multiplying
#pragma unroll
        for (int s = 0; s < kKS; ++s) {
          acc = fast_mfma(A.v[s], Bs.v[s], acc);
          A.v[s] = fast_ld_a(wf, g.Kd, min(ks0 + base + kKS + s, ks_last));
          Bs.v[s] = fast_ld_b(g.b, g.Kd, ks0, base + kKS + s, ns, lr, lg);
        }
      } else {
#pragma unroll
        for (int s = 0; s < kKS; ++s) acc = fast_mfma(A.v[s], Bs.v[s], acc);
      }
    }
    lds_barrier();
    if (e == 0) fast_row_scales_finish(g, sp, scale_s, wave, lane);
    *reinterpret_cast<f32x4 *>(red + ((size_t)(wave * kMaxT) * 64 + lane) * 4) = acc;
    lds_barrier();
    fast_epilogue(g, wg, nwg, e, 1, red, scale_s, ep, tid);
    lds_barrier();
  }
}

// ---- embedding: x = E[id] (fp32, owner-private), plane records of x*gain, partial sums of squares ----
// One 16-column tile per call; the first 64 threads of the workgroup work: thread (c2, m).
__device__ __forceinline__ void fast_embed_tile(const int32_t *ids, const uint16_t *emb, int vocab, int d, int M, int tile,
                                                const float *gain, float *x, uint16_t *planes, float *ssq_out, int tid) {
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
  q = sum8(q);
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

constexpr int kAttnR = 10;   // prefix rows a value stream requests at once
constexpr int kAttnKT = 3;   // tiles of 16 prefix keys a wave requests at once (8 waves: 384 keys)

inline size_t fast_attn_lds(int hd, int cap) {
  return sizeof(float) * ((size_t)hd * (1 + 8 + 8) + (size_t)cap + 32 + (size_t)kFastWaves * hd + (size_t)hd) + 16;
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
  u32x4 k[kAttnKT * 4];      // key tiles wave, wave + 8, ... as MFMA A fragments: [tile][k-step of 32 channels]
  uint4 v[kAttnR];
};

// The cache stores a key as HD consecutive bf16: lane l's 16 bytes at channel 32 ks + 8 (l / 16) of key 16 t + l % 16
// are its piece of the A operand of v_mfma_f32_16x16x32_bf16 for key tile t, k-step ks.
template <int HD>
__device__ __forceinline__ u32x4 fast_attn_key_frag(const uint16_t *kc, int tile, int ks, int P, int lane) {
  const int r = 16 * tile + (lane & 15);
  return r < P ? *reinterpret_cast<const u32x4 *>(kc + (size_t)r * HD + 32 * ks + 8 * (lane >> 4)) : u32x4{0u, 0u, 0u, 0u};
}

// Request the first kAttnKT key tiles of this wave and the first kAttnR value rows of this lane's stream (no
// dependence on the current step's activations: may be called before the grid barrier that publishes q/k/v).
template <int HD>
__device__ __forceinline__ void fast_attn_prefetch(const FastAttn &a, int b, int h, AttnPre &pre, int tid) {
  constexpr int LPK = HD / 8, G = kFastThreads / LPK, KS = HD / 32;
  const int li = tid % LPK, g = tid / LPK;
  int P = a.prefix_len[b];
  P = max(0, min(P, a.cap - a.K));
  const bool skip = episode_sits_out(a.skip, a.prefix_len, b, a.K, a.cap);
  const uint16_t *kc = a.k_cache + ((size_t)(b * a.H + h) * a.cap) * HD;
  const uint16_t *vc = a.v_cache + ((size_t)(b * a.H + h) * a.cap) * HD;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), Pk = skip ? 0 : P;
#pragma unroll
  for (int tt = 0; tt < kAttnKT; ++tt)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) pre.k[tt * KS + ks] = fast_attn_key_frag<HD>(kc, wave + 8 * tt, ks, Pk, tid & 63);
#pragma unroll
  for (int u = 0; u < kAttnR; ++u) {
    const int r = u * G + g;
    const bool ok = !skip && r < P;
    pre.v[u] = ok ? *reinterpret_cast<const uint4 *>(vc + (size_t)r * HD + li * 8) : make_uint4(0, 0, 0, 0);
  }
}

// Query jq (< K <= 8) of episode b, head h: one workgroup.  512 threads = 512/(HD/8) key streams;
// `pre` holds the first kAttnR prefix rows of each stream.  The unit rotates the block's keys
// 0..jq itself (fp32, LDS) and appends row jq to the cache; scores live in LDS; the softmax is a
// workgroup reduction; only the stored cache rows are rounded to bf16.  The unit's barriers order LDS
// traffic only (lds_barrier): what the waves exchange goes through LDS, and a full barrier would also wait for
// the acknowledgement of the appended cache rows and of the output records, on the unit's critical path.
struct NoHook {
  __device__ __forceinline__ void operator()() const {}
};
// `after_loads` is called once the unit's q/k/v records are in LDS (nothing of this step's activations
// is requested after that point when the prefix fits the prefetched rows): the persistent kernel
// starts bulk transfers there, behind which the unit's own loads must not queue.
template <int HD, class Hook = NoHook>
__device__ __forceinline__ void fast_attn_unit(const FastAttn &a, int b, int h, int jq, unsigned char *smem,
                                               const AttnPre &pre, int tid, Hook after_loads = Hook()) {
  constexpr int HALF = HD / 2;
  constexpr int LPK = HD / 8;
  constexpr int G = kFastThreads / LPK;
  constexpr int TPH = HD / 16;                      // 16-column tiles per head
  float *qs = reinterpret_cast<float *>(smem);     // [HD] rotated, scaled query
  float *kb = qs + HD;                              // [8][HD] rotated keys of the block
  float *vb = kb + 8 * HD;                          // [8][HD] values of the block
  float *sc = vb + 8 * HD;                          // [cap]
  float *wred = sc + a.cap;                         // [32] per-wave partials
  float *ored = wred + 32;                          // [waves][HD]
  uint16_t *qh = reinterpret_cast<uint16_t *>((reinterpret_cast<uintptr_t>(ored + kFastWaves * HD) + 15) & ~(uintptr_t)15);
                                                                         // [HD] bf16 head of the query (16-byte aligned) ...
  uint16_t *ql = qh + HD;                                                // [HD] ... and bf16 tail
  const int lane = tid & 63, wave = tid >> 6;
  const int K = a.K, d = a.d, cap = a.cap;
  const int m = b * K + jq;                         // activation row of this query
  const int li = tid % LPK, g = tid / LPK;
  if (episode_sits_out(a.skip, a.prefix_len, b, K, cap)) {
    for (int c2 = tid; c2 < HALF; c2 += kFastThreads) {     // zero this row's slice of the records
      const int c = c2 * 2;
      uint32_t *rec = reinterpret_cast<uint32_t *>(a.o_planes + (size_t)(h * TPH + c / 16) * 256);
      st_dev(rec + (m * 16 + (c & 15)) / 2, 0u);
      st_dev(rec + ((m + 8) * 16 + (c & 15)) / 2, 0u);
    }
    after_loads();
    return;
  }
  int P = a.prefix_len[b];
  P = max(0, min(P, cap - K));
  uint16_t *kc = a.k_cache + ((size_t)(b * a.H + h) * cap) * HD;
  uint16_t *vc = a.v_cache + ((size_t)(b * a.H + h) * cap) * HD;
  const int n_t = d / 16;

  // rotate keys 0..jq into LDS, copy values, rotate + scale the query; append row jq (bf16)
  for (int idx = tid; idx < (jq + 1) * HALF; idx += kFastThreads) {
    const int j = idx / HALF, i = idx - j * HALF;
    const int mj = b * K + j;
    const float *qa = a.qkv + (size_t)(h * TPH + i / 16) * 128 + mj * 16 + (i & 15);
    const float *qb = a.qkv + (size_t)(h * TPH + (i + HALF) / 16) * 128 + mj * 16 + ((i + HALF) & 15);
    const size_t ko = (size_t)n_t * 128, vo = (size_t)2 * n_t * 128;
    const float2 cs = a.rope[(size_t)(P + j) * HALF + i];
    const float k1 = qa[ko], k2 = qb[ko], v1 = qa[vo], v2 = qb[vo];
    const float kr1 = k1 * cs.x - k2 * cs.y, kr2 = k2 * cs.x + k1 * cs.y;
    kb[j * HD + i] = kr1;
    kb[j * HD + i + HALF] = kr2;
    vb[j * HD + i] = v1;
    vb[j * HD + i + HALF] = v2;
    if (j == jq) {
      const float q1 = qa[0], q2 = qb[0];
      const float r1 = (q1 * cs.x - q2 * cs.y) * a.scale, r2 = (q2 * cs.x + q1 * cs.y) * a.scale;
      qs[i] = r1;
      qs[i + HALF] = r2;
      uint32_t h1, l1, h2, l2;
      split_bf16(r1, h1, l1);
      split_bf16(r2, h2, l2);
      qh[i] = (uint16_t)h1; ql[i] = (uint16_t)l1;
      qh[i + HALF] = (uint16_t)h2; ql[i + HALF] = (uint16_t)l2;
      uint16_t *kr = kc + (size_t)(P + j) * HD;
      kr[i] = (uint16_t)f32_to_bf16_bits(kr1);
      kr[i + HALF] = (uint16_t)f32_to_bf16_bits(kr2);
      uint16_t *vr = vc + (size_t)(P + j) * HD;
      vr[i] = (uint16_t)f32_to_bf16_bits(v1);
      vr[i + HALF] = (uint16_t)f32_to_bf16_bits(v2);
    }
  }
  lds_barrier();
  after_loads();
  float qf[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) qf[i] = qs[li * 8 + i];

  auto score_row = [&](const float (&kf)[8], int r) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) t = fmaf(qf[i], kf[i], t);
    t = LPK == 16 ? sum16(t) : sum8(t);
    if (li == 0) sc[r] = t;
  };
  // ---- pass 1: scores of the prefix keys on the matrix cores, then of the block's keys 0..jq with FMAs ----
  // A = a tile of 16 cached keys (bf16, straight from the cache), B = the query: its bf16 head in column 0 and
  // its bf16 tail in column 1 (q = head + tail to 16 mantissa bits; the products are exact in fp32), the other
  // columns zero.  Output element (key 4 (l / 16) + i, column l % 16) is register i of lane l: lanes 0, 16, 32, 48
  // add their neighbour's column and store four scores each.
  {
    constexpr int KS = HD / 32;
    const int lr = lane & 15, lg = lane >> 4, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    u32x4 bq[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const u32x4 qv = *reinterpret_cast<const u32x4 *>((lr == 0 ? qh : ql) + 32 * ks + 8 * lg);
      bq[ks] = lr < 2 ? qv : u32x4{0u, 0u, 0u, 0u};
    }
    const int n_kt = (P + 15) >> 4;
    auto emit = [&](int tile, const f32x4 acc) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float t = acc[i] + dpp_move<kDppNext>(acc[i]);
        const int r = 16 * tile + 4 * lg + i;
        if (lr == 0 && r < P) sc[r] = t;
      }
    };
#pragma unroll
    for (int tt = 0; tt < kAttnKT; ++tt) {
      const int tile = wv + 8 * tt;
      if (tile < n_kt) {                                  // wave-uniform
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc = fast_mfma(pre.k[tt * KS + ks], bq[ks], acc);
        emit(tile, acc);
      }
    }
    for (int tile = wv + 8 * kAttnKT; tile < n_kt; tile += 8) {
      u32x4 kf[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[ks] = fast_attn_key_frag<HD>(kc, tile, ks, P, lane);
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc = fast_mfma(kf[ks], bq[ks], acc);
      emit(tile, acc);
    }
  }
  if (g <= jq) {
    float kf[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) kf[i] = kb[g * HD + li * 8 + i];
    score_row(kf, P + g);
  }
  lds_barrier();
  const int nkeys = P + jq + 1;
  // ---- softmax over the visible keys (workgroup reduction) ----
  float mx = -INFINITY;
  for (int r = tid; r < nkeys; r += kFastThreads) mx = fmaxf(mx, sc[r]);
  mx = wave_max(mx);
  if (lane == 0) wred[wave] = mx;
  lds_barrier();
  mx = wred[0];
#pragma unroll
  for (int w = 1; w < kFastWaves; ++w) mx = fmaxf(mx, wred[w]);
  float sum = 0.f;
  for (int r = tid; r < nkeys; r += kFastThreads) {
    const float pr = expf(sc[r] - mx);
    sc[r] = pr;
    sum += pr;
  }
  sum = wave_sum(sum);
  if (lane == 0) wred[8 + wave] = sum;
  lds_barrier();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < kFastWaves; ++w) tot += wred[8 + w];
  const float inv_l = 1.0f / tot;
  // ---- pass 2: weighted sum of the value rows ----
  float o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = 0.f;
#pragma unroll
  for (int u = 0; u < kAttnR; ++u) {
    const int r = u * G + g;
    if (r < P) {
      float vf[8];
      unpack8(pre.v[u], vf);
      const float pr = sc[r];
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = fmaf(pr, vf[i], o[i]);
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
        const float pr = sc[r];
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = fmaf(pr, vf[i], o[i]);
      }
    }
  }
  if (g <= jq) {
    const float pr = sc[P + g];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = fmaf(pr, vb[g * HD + li * 8 + i], o[i]);
  }
#pragma unroll
  for (int off = LPK; off < kWave; off <<= 1)
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] += __shfl_xor(o[i], off, kWave);
  if (lane < LPK) {
#pragma unroll
    for (int i = 0; i < 8; ++i) ored[wave * HD + lane * 8 + i] = o[i];
  }
  lds_barrier();
  for (int c2 = tid; c2 < HALF; c2 += kFastThreads) {      // two adjacent channels per thread
    const int c = c2 * 2;
    float t0 = 0.f, t1 = 0.f;
#pragma unroll
    for (int w = 0; w < kFastWaves; ++w) {
      t0 += ored[w * HD + c];
      t1 += ored[w * HD + c + 1];
    }
    uint32_t h0, l0, h1, l1;
    split_bf16(t0 * inv_l, h0, l0);
    split_bf16(t1 * inv_l, h1, l1);
    uint32_t *rec = reinterpret_cast<uint32_t *>(a.o_planes + (size_t)(h * TPH + c / 16) * 256);
    st_dev(rec + (m * 16 + (c & 15)) / 2, h0 | (h1 << 16));
    st_dev(rec + ((m + 8) * 16 + (c & 15)) / 2, l0 | (l1 << 16));
  }
  lds_barrier();
}

// ---- one launch per phase ---------------------------------------------------------------------

// KC names the projection (a kernel class id); it changes no code, it only gives each projection
// its own kernel symbol so that profilers report them apart.
template <int KC>
__global__ __launch_bounds__(kFastThreads) void fast_gemm_kernel(FastGemm g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  Frag16 A;
  // The first weight fragments are requested before anything else: the phase's loop over passes begins
  // with a wait for every request made so far (the compiler cannot count requests across the loop's
  // back edge), so whatever is requested after that wait starts one memory round trip late.
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  fast_issue16(A, g, blockIdx.x, gridDim.x, 0, wave, lane & 15, lane >> 4);
  fast_gemm_phase(g, blockIdx.x, gridDim.x, smem, A, true);
}

template <int KC>
__global__ __launch_bounds__(kFastThreads) void fast_gemm_stream_kernel(FastGemm g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  Frag16 A;
  fast_gemm_stream_phase(g, blockIdx.x, gridDim.x, smem, A, false);
}

template <int HD>
__global__ __launch_bounds__(kFastThreads) void fast_attn_kernel(FastAttn a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  AttnPre pre;
  const int b = blockIdx.y / a.K, jq = blockIdx.y - b * a.K;     // grid (H, batch*K)
  fast_attn_prefetch<HD>(a, b, blockIdx.x, pre, threadIdx.x);
  fast_attn_unit<HD>(a, b, blockIdx.x, jq, smem, pre, threadIdx.x);
}

__global__ __launch_bounds__(64) void fast_embed_kernel(const int32_t *ids, const uint16_t *emb, int vocab, int d, int M,
                                                       const float *gain, float *x, uint16_t *planes, float *ssq_out) {
  fast_embed_tile(ids, emb, vocab, d, M, blockIdx.x, gain, x, planes, ssq_out, threadIdx.x);
}

}  // namespace heisd
