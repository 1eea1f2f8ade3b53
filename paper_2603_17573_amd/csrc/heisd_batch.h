// Verify forward for M = batch*K > 8 rows (several episodes verified in one pass: paper Sec. 2.2
// "parallel verification", batched over episodes).
//
// Same exchange format as the M <= 8 kernels, widened by a column-tile index: the activation rows
// are cut into column tiles of 8 rows, and for every 16-wide k-tile and every column tile there is
// one 512-byte record [16][16] of bf16 (rows 0-7 = bf16 heads of the 8 activation rows, rows
// 8-15 = tails, columns = 16 consecutive k), laid out [k-tile][column tile][16][16].  A record row
// is a piece of one column of the MFMA B operand, so a lane loads its B fragment with one 16-byte
// read.  Producers split every element once; no consumer converts anything.
//
// GEMM: a workgroup owns a list of 16-row weight tiles and multiplies up to NT of them per pass.
// Its 8 waves are arranged MW x KW: MW groups of MC column tiles each, KW shares of the k-steps, so
// few rows mean a deep k split (every wave streams different weight bytes) and many rows mean all
// waves multiply the same weight fragments with different rows.  Weight fragments go from global
// memory straight into the MFMA A layout through a ring kBatRing k-steps deep, and the B fragments
// travel through the same ring.  The KW partial sums meet in LDS in a fixed order.  RMSNorm is
// folded in as in the M <= 8 kernels: records hold x*gain, a small kernel turns per-tile partial sums of squares
// into 1/rms per row, and the consuming GEMM scales its output rows.
#pragma once
#include "heisd_fast.h"

namespace heisd {

constexpr int kBatThreads = 512;
constexpr int kBatWaves = 8;
constexpr int kBatRing = 3;       // k-steps of fragments (weights and activations) requested ahead

struct BatGemm {
  int epi;                // FEPI_STORE_ROWS, FEPI_RESID_NORM or FEPI_SWIGLU
  const uint16_t *w[3];   // weight segments, bf16, in the packed fragment order of fast_pack_weights
  int seg_tiles;          // n-tiles per segment
  int n_units;            // n-tiles, or (gate, up) pairs for FEPI_SWIGLU
  int Kd;
  const uint16_t *b;      // records [2*ceil(Kd/32) + 2][CTS][16][16]; the k-tiles past Kd/16 are all zero
  int CT;                 // column tiles in use = ceil(M/8)
  int CTS;                // column tiles allocated per k-tile (the stride; fixed at init, so that the
                          // zero k-tile stays where it is when M changes between calls)
  int M;
  // A projection of a normalised input (QKV, gate/up, LM head) multiplies its output rows by 1/rms.  The
  // scales are computed inside the consuming launch (bat_scales_produce) and handed to its epilogues
  // through epoch-tagged words (bat_row_scale); scale_tag == nullptr: the input is not normalised.
  const float *ssq_in;    // [ssq_tiles][CTS*8] partial sums of squares of the raw input rows
  int ssq_tiles;          // Kd / 16
  float eps;
  unsigned long long *scale_tag;   // [CTS*8] low word: bits of 1/rms of the row, high word: epoch of the launch that wrote it
  unsigned scale_epoch;   // this launch's epoch (unique per consuming projection; never 0)
  unsigned *err;          // device error word (a scale that never arrives raises kErrBarrier)
  int scale_spin;         // polls an epilogue makes for a row's word before it gives up (kScaleSpin unless a test lowers it)
  int scale_skip;         // != 0 (tests of the give-up path only): the launch does not produce the words
  float *out;             // STORE_ROWS: [M][ldo]; RESID_NORM: residual stream x [M][ldo], updated in place
  int ldo;
  const float *next_gain; // RESID_NORM: gain of the norm that consumes x next
  uint16_t *o_planes;     // RESID_NORM / SWIGLU: records [unit][CTS][16][16]
  float *ssq_out;         // RESID_NORM: [n_units][CTS*8] partial sums of squares of the new x
  int single;             // activations as ONE bf16 each (bat_gemm_wide, bat_gemm_ns, bat_split_finish, bat_embed and the
                          // attention kernels; not bat_gemm): a record then holds the bf16 values of 16 activation rows, a column tile
                          // is 16 rows, CT = ceil(M/16), and the 16 columns of an accumulator tile are 16 rows'
                          // results (nothing to add up).  0: head + tail of 8 rows, as described above
  int MW;                 // bat_gemm: waves across column tiles (1, 2, 4 or 8); the other 8/MW split k
  int NW;                 // bat_gemm_ns: computing waves across weight tiles (6 or 3); set by the launcher
};

// 1/rms of every row in use, by the first workgroups of the launch that consumes them: wave w of workgroup
// b takes rows 8 b + w, 8 b + w + 8 * workgroups, ...; the partial sums are added in a fixed order (lanes
// stride over the producer's tiles, butterfly sum).  Called first thing by every GEMM kernel, before any
// workgroup leaves: the epilogues of ALL workgroups wait for these words, and the workgroups with the lowest
// ids are dispatched first and wait for nobody, so the wait ends.  A launch that only stores partial sums
// for a finishing launch produces the scales for that launch (same epoch, already there when it starts).
constexpr int kScaleSpin = 1 << 20;
__device__ __forceinline__ void bat_scales_produce(const BatGemm &g) {
  if (!g.scale_tag || g.scale_skip) return;
  const int rows = g.CT * (g.single ? 16 : 8), stride = g.CTS * 8;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  int m = blockIdx.x * nw + wave;
  if (m >= rows) return;                                     // uniform over the wave
  for (; m < rows; m += gridDim.x * nw) {
    float t = 0.f;
    for (int p = lane; p < g.ssq_tiles; p += kWave) t += g.ssq_in[(size_t)p * stride + m];
    t = wave_sum(t);
    const unsigned long long v = ((unsigned long long)g.scale_epoch << 32) | __float_as_uint(rsqrtf(t / (float)g.Kd + g.eps));
    if (lane == 0) __hip_atomic_store(g.scale_tag + m, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  wait_vmcnt_all();                                          // nothing of this is pending when the counted waits begin
}
// The scale of row m (bounded wait for this launch's epoch; 1 if the input is not normalised).
__device__ __forceinline__ float bat_row_scale(const BatGemm &g, int m) {
  if (!g.scale_tag) return 1.0f;
  if (m >= g.CT * (g.single ? 16 : 8)) return 0.f;
  for (int spin = 0; spin < g.scale_spin; ++spin) {
    const unsigned long long v = __hip_atomic_load(g.scale_tag + m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((unsigned)(v >> 32) == g.scale_epoch) return __uint_as_float((unsigned)v);
    __builtin_amdgcn_s_sleep(4);
  }
  __hip_atomic_fetch_or(g.err, kErrBarrier, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return 0.f;
}

template <int MC>
constexpr size_t bat_lds_bytes() {
  return (size_t)2 * kBatWaves * MC * 64 * 16;     // two tiles (gate and up) of per-wave accumulators
}

// Tile entry e of workgroup wg: weight rows and output unit.
__device__ __forceinline__ void bat_tile(const BatGemm &g, int wg, int nwg, int e, const uint16_t *&wbase, int &wrow0,
                                         int &unit) {
  if (g.epi == FEPI_SWIGLU) {
    unit = wg + (e >> 1) * nwg;
    wbase = (e & 1) ? g.w[1] : g.w[0];
    wrow0 = unit * 16;
    return;
  }
  unit = wg + e * nwg;
  const int seg = unit / g.seg_tiles;
  wbase = seg == 0 ? g.w[0] : (seg == 1 ? g.w[1] : g.w[2]);
  wrow0 = (unit - seg * g.seg_tiles) * 16;
}

// The projection's epilogue for one output pair: row m = 8*ct + jm, columns 2*c2, 2*c2+1 of unit
// `unit`; (s0, s1) = the sums, (u0, u1) = the sums of the up tile (SwiGLU).  The 8 lanes c2 = 0..7 of
// a row must call this together (they add up the row's partial sum of squares).  In two halves, so
// that a caller with many pairs can request everything they read before the first store (a load
// after a store to memory the compiler cannot tell apart waits for that store).
struct EmitPre {
  float sc;       // 1/rms of the row (1 if the projection's input is not normalised)
  float2 xo;      // RESID_NORM: the residual stream's old values
  float2 gn;      // RESID_NORM: the next norm's gains
};
// hh: with single-bf16 activations a column tile has 16 rows and lane (jm, c2) serves rows jm (hh = 0) and jm + 8
// (hh = 1) of it, from accumulator columns jm and jm + 8; otherwise hh = 0.
__device__ __forceinline__ int bat_row_of(const BatGemm &g, int ct, int jm, int hh) {
  return g.single ? ct * 16 + hh * 8 + jm : ct * 8 + jm;
}
// tab (optional): the scales of rows tab_m0 .. tab_m0 + kScaleTab - 1 in LDS, read once by the caller (a wait
// for a tagged word is a round trip to the L2, the table is not).
constexpr int kScaleTab = 128;
__device__ __forceinline__ EmitPre bat_emit_load(const BatGemm &g, int unit, int ct, int jm, int c2, int hh = 0,
                                                 const float *tab = nullptr, int tab_m0 = 0) {
  const int i = 2 * c2, m = bat_row_of(g, ct, jm, hh);
  EmitPre p;
  p.sc = !g.scale_tag ? 1.0f : (tab ? tab[max(0, min(m - tab_m0, kScaleTab - 1))] : bat_row_scale(g, m));
  p.xo = make_float2(0.f, 0.f);
  p.gn = make_float2(0.f, 0.f);
  if (g.epi == FEPI_RESID_NORM) {
    if (m < g.M) p.xo = *reinterpret_cast<const float2 *>(g.out + (size_t)m * g.ldo + unit * 16 + i);
    p.gn = *reinterpret_cast<const float2 *>(g.next_gain + unit * 16 + i);
  }
  return p;
}
__device__ __forceinline__ void bat_emit_apply(const BatGemm &g, int unit, int ct, int jm, int c2, float s0, float s1,
                                               float u0, float u1, const EmitPre &pre, int hh = 0) {
  const int i = 2 * c2;
  const int m = bat_row_of(g, ct, jm, hh);
  const bool live = m < g.M;
  const float sc = pre.sc;
  if (g.epi == FEPI_STORE_ROWS) {
    if (live) *reinterpret_cast<float2 *>(g.out + (size_t)m * g.ldo + unit * 16 + i) = make_float2(s0 * sc, s1 * sc);
    return;
  }
  float a0 = 0.f, a1 = 0.f;
  if (g.epi == FEPI_SWIGLU) {
    const float g0 = s0 * sc, g1 = s1 * sc;
    if (live) {
      a0 = g0 / (1.0f + expf(-g0)) * (u0 * sc);
      a1 = g1 / (1.0f + expf(-g1)) * (u1 * sc);
    }
  } else {
    if (live) {
      a0 = pre.xo.x + s0 * sc;
      a1 = pre.xo.y + s1 * sc;
      *reinterpret_cast<float2 *>(g.out + (size_t)m * g.ldo + unit * 16 + i) = make_float2(a0, a1);
    }
    float q = a0 * a0 + a1 * a1;          // over the tile's 16 columns: 8 adjacent lanes
    q = sum8(q);
    if (c2 == 0) g.ssq_out[(size_t)unit * (g.CTS * 8) + m] = q;
    a0 *= pre.gn.x;
    a1 *= pre.gn.y;
  }
  uint32_t h0, l0, h1, l1;
  split_bf16(a0, h0, l0);
  split_bf16(a1, h1, l1);
  uint32_t *rec = reinterpret_cast<uint32_t *>(g.o_planes + ((size_t)unit * g.CTS + ct) * 256);
  if (g.single) {
    rec[((jm + 8 * hh) * 16 + i) / 2] = h0 | (h1 << 16);         // the value rounded to bf16, nothing else
  } else {
    rec[(jm * 16 + i) / 2] = h0 | (h1 << 16);
    rec[((jm + 8) * 16 + i) / 2] = l0 | (l1 << 16);
  }
}
__device__ __forceinline__ void bat_emit(const BatGemm &g, int unit, int ct, int jm, int c2, float s0, float s1, float u0,
                                         float u1, int hh = 0, const float *tab = nullptr, int tab_m0 = 0) {
  const EmitPre pre = bat_emit_load(g, unit, ct, jm, c2, hh, tab, tab_m0);
  bat_emit_apply(g, unit, ct, jm, c2, s0, s1, u0, u1, pre, hh);
}

// First column tile of wave group mw in the block that starts at cb: groups that would run past
// the last tile are moved back so that every tile they read exists (tiles are then computed twice;
// the epilogue takes each from the group bat_group_of names).  Needs CTS >= MC.
template <int MC>
__device__ __forceinline__ int bat_c0(int cb, int mw, int CT) {
  return max(0, min(cb + mw * MC, CT - MC));
}

// One output pair (row rr of this workgroup's row block, columns 2*c2, 2*c2+1) of tile entry e:
// sum of the k shares and of head and tail columns, then the projection's epilogue.
template <int MC>
__device__ __forceinline__ void bat_epilogue(const BatGemm &g, int wg, int nwg, int e, int cb, const float *red) {
  const int MW = g.MW, KW = kBatWaves / MW;
  const int pairs = MW * MC * 64;                        // 8 rows x 8 pairs per column tile
  const uint16_t *wbase;
  int wrow0, unit;
  bat_tile(g, wg, nwg, e, wbase, wrow0, unit);
  for (int o = threadIdx.x; o < pairs; o += kBatThreads) {
    const int c2 = o & 7, jm = (o >> 3) & 7, cc = o >> 6;
    const int ct = cb + cc;
    if (ct >= g.CT) continue;                                          // uniform over the 8 lanes of a row
    const int mw = cc / MC, c = ct - bat_c0<MC>(cb, mw, g.CT);         // the wave group that holds tile ct, and where
    const int i = 2 * c2;
    const int l_hi = (i >> 2) * 16 + jm, r = i & 3;
    float s0 = 0.f, s1 = 0.f, u0 = 0.f, u1 = 0.f;
    for (int kw = 0; kw < KW; ++kw) {
      const float *p = red + ((size_t)((kw * MW + mw) * MC + c) * 64) * 4;
      const float2 a = *reinterpret_cast<const float2 *>(p + l_hi * 4 + r);
      const float2 b = *reinterpret_cast<const float2 *>(p + (l_hi + 8) * 4 + r);
      s0 += a.x + b.x;
      s1 += a.y + b.y;
      if (g.epi == FEPI_SWIGLU) {
        const float *q = p + (size_t)kBatWaves * MC * 256;
        const float2 cg = *reinterpret_cast<const float2 *>(q + l_hi * 4 + r);
        const float2 dg = *reinterpret_cast<const float2 *>(q + (l_hi + 8) * 4 + r);
        u0 += cg.x + dg.x;
        u1 += cg.y + dg.y;
      }
    }
    bat_emit(g, unit, ct, jm, c2, s0, s1, u0, u1);
  }
}

template <int MC, int NT>
__global__ __launch_bounds__(kBatThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void bat_gemm(BatGemm g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float *red = reinterpret_cast<float *>(smem);
  const int wg = blockIdx.x, nwg = gridDim.x;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lr = lane & 15, lg = lane >> 4;
  bat_scales_produce(g);
  const int MW = g.MW, KW = kBatWaves / MW;
  const int mw = wave % MW, kw = wave / MW;
  const int total = (g.Kd + 31) / 32;
  const int ksw = (total + KW - 1) / KW;
  const int ks0 = kw * ksw;
  const int ns = max(0, min(ksw, total - ks0));
  const bool swiglu = g.epi == FEPI_SWIGLU;
  const int UT = swiglu ? 2 : 1;
  const int my_units = g.n_units > wg ? (g.n_units - wg + nwg - 1) / nwg : 0;
  const int my_entries = my_units * UT;
  if (my_entries == 0) return;
  const size_t bstep = (size_t)2 * g.CTS * 256;          // elements per k-step (two k-tiles)

  for (int cb = 0; cb < g.CT; cb += MW * MC) {            // more than MW*MC column tiles: weights are streamed again
    // this lane's piece of the B fragment of column tile c0 + c at k-step ks: bfrag + ks*bstep + c*256
    const uint16_t *bfrag = g.b + ((size_t)(lg >> 1) * g.CTS + bat_c0<MC>(cb, mw, g.CT)) * 256 + lr * 16 + (lg & 1) * 8;
    for (int e0 = 0; e0 < my_entries; e0 += NT) {
      const uint16_t *wf[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const uint16_t *wbase;
        int wrow0, unit;
        bat_tile(g, wg, nwg, min(e0 + t, my_entries - 1), wbase, wrow0, unit);
        wf[t] = fast_wfrag(wbase, wrow0, g.Kd, lane);
      }
      f32x4 acc[NT][MC];
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int c = 0; c < MC; ++c) acc[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
      // One ring for both operands, kBatRing k-steps deep: the fragments of step s + kBatRing are
      // requested into the registers step s has just released.  (Loads return in order, so the two
      // operands must be requested equally far ahead: a B fragment requested late would make the
      // wait for it cover every weight fragment requested before it.)
      // The loop body has no branch: steps past this wave's share read the all-zero k-step of the
      // record buffer (and a clamped, valid weight address), so the trip count can be rounded up
      // and the compiler's count of outstanding loads stays exact across the back edge.
      u32x4 A[kBatRing][NT], B[kBatRing][MC];
      if (ns > 0) {
#pragma unroll
        for (int u = 0; u < kBatRing; ++u) {
          const int ksb = u < ns ? ks0 + u : total;
#pragma unroll
          for (int t = 0; t < NT; ++t) A[u][t] = fast_ld_a(wf[t], g.Kd, ks0 + u);
#pragma unroll
          for (int c = 0; c < MC; ++c) B[u][c] = ld_g(bfrag + (size_t)ksb * bstep + c * 256);
          __builtin_amdgcn_sched_barrier(0);        // same request order as in the loop body
        }
        for (int s0 = 0; s0 < ns; s0 += kBatRing) {
#pragma unroll
          for (int u = 0; u < kBatRing; ++u) {
            const int sn = s0 + u + kBatRing;
            const int ksn = sn < ns ? ks0 + sn : total;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
#pragma unroll
              for (int c = 0; c < MC; ++c) acc[t][c] = fast_mfma(A[u][t], B[u][c], acc[t][c]);
              A[u][t] = fast_ld_a(wf[t], g.Kd, ks0 + sn);
            }
#pragma unroll
            for (int c = 0; c < MC; ++c) B[u][c] = ld_g(bfrag + (size_t)ksn * bstep + c * 256);
            __builtin_amdgcn_sched_barrier(0);      // the requests stay in this step: the scheduler may not
          }                                         // sink them towards their use to save registers
        }
      }
      // the KW partial sums meet in LDS; SwiGLU needs gate and up together, the others go tile by tile
      if (swiglu) {
        __syncthreads();
#pragma unroll
        for (int t = 0; t < 2 && t < NT; ++t)
#pragma unroll
          for (int c = 0; c < MC; ++c)
            *reinterpret_cast<f32x4 *>(red + ((size_t)((t * kBatWaves + wave) * MC + c) * 64 + lane) * 4) = acc[t][c];
        __syncthreads();
        bat_epilogue<MC>(g, wg, nwg, e0, cb, red);
      } else {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          if (e0 + t < my_entries) {
            __syncthreads();
#pragma unroll
            for (int c = 0; c < MC; ++c)
              *reinterpret_cast<f32x4 *>(red + ((size_t)(wave * MC + c) * 64 + lane) * 4) = acc[t][c];
            __syncthreads();
            bat_epilogue<MC>(g, wg, nwg, e0 + t, cb, red);
          }
        }
      }
    }
  }
}

// ---- M <= 64 rows: the waves split the weight tiles and share the activation fragments through LDS ----
// With few rows bat_gemm gives every wave its own part of the reduction, so every workgroup reads ALL
// activation records once per pass (0.9 MB at M = 56 against 0.4 MB of weights): L2 traffic, not HBM,
// bounds it.  Here kNsCompute waves of a workgroup multiply different weight tiles over the same
// k-steps (arranged NW tiles x KW shares of the reduction), and the B fragments of those steps are
// brought into LDS once per workgroup, double buffered in chunks of kNsSlots k-steps, by the other
// two waves with direct global -> LDS transfers.  The split of roles matters: a wave's memory
// operations complete in order, so a wave that streamed weights AND waited for B transfers would
// drain its weight requests at every chunk; the computing waves meet the filling waves only at
// workgroup barriers.  Record traffic drops with the number of workgroups, n_units/NW.  One unit
// per computing wave and pass: a tile, or a (gate, up) pair.
constexpr int kNsSlots = 4;                       // k-steps (over all shares) per chunk
constexpr int kNsBufs = 4;                        // chunks resident in LDS: three in flight while one is multiplied
constexpr int kNsCompute = 6;
template <int MC>
constexpr size_t bat_ns_lds_bytes() {
  return (size_t)kNsBufs * kNsSlots * MC * 1024   // the ring; reused for the waves' accumulators at the end
         + kScaleTab * sizeof(float);             // the rows' 1/rms
}

template <int MC, int NT, int KW>
__global__ __launch_bounds__(kBatThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void bat_gemm_ns(BatGemm g) {
  constexpr int NW = kNsCompute / KW;
  constexpr int S = kNsSlots / KW;                  // k-steps per chunk and share
  constexpr int R = 8 / NT;                         // k-steps of weight fragments requested ahead (deeper measured slower)
  constexpr int NF = kBatWaves - kNsCompute;        // filling waves
  static_assert(R % S == 0, "a ring revolution is a whole number of chunks");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const uint32_t smem_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
  const int wg = blockIdx.x, nwg = gridDim.x;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lr = lane & 15, lg = lane >> 4;
  bat_scales_produce(g);
  const bool filler = wave >= kNsCompute;
  const int nw = wave % NW, kw = filler ? 0 : wave / NW;
  const int total = (g.Kd + 31) / 32;
  const int ksw = (total + KW - 1) / KW;
  const int ks0 = kw * ksw;
  const int ns = max(0, min(ksw, total - ks0));
  const int ks_last = min(ks0 + max(ns, 1) - 1, total - 1);
  const int n_chunks = (ksw + S - 1) / S;
  const int n_groups = (g.n_units + NW - 1) / NW;
  const bool swiglu = g.epi == FEPI_SWIGLU;
  const uint16_t *bsrc = g.b + (size_t)(lg >> 1) * g.CTS * 256 + lr * 16 + (lg & 1) * 8;     // + ks*bstep + ct*256
  const size_t bstep = (size_t)2 * g.CTS * 256;
  // filling wave f moves slots f, f+NF, ... of a chunk: slot = share*S + step.  Chunks past the end are moved
  // too (from the all-zero k-step), so that the count of transfers in flight is the same at every wait.
  constexpr int OPS = kNsSlots / NF * MC;           // transfers per filling wave and chunk
  static_assert(kNsSlots % NF == 0 && sizeof(float) * kNsCompute * NT * MC * 256 <= bat_ns_lds_bytes<MC>(), "ring arithmetic");
  auto fill = [&](int c) __attribute__((always_inline)) {
    const int buf = c % kNsBufs;
#pragma unroll 1
    for (int slot = wave - kNsCompute; slot < kNsSlots; slot += NF) {     // rolled: unrolled it takes the registers the products need
      const int skw = slot / S, j = c * S + slot % S;
      const int s_ns = max(0, min(ksw, total - skw * ksw));
      const int ks = j < s_ns ? skw * ksw + j : total;          // past the share: the all-zero k-step
      const uint16_t *src = bsrc + (size_t)ks * bstep;
#pragma unroll
      for (int ct = 0; ct < MC; ++ct)
        lds_dma16(src + ct * 256, __builtin_amdgcn_readfirstlane(smem_lds + (uint32_t)(((buf * kNsSlots + slot) * MC + ct) * 1024)));
    }
  };

  for (int grp = wg; grp < n_groups; grp += nwg) {
    const int unit = grp * NW + nw;
    const bool valid = !filler && unit < g.n_units;
    const int ucl = unit < g.n_units ? unit : g.n_units - 1;     // surplus waves multiply a valid tile, results dropped
    const uint16_t *wf[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const uint16_t *wbase;
      int wrow0;
      if (swiglu) {
        wbase = t ? g.w[1] : g.w[0];
        wrow0 = ucl * 16;
      } else {
        const int seg = ucl / g.seg_tiles;
        wbase = seg == 0 ? g.w[0] : (seg == 1 ? g.w[1] : g.w[2]);
        wrow0 = (ucl - seg * g.seg_tiles) * 16;
      }
      wf[t] = fast_wfrag(wbase, wrow0, g.Kd, lane);
    }
    f32x4 acc[NT][MC];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int c = 0; c < MC; ++c) acc[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (filler) {
      wait_vmcnt_all();                               // no wait of the compiler's between the transfers
#pragma unroll 1
      for (int c = 0; c < kNsBufs - 1; ++c) fill(c);
      wait_vmcnt<(kNsBufs - 2) * OPS>();              // chunk 0 has arrived
      lds_barrier();
      for (int c = 0; c < n_chunks; ++c) {
        fill(c + kNsBufs - 1);                        // into the buffer chunk c-1 was read from
        wait_vmcnt<(kNsBufs - 2) * OPS>();            // chunk c+1 has arrived
        lds_barrier();
      }
      wait_vmcnt<0>();                                // nothing may land in LDS after the buffers change hands
    } else {
      u32x4 A[R][NT];
#pragma unroll
      for (int u = 0; u < R; ++u)
#pragma unroll
        for (int t = 0; t < NT; ++t) A[u][t] = fast_ld_a(wf[t], g.Kd, min(ks0 + u, ks_last));
      lds_barrier();                                  // chunk 0 is in LDS
      for (int c0 = 0; c0 < n_chunks; c0 += R / S) {
#pragma unroll
        for (int cc = 0; cc < R / S; ++cc) {
          const int c = c0 + cc;
          if (c < n_chunks) {
            const unsigned char *bl = smem + ((size_t)((c % kNsBufs) * kNsSlots + kw * S) * MC) * 1024 + lane * 16;
#pragma unroll
            for (int s = 0; s < S; ++s) {
              const int u = cc * S + s;               // ring slot of step c*S + s
              u32x4 Bf[MC];
#pragma unroll
              for (int ct = 0; ct < MC; ++ct) Bf[ct] = *reinterpret_cast<const u32x4 *>(bl + (size_t)(s * MC + ct) * 1024);
#pragma unroll
              for (int t = 0; t < NT; ++t) {
#pragma unroll
                for (int ct = 0; ct < MC; ++ct) acc[t][ct] = fast_mfma(A[u][t], Bf[ct], acc[t][ct]);
                A[u][t] = fast_ld_a(wf[t], g.Kd, min(ks0 + c * S + s + R, ks_last));
              }
            }
            lds_barrier();                            // chunk c+1 complete in LDS; everybody is done reading chunk c
          }
        }
      }
    }
    lds_barrier();                                    // every transfer has landed: the ring is free
    // the shares of the reduction meet in LDS; the wave with share 0 finishes the unit
    float *red = reinterpret_cast<float *>(smem);
    float *sc_tab = reinterpret_cast<float *>(smem + (size_t)kNsBufs * kNsSlots * MC * 1024);
    if (grp == wg && g.scale_tag && threadIdx.x < kScaleTab) sc_tab[threadIdx.x] = bat_row_scale(g, threadIdx.x);   // once per workgroup
    if (!filler) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int ct = 0; ct < MC; ++ct)
          *reinterpret_cast<f32x4 *>(red + ((size_t)((wave * NT + t) * MC + ct) * 64 + lane) * 4) = acc[t][ct];
    }
    lds_barrier();
    if (kw == 0 && valid) {
#pragma unroll
      for (int ct = 0; ct < MC; ++ct) {
        if (ct < g.CT) {
          const int c2 = lane & 7, jm = lane >> 3;
          const int i = 2 * c2;
          const int l_hi = (i >> 2) * 16 + jm, r = i & 3;
          float s0 = 0.f, s1 = 0.f, u0 = 0.f, u1 = 0.f, t0 = 0.f, t1 = 0.f, w0 = 0.f, w1 = 0.f;
#pragma unroll
          for (int kk = 0; kk < KW; ++kk) {
            const float *p = red + ((size_t)(((kk * NW + nw) * NT) * MC + ct) * 64) * 4;
            const float2 a = *reinterpret_cast<const float2 *>(p + l_hi * 4 + r);
            const float2 b = *reinterpret_cast<const float2 *>(p + (l_hi + 8) * 4 + r);
            s0 += a.x;
            s1 += a.y;
            t0 += b.x;
            t1 += b.y;
            if (NT == 2) {
              const float *q = p + (size_t)MC * 256;
              const float2 cg = *reinterpret_cast<const float2 *>(q + l_hi * 4 + r);
              const float2 dg = *reinterpret_cast<const float2 *>(q + (l_hi + 8) * 4 + r);
              u0 += cg.x;
              u1 += cg.y;
              w0 += dg.x;
              w1 += dg.y;
            }
          }
          if (g.single) {                             // accumulator columns jm and jm + 8 are two rows' results
            bat_emit(g, unit, ct, jm, c2, s0, s1, u0, u1, 0, sc_tab);
            bat_emit(g, unit, ct, jm, c2, t0, t1, w0, w1, 1, sc_tab);
          } else {
            bat_emit(g, unit, ct, jm, c2, s0 + t0, s1 + t1, u0 + w0, u1 + w1, 0, sc_tab);
          }
        }
      }
    }
    lds_barrier();                                    // the buffers are refilled by the next group
  }
}

// ---- M >= 128 rows: two-dimensional tiles, activation fragments shared through LDS -----------------
// With many rows bat_gemm is bound by the vector-memory path of a compute unit: every wave fetches its
// own activation fragments (8 KB per k-step against 3 KB of weights) and nothing is shared.  Here a
// workgroup owns 12 weight tiles x 16 column tiles (192 weight rows x 128 activation rows): six
// computing waves arranged 3 x 2, each 4 weight tiles x 8 column tiles (32 accumulator tiles), read
// their B fragments from LDS, where two filling waves put every k-step's 16 column tiles once with
// direct global -> LDS transfers: a ring of four chunks of 2 k-steps, three of them in flight (one
// chunk ahead is not enough: a transfer's round trip is about as long as two chunks of products).  The weights still go
// straight from global memory into the MFMA A layout.  Workgroups are numbered so that the row blocks
// of one weight group run next to each other on one XCD and find its weights in that L2.
// With MW = 1 the six computing waves all take different weight tiles of one block of 8 column tiles:
// the arrangement for up to 64 rows.  MC, the column tiles per wave, is 8 unless fewer leave less padding:
// 448 rows are 56 column tiles, 4 blocks of 2 x 7 instead of 4 blocks of 2 x 8 (an eighth fewer products
// and transfers); 56 rows are one block of 7.
constexpr int kWdMC = 8;
constexpr int kWdS = 2, kWdNB = 4;                       // k-steps per chunk of B fragments, chunks resident in LDS
constexpr int kWdRA = 4;                                 // k-steps of weight fragments requested ahead
constexpr int kWdCompute = 6;                            // of the 8 waves: 3 x 2 (weight tiles x column tiles) or 6 x 1
constexpr int kWdCols = 2 * kWdMC;                       // 16 column tiles per workgroup in the 3 x 2 arrangement
constexpr size_t kBatWideLds = (size_t)kWdNB * kWdS * kWdCols * 1024;  // 128 KB: four chunks of B fragments (3 x 2); at
                                                         // the end 16 KB per computing wave to turn its tiles around

// The end of a wide-GEMM wave: its NT x 8 accumulator tiles are turned around through `mine` (16 KB of LDS
// of its own: room for 2 x 8 tiles), two weight tiles at a time, so that a lane holds the pairs the epilogue works on; then the
// projection's epilogue, or, in a split reduction, the store of the run's sums.  ctg0: first of the wave's MC
// column tiles.
template <int NT, int MC>
__device__ __forceinline__ void bat_wide_finish_wave(const BatGemm &g, f32x4 (&acc)[NT][MC], const int (&unit_of)[NT], float *mine,
                                                     int ctg0, int lane, bool swiglu, int split, int ksplit, float2 *part,
                                                     const float *tab, int tab_m0) {
  const int c2 = lane & 7, jm = lane >> 3, i = 2 * c2;
  const int l_hi = (i >> 2) * 16 + jm, r = i & 3;
#pragma unroll
  for (int h = 0; h < NT / 2; ++h) {                  // two tiles at a time: 16 KB of LDS per wave
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int ct = 0; ct < MC; ++ct)
        *reinterpret_cast<f32x4 *>(mine + ((size_t)(tt * MC + ct) * 64 + lane) * 4) = acc[2 * h + tt][ct];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      if (swiglu && tt == 1) break;                   // a pair is emitted once, from its gate tile
      const int unit = unit_of[2 * h + tt];
      if (unit >= g.n_units) continue;                // uniform over the wave
      if (ksplit > 1) {                               // uniform: the sums go to bat_split_finish
#pragma unroll
        for (int ct = 0; ct < MC; ++ct) {
          const int ctg = ctg0 + ct;
          if (ctg >= g.CT) continue;
          const float *p = mine + ((size_t)(tt * MC + ct) * 64) * 4;
          const float2 a = *reinterpret_cast<const float2 *>(p + l_hi * 4 + r);
          const float2 b = *reinterpret_cast<const float2 *>(p + (l_hi + 8) * 4 + r);
          if (g.single) {                             // two rows' sums, kept apart
            float2 *dst = part + ((((size_t)split * g.n_units + unit) * g.CT + ctg) * 2) * 64 + lane;
            dst[0] = a;
            dst[64] = b;
          } else {
            part[(((size_t)split * g.n_units + unit) * g.CT + ctg) * 64 + lane] = make_float2(a.x + b.x, a.y + b.y);
          }
        }
        continue;
      }
      const int n_half = g.single ? 2 : 1;
#pragma unroll 1
      for (int hh = 0; hh < n_half; ++hh) {
        EmitPre pre[MC];                              // everything the tile's 8 column tiles read, requested before the first store
#pragma unroll
        for (int ct = 0; ct < MC; ++ct) pre[ct] = bat_emit_load(g, unit, min(ctg0 + ct, g.CT - 1), jm, c2, hh, tab, tab_m0);
#pragma unroll
        for (int ct = 0; ct < MC; ++ct) {
          const int ctg = ctg0 + ct;
          if (ctg >= g.CT) continue;                  // uniform over the wave
          const float *p = mine + ((size_t)(tt * MC + ct) * 64) * 4;
          const float2 a = *reinterpret_cast<const float2 *>(p + l_hi * 4 + r);
          const float2 b = *reinterpret_cast<const float2 *>(p + (l_hi + 8) * 4 + r);
          float2 cg = make_float2(0.f, 0.f), dg = make_float2(0.f, 0.f);
          if (swiglu) {
            const float *qq = p + (size_t)MC * 256;
            cg = *reinterpret_cast<const float2 *>(qq + l_hi * 4 + r);
            dg = *reinterpret_cast<const float2 *>(qq + (l_hi + 8) * 4 + r);
          }
          if (g.single) {
            const float2 s = hh ? b : a, u = hh ? dg : cg;
            bat_emit_apply(g, unit, ctg, jm, c2, s.x, s.y, u.x, u.y, pre[ct], hh);
          } else {
            bat_emit_apply(g, unit, ctg, jm, c2, a.x + b.x, a.y + b.y, cg.x + dg.x, cg.y + dg.y, pre[ct]);
          }
        }
      }
    }
  }
}

// NT: weight tiles per computing wave, 4 or 2 (2: half as many rows per workgroup, for projections with few tiles).
// ksplit > 1: the reduction is cut into ksplit equal runs of chunks, one workgroup each; a workgroup then
// stores its sums (part[split][unit][column tile][lane], the pair a lane would hand to the epilogue) and
// bat_split_finish adds them in the order of the splits and applies the epilogue.  For projections with
// so few weight tiles that one workgroup per tile group leaves most compute units idle (O-proj, down).
template <int NT, bool WHOLE, int MW, int MC>
__global__ __launch_bounds__(kBatThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void bat_gemm_wide(BatGemm g, int n_blk, int ksplit,
                                                                                                          float2 *part) {
  constexpr int S = kWdS;
  static_assert(MC >= 5 && MC <= kWdMC && (S * MW * MC) % (kBatWaves - kWdCompute) == 0, "column tiles per wave");
  constexpr int NWV = kWdCompute / MW, COLS = MW * MC;     // waves across weight tiles; column tiles per workgroup
  static_assert(MW == 1 || MW == 2, "wave arrangements");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const uint32_t smem_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lr = lane & 15, lg = lane >> 4;
  bat_scales_produce(g);
  const bool filler = wave >= kWdCompute;
  const int nwv = wave % NWV, mwv = filler ? 0 : wave / NWV;
  const bool swiglu = g.epi == FEPI_SWIGLU;
  const int upg = swiglu ? NWV * (NT / 2) : NWV * NT;          // units (tiles, or gate/up pairs) per workgroup
  const int n_groups = (g.n_units + upg - 1) / upg;
  // workgroup -> (weight group, row block): the row blocks of a group differ by 8 in the launch order
  const int id = blockIdx.x, q = id >> 3;
  const int inner = q % (n_blk * ksplit);
  const int blk = inner % n_blk, split = inner / n_blk, grp = (q / (n_blk * ksplit)) * 8 + (id & 7);
  if (grp >= n_groups) return;
  const int total = (g.Kd + 31) / 32;
  const int all_chunks = (total + S - 1) / S, per = (all_chunks + ksplit - 1) / ksplit;
  const int n_chunks = max(0, min(per, all_chunks - split * per)); // of this split (the last one may be shorter)
  const int kbase = split * per * S;                               // its first k-step
  const size_t bstep = (size_t)2 * g.CTS * 256;
  // units of this wave's NT tiles (SwiGLU: tile t is matrix t & 1 of pair t >> 1)
  int unit_of[NT];
  const uint16_t *wf[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int u = swiglu ? grp * upg + nwv * (NT / 2) + (t >> 1) : grp * upg + nwv * NT + t;
    unit_of[t] = u;
    const int ucl = u < g.n_units ? u : g.n_units - 1;               // surplus tiles multiply a valid one, results dropped
    const uint16_t *wbase;
    int wrow0;
    if (swiglu) {
      wbase = (t & 1) ? g.w[1] : g.w[0];
      wrow0 = ucl * 16;
    } else {
      const int seg = ucl / g.seg_tiles;
      wbase = seg == 0 ? g.w[0] : (seg == 1 ? g.w[1] : g.w[2]);
      wrow0 = (ucl - seg * g.seg_tiles) * 16;
    }
    wf[t] = fast_wfrag(wbase, wrow0, g.Kd, lane);
  }
  f32x4 acc[NT][MC];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int c = 0; c < MC; ++c) acc[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};

  if (filler) {
    wait_vmcnt_all();                                 // no wait of the compiler's between the transfers
    // this lane's piece of the B fragment of (k-step ks, column tile blk*16 + ct): bsrc + ks*bstep + ct*256
    const uint16_t *bsrc = g.b + ((size_t)(lg >> 1) * g.CTS + (size_t)blk * COLS) * 256 + lr * 16 + (lg & 1) * 8;
    constexpr int NF = kBatWaves - kWdCompute;                    // 2 filling waves
    constexpr int OPS = S * COLS / NF;                         // transfers per wave and chunk
    // Chunks past the end are transferred too (from the all-zero k-step), so that the count of
    // transfers in flight is the same at every wait.
    auto fill = [&](int c) __attribute__((always_inline)) {
      const int buf = c % kWdNB;
#pragma unroll
      for (int o = 0; o < OPS; ++o) {
        const int op = o * NF + (wave - kWdCompute);
        const int slot = op / COLS, ct = op % COLS;
        const int ksl = c * S + slot;
        const int ks = (ksl < n_chunks * S && kbase + ksl < total) ? kbase + ksl : total;
        lds_dma16(bsrc + (size_t)ks * bstep + ct * 256,
                  __builtin_amdgcn_readfirstlane(smem_lds + (uint32_t)(((buf * S + slot) * COLS + ct) * 1024)));
      }
    };
#pragma unroll
    for (int c = 0; c < kWdNB - 1; ++c) fill(c);
    wait_vmcnt<(kWdNB - 2) * OPS>();                              // chunk 0 has arrived
    lds_barrier();
    for (int c = 0; c < n_chunks; ++c) {
      fill(c + kWdNB - 1);                                        // into the buffer chunk c-1 was read from
      wait_vmcnt<(kWdNB - 2) * OPS>();                            // chunk c+1 has arrived
      lds_barrier();
    }
    wait_vmcnt<0>();                                              // nothing may land in LDS after the buffers change hands
  } else {
    u32x4 A[kWdRA][NT];
#pragma unroll
    for (int u = 0; u < kWdRA; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t) A[u][t] = fast_ld_a(wf[t], g.Kd, kbase + u);
    lds_barrier();                                    // chunk 0 is in LDS
    constexpr int CPR = kWdRA / S;                    // chunks per revolution of the weight ring
    auto chunk = [&](int c, int cc) __attribute__((always_inline)) {
      const unsigned char *bl = smem + ((size_t)((c % kWdNB) * S * COLS + mwv * MC)) * 1024 + lane * 16;
#pragma unroll
      for (int s = 0; s < S; ++s) {
        const int u = cc * S + s;                     // ring slot of k-step c*S + s
        u32x4 Bf[MC];
#pragma unroll
        for (int ct = 0; ct < MC; ++ct) Bf[ct] = *reinterpret_cast<const u32x4 *>(bl + (size_t)(s * COLS + ct) * 1024);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
          for (int ct = 0; ct < MC; ++ct) acc[t][ct] = fast_mfma(A[u][t], Bf[ct], acc[t][ct]);
          A[u][t] = fast_ld_a(wf[t], g.Kd, kbase + c * S + s + kWdRA);   // clamped into the matrix; never used past the end
        }
      }
      lds_barrier();                                  // chunk c+1 complete in LDS; everybody is done reading chunk c
    };
    // WHOLE (the chunk count is a whole number of revolutions): no branch inside the loop, so the waits
    // the compiler places before each weight fragment count every younger request of the ring; with a
    // branch it can only count those of the current chunk, which halves the distance the weights are
    // requested ahead.
    for (int c0 = 0; c0 < n_chunks; c0 += CPR) {
#pragma unroll
      for (int cc = 0; cc < CPR; ++cc)
        if (WHOLE || c0 + cc < n_chunks) chunk(c0 + cc, cc);   // uniform over the workgroup
    }
  }
  lds_barrier();                                      // the B buffers are free: every wave turns its own tiles around in them
  if (filler) return;
  // the 1/rms of this wave's rows, once, into a table of its own above the computing waves' 16 KB each
  const float *tab = nullptr;
  int tab_m0 = 0;
  if (ksplit == 1 && g.scale_tag) {
    static_assert((size_t)kWdCompute * (2 * kWdMC * 1024) + kWdCompute * kScaleTab * sizeof(float) <= kBatWideLds, "room for the tables");
    float *t = reinterpret_cast<float *>(smem + (size_t)kWdCompute * (2 * kWdMC * 1024)) + wave * kScaleTab;
    const int rpt = g.single ? 16 : 8;
    tab_m0 = (blk * COLS + mwv * MC) * rpt;
    for (int i = lane; i < MC * rpt; i += kWave) t[i] = bat_row_scale(g, tab_m0 + i);
    tab = t;
  }
  bat_wide_finish_wave<NT, MC>(g, acc, unit_of, reinterpret_cast<float *>(smem + (size_t)wave * (2 * kWdMC * 1024)), blk * COLS + mwv * MC,
                           lane, swiglu, split, ksplit, part, tab, tab_m0);
}

// Second half of a split reduction: one wave per (column tile, unit); lane (jm, c2) adds the pair of every
// split in the order of the splits and applies the projection's epilogue (not SwiGLU: never split).
__global__ __launch_bounds__(256) void bat_split_finish(BatGemm g, int ksplit, const float2 *part) {
  const int lane = threadIdx.x & 63;
  const int tile = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tile >= g.n_units * g.CT) return;               // uniform over the wave
  const int ct = tile / g.n_units, unit = tile - ct * g.n_units;     // neighbouring waves: neighbouring columns of the same rows
  const int c2 = lane & 7, jm = lane >> 3;
  const int n_half = g.single ? 2 : 1;                // single-bf16 activations: two rows' sums per lane and tile
  // eight runs are requested together (one round trip, not one per run) and added in the order of the runs
  const size_t run_stride = (size_t)g.n_units * g.CT * 64 * n_half;
  for (int hh = 0; hh < n_half; ++hh) {
    const EmitPre pre = bat_emit_load(g, unit, ct, jm, c2, hh);
    const float2 *mine = part + (((size_t)unit * g.CT + ct) * n_half + hh) * 64 + lane;
    float2 s = make_float2(0.f, 0.f);
    for (int k0 = 0; k0 < ksplit; k0 += 8) {
      float2 v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = mine[(size_t)min(k0 + k, ksplit - 1) * run_stride];
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (k0 + k < ksplit) {
          s.x += v[k].x;
          s.y += v[k].y;
        }
    }
    bat_emit_apply(g, unit, ct, jm, c2, s.x, s.y, 0.f, 0.f, pre, hh);
  }
}

// ---- embedding: x rows (fp32), records of x*gain, partial sums of squares --------------------------
// One 16-column tile per workgroup (64 threads); thread (c2, jm) walks the column tiles (those of its share
// when the grid has a second dimension: with many rows one walk is a long chain of dependent gathers).  With `rows`
// given the input rows are taken from there (fp32 [M][d]: visual tokens arrive as embeddings, App. A.1)
// instead of being looked up; with both `ids` and `rows`, row m is looked up if ids[m] >= 0 and taken from
// `rows` otherwise.
__global__ __launch_bounds__(64) void bat_embed(const int32_t *ids, const float *rows, const uint16_t *emb, int vocab, int d,
                                                int M, int CT, int CTS, const float *gain, float *x, uint16_t *planes,
                                                float *ssq_out, int single, unsigned long long *scale_tag) {
  const int tile = blockIdx.x, tid = threadIdx.x;
  const int c2 = tid & 7, jm = tid >> 3;
  const int col = tile * 16 + 2 * c2;
  const float2 gn = *reinterpret_cast<const float2 *>(gain + col);
  const int n_half = single ? 2 : 1;                          // single-bf16 records: 16 rows per column tile
  // The step's first launch clears the tagged row scales (BatGemm::scale_tag): a step replayed from a HIP
  // graph carries the epochs of its capture, and a projection must not take last replay's words for its own.
  if (blockIdx.x == 0 && blockIdx.y == 0)
    for (int i = tid; i < CT * 8 * n_half; i += 64) scale_tag[i] = 0ull;
  for (int cth = blockIdx.y; cth < CT * n_half; cth += gridDim.y) {       // the grid's second dimension shares the column tiles
    const int ct = cth / n_half, hh = cth - ct * n_half;
    const int m = single ? ct * 16 + hh * 8 + jm : ct * 8 + jm;
    float v0 = 0.f, v1 = 0.f;
    if (m < M) {
      if (rows && (!ids || ids[m] < 0)) {           // both given: a negative id takes the row's embedding
        const float2 r = *reinterpret_cast<const float2 *>(rows + (size_t)m * d + col);
        v0 = r.x;
        v1 = r.y;
      } else {
        int id = ids[m];
        id = max(0, min(id, vocab - 1));
        const uint32_t pr = *reinterpret_cast<const uint32_t *>(emb + (size_t)id * d + col);
        v0 = __uint_as_float(pr << 16);
        v1 = __uint_as_float(pr & 0xFFFF0000u);
      }
      *reinterpret_cast<float2 *>(x + (size_t)m * d + col) = make_float2(v0, v1);
    }
    float q = v0 * v0 + v1 * v1;
    q = sum8(q);
    if (c2 == 0) ssq_out[(size_t)tile * (CTS * 8) + m] = q;
    uint32_t h0, l0, h1, l1;
    split_bf16(v0 * gn.x, h0, l0);
    split_bf16(v1 * gn.y, h1, l1);
    uint32_t *rec = reinterpret_cast<uint32_t *>(planes + ((size_t)tile * CTS + ct) * 256);
    if (single) {
      rec[((jm + 8 * hh) * 16 + 2 * c2) / 2] = h0 | (h1 << 16);
    } else {
      rec[(jm * 16 + 2 * c2) / 2] = h0 | (h1 << 16);
      rec[((jm + 8) * 16 + 2 * c2) / 2] = l0 | (l1 << 16);
    }
  }
}

}  // namespace heisd
