// Weight-streaming skinny GEMM  y[M,N] = act[M,Kd] . W[N,Kd]^T  for the decoder's linear
// layers (the K draft tokens of a verify step, M = batch*K rows; paper Sec. 2.2 "parallel
// verification", App. A.1 backbone).  The weights are read from HBM exactly once per row
// block; everything else lives in LDS/registers.
//
// Mapping (gfx950, wave64, v_mfma_f32_16x16x32_bf16):
//   * A operand = a 16-row x 32-k tile of W, loaded straight from global memory into the
//     MFMA register layout: lane l reads 16 bytes at W[n0 + l%16][k0 + 8*(l/16)].
//   * B operand = activations.  Each fp32 activation is split into a bf16 head and a bf16
//     tail; one 16-column B tile carries 8 activation rows: columns 0-7 the heads, columns
//     8-15 the tails.  The two partial products are added in the epilogue, so activations
//     keep ~16 mantissa bits although the matrix core multiplies bf16.
//   * A workgroup (8 waves) owns NT n-tiles over the whole reduction; its waves split the
//     k-steps and are reduced through LDS in a fixed order (deterministic, no atomics).
//   * Optional RMSNorm prologue: the B tile holds x*g and the row's sum of squares is
//     accumulated while staging; 1/rms is applied to the accumulator in the epilogue.
//   * Epilogues: store (+ residual), or SwiGLU over (gate tile, up tile) pairs.
#pragma once
#include "heisd_common.h"

namespace heisd {

constexpr int kGemmThreads = 512;
constexpr int kGemmWaves = 8;
constexpr int kGemmChunkK = 4096;  // k elements staged per chunk when MC == 1

enum { EPI_STORE = 0, EPI_SWIGLU = 1 };

struct GemmArgs {
  const float *act;     // [M][Kd] fp32
  const float *gain;    // [Kd] RMSNorm gain, or nullptr for no norm
  const uint16_t *w[3]; // weight segments, bf16 row-major [rows][Kd]
  int seg_tiles;        // n-tiles (16 rows) per segment
  int n_units;          // n-tiles (EPI_STORE) or (gate,up) tile pairs (EPI_SWIGLU) in total
  int M, Kd;
  float eps;
  float *out;           // [M][ldo]
  int ldo;
  const float *resid;   // [M][ldo] added in the epilogue, or nullptr (may alias out)
};

template <int MC>
constexpr size_t gemm_lds_bytes() {
  return (size_t)16 * MC * (kGemmChunkK / MC + 8) * 2 + 8 * MC * sizeof(float);
}

template <int U, int NT>
__device__ __forceinline__ void gemm_load_group(uint4 (&A)[U][NT], const uint16_t *const (&wrow)[NT],
                                                const bool (&tvalid)[NT], int s_first, int s_end,
                                                int kc0, int k_lane, int Kd) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int s = s_first + u;
    const int k = kc0 + s * 32;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const bool ok = (s < s_end) && tvalid[t] && (k + k_lane + 8 <= Kd);
      A[u][t] = ok ? *reinterpret_cast<const uint4 *>(wrow[t] + k) : make_uint4(0, 0, 0, 0);
    }
  }
}

template <int U, int NT, int MC, int KCP>
__device__ __forceinline__ void gemm_compute_group(const uint4 (&A)[U][NT], f32x4 (&acc)[NT][MC],
                                                   const uint16_t *Bs, int s_first, int s_end, int lr,
                                                   int lg) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int s = s_first + u;
    if (s < s_end) {
      bf16x8 b[MC];
#pragma unroll
      for (int c = 0; c < MC; ++c)
        b[c] = *reinterpret_cast<const bf16x8 *>(Bs + (size_t)(c * 16 + lr) * KCP + s * 32 + lg * 8);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, A[u][t]);
#pragma unroll
        for (int c = 0; c < MC; ++c) acc[t][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b[c], acc[t][c], 0, 0, 0);
      }
    }
  }
}

template <int MC, int NT, int EPI>
__global__ __launch_bounds__(kGemmThreads) void gemm_skinny(GemmArgs a) {
  static_assert(EPI == EPI_STORE || (NT % 2) == 0, "SwiGLU needs tile pairs");
  constexpr int KC = kGemmChunkK / MC;
  constexpr int KCP = KC + 8;  // +16 bytes per row: consecutive columns land in different banks
  constexpr int U = NT >= 3 ? 4 : (NT == 2 ? 8 : 16);  // weight tiles in flight per wave: 2*U*NT KB
  static_assert(NT * MC <= 16, "reduction buffer must fit in the staging area");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t *Bs = reinterpret_cast<uint16_t *>(smem);
  float *sumsq = reinterpret_cast<float *>(smem + (size_t)16 * MC * KCP * 2);
  float *red = reinterpret_cast<float *>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int Kd = a.Kd, M = a.M;

  // unit -> (valid, first weight row inside its matrix, matrix, output column)
  auto unit_of = [&](int t, bool &valid, int &wrow0, const uint16_t *&wbase, int &col) {
    if (EPI == EPI_STORE) {
      const int g = blockIdx.x * NT + t;
      valid = g < a.n_units;
      const int gg = valid ? g : 0;
      const int seg = gg / a.seg_tiles;
      wrow0 = (gg - seg * a.seg_tiles) * 16;
      wbase = seg == 0 ? a.w[0] : (seg == 1 ? a.w[1] : a.w[2]);
      col = gg * 16;
    } else {
      const int p = blockIdx.x * (NT / 2) + (t >> 1);
      valid = p < a.n_units;
      wrow0 = (valid ? p : 0) * 16;
      wbase = (t & 1) ? a.w[1] : a.w[0];
      col = wrow0;
    }
  };
  const uint16_t *wrow[NT];
  bool tvalid[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    int wrow0, col;
    const uint16_t *wbase;
    unit_of(t, tvalid[t], wrow0, wbase, col);
    wrow[t] = wbase + (size_t)(wrow0 + lr) * Kd + lg * 8;
  }

  f32x4 acc[NT][MC];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int c = 0; c < MC; ++c) acc[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
  float ss[MC];
#pragma unroll
  for (int c = 0; c < MC; ++c) ss[c] = 0.f;

  for (int kc0 = 0; kc0 < Kd; kc0 += KC) {
    const int kc_len = min(KC, Kd - kc0);
    const int ksteps = (kc_len + 31) >> 5;
    // this wave's share of the k-steps; its first weight tiles are requested before the
    // activations are staged, so the HBM latency overlaps the staging
    const int s0 = wave * ksteps / kGemmWaves, s1 = (wave + 1) * ksteps / kGemmWaves;
    uint4 A0[U][NT], A1[U][NT];
    gemm_load_group<U, NT>(A0, wrow, tvalid, s0, s1, kc0, lg * 8, Kd);
    __syncthreads();
    // ---- stage the activations of this k-chunk: wave w owns rows c*8 + w ----
#pragma unroll
    for (int c = 0; c < MC; ++c) {
      const int m = c * 8 + wave;
      uint16_t *hi = Bs + (size_t)(c * 16 + wave) * KCP;
      uint16_t *lo = hi + (size_t)8 * KCP;
      for (int k = lane * 4; k < ksteps * 32; k += 256) {
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (m < M && k < kc_len) {
          x = *reinterpret_cast<const float4 *>(a.act + (size_t)m * Kd + kc0 + k);
          if (a.gain) {
            ss[c] += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
            const float4 g = *reinterpret_cast<const float4 *>(a.gain + kc0 + k);
            x.x *= g.x; x.y *= g.y; x.z *= g.z; x.w *= g.w;
          }
        }
        uint32_t h0, h1, h2, h3, l0, l1, l2, l3;
        split_bf16(x.x, h0, l0); split_bf16(x.y, h1, l1);
        split_bf16(x.z, h2, l2); split_bf16(x.w, h3, l3);
        *reinterpret_cast<uint2 *>(hi + k) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
        *reinterpret_cast<uint2 *>(lo + k) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
      }
    }
    __syncthreads();
    // ---- stream the weight tiles ----
    for (int s = s0; s < s1; s += 2 * U) {
      gemm_load_group<U, NT>(A1, wrow, tvalid, s + U, s1, kc0, lg * 8, Kd);
      gemm_compute_group<U, NT, MC, KCP>(A0, acc, Bs, s, s1, lr, lg);
      gemm_load_group<U, NT>(A0, wrow, tvalid, s + 2 * U, s1, kc0, lg * 8, Kd);
      gemm_compute_group<U, NT, MC, KCP>(A1, acc, Bs, s + U, s1, lr, lg);
    }
  }

  // ---- fixed-order reduction over the 8 waves, then the epilogue ----
  __syncthreads();
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int c = 0; c < MC; ++c)
      *reinterpret_cast<f32x4 *>(red + ((size_t)((wave * NT + t) * MC + c) * 64 + lane) * 4) = acc[t][c];
  if (a.gain) {
#pragma unroll
    for (int c = 0; c < MC; ++c) {
      const float tot = wave_sum(ss[c]);
      if (lane == 0) sumsq[c * 8 + wave] = tot;
    }
  }
  __syncthreads();

  auto tile_sum = [&](int t, int c, int i, int jm) -> float {
    const int l_hi = (i >> 2) * 16 + jm, r = i & 3;
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < kGemmWaves; ++w) {
      const float *p = red + ((size_t)((w * NT + t) * MC + c) * 64) * 4;
      s += p[l_hi * 4 + r] + p[(l_hi + 8) * 4 + r];
    }
    return s;
  };
  const float inv_k = 1.0f / (float)Kd;
  constexpr int UNITS = (EPI == EPI_STORE) ? NT : NT / 2;
  for (int o = tid; o < UNITS * MC * 128; o += kGemmThreads) {
    const int i = o & 15, jm = (o >> 4) & 7;
    const int c = (o >> 7) % MC, un = (o >> 7) / MC;
    const int m = c * 8 + jm;
    const int t = (EPI == EPI_STORE) ? un : 2 * un;
    bool valid;
    int wrow0, col;
    const uint16_t *wbase;
    unit_of(t, valid, wrow0, wbase, col);
    if (m >= M || !valid) continue;
    const float scale = a.gain ? rsqrtf(sumsq[m] * inv_k + a.eps) : 1.0f;
    const size_t idx = (size_t)m * a.ldo + col + i;
    if (EPI == EPI_STORE) {
      float v = tile_sum(t, c, i, jm) * scale;
      if (a.resid) v += a.resid[idx];
      a.out[idx] = v;
    } else {
      const float g = tile_sum(t, c, i, jm) * scale;
      const float u = tile_sum(t + 1, c, i, jm) * scale;
      a.out[idx] = g / (1.0f + expf(-g)) * u;
    }
  }
}

}  // namespace heisd
