// The whole decoder forward of a verify step (M = batch*K <= 8 rows) as ONE persistent kernel:
// one workgroup per compute unit interprets a short phase program - embedding, then per layer
// {QKV, attention, O-proj, gate/up, down}, then the LM-head slice - with a grid barrier after each
// phase.  There is one copy of each phase body; the program entries are data.
//
// Why: at 7B shape one layer is five dependent phases of 4-23 microseconds of HBM time each.
// Launching them one by one costs a ramp-up and a drain per phase; here every workgroup requests
// the first weight tile of the NEXT GEMM phase right after it has published its outputs, so HBM
// keeps streaming while the workgroups wait for each other and fetch their activations.
//
// Grid barrier: one 64-byte-padded flag per workgroup holding the last epoch it reached; wave 0 of
// every workgroup publishes its flag and polls all flags with device-scope loads.  No L2
// write-back/invalidate: all exchanged data is written with device-scope stores into per-layer
// buffers (see heisd_fast.h).  The spin is bounded; on expiry the workgroup raises the error word
// and leaves, and so does every other workgroup at its next barrier.
#pragma once
#include "heisd_fast.h"

namespace heisd {

constexpr int kFlagStride = 16;          // uint32 per flag slot (64 bytes)
constexpr int kSpinLimit = 1 << 22;

// The step is a short program: one entry per phase, built once at init and kept in device memory.
enum { PH_EMBED = 0, PH_GEMM = 1, PH_GEMM_STREAM = 2, PH_ATTN = 3 };

struct Phase {
  int kind;        // PH_*
  int layer;       // PH_ATTN: decoder layer (selects the KV-cache slab)
  int next_gemm;   // index of the GEMM phase whose first weight tile this phase requests when its own
                   // weights have been consumed (-1: none)
  int pad;
  FastGemm g;      // PH_GEMM*: the GEMM.  PH_EMBED: next_gain, out (x), o_planes, ssq_out.
                   // PH_ATTN: b = q/k/v records (fp32), o_planes = attention output records.
};

struct PersistArgs {
  const Phase *prog;
  int n_phases;
  int d, H, vocab, cap;
  const uint16_t *tok_emb;
  float scale;
  const float2 *rope;
  // step inputs
  const int32_t *ids;
  uint16_t *k_cache, *v_cache;
  size_t kv_layer_stride;
  const int32_t *prefix_len;
  const uint8_t *skip;
  int K, batch;
  float *logits;                         // [M][n_bins]
  unsigned *flags;                       // [nwg][kFlagStride]
  unsigned epoch0;                       // flags hold values <= epoch0 when the kernel starts
  unsigned *err;
  unsigned long long *trace;             // optional [n_phases][8] timestamps of workgroup 0 (measurement aid)
};

// Grid barrier, split in two so that weight prefetches can be slotted in between.
// Arrive: every wave waits for its own device-scope stores (nothing else is outstanding at that
// point), then the workgroup publishes the epoch.
__device__ __forceinline__ void grid_arrive(const PersistArgs &p, int wg, unsigned epoch) {
  __builtin_amdgcn_s_waitcnt(0);
  lds_barrier();
  if (threadIdx.x == 0)
    __hip_atomic_store(&p.flags[wg * kFlagStride], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Wait: wave 0 polls every workgroup's flag (it must not have loads of its own in flight, its polls
// would queue behind them); the other waves just meet it at the workgroup barrier, their
// prefetched loads still flying.  Returns false if the wait gave up (error word raised) or an
// error was seen.
__device__ __forceinline__ bool grid_wait(const PersistArgs &p, int nwg, unsigned epoch) {
  __shared__ int s_ok;
  if (threadIdx.x < kWave) {
    const int lane = threadIdx.x;
    int spins = 0;
    bool good = true;
    while (true) {
      bool ok = true;
      for (int i = lane; i < nwg; i += kWave) {
        const unsigned f = __hip_atomic_load(&p.flags[i * kFlagStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok = ok && ((int)(f - epoch) >= 0);
      }
      if (__all(ok)) break;
      if (++spins > kSpinLimit ||
          ((spins & 255) == 0 && __hip_atomic_load(p.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
        good = false;
        break;
      }
    }
    if (!good && lane == 0) __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (lane == 0) s_ok = good ? 1 : 0;
  }
  lds_barrier();
  const bool r = s_ok != 0;
  lds_barrier();          // s_ok may be rewritten only after everybody has read it
  return r;
}

// Attention unit t (t = 0, 1, ...) of workgroup wg: queries of one head stay on one XCD (workgroup
// ids are dealt to the 8 XCDs round-robin), so its K/V rows are fetched from HBM once.
__device__ __forceinline__ bool attn_unit_of(const PersistArgs &p, int wg, int nwg, int t, int &b, int &h, int &jq) {
  const int n_heads_total = p.batch * p.H;
  if ((nwg & 7) == 0) {
    const int x = wg & 7, per = nwg >> 3;
    const int slot = (wg >> 3) + t * per;
    const int hh = slot / p.K;
    jq = slot - hh * p.K;
    const int bh = hh * 8 + x;
    b = bh / p.H;
    h = bh - b * p.H;
    return bh < n_heads_total;
  }
  const int u = wg + t * nwg;
  const int bh = u / p.K;
  jq = u - bh * p.K;
  b = bh / p.H;
  h = bh - b * p.H;
  return bh < n_heads_total;
}

// Program entry with the step's own values filled in.
__device__ __forceinline__ FastGemm phase_gemm(const PersistArgs &p, int ph) {
  FastGemm g = p.prog[ph].g;
  g.M = p.batch * p.K;
  if (g.epi == FEPI_STORE_ROWS) g.out = p.logits;
  return g;
}

template <int HD>
__global__ __launch_bounds__(kFastThreads) void persist_forward(PersistArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int wg = blockIdx.x, nwg = gridDim.x;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lr = lane & 15, lg = lane >> 4;
  Frag16 A;                                // the weight ring, carried across phases and barriers
  unsigned epoch = p.epoch0;

  auto stamp = [&](int ph, int slot) __attribute__((always_inline)) {
    if (p.trace && wg == 0 && threadIdx.x == 0) p.trace[ph * 8 + slot] = wall_clock64();
  };
  for (int ph = 0; ph < p.n_phases; ++ph) {
    const int kind = p.prog[ph].kind;
    stamp(ph, 0);
    if (kind == PH_GEMM) {
      const FastGemm g = phase_gemm(p, ph);
      fast_gemm_phase(g, wg, nwg, smem, A, true);
    } else if (kind == PH_GEMM_STREAM) {
      const FastGemm g = phase_gemm(p, ph);
      fast_gemm_stream_phase(g, wg, nwg, smem, A, true);
    } else if (kind == PH_ATTN) {
      const Phase &P = p.prog[ph];
      FastAttn at{};
      at.qkv = reinterpret_cast<const float *>(P.g.b);
      at.k_cache = p.k_cache + (size_t)P.layer * p.kv_layer_stride;
      at.v_cache = p.v_cache + (size_t)P.layer * p.kv_layer_stride;
      at.prefix_len = p.prefix_len; at.skip = p.skip; at.rope = p.rope;
      at.o_planes = P.g.o_planes;
      at.K = p.K; at.H = p.H; at.cap = p.cap; at.d = p.d; at.batch = p.batch; at.scale = p.scale;
      for (int t = 0;; ++t) {
        int ab, ah, aj;
        if (!attn_unit_of(p, wg, nwg, t, ab, ah, aj)) break;
        AttnPre pre;
        fast_attn_prefetch<HD>(at, ab, ah, pre);
        fast_attn_unit<HD>(at, ab, ah, aj, smem, pre);
      }
    } else {
      const Phase &P = p.prog[ph];
      for (int tile = wg; tile < p.d / 16; tile += nwg)
        fast_embed_tile(p.ids, p.tok_emb, p.vocab, p.d, p.batch * p.K, tile, P.g.next_gain, P.g.out, P.g.o_planes,
                        P.g.ssq_out);
    }
    stamp(ph, 1);
    if (ph + 1 == p.n_phases) break;
    // barrier; the first weight tile of the next GEMM phase is requested while waiting
    ++epoch;
    grid_arrive(p, wg, epoch);
    // (the polls of wave 0 queue behind these loads in the compute unit's memory pipeline: the
    // barrier is seen once they have drained, and HBM stays busy meanwhile)
    const int ng = p.prog[ph].next_gemm;
    if (ng >= 0) {
      const FastGemm gn = phase_gemm(p, ng);
      fast_issue16(A, gn, wg, nwg, 0, wave, lr, lg);
    }
    stamp(ph, 2);
    if (!grid_wait(p, nwg, epoch)) return;
    stamp(ph, 3);
  }
}

// epochs one launch consumes
inline unsigned persist_epochs(int n_phases) { return (unsigned)(n_phases - 1); }

}  // namespace heisd
