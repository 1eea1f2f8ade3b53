// The whole decoder forward of a verify step (M = batch*K <= 8 rows; paper Sec. 2.2, Eq. 2-2: one
// teacher-forced pass of the target model over the drafts) as ONE persistent kernel: one workgroup
// per compute unit walks a short phase program - embedding, then per layer {QKV, attention, O-proj,
// gate/up, down}, then the LM-head slice - and the workgroups meet at a grid barrier between phases.
//
// Why: at the 7B shape a layer is five dependent phases of 5-28 microseconds of HBM time each, and a
// kernel boundary between two of them costs 4-5 microseconds in which no weights move.  Here the
// weight stream runs across the phase boundaries:
//   * When a workgroup has multiplied its last weight tile of a GEMM phase, two of its waves start
//     direct global -> LDS transfers of the first kPF k-steps of every wave's first tile of the NEXT
//     GEMM phase (96 KB per compute unit, 24 MB on the chip), before the reduction, the epilogue and
//     the barrier.  Nothing but LDS is carried from one phase to the next, so every phase body keeps
//     its own register allocation.
//   * A phase requests what does not depend on the previous phase's outputs (the rest of its first
//     weight tile; the prefix keys and values of an attention unit) BEFORE it waits at the barrier.
// The O-projection's hand-over is started at the end of the attention phase (in front of the attention
// units' own loads and stores it cost them more than it saved the projection).
//
// Grid barrier: one word per workgroup holding the last epoch it published (packed: 1 KB for 256
// workgroups); wave 0 polls all flags with device-scope loads (it keeps no other load in flight before the wait, its polls would
// queue behind them).  Phase ph waits for epoch0 + ph.  No L2 write-back or invalidate: all exchanged
// data is written with device-scope stores into per-layer buffers (see heisd_fast.h).  The spin is
// bounded; on expiry the workgroup raises the error word and leaves, and every other workgroup leaves
// at its next barrier.
#pragma once
#include "heisd_fast.h"
#include "heisd_misc.h"

namespace heisd {

constexpr int kFlagStride = 1;           // flags are packed: a poll of all of them is 8 cache lines, not one per workgroup
constexpr int kSpinLimit = 1 << 22;
// 256 workgroups polling ONE kilobyte of uncached memory queue on the memory channel that holds it.  In a slot of
// uncached memory the flag array exists eight times: a workgroup stores its flag into every copy (eight lanes, one
// store each) and polls copy wg % 8, its XCD's, so that 32 workgroups share a copy: 2.799 -> 2.758 ms per step at
// the 7B shape (16 / 32 copies: 2.749 / 2.754 ms against 2.751 ms with 8 in the same run).
constexpr int kFlagCopies = 8, kFlagCopyWords = 1024 + 64;     // copies of the flag array (uncached slot only) and their distance in words

// Publish a flag: into every copy (lanes 0 .. copies-1 of the calling wave store one each).
__device__ __forceinline__ void p2_store_flag(unsigned *flags, int copies, int wg, unsigned value, int lane) {
  if (lane < copies)
    __hip_atomic_store(flags + (size_t)lane * kFlagCopyWords + wg * kFlagStride, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kPF = kKS;                 // k-steps of a wave's first weight tile handed over through LDS: a whole ring
constexpr int kPfBefore = 12;            // of those, handed over BEFORE the barrier; the rest follows when the barrier is passed (16 / 12 / 8 / 4
                                         // before it: 2.905 / 2.887 / 2.914 / 3.030 ms per step at the 7B shape; with the flags in uncached memory 16 / 12 / 8: 2.798 / 2.776 / 2.827 ms)
constexpr int kPfWave0 = 6;              // waves kPfWave0 .. 7 issue the transfers (they never store in a GEMM epilogue)
// LDS map.  The hand-over region (128 KB) and the reduction buffer share their bytes: a phase reads what was
// handed over into registers when it starts and reduces through the same bytes when it ends, and the next
// hand-over is started only after every storing wave has read its sums (p2_wait_words).  The attention
// units work above both, so that the O-projection's hand-over may sit in LDS while they run.
constexpr size_t kPfOff = 0;
constexpr size_t kPfBytes = (size_t)kFastWaves * kPF * 1024;
constexpr size_t kCtlOff = kPfBytes;                                 // 16 floats: the rows' 1/rms
constexpr size_t kSyncOff = kCtlOff + 64;                            // 8 words: what each wave has published (see gemm_publish)
constexpr size_t kOkOff = kCtlOff + 128;                             // 1 word: outcome of the last grid wait
constexpr size_t kAttnOff = kCtlOff + 256;                           // the attention units' buffers (fast_attn_lds bytes)
inline size_t persist_lds_bytes(int hd, int cap) { return kAttnOff + fast_attn_lds(hd, cap); }
static_assert(kPfBytes >= kFastRedBytes, "the reduction buffer lies inside the hand-over region");
static_assert(kPfBefore % 4 == 0 && kPfBefore >= 4 && kPfBefore <= kPF, "the products read LDS four steps at a time");
static_assert(kMaxT <= kPfWave0, "the waves that issue transfers must not take part in epilogue stores");
static_assert(kFastWaves % (kFastWaves - kPfWave0) == 0 && kPF <= 31, "an issuing wave serves a whole number of wave shares");

enum { PHF_IN_LDS = 1,    // an earlier phase has handed steps 0 .. kPF-1 of every wave share over in LDS
       PHF_EARLY = 2 };   // the steps not handed over are requested before the wait at the barrier (not by wave 0)

// The step is a short program: one entry per phase, built once at init and kept in device memory.
enum { PH_EMBED = 0, PH_GEMM = 1, PH_GEMM_STREAM = 2, PH_ATTN = 3 };

struct Phase {
  int kind;        // PH_*
  int layer;       // PH_ATTN: decoder layer (selects the KV-cache slab)
  int next_gemm;   // index of the GEMM phase whose first weight steps this phase hands over in LDS (-1: none)
  int first_tile;  // PH_GEMM*: PHF_* bits - where the first weight tile's fragments come from
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
  unsigned long long *trace;             // optional [n_phases][workgroups][8] timestamps (measurement aid)
  const int *attn_prod;                  // [H][n_prod]: the workgroups that produce head h's q/k/v in a QKV phase
  int n_prod;                            // 3 * head_dim / 16 (at most 64)
  int flag_copies;                       // 1, or 8: every workgroup writes its flag into 8 copies of the array and polls copy wg % 8
  int spin_limit;                        // polls a grid wait makes before it gives up (kSpinLimit unless a test lowers it)
  AcceptArgs acc;                        // greedy bins + acceptance scan of the step (paper Sec. 4.2), run by workgroups 0 .. batch-1
};

// The thread index as a value the optimiser cannot trace back to the hardware register: what a phase
// derives from it (lane offsets, row and column indices of the epilogues, the attention unit's key
// streams) is then recomputed inside that phase instead of being hoisted out of the loop over phases,
// where dozens of such per-lane values would stay live across every phase and spill.
__device__ __forceinline__ int p2_tid() {
  int t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}

__device__ __forceinline__ void p2_stamp(const PersistArgs &p, int wg, int ph, int slot) {
  if (p.trace && p2_tid() == 0) p.trace[((size_t)ph * gridDim.x + wg) * 8 + slot] = wall_clock64();
}

// Publish: this workgroup's outputs of the phase are in memory.  Every wave that may have stored waits
// for its stores (with only_storing the transfer-issuing waves are left out: they have stored nothing,
// and waiting would make the flag wait for their transfers), then thread 0 sets the flag.
__device__ __forceinline__ void grid_arrive(const PersistArgs &p, int wg, unsigned epoch, bool only_storing) {
  const int tid = p2_tid(), wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (!only_storing || wave < kPfWave0) wait_vmcnt_all();
  lds_barrier();
  if (tid < kWave) p2_store_flag(p.flags, p.flag_copies, wg, epoch, tid);
}

// A compute unit serves its waves' vector memory operations in the order they were issued, and the memory
// system behind it is a queue too.  The 128 transfers of a hand-over take microseconds to drain, and
// epilogue stores issued behind them - or merely while they are in flight - are acknowledged late
// (measured: 4-7 us from the last product to the published flag with the hand-over in front of the stores,
// 2-4 us with the hand-over started once the stores were issued, against 0.4 us for a phase that hands
// nothing over).  So the hand-over starts when the workgroup's stores have been ACKNOWLEDGED: every wave
// says so in LDS (gemm_publish, attn_publish), and the issuing waves wait for those words (p2_wait_words).  (Waiting for
// the flag's acknowledgement as well measured slower again: the hand-over then starts too late.)
// Spin (bounded) until the sync words of waves lo .. hi-1 have reached `token`.  The words are compared as
// "this epoch or a later one": a workgroup without an attention unit passes no workgroup barrier between its
// QKV and attention phases, so a wave may already have written the next phase's token when a slower wave
// looks.  If the bound expires the error word is raised (every workgroup then leaves at its next barrier).
__device__ __forceinline__ void p2_wait_words(const PersistArgs &p, unsigned char *smem, unsigned token, int tid, int lo,
                                              int hi) {
  volatile unsigned *w = reinterpret_cast<volatile unsigned *>(smem + kSyncOff);
  const int lane = tid & 63;
  for (int spins = 0; spins < kSpinLimit; ++spins) {
    const unsigned v = w[lane & 7];                  // (read unconditionally: a load through a selected address
    if (__all(lane < lo || lane >= hi || (int)(v - token) >= 0)) return;   //  would put `token` on the stack)
  }
  if (lane == 0) __hip_atomic_fetch_or(p.err, kErrBarrier, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The same for the end of a GEMM phase, without a workgroup barrier: the transfer-issuing waves are still
// busy handing the next phase's weights over (a wave's transfers leave at the pace HBM serves them, so
// the last ones are issued microseconds after the first) and must not hold the flag back.  Each of the
// other waves waits for its own stores and says so in LDS; wave 0 collects the words and sets the flag.
// `token` is the epoch being published: a value no earlier phase has written.
__device__ __forceinline__ void gemm_publish(const PersistArgs &p, int wg, unsigned token, unsigned char *smem, int tid) {
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  if (wave >= kPfWave0) return;
  volatile unsigned *sync_s = reinterpret_cast<volatile unsigned *>(smem + kSyncOff);
  wait_vmcnt_all();
  if (lane == 0) sync_s[wave] = token;
  if (wave != 0) return;
  p2_wait_words(p, smem, token, tid, 1, kPfWave0);
  p2_store_flag(p.flags, p.flag_copies, wg, token, lane);
}

__device__ __forceinline__ void p2_handover_issue(const PersistArgs &p, int ng, int wg, int nwg, uint32_t pf_lds);

// End of an attention phase: every wave may have stored (output records, appended cache rows).  Each
// waits for its own stores and says so; the issuing waves then start the O-projection's hand-over, and
// wave 0 sets the flag once the other seven words are in - again without a workgroup barrier.
__device__ __forceinline__ void attn_publish(const PersistArgs &p, int wg, int nwg, int ng, unsigned token,
                                             unsigned char *smem, uint32_t pf_lds, int tid) {
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  volatile unsigned *sync_s = reinterpret_cast<volatile unsigned *>(smem + kSyncOff);
  wait_vmcnt_all();
  if (lane == 0) sync_s[wave] = token;
  if (wave != 0) {
    if (wave >= kPfWave0) {
      p2_wait_words(p, smem, token, tid, 0, kFastWaves);
      p2_handover_issue(p, ng, wg, nwg, pf_lds);
    }
    return;
  }
  p2_wait_words(p, smem, token, tid, 1, kFastWaves);
  p2_store_flag(p.flags, p.flag_copies, wg, token, lane);
}

// Wait until every workgroup has published `epoch` - or, with `subset` (n_subset <= 64 workgroup indices), until
// those workgroups have.  Wave 0 polls; the others meet it at the workgroup
// barrier with their requested loads still in flight - except that with land_transfers the issuing
// waves first wait for their global -> LDS transfers, so that after the barrier every wave may read
// what was handed over.  Returns false if the wait gave up (error word raised) or an error was seen.
__device__ __forceinline__ bool grid_wait(const PersistArgs &p, int nwg, unsigned epoch, bool land_transfers,
                                          unsigned char *smem, const int *subset = nullptr, int n_subset = 0) {
  volatile int &s_ok = *reinterpret_cast<volatile int *>(smem + kOkOff);
  const int tid = p2_tid(), wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (wave == 0) {
    const int lane = tid;
    int spins = 0;
    bool good = true;
    const unsigned *my_flags = p.flags + (p.flag_copies > 1 ? (size_t)(blockIdx.x & (kFlagCopies - 1)) * kFlagCopyWords : 0);   // this XCD's copy
    const unsigned long long *f64 = reinterpret_cast<const unsigned long long *>(my_flags);
    const int mine = (subset && lane < n_subset) ? subset[lane] : 0;      // one flag per lane
    while (true) {
      bool ok = true;
      if (subset) {
        if (lane < n_subset) {      // (the other lanes load nothing: 200 workgroups polling one spare word would queue on it)
          const unsigned f = __hip_atomic_load(my_flags + mine * kFlagStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ok = (int)(f - epoch) >= 0;
        }
      } else {
        for (int i = lane; 2 * i < nwg; i += kWave) {       // two flags per load
          const unsigned long long f = __hip_atomic_load(f64 + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ok = ok && ((int)((unsigned)f - epoch) >= 0) && (2 * i + 1 >= nwg || (int)((unsigned)(f >> 32) - epoch) >= 0);
        }
      }
      if (__all(ok)) break;
      __builtin_amdgcn_s_sleep(2);      // 256 pollers at full rate slow the loads they wait for (1 % of the step; with the flags
                                        // in uncached memory pauses of 2 / 4 / 8 / 16 measured 2.773 / 2.777 / 2.777 / 2.780 ms)
      if (++spins > p.spin_limit ||
          ((spins & 255) == 0 && (__hip_atomic_load(p.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kErrBarrier) != 0u)) {
        good = false;
        break;
      }
    }
    if (p.trace && lane == 0)      // slot 6: the polls have seen every flag (slot 1, taken after this function, includes
      p.trace[((size_t)(epoch - p.epoch0) * gridDim.x + blockIdx.x) * 8 + 6] = wall_clock64();   // the transfers' landing)
    if (!good && lane == 0) __hip_atomic_fetch_or(p.err, kErrBarrier, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (lane == 0) s_ok = good ? 1 : 0;
  } else if (land_transfers && wave >= kPfWave0) {
    wait_vmcnt_all();
  }
  lds_barrier();
  const bool r = __builtin_amdgcn_readfirstlane(s_ok) != 0;     // the same word for every lane: keep the branch on it scalar
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

// The phase program never changes while a step runs: it is read through the constant address space, so
// that the (wave-uniform) descriptor fields arrive in scalar registers by scalar loads.  A plain copy of
// a descriptor out of global memory is made with vector loads into a stack object instead, and every
// later field access becomes a scratch access.
typedef const Phase __attribute__((address_space(4))) *cphase_t;
__device__ __forceinline__ cphase_t p2_phase(const PersistArgs &p, int ph) {
  return reinterpret_cast<cphase_t>(reinterpret_cast<uintptr_t>(p.prog + ph));
}

// Program entry with the step's own values filled in.
__device__ __forceinline__ FastGemm phase_gemm(const PersistArgs &p, int ph) {
  const cphase_t P = p2_phase(p, ph);
  FastGemm g;
  g.epi = P->g.epi;
  g.w[0] = P->g.w[0];
  g.w[1] = P->g.w[1];
  g.w[2] = P->g.w[2];
  g.seg_tiles = P->g.seg_tiles;
  g.n_units = P->g.n_units;
  g.Kd = P->g.Kd;
  g.b = P->g.b;
  g.ssq = P->g.ssq;
  g.n_ssq = P->g.n_ssq;
  g.eps = P->g.eps;
  g.M = p.batch * p.K;
  g.out = g.epi == FEPI_STORE_ROWS ? p.logits : P->g.out;
  g.ldo = P->g.ldo;
  g.next_gain = P->g.next_gain;
  g.o_planes = P->g.o_planes;
  g.ssq_out = P->g.ssq_out;
  g.xcd_heads = P->g.xcd_heads;
  return g;
}

// Addresses in these phase bodies are written as a wave-uniform 64-bit base (scalar registers, scalar
// arithmetic) plus one 32-bit per-lane byte offset that every load of a ring shares: a load then needs
// no vector address arithmetic and no vector register pair of its own.
// (The empty asm hides the offset from the optimiser, which would otherwise fold it into a loop-invariant
// per-lane 64-bit base and add the uniform part with vector instructions for every load.)
__device__ __forceinline__ u32x4 ld_gs(const void *sbase, uint32_t lane_off) {
  uint32_t o = lane_off;
  asm("" : "+v"(o));
  return *reinterpret_cast<gptr_u4>(reinterpret_cast<uintptr_t>(sbase) + (uint64_t)o);
}
// A wave-uniform pointer moved into scalar registers.  (Uniform values that come out of vector-only
// arithmetic - an integer division by a run-time value, say - stay in vector registers otherwise, and
// so does every address computed from them.)
template <typename T>
__device__ __forceinline__ const T *p2_scalar(const T *p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const T *>(((uint64_t)hi << 32) | lo);
}
// k-step 0 of tile entry e of this workgroup, lane 0 (wave-uniform).
__device__ __forceinline__ const uint16_t *p2_tile_base(const FastGemm &g, int wg, int nwg, int e) {
  const uint16_t *wbase;
  int wrow0, unit;
  fast_tile(g, wg, nwg, e, wbase, wrow0, unit);
  return p2_scalar(wbase + (size_t)(wrow0 >> 4) * (size_t)((g.Kd + 31) / 32) * 512);
}
// Weight fragment of k-step ks (wave-uniform, already clamped into the matrix); lane_off = 16 * lane.
__device__ __forceinline__ u32x4 p2_ld_a(const uint16_t *tbase, int ks, uint32_t lane_off) {
  return ld_gs(tbase + (size_t)ks * 512, lane_off);
}
// The k-step that step s of wave share w of a tile reads (the clamps of fast_gemm_phase and of
// fast_gemm_stream_phase: past the matrix, respectively past the wave's own share, re-read the last step).
__device__ __forceinline__ int p2_a_step(int Kd, bool stream, int w, int s) {
  const int total = (Kd + 31) / 32, ks0 = w * fast_ksw(Kd);
  int ks = ks0 + s;
  if (stream) ks = min(ks, ks0 + max(fast_steps(Kd, w), 1) - 1);
  return min(ks, total - 1);
}
// Activation fragment of step s of a wave that owns ns steps from ks0 (the zero records past them);
// b_off = this lane's byte offset inside a k-step's two records: record lg/2, row lr, half lg&1.
__device__ __forceinline__ uint32_t p2_b_lane_off(int lr, int lg) {
  return (uint32_t)(((lg >> 1) * 256 + lr * 16 + (lg & 1) * 8) * 2);
}
__device__ __forceinline__ u32x4 p2_ld_b(const uint16_t *planes, int Kd, int ks0, int s, int ns, uint32_t b_off) {
  const int total = (Kd + 31) / 32;
  const int ks = (s < ns) ? ks0 + s : total;
  return ld_gs(planes + (size_t)ks * 512, b_off);
}

// Hand-over for the GEMM of phase `ng` (-1: none): the issuing waves start the transfers of steps
// 0 .. kPF-1 of every wave share of this workgroup's first tile into the LDS region at pf_lds,
// fragment (w, s) at (w*kPF + s) KB - the k-steps p2_a_step names.
// The region must be free (every wave past its reads of it).  Everything but the lane's 16-byte slot
// is wave-uniform, so the addresses are scalar arithmetic.
__device__ __forceinline__ void p2_handover_issue(const PersistArgs &p, int ng, int wg, int nwg, uint32_t pf_lds) {
  const int tid = p2_tid(), wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  if (ng < 0 || wave < kPfWave0) return;
  const cphase_t N = p2_phase(p, ng);
  const int Kd = N->g.Kd, n_units = N->g.n_units, epi = N->g.epi, seg_tiles = N->g.seg_tiles;
  if (wg >= n_units) return;                                   // no tile of that GEMM is this workgroup's
  const bool stream = N->kind == PH_GEMM_STREAM;
  // tile entry 0 of workgroup wg is unit wg: the gate tile of pair wg, or tile wg of the segmented matrix
  const int seg = epi == FEPI_SWIGLU ? 0 : wg / seg_tiles;
  const uint16_t *wbase = seg == 0 ? N->g.w[0] : (seg == 1 ? N->g.w[1] : N->g.w[2]);
  int tile = epi == FEPI_SWIGLU ? wg : wg - seg * seg_tiles;
  if (N->g.xcd_heads && nwg == 256) tile = fast_xcd_tile(wg);          // as fast_tile deals them
  const int total = (Kd + 31) / 32;
  const uint16_t *tbase = p2_scalar(wbase + (size_t)tile * (size_t)total * 512);      // k-step 0 of the tile, lane 0
  constexpr int SH = kFastWaves / (kFastWaves - kPfWave0);     // wave shares per issuing wave
  const uint32_t lane_off = (uint32_t)lane * 16u;
  wait_vmcnt_all();                                            // nothing of this wave's own is pending
#pragma unroll 1
  for (int i = 0; i < SH; ++i) {
    const int w = (wave - kPfWave0) * SH + i;
    if ((i + 1) * kPfBefore > 63) wait_vmcnt<63 - kPfBefore>();   // a wave keeps at most 63 memory operations outstanding
#pragma unroll
    for (int s = 0; s < kPfBefore; ++s) {
      const int ks = __builtin_amdgcn_readfirstlane(p2_a_step(Kd, stream, w, s));
      lds_dma16_s(tbase + (size_t)ks * 512, lane_off,
                  __builtin_amdgcn_readfirstlane(pf_lds + (uint32_t)((w * kPF + s) * 1024)));
    }
  }
}

// The rest of the hand-over (steps kPfBefore .. kPF-1), started by every wave for its own share when the barrier
// is passed, in front of its other requests: what the wave reads from LDS at those steps it reads behind
// activation fragments requested later, so the transfers have landed by then (a wave's memory operations
// complete in order).
__device__ __forceinline__ void p2_handover_rest(const uint16_t *tb0, int Kd, bool stream, int wave, int lane, uint32_t pf_lds) {
  if (kPfBefore >= kPF) return;
  const uint32_t lane_off = (uint32_t)lane * 16u;
#pragma unroll
  for (int s = kPfBefore; s < kPF; ++s) {
    const int ks = __builtin_amdgcn_readfirstlane(p2_a_step(Kd, stream, wave, s));
    lds_dma16_s(tb0 + (size_t)ks * 512, lane_off, __builtin_amdgcn_readfirstlane(pf_lds + (uint32_t)((wave * kPF + s) * 1024)));
  }
}

__device__ __forceinline__ uint32_t p2_lds_addr(const unsigned char *smem) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char *)smem;
}

// One resident-B GEMM phase (Kd <= 4096).  Same arithmetic, order of additions included, as
// fast_gemm_phase; the differences are where the first ring comes from and what happens around the
// barrier.  Returns false if the barrier gave up.
__device__ __forceinline__ bool p2_gemm_phase(const PersistArgs &p, int ph, int wg, int nwg, unsigned char *smem,
                                              unsigned wait_epoch) {
  const FastGemm g = phase_gemm(p, ph);
  const int ng = p2_phase(p, ph)->next_gemm;
  float *red = reinterpret_cast<float *>(smem);
  float *scale_s = reinterpret_cast<float *>(smem + kCtlOff);
  const u32x4 *pf = reinterpret_cast<const u32x4 *>(smem + kPfOff);
  const uint32_t pf_lds = p2_lds_addr(smem) + (uint32_t)kPfOff;
  const int tid = p2_tid(), lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t a_off = (uint32_t)lane * 16u, b_off = p2_b_lane_off(lane & 15, lane >> 4);
  const int my_entries = fast_my_entries(g, wg, nwg);
  const int ks0 = wave * fast_ksw(g.Kd), ns = fast_steps(g.Kd, wave);
  const uint16_t *tb0 = my_entries > 0 ? p2_tile_base(g, wg, nwg, 0) : g.w[0];
  Frag16 A;
  const int ft = p2_phase(p, ph)->first_tile;
  const bool in_lds = (ft & PHF_IN_LDS) != 0, early = (ft & PHF_EARLY) != 0;
  // The first request into the register ring: the first tile - or, when that one was handed over in LDS, the
  // second, so that weights stream while the activation fragments are still on their way.
  const uint16_t *tb_ring = in_lds ? (my_entries > 1 ? p2_tile_base(g, wg, nwg, 1) : nullptr) : tb0;
  if (my_entries > 0 && wave != 0 && early && tb_ring) {     // the polling wave keeps nothing in flight
#pragma unroll
    for (int s = 0; s < kKS; ++s) A.v[s] = p2_ld_a(tb_ring, p2_a_step(g.Kd, false, wave, s), a_off);
  }
  if (!grid_wait(p, nwg, wait_epoch, true, smem)) return false;
  p2_stamp(p, wg, ph, 1);
  if (my_entries == 0) {
    p2_handover_issue(p, ng, wg, nwg, pf_lds);
    gemm_publish(p, wg, wait_epoch + 1, smem, tid);
    return true;
  }
  if (in_lds) p2_handover_rest(tb0, g.Kd, false, wave, lane, pf_lds);
  const bool ring_now = (wave == 0 || !early) && tb_ring;
  if (ring_now && !in_lds) {
#pragma unroll
    for (int s = 0; s < kKS; ++s) A.v[s] = p2_ld_a(tb_ring, p2_a_step(g.Kd, false, wave, s), a_off);
  }
  const SsqPre sp = fast_row_scales_issue(g, wave, lane);
  Frag16 Bf;
#pragma unroll
  for (int s = 0; s < kKS; ++s) Bf.v[s] = p2_ld_b(g.b, g.Kd, ks0, s, ns, b_off);
  if (ring_now && in_lds) {                                  // behind the activation fragments, which are needed first
#pragma unroll
    for (int s = 0; s < kKS; ++s) A.v[s] = p2_ld_a(tb_ring, p2_a_step(g.Kd, false, wave, s), a_off);
  }
  for (int e0 = 0; e0 < my_entries; e0 += kMaxT) {
    f32x4 acc[kMaxT];
#pragma unroll
    for (int t = 0; t < kMaxT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    const EpiPre ep = fast_epilogue_preload(g, wg, nwg, e0, min(kMaxT, my_entries - e0), tid);
    asm volatile("" ::: "memory");       // the epilogue's loads are requested here, not moved down to their use
    if (e0 > 0) {
      const uint16_t *tb = p2_tile_base(g, wg, nwg, e0);
#pragma unroll
      for (int s = 0; s < kKS; ++s) A.v[s] = p2_ld_a(tb, p2_a_step(g.Kd, false, wave, s), a_off);
    }
#pragma unroll
    for (int t = 0; t < kMaxT; ++t) {
      if (t == 0 && e0 == 0 && in_lds) {
#pragma unroll
        for (int s = 0; s < kKS; ++s) {
          acc[0] = fast_mfma(pf[(wave * kPF + s) * 64 + lane], Bf.v[s], acc[0]);
          if ((s & 1) == 1) __builtin_amdgcn_sched_barrier(0);     // two fragments out of LDS at a time, not all sixteen
        }
      } else if (e0 + t < my_entries) {
        if (t + 1 < kMaxT && e0 + t + 1 < my_entries) {
          const uint16_t *tb = p2_tile_base(g, wg, nwg, e0 + t + 1);
#pragma unroll
          for (int s = 0; s < kKS; ++s) {
            acc[t] = fast_mfma(A.v[s], Bf.v[s], acc[t]);
            A.v[s] = p2_ld_a(tb, p2_a_step(g.Kd, false, wave, s), a_off);
          }
        } else {
#pragma unroll
          for (int s = 0; s < kKS; ++s) acc[t] = fast_mfma(A.v[s], Bf.v[s], acc[t]);
        }
      }
      // 1/rms of the rows, summed behind the first tile's products (the partial sums, requested before the
      // activation fragments, are here by then): off the path from the last product to the published outputs
      if (t == 0 && e0 == 0) fast_row_scales_finish(g, sp, scale_s, wave, lane);
    }
    lds_barrier();
    const bool last = e0 + kMaxT >= my_entries;
    if (last) p2_stamp(p, wg, ph, 2);
#pragma unroll
    for (int t = 0; t < kMaxT; ++t)
      *reinterpret_cast<f32x4 *>(red + ((size_t)(wave * kMaxT + t) * 64 + lane) * 4) = acc[t];
    lds_barrier();
    if (!last) {
      fast_epilogue(g, wg, nwg, e0, min(kMaxT, my_entries - e0), red, scale_s, ep, tid);
      lds_barrier();
    } else if (wave >= kPfWave0) {
      // last pass: the weights are consumed and the hand-over region is free.  From here to the next
      // phase's barrier the issuing waves and the storing waves go separate ways (no workgroup barrier).
      p2_wait_words(p, smem, wait_epoch + 1, tid, 0, kPfWave0);
      p2_handover_issue(p, ng, wg, nwg, pf_lds);
    } else {
      p2_stamp(p, wg, ph, 4);
      fast_epilogue(g, wg, nwg, e0, min(kMaxT, my_entries - e0), red, scale_s, ep, tid);
      p2_stamp(p, wg, ph, 5);
    }
  }
  gemm_publish(p, wg, wait_epoch + 1, smem, tid);
  return true;
}

// One streaming GEMM phase (long reductions: the down projection), arithmetic as fast_gemm_stream_phase.
__device__ __forceinline__ bool p2_gemm_stream_phase(const PersistArgs &p, int ph, int wg, int nwg, unsigned char *smem,
                                                     unsigned wait_epoch) {
  const FastGemm g = phase_gemm(p, ph);
  const int ng = p2_phase(p, ph)->next_gemm;
  float *red = reinterpret_cast<float *>(smem);
  float *scale_s = reinterpret_cast<float *>(smem + kCtlOff);
  const u32x4 *pf = reinterpret_cast<const u32x4 *>(smem + kPfOff);
  const uint32_t pf_lds = p2_lds_addr(smem) + (uint32_t)kPfOff;
  const int tid = p2_tid(), lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t a_off = (uint32_t)lane * 16u, b_off = p2_b_lane_off(lane & 15, lane >> 4);
  const int my_entries = fast_my_entries(g, wg, nwg);
  const int ksw = fast_ksw(g.Kd), ks0 = wave * ksw, ns = fast_steps(g.Kd, wave);
  const uint16_t *tb0 = my_entries > 0 ? p2_tile_base(g, wg, nwg, 0) : g.w[0];
  Frag16 A;
  const int ft = p2_phase(p, ph)->first_tile;
  const bool in_lds = (ft & PHF_IN_LDS) != 0, early = (ft & PHF_EARLY) != 0;
  if (my_entries > 0 && wave != 0 && early) {     // the polling wave keeps nothing in flight
#pragma unroll
    for (int s = 0; s < kKS; ++s)
      if (s >= kPF || !in_lds) A.v[s] = p2_ld_a(tb0, p2_a_step(g.Kd, true, wave, s), a_off);
  }
  if (!grid_wait(p, nwg, wait_epoch, true, smem)) return false;
  p2_stamp(p, wg, ph, 1);
  if (my_entries == 0) {
    p2_handover_issue(p, ng, wg, nwg, pf_lds);
    gemm_publish(p, wg, wait_epoch + 1, smem, tid);
    return true;
  }
  if (in_lds) p2_handover_rest(tb0, g.Kd, true, wave, lane, pf_lds);
  if (wave == 0 || !early) {
#pragma unroll
    for (int s = 0; s < kKS; ++s)
      if (s >= kPF || !in_lds) A.v[s] = p2_ld_a(tb0, p2_a_step(g.Kd, true, wave, s), a_off);
  }
  const SsqPre sp = fast_row_scales_issue(g, wave, lane);
  for (int e = 0; e < my_entries; ++e) {
    const uint16_t *tb = p2_tile_base(g, wg, nwg, e);
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    Frag16 Bs;
    const EpiPre ep = fast_epilogue_preload(g, wg, nwg, e, 1, tid);
    asm volatile("" ::: "memory");       // the epilogue's loads are requested here, not moved down to their use
#pragma unroll
    for (int s = 0; s < kKS; ++s) Bs.v[s] = p2_ld_b(g.b, g.Kd, ks0, s, ns, b_off);
    if (e == 0 && in_lds) {
#pragma unroll
      for (int s = 0; s < kPfBefore; ++s) A.v[s] = pf[(wave * kPF + s) * 64 + lane];
      if (kPfBefore < kPF) {               // the rest was requested in front of the fragments above: wait for those
        wait_vmcnt_all();
        asm volatile("" ::: "memory");
#pragma unroll
        for (int s = kPfBefore; s < kPF; ++s) A.v[s] = pf[(wave * kPF + s) * 64 + lane];
      }
    } else if (e > 0) {
#pragma unroll
      for (int s = 0; s < kKS; ++s) A.v[s] = p2_ld_a(tb, p2_a_step(g.Kd, true, wave, s), a_off);
    }
    for (int base = 0; base < ksw; base += kKS) {
      if (base + kKS < ksw) {
#pragma unroll
        for (int s = 0; s < kKS; ++s) {
          acc = fast_mfma(A.v[s], Bs.v[s], acc);
          A.v[s] = p2_ld_a(tb, p2_a_step(g.Kd, true, wave, base + kKS + s), a_off);
          Bs.v[s] = p2_ld_b(g.b, g.Kd, ks0, base + kKS + s, ns, b_off);
        }
      } else {
#pragma unroll
        for (int s = 0; s < kKS; ++s) acc = fast_mfma(A.v[s], Bs.v[s], acc);
      }
    }
    lds_barrier();
    const bool last = e + 1 == my_entries;
    if (last) p2_stamp(p, wg, ph, 2);
    if (e == 0) fast_row_scales_finish(g, sp, scale_s, wave, lane);
    *reinterpret_cast<f32x4 *>(red + ((size_t)(wave * kMaxT) * 64 + lane) * 4) = acc;
    lds_barrier();
    if (!last) {
      fast_epilogue(g, wg, nwg, e, 1, red, scale_s, ep, tid);
      lds_barrier();
    } else if (wave >= kPfWave0) {                    // as in p2_gemm_phase: no workgroup barrier from here on
      p2_wait_words(p, smem, wait_epoch + 1, tid, 0, kPfWave0);
      p2_handover_issue(p, ng, wg, nwg, pf_lds);
    } else {
      p2_stamp(p, wg, ph, 4);
      fast_epilogue(g, wg, nwg, e, 1, red, scale_s, ep, tid);
      p2_stamp(p, wg, ph, 5);
    }
  }
  gemm_publish(p, wg, wait_epoch + 1, smem, tid);
  return true;
}

template <int HD>
__device__ __forceinline__ bool p2_attn_phase(const PersistArgs &p, int ph, int wg, int nwg, unsigned char *smem,
                                              unsigned wait_epoch) {
  const cphase_t P = p2_phase(p, ph);
  const int layer = P->layer;
  FastAttn at;
  at.qkv = reinterpret_cast<const float *>(P->g.b);
  at.k_cache = p.k_cache + (size_t)layer * p.kv_layer_stride;
  at.v_cache = p.v_cache + (size_t)layer * p.kv_layer_stride;
  at.prefix_len = p.prefix_len; at.rope = p.rope;
  {   // the test of this pointer against NULL is made here, per phase: hoisted out of the loop over phases the
      // outcome is one more value that lives across every phase body (it ended up in scratch)
    const uint8_t *sk = p.skip;
    asm volatile("" : "+s"(sk));
    at.skip = sk;
  }
  at.o_planes = P->g.o_planes;
  at.K = p.K; at.H = p.H; at.cap = p.cap; at.d = p.d; at.batch = p.batch; at.scale = p.scale;
  const int tid = p2_tid();
  int ab, ah, aj;
  const bool have = attn_unit_of(p, wg, nwg, 0, ab, ah, aj);
  AttnPre pre;
  if (have) fast_attn_prefetch<HD>(at, ab, ah, pre, tid);       // cached rows: no dependence on this step's q/k/v
  // (the polling wave included: leaving its rows for after the wait, so that its polls do not return behind
  //  them, measured 0.3 % slower)
  // An attention unit needs the q/k/v of ONE head: it waits for the workgroups that own that head's rows of
  // the QKV weights (p.attn_prod), not for all of them - neither for the last workgroup of the whole QKV phase
  // nor for a poll of every flag.  A workgroup without a unit waits for nothing.  (What an early unit writes -
  // output records, appended cache rows - is read only behind the next barrier, which is a full one.)
  if (have && !grid_wait(p, nwg, wait_epoch, false, smem, p.attn_prod + ah * p.n_prod, p.n_prod)) return false;
  p2_stamp(p, wg, ph, 1);
  const int ng = P->next_gemm;
  const uint32_t pf_lds = p2_lds_addr(smem) + (uint32_t)kPfOff;
  if (have) {
    fast_attn_unit<HD>(at, ab, ah, aj, smem + kAttnOff, pre, tid);
    for (int t = 1; attn_unit_of(p, wg, nwg, t, ab, ah, aj); ++t) {
      fast_attn_prefetch<HD>(at, ab, ah, pre, tid);
      if (!grid_wait(p, nwg, wait_epoch, false, smem, p.attn_prod + ah * p.n_prod, p.n_prod)) return false;
      fast_attn_unit<HD>(at, ab, ah, aj, smem + kAttnOff, pre, tid);
    }
  }
  p2_stamp(p, wg, ph, 2);
  attn_publish(p, wg, nwg, ng, wait_epoch + 1, smem, pf_lds, tid);
  return true;
}

template <int HD>
__global__ __launch_bounds__(kFastThreads) void persist_forward(PersistArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int wg = blockIdx.x, nwg = gridDim.x;
  const uint32_t pf_lds = p2_lds_addr(smem) + (uint32_t)kPfOff;
  if (threadIdx.x < kFastWaves) {      // the waves' words start at a value no phase of this launch publishes
    reinterpret_cast<volatile unsigned *>(smem + kSyncOff)[threadIdx.x] = p.epoch0;
  }
  lds_barrier();
  for (int ph = 0; ph < p.n_phases; ++ph) {
    const int kind = p2_phase(p, ph)->kind;
    const unsigned wait_epoch = p.epoch0 + (unsigned)ph;     // published by every workgroup after phase ph-1
    p2_stamp(p, wg, ph, 0);
    bool ok = true;
    if (kind == PH_GEMM) {
      ok = p2_gemm_phase(p, ph, wg, nwg, smem, wait_epoch);
    } else if (kind == PH_GEMM_STREAM) {
      ok = p2_gemm_stream_phase(p, ph, wg, nwg, smem, wait_epoch);
    } else if (kind == PH_ATTN) {
      ok = p2_attn_phase<HD>(p, ph, wg, nwg, smem, wait_epoch);
    } else {                                                  // PH_EMBED: the first phase, nothing to wait for
      const cphase_t P = p2_phase(p, ph);
      p2_handover_issue(p, P->next_gemm, wg, nwg, pf_lds);
      for (int tile = wg; tile < p.d / 16; tile += nwg)
        fast_embed_tile(p.ids, p.tok_emb, p.vocab, p.d, p.batch * p.K, tile, P->g.next_gain, P->g.out, P->g.o_planes,
                        P->g.ssq_out, p2_tid());
      grid_arrive(p, wg, wait_epoch + 1, true);
    }
    if (!ok) {                 // a wait gave up: nothing of this workgroup's may still be on its way into LDS when it ends
      wait_vmcnt_all();
      return;
    }
    p2_stamp(p, wg, ph, 3);
  }
  // Greedy bins and the acceptance scan: workgroup b judges episode b once every workgroup has published its
  // part of the logits (the epoch after the last phase).  The logits were written with device-scope stores
  // into lines nobody has read in this launch, so plain loads see them.
  if (wg < p.batch && p.acc.accepted_len) {      // (a prefill chunk or decode step has no drafts to judge)
    if (!grid_wait(p, nwg, p.epoch0 + (unsigned)p.n_phases, false, smem)) return;
    accept_episode<kFastThreads>(p.acc, wg, p2_tid());
  }
}

// epochs one launch consumes
inline unsigned persist_epochs(int n_phases) { return (unsigned)n_phases; }

}  // namespace heisd
