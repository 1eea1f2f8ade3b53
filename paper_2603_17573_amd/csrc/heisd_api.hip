// C ABI of the verify step: context, argument checks, workspace layout and the launch
// sequence of one step.  All arithmetic happens in the kernels included below.
#include "../../include/heisd_verify.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "heisd_attn.h"
#include "heisd_fast.h"
#include "heisd_persist.h"
#include "heisd_batch.h"
#include "heisd_gemm.h"
#include "heisd_misc.h"
#include "heisd_skip.h"
#include "heisd_retrieve.h"
#include "heisd_measure.h"

using namespace heisd;

struct heisd_verify_ctx {
  heisd_model_desc d;
  std::vector<const void *> wq, wk, wv, wo, w_gate, w_up, w_down;
  std::vector<const float *> attn_norm, ffn_norm;
  // copies of the matrices in MFMA fragment order (see fast_pack_weights), in the workspace
  std::vector<const uint16_t *> pq, pk, pv, po, pg, pu, pd;
  const uint16_t *plm = nullptr;       // the n_bins LM-head rows
  // workspace carve-up
  float2 *rope;
  float *x, *qkv, *attn_o, *act, *logits;
  int32_t *tbins;
  int32_t *tree_depth, *tree_path;     // tree steps: depth of every token, accepted path when the caller wants none
  unsigned long long *tree_anc;        // tree steps: visibility bits [rows][4]
  unsigned char *fscr;                 // fast path: per-layer exchange records (see FastScratch)
  unsigned char *bscr;                 // batched path (M > 8): records and row statistics (see BatScratch)
  Phase *prog;                         // persistent kernel: the phase program in device memory
  int n_phases = 0;
  unsigned *flags, *dev_err;           // persistent kernel: barrier flags [n_cu], error word
  unsigned *lm_done = nullptr;         // fused LM head + acceptance: arrival counter of its workgroups
  unsigned epoch = 0;                  // last barrier epoch handed out
  bool persist_ok = false;
  int *attn_prod = nullptr;            // persistent kernel: [n_heads][3 * head_dim / 16] producer workgroups of a head's q/k/v
  int qkv_xcd_heads = 0;               // persistent kernel: QKV tiles dealt so that a head is produced on the XCD that consumes it
  int act_bf16 = 0;                    // batch path from kActBf16MinRows rows: activations enter the GEMMs as one bf16 each (opt-in)
  int wait_limit = kSpinLimit, scale_spin = kScaleSpin;   // bounds of the in-kernel waits (heisd_debug_set_wait_limits)
  bool skip_scales = false;
  unsigned *sflags = nullptr;          // persistent kernel: barrier flags in uncached memory (flag_slot_acquire), or nullptr
  int sflag_slot = -1, sflag_dev = -1;
  unsigned scale_epoch = 0;            // batch path: epoch of the last projection of a normalised input (see BatGemm::scale_tag)
  int handover_mode = 0;               // persistent kernel: what crosses a grid barrier (see persist_build_program)
  unsigned long long *trace = nullptr; // device buffer [n_phases][8] when tracing is on
  bool trace_on = false;
  int n_cu = 256;
  int path = 0;                        // HEISD_PATH_*
  bool fast_ok = false;                // the shape fits the fast kernels
  bool originals_gone = false;         // heisd_verify_release_projections: the caller's projection matrices may be freed
  char err[256];
  // optional per-launch event timing
  bool prof_on = false;
  std::vector<hipEvent_t> ev;      // pairs (start, stop)
  std::vector<int> ev_class;       // kernel class of each recorded pair
  size_t ev_used = 0;
  int prof_steps = 0;
};

// Brackets the launches issued between its construction and destruction with two events.
struct ProfScope {
  heisd_verify_ctx *c;
  hipStream_t st;
  size_t slot;
  bool on;
  ProfScope(heisd_verify_ctx *ctx, int kclass, hipStream_t s, bool enabled) : c(ctx), st(s), slot(0), on(false) {
    if (!enabled || c->ev_used + 2 > c->ev.size()) return;
    on = true;
    slot = c->ev_used;
    c->ev_used += 2;
    c->ev_class.push_back(kclass);
    (void)hipEventRecord(c->ev[slot], st);
  }
  ~ProfScope() {
    if (on) (void)hipEventRecord(c->ev[slot + 1], st);
  }
};

static thread_local char g_init_err[256] = "";

static int fail(heisd_verify_ctx *ctx, int code, const char *fmt, ...) {
  char *dst = ctx ? ctx->err : g_init_err;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, 256, fmt, ap);
  va_end(ap);
  return code;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct WsLayout {
  size_t rope, x, qkv, attn_o, act, logits, tbins, tree_depth, tree_path, tree_anc, fscr, fscr_bytes, bscr, bscr_bytes, players, attn_prod, flags, trace, packed, packed_bytes, total;
};

// Buffers of the batched path (M > 8 rows).  One launch per phase, so one set serves every layer.
constexpr int kSplitMax = 16;         // runs a reduction is cut into at most (bat_gemm_wide)

struct BatScratch {
  int CTS;                         // column tiles allocated: those of max_batch*max_k rows, at least 8
  size_t rec_x, rec_o, rec_act, ssq, inv_rms, part, total;
  int part_tiles() const { return 4 * CTS > 128 ? 4 * CTS : 128; }   // 16 runs at up to 64 rows, 4 runs at any row count
  explicit BatScratch(const heisd_model_desc *d) {
    const size_t M = (size_t)d->max_batch * d->max_k;
    CTS = (int)((M + 7) / 8);
    if (CTS < 8) CTS = 8;
    // the wide kernel reads whole blocks of column tiles; one tile more keeps the distance between k-steps
    // from being a multiple of 8 KB (with that, workloads that use a few of the tiles read from few channels)
    if (CTS > 8) CTS = (CTS + kWdCols - 1) / kWdCols * kWdCols + 1;
    const size_t kd = 2 * (((size_t)d->d_model + 31) / 32) + 2, kf = 2 * (((size_t)d->d_ffn + 31) / 32) + 2;   // + a zero k-step
    size_t off = 0;
    rec_x = off;   off += kd * CTS * 512;
    rec_o = off;   off += kd * CTS * 512;
    rec_act = off; off += kf * CTS * 512;
    ssq = off;     off += align256((size_t)(d->d_model / 16) * CTS * 8 * sizeof(float));
    inv_rms = off; off += align256((size_t)CTS * 8 * sizeof(unsigned long long));   // epoch-tagged 1/rms of the rows
    // sums of split reductions (bat_gemm_wide): up to 3*d_model/16 units (QKV) x part_tiles() column tiles
    // (runs x tiles in use) x 64 lanes x float2
    part = off;    off += (size_t)(3 * d->d_model / 16) * part_tiles() * 512;
    total = align256(off);
  }
};

// Per-layer exchange buffers of the fast path.  Every buffer is written once per step, so an
// address is never re-read with stale contents inside one launch.
struct FastScratch {
  size_t rec_x_a, ssq_a, qkv, rec_attn, rec_x_b, ssq_b, rec_act, stride;
  explicit FastScratch(const heisd_model_desc *d) {
    const size_t nt = d->d_model / 16;
    // plane buffers end with all-zero records that out-of-range k-steps are pointed at
    const size_t pd = (size_t)fast_plane_records(d->d_model), pf = (size_t)fast_plane_records(d->d_ffn);
    size_t off = 0;
    rec_x_a = off;  off += pd * 512;
    ssq_a = off;    off += nt * kSsqStride * sizeof(float);
    qkv = off;      off += 3 * nt * 512;
    rec_attn = off; off += pd * 512;
    rec_x_b = off;  off += pd * 512;
    ssq_b = off;    off += nt * kSsqStride * sizeof(float);
    rec_act = off;  off += pf * 512;
    stride = align256(off);
  }
};

static hipError_t bat_prepare();
static hipError_t bat_ns_prepare();

static bool shape_ok(const heisd_model_desc *d) {
  return d && d->n_layers > 0 && d->d_model > 0 && d->n_heads > 0 && d->head_dim > 0 && d->d_ffn > 0 &&
         d->vocab > 0 && d->n_bins > 0 && d->max_batch > 0 && d->max_k > 0 && d->kv_capacity > 0 &&
         (int64_t)d->n_heads * d->head_dim == d->d_model && d->bin_token_base >= 0 &&
         (int64_t)d->bin_token_base + d->n_bins <= d->vocab;
}

static WsLayout ws_layout(const heisd_model_desc *d) {
  WsLayout w;
  const size_t M = (size_t)d->max_batch * d->max_k;
  size_t off = 0;
  w.rope = off;   off += align256((size_t)d->kv_capacity * (d->head_dim / 2) * sizeof(float2));
  w.x = off;      off += align256(M * d->d_model * sizeof(float));
  w.qkv = off;    off += align256(M * 3 * d->d_model * sizeof(float));
  w.attn_o = off; off += align256(M * d->d_model * sizeof(float));
  w.act = off;    off += align256(M * d->d_ffn * sizeof(float));
  w.logits = off; off += align256(M * d->n_bins * sizeof(float));
  w.tbins = off;  off += align256((size_t)d->max_batch * (d->max_k + 1) * sizeof(int32_t));
  w.tree_depth = off; off += align256(M * sizeof(int32_t));
  w.tree_path = off;  off += align256(M * sizeof(int32_t));
  w.tree_anc = off;   off += align256(M * 4 * sizeof(unsigned long long));
  w.fscr = off;
  w.fscr_bytes = FastScratch(d).stride * (size_t)(d->n_layers + 1);
  off += w.fscr_bytes;
  w.bscr = off;
  w.bscr_bytes = BatScratch(d).total;
  off += w.bscr_bytes;
  w.players = off; off += align256((size_t)(5 * d->n_layers + 2) * sizeof(Phase));
  w.attn_prod = off; off += align256((size_t)d->n_heads * (3 * d->head_dim / 16) * sizeof(int));
  w.flags = off;   off += align256((size_t)(1024 + 64) * sizeof(unsigned));   // barrier flags, error word, LM-head arrival counter
  w.trace = off;   off += align256((size_t)(5 * d->n_layers + 2) * 1024 * 8 * sizeof(unsigned long long));   // [phase][workgroup][8]
  w.packed = off;
  const size_t per_layer = 4 * align256(fast_packed_elems(d->d_model, d->d_model) * 2) +
                           2 * align256(fast_packed_elems(d->d_ffn, d->d_model) * 2) +
                           align256(fast_packed_elems(d->d_model, d->d_ffn) * 2);
  w.packed_bytes = per_layer * (size_t)d->n_layers + align256(fast_packed_elems(d->n_bins, d->d_model) * 2);
  off += w.packed_bytes;
  w.total = off;
  return w;
}

extern "C" size_t heisd_verify_workspace_bytes(const heisd_model_desc *desc) {
  if (!shape_ok(desc)) return 0;
  return ws_layout(desc).total;
}

// ---- GEMM dispatch -------------------------------------------------------------------

template <int MC, int NT, int EPI>
static hipError_t gemm_prepare() {
  return hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_skinny<MC, NT, EPI>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_lds_bytes<MC>());
}

template <int MC>
static hipError_t gemm_prepare_mc() {
  hipError_t e;
  if ((e = gemm_prepare<MC, 1, EPI_STORE>()) != hipSuccess) return e;
  if ((e = gemm_prepare<MC, 2, EPI_SWIGLU>()) != hipSuccess) return e;
  if (MC <= 4)
    if ((e = gemm_prepare<(MC <= 4 ? MC : 1), 3, EPI_STORE>()) != hipSuccess) return e;
  return hipSuccess;
}

template <int MC>
static void gemm_launch_mc(const GemmArgs &a, int epi, hipStream_t st) {
  const size_t lds = gemm_lds_bytes<MC>();
  if (epi == EPI_SWIGLU) {
    gemm_skinny<MC, 2, EPI_SWIGLU><<<dim3(a.n_units), dim3(kGemmThreads), lds, st>>>(a);
  } else if (MC <= 4 && a.n_units >= 768 && a.n_units % 3 == 0) {
    gemm_skinny<(MC <= 4 ? MC : 1), 3, EPI_STORE><<<dim3(a.n_units / 3), dim3(kGemmThreads), lds, st>>>(a);
  } else {
    gemm_skinny<MC, 1, EPI_STORE><<<dim3(a.n_units), dim3(kGemmThreads), lds, st>>>(a);
  }
}

// y = act . W^T for all M rows, in row blocks of at most 64 rows (each block streams W once).
static void gemm_launch(GemmArgs a, int M, int epi, hipStream_t st) {
  const float *act = a.act;
  float *out = a.out;
  const float *resid = a.resid;
  for (int m0 = 0; m0 < M; m0 += 64) {
    const int mb = M - m0 < 64 ? M - m0 : 64;
    a.act = act + (size_t)m0 * a.Kd;
    a.out = out + (size_t)m0 * a.ldo;
    a.resid = resid ? resid + (size_t)m0 * a.ldo : nullptr;
    a.M = mb;
    if (mb <= 8) gemm_launch_mc<1>(a, epi, st);
    else if (mb <= 16) gemm_launch_mc<2>(a, epi, st);
    else if (mb <= 32) gemm_launch_mc<4>(a, epi, st);
    else gemm_launch_mc<8>(a, epi, st);
  }
}

// ---- any-M attention: workgroup size by the number of (episode, head) pairs ----------------

constexpr size_t kLdsPerWorkgroup = 160 * 1024;

template <int HD, int THREADS, bool TREE, bool SPLIT>
static hipError_t attn_prepare_one(int cap) {
  if (attn_lds_bytes(HD, cap, THREADS / 64) > kLdsPerWorkgroup) return hipSuccess;   // variant not used at this capacity
  return hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_verify<HD, THREADS, TREE, SPLIT>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_lds_bytes(HD, cap, THREADS / 64));
}
template <int HD, bool TREE>
static hipError_t attn_prepare_mode(int cap) {
  hipError_t e;
  if ((e = attn_prepare_one<HD, 256, TREE, false>(cap)) != hipSuccess) return e;
  if ((e = attn_prepare_one<HD, 512, TREE, false>(cap)) != hipSuccess) return e;
  if ((e = attn_prepare_one<HD, 256, TREE, true>(cap)) != hipSuccess) return e;
  return attn_prepare_one<HD, 512, TREE, true>(cap);
}
static hipError_t attn_prepare(int hd, int cap) {
  hipError_t e = hd == 128 ? attn_prepare_mode<128, false>(cap) : attn_prepare_mode<64, false>(cap);
  if (e != hipSuccess) return e;
  return hd == 128 ? attn_prepare_mode<128, true>(cap) : attn_prepare_mode<64, true>(cap);
}

// One workgroup per (head, episode) while an episode has at most 8 new rows (one block of queries);
// otherwise the append runs as a launch of its own and every block of 8 queries gets a workgroup.
template <int HD, bool TREE>
static void attn_launch_mode(const AttnArgs &a, int H, int batch, int cap, int n_cu, hipStream_t st) {
  const int nqb = (a.K + kAttnQB - 1) / kAttnQB;
  // at most one workgroup per compute unit: 512 threads each hide more latency (if their LDS fits)
  const bool big = H * batch * nqb <= n_cu && attn_lds_bytes(HD, cap, 8) <= kLdsPerWorkgroup;
  if (nqb == 1) {
    const dim3 grid(H, batch);
    if (big) attn_verify<HD, 512, TREE, false><<<grid, dim3(512), attn_lds_bytes(HD, cap, 8), st>>>(a);
    else attn_verify<HD, 256, TREE, false><<<grid, dim3(256), attn_lds_bytes(HD, cap, 4), st>>>(a);
    return;
  }
  attn_append<HD, TREE><<<dim3(H, batch, nqb), dim3(256), 0, st>>>(a);
  const dim3 grid(H, batch, nqb);
  if (big) attn_verify<HD, 512, TREE, true><<<grid, dim3(512), attn_lds_bytes(HD, cap, 8), st>>>(a);
  else attn_verify<HD, 256, TREE, true><<<grid, dim3(256), attn_lds_bytes(HD, cap, 4), st>>>(a);
}
static void attn_launch(const AttnArgs &a, int hd, int H, int batch, int cap, int n_cu, hipStream_t st) {
  const bool tree = a.depth != nullptr && a.anc != nullptr;
  if (hd == 128) {
    if (tree) attn_launch_mode<128, true>(a, H, batch, cap, n_cu, st);
    else attn_launch_mode<128, false>(a, H, batch, cap, n_cu, st);
  } else {
    if (tree) attn_launch_mode<64, true>(a, H, batch, cap, n_cu, st);
    else attn_launch_mode<64, false>(a, H, batch, cap, n_cu, st);
  }
}

// ---- weights in fragment order ------------------------------------------------------------

static hipError_t pack_one(const void *src, int rows, int Kd, unsigned char *&cursor, const uint16_t *&out) {
  uint16_t *dst = reinterpret_cast<uint16_t *>(cursor);
  const size_t pieces = fast_packed_elems(rows, Kd) / 8;
  const unsigned grid = (unsigned)((pieces + 255) / 256 < 65535 * 16 ? (pieces + 255) / 256 : 65535 * 16);
  fast_pack_weights<<<dim3(grid), dim3(256)>>>(static_cast<const uint16_t *>(src), rows, Kd, dst);
  out = dst;
  cursor += align256(fast_packed_elems(rows, Kd) * 2);
  return hipGetLastError();
}

// Copies every matrix the record kernels multiply into the workspace, in fragment order (init only).
static hipError_t pack_all(heisd_verify_ctx *c, unsigned char *cursor) {
  const heisd_model_desc &d = c->d;
  const int L = d.n_layers, dm = d.d_model, F = d.d_ffn;
  c->pq.resize(L); c->pk.resize(L); c->pv.resize(L); c->po.resize(L); c->pg.resize(L); c->pu.resize(L); c->pd.resize(L);
  hipError_t e = hipSuccess;
  for (int l = 0; l < L && e == hipSuccess; ++l) {
    e = pack_one(c->wq[l], dm, dm, cursor, c->pq[l]);
    if (e == hipSuccess) e = pack_one(c->wk[l], dm, dm, cursor, c->pk[l]);
    if (e == hipSuccess) e = pack_one(c->wv[l], dm, dm, cursor, c->pv[l]);
    if (e == hipSuccess) e = pack_one(c->wo[l], dm, dm, cursor, c->po[l]);
    if (e == hipSuccess) e = pack_one(c->w_gate[l], F, dm, cursor, c->pg[l]);
    if (e == hipSuccess) e = pack_one(c->w_up[l], F, dm, cursor, c->pu[l]);
    if (e == hipSuccess) e = pack_one(c->w_down[l], dm, F, cursor, c->pd[l]);
  }
  if (e == hipSuccess)
    e = pack_one(static_cast<const uint16_t *>(d.lm_head) + (size_t)d.bin_token_base * dm, d.n_bins, dm, cursor, c->plm);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  return e;
}

// ---- fast path (M <= 8 rows) ------------------------------------------------------------

static hipError_t fast_prepare(int hd, int cap) {
  hipError_t e;
  const int lds = (int)kFastLds;
  const void *fns[] = {reinterpret_cast<const void *>(&fast_gemm_kernel<HEISD_KC_QKV>),
                       reinterpret_cast<const void *>(&fast_gemm_kernel<HEISD_KC_OPROJ>),
                       reinterpret_cast<const void *>(&fast_gemm_kernel<HEISD_KC_GATEUP>),
                       reinterpret_cast<const void *>(&fast_gemm_kernel<HEISD_KC_DOWN>),
                       reinterpret_cast<const void *>(&fast_gemm_kernel<HEISD_KC_LMHEAD>),
                       reinterpret_cast<const void *>(&fast_gemm_stream_kernel<HEISD_KC_DOWN>),
                       reinterpret_cast<const void *>(&fast_lmhead_accept_kernel)};
  for (const void *f : fns)
    if ((e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds)) != hipSuccess) return e;
  const int alds = (int)fast_attn_lds(hd, cap);
  if (hd == 128)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fast_attn_kernel<128>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, alds);
  else
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fast_attn_kernel<64>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, alds);
  return e;
}

// GEMM descriptors of layer l (and of the LM head for l == n_layers), shared by both fast drivers.
struct FastLayerDescs {
  FastGemm qkv, oproj, gateup, down;
  FastAttn attn;
};

static FastGemm fast_lm_desc(const heisd_verify_ctx *ctx, int M, float *logits) {
  const heisd_model_desc &d = ctx->d;
  const FastScratch fs(&d);
  unsigned char *base = ctx->fscr + fs.stride * (size_t)d.n_layers;
  FastGemm g{};
  g.epi = FEPI_STORE_ROWS;
  g.w[0] = ctx->plm;
  g.seg_tiles = d.n_bins / 16; g.n_units = d.n_bins / 16; g.Kd = d.d_model;
  g.b = reinterpret_cast<const uint16_t *>(base + fs.rec_x_a);
  g.ssq = reinterpret_cast<const float *>(base + fs.ssq_a);
  g.n_ssq = d.d_model / 16; g.eps = d.rms_eps; g.M = M; g.out = logits; g.ldo = d.n_bins;
  return g;
}

static FastLayerDescs fast_layer_descs(const heisd_verify_ctx *ctx, const heisd_kv_desc *kv, int l, int K, int batch,
                                       const uint8_t *skip_mask) {
  const heisd_model_desc &d = ctx->d;
  const int M = batch * K, dm = d.d_model, F = d.d_ffn, H = d.n_heads, HD = d.head_dim, cap = d.kv_capacity;
  const FastScratch fs(&d);
  unsigned char *base = ctx->fscr + fs.stride * (size_t)l;
  unsigned char *nbase = ctx->fscr + fs.stride * (size_t)(l + 1);
  FastLayerDescs L{};
  FastGemm &q = L.qkv;
  q.epi = FEPI_STORE_REC;
  q.w[0] = ctx->pq[l];
  q.w[1] = ctx->pk[l];
  q.w[2] = ctx->pv[l];
  q.seg_tiles = dm / 16; q.n_units = 3 * dm / 16; q.Kd = dm;
  q.b = reinterpret_cast<const uint16_t *>(base + fs.rec_x_a);
  q.ssq = reinterpret_cast<const float *>(base + fs.ssq_a);
  q.n_ssq = dm / 16; q.eps = d.rms_eps; q.M = M;
  q.out = reinterpret_cast<float *>(base + fs.qkv);
  FastAttn &a = L.attn;
  const size_t layer_stride = (size_t)batch * H * cap * HD;
  a.qkv = reinterpret_cast<const float *>(base + fs.qkv);
  a.k_cache = static_cast<uint16_t *>(kv->k_cache) + (size_t)l * layer_stride;
  a.v_cache = static_cast<uint16_t *>(kv->v_cache) + (size_t)l * layer_stride;
  a.prefix_len = kv->prefix_len; a.skip = skip_mask; a.rope = ctx->rope;
  a.o_planes = reinterpret_cast<uint16_t *>(base + fs.rec_attn);
  a.K = K; a.H = H; a.cap = cap; a.d = dm; a.batch = batch; a.scale = 1.0f / std::sqrt((float)HD);
  FastGemm &o = L.oproj;
  o.epi = FEPI_RESID_NORM;
  o.w[0] = ctx->po[l];
  o.seg_tiles = dm / 16; o.n_units = dm / 16; o.Kd = dm;
  o.b = reinterpret_cast<const uint16_t *>(base + fs.rec_attn);
  o.ssq = nullptr; o.M = M; o.out = ctx->x; o.ldo = dm; o.next_gain = ctx->ffn_norm[l];
  o.o_planes = reinterpret_cast<uint16_t *>(base + fs.rec_x_b);
  o.ssq_out = reinterpret_cast<float *>(base + fs.ssq_b);
  FastGemm &g = L.gateup;
  g.epi = FEPI_SWIGLU;
  g.w[0] = ctx->pg[l];
  g.w[1] = ctx->pu[l];
  g.seg_tiles = F / 16; g.n_units = F / 16; g.Kd = dm;
  g.b = reinterpret_cast<const uint16_t *>(base + fs.rec_x_b);
  g.ssq = reinterpret_cast<const float *>(base + fs.ssq_b);
  g.n_ssq = dm / 16; g.eps = d.rms_eps; g.M = M;
  g.o_planes = reinterpret_cast<uint16_t *>(base + fs.rec_act);
  FastGemm &w = L.down;
  w.epi = FEPI_RESID_NORM;
  w.w[0] = ctx->pd[l];
  w.seg_tiles = dm / 16; w.n_units = dm / 16; w.Kd = F;
  w.b = reinterpret_cast<const uint16_t *>(base + fs.rec_act);
  w.ssq = nullptr; w.M = M; w.out = ctx->x; w.ldo = dm;
  w.next_gain = (l + 1 < d.n_layers) ? ctx->attn_norm[l + 1] : d.final_norm;
  w.o_planes = reinterpret_cast<uint16_t *>(nbase + fs.rec_x_a);
  w.ssq_out = reinterpret_cast<float *>(nbase + fs.ssq_a);
  return L;
}

// The decoder forward for M <= 8 rows, one launch per phase; leaves the bin logits in `logits`.
// With `accept` the LM-head launch also takes the greedy bins and runs the acceptance scan.
static void fast_forward(heisd_verify_ctx *ctx, const heisd_kv_desc *kv, const int32_t *draft_tokens, int K,
                         int batch, const uint8_t *skip_mask, float *logits, hipStream_t st, bool prof,
                         const AcceptArgs *accept = nullptr) {
  const heisd_model_desc &d = ctx->d;
  const int M = batch * K, dm = d.d_model, H = d.n_heads, HD = d.head_dim, cap = d.kv_capacity;
  const int ncu = ctx->n_cu;
  const FastScratch fs(&d);
  auto grid_for = [&](int units) { return dim3(units < ncu ? units : ncu); };
  {
    ProfScope ps(ctx, HEISD_KC_EMBED, st, prof);
    fast_embed_kernel<<<dim3(dm / 16), dim3(64), 0, st>>>(
        draft_tokens, static_cast<const uint16_t *>(d.tok_emb), d.vocab, dm, M, ctx->attn_norm[0], ctx->x,
        reinterpret_cast<uint16_t *>(ctx->fscr + fs.rec_x_a), reinterpret_cast<float *>(ctx->fscr + fs.ssq_a));
  }
  const size_t alds = fast_attn_lds(HD, cap);
  const bool stream_down = d.d_ffn > kFastWaves * kKS * 32;
  const FastGemm lm = fast_lm_desc(ctx, M, logits);
  for (int l = 0; l < d.n_layers; ++l) {
    const FastLayerDescs L = fast_layer_descs(ctx, kv, l, K, batch, skip_mask);
    {
      ProfScope ps(ctx, HEISD_KC_QKV, st, prof);
      fast_gemm_kernel<HEISD_KC_QKV><<<grid_for(L.qkv.n_units), dim3(kFastThreads), kFastLds, st>>>(L.qkv);
    }
    {
      ProfScope ps(ctx, HEISD_KC_ATTN, st, prof);
      if (HD == 128) fast_attn_kernel<128><<<dim3(H, batch * K), dim3(kFastThreads), alds, st>>>(L.attn);
      else fast_attn_kernel<64><<<dim3(H, batch * K), dim3(kFastThreads), alds, st>>>(L.attn);
    }
    {
      ProfScope ps(ctx, HEISD_KC_OPROJ, st, prof);
      fast_gemm_kernel<HEISD_KC_OPROJ><<<grid_for(L.oproj.n_units), dim3(kFastThreads), kFastLds, st>>>(L.oproj);
    }
    {
      ProfScope ps(ctx, HEISD_KC_GATEUP, st, prof);
      fast_gemm_kernel<HEISD_KC_GATEUP><<<grid_for(L.gateup.n_units), dim3(kFastThreads), kFastLds, st>>>(L.gateup);
    }
    {
      ProfScope ps(ctx, HEISD_KC_DOWN, st, prof);
      if (stream_down)
        fast_gemm_stream_kernel<HEISD_KC_DOWN><<<grid_for(L.down.n_units), dim3(kFastThreads), kFastLds, st>>>(L.down);
      else
        fast_gemm_kernel<HEISD_KC_DOWN><<<grid_for(L.down.n_units), dim3(kFastThreads), kFastLds, st>>>(L.down);
    }
  }
  {
    ProfScope ps(ctx, HEISD_KC_LMHEAD, st, prof);
    if (accept)
      fast_lmhead_accept_kernel<<<grid_for(lm.n_units), dim3(kFastThreads), kFastLds, st>>>(lm, *accept, batch, ctx->lm_done);
    else
      fast_gemm_kernel<HEISD_KC_LMHEAD><<<grid_for(lm.n_units), dim3(kFastThreads), kFastLds, st>>>(lm);
  }
}

// ---- persistent whole-step kernel ----------------------------------------------------------

// Barrier flags that scalar loads can poll: one allocation of uncached device memory per device, made on first
// use, cut into slots of 64 KB (eight copies of 1024 flags + spare), handed to contexts at init and taken back at heisd_free.  The
// allocation itself is never freed (memory of this kind that a kernel has read must outlive the process's
// other allocations).  A context that gets no slot keeps its flags in the workspace and polls them with vector
// loads.
constexpr int kFlagSlots = 32, kFlagDevices = 16;
constexpr size_t kFlagSlotBytes = 65536;      // room for kFlagCopies copies of the flag array
static_assert((size_t)kFlagCopies * kFlagCopyWords * 4 <= kFlagSlotBytes, "the copies fit a slot");
struct FlagPool {
  unsigned char *base = nullptr;
  bool tried = false;
  uint32_t used = 0;
};
static FlagPool g_flag_pool[kFlagDevices];
static std::mutex g_flag_mutex;

static unsigned *flag_slot_acquire(int dev, int *slot) {
  std::lock_guard<std::mutex> lock(g_flag_mutex);
  *slot = -1;
  if (dev < 0 || dev >= kFlagDevices) return nullptr;
  FlagPool &pool = g_flag_pool[dev];
  if (!pool.tried) {
    pool.tried = true;
    void *p = nullptr;
    if (hipExtMallocWithFlags(&p, kFlagSlots * kFlagSlotBytes, hipDeviceMallocUncached) == hipSuccess) pool.base = static_cast<unsigned char *>(p);
    else (void)hipGetLastError();
  }
  if (!pool.base) return nullptr;
  for (int s = 0; s < kFlagSlots; ++s)
    if (!(pool.used & (1u << s))) {
      unsigned char *q = pool.base + (size_t)s * kFlagSlotBytes;
      if (hipMemset(q, 0, kFlagSlotBytes) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
      }
      pool.used |= 1u << s;
      *slot = s;
      return reinterpret_cast<unsigned *>(q);
    }
  return nullptr;
}
static void flag_slot_release(int dev, int slot) {
  std::lock_guard<std::mutex> lock(g_flag_mutex);
  if (dev >= 0 && dev < kFlagDevices && slot >= 0 && slot < kFlagSlots) g_flag_pool[dev].used &= ~(1u << slot);
}

static const void *persist_pick(const heisd_verify_ctx *c) {
  return c->d.head_dim == 128 ? reinterpret_cast<const void *>(&persist_forward<128>)
                              : reinterpret_cast<const void *>(&persist_forward<64>);
}

static size_t persist_lds(const heisd_verify_ctx *c) { return persist_lds_bytes(c->d.head_dim, c->d.kv_capacity); }

// The persistent kernel needs every workgroup resident at once: one per compute unit.
static hipError_t persist_prepare(heisd_verify_ctx *c) {
  c->persist_ok = false;
  if (!c->fast_ok || c->n_cu > 512) return hipSuccess;      // a barrier poll covers 512 flags
  if (persist_lds(c) > kLdsPerWorkgroup) return hipSuccess;
  const void *fn = persist_pick(c);
  hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)persist_lds(c));
  if (e != hipSuccess) return e;
  int per_cu = 0;
  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kFastThreads, persist_lds(c));
  if (e != hipSuccess) return e;
  c->persist_ok = per_cu >= 1;
  return hipSuccess;
}

static bool qkv_xcd_eligible(const heisd_verify_ctx *c) {
  return c->n_cu == 256 && c->d.d_model == 4096 && c->d.head_dim == 128;
}

// The phase program of one step (everything that does not change from step to step).
// ctx->handover_mode (heisd_verify_set_handover; default 0):
//   0  every GEMM phase gets its first weight steps handed over in LDS by the phase before it (the
//      O-projection by the attention phase, at its end) and requests the rest before the barrier
//   1  as 0, but the O-projection's hand-over starts at the end of the QKV phase
//   2  no LDS hand-over: the whole first tile is requested into registers before the barrier
//   3  nothing is requested across a barrier
//   4  as 0, and the second weight tile is requested into registers before the barrier
//   5  as 0, with the QKV tiles dealt to the workgroups in their plain order (see fast_xcd_tile)
static hipError_t persist_build_program(heisd_verify_ctx *ctx) {
  const heisd_model_desc &d = ctx->d;
  const int L = d.n_layers;
  const FastScratch fs(&d);
  const bool stream_down = d.d_ffn > kFastWaves * kKS * 32;
  const int mode = ctx->handover_mode;
  const bool lds = mode == 0 || mode == 1 || mode == 4 || mode == 5;
  const int ft = (lds ? PHF_IN_LDS : 0) | (mode == 2 || mode == 4 ? PHF_EARLY : 0);
  auto nx = [&](int idx) { return lds ? idx : -1; };
  std::vector<Phase> prog;
  heisd_kv_desc no_kv{};
  Phase e{};
  e.kind = PH_EMBED; e.next_gemm = nx(1);
  e.g.next_gain = ctx->attn_norm[0]; e.g.out = ctx->x;
  e.g.o_planes = reinterpret_cast<uint16_t *>(ctx->fscr + fs.rec_x_a);
  e.g.ssq_out = reinterpret_cast<float *>(ctx->fscr + fs.ssq_a);
  prog.push_back(e);
  for (int l = 0; l < L; ++l) {
    const FastLayerDescs D = fast_layer_descs(ctx, &no_kv, l, 1, 1, nullptr);
    const int base = 1 + 5 * l;
    Phase q{}; q.kind = PH_GEMM; q.g = D.qkv; q.g.xcd_heads = ctx->qkv_xcd_heads; q.first_tile = ft; q.next_gemm = mode == 1 ? base + 2 : -1; prog.push_back(q);
    Phase a{}; a.kind = PH_ATTN; a.layer = l; a.next_gemm = mode == 0 || mode == 4 || mode == 5 ? base + 2 : -1;
    a.g.b = reinterpret_cast<const uint16_t *>(D.attn.qkv); a.g.o_planes = D.attn.o_planes; prog.push_back(a);
    Phase o{}; o.kind = PH_GEMM; o.g = D.oproj; o.first_tile = ft; o.next_gemm = nx(base + 3); prog.push_back(o);
    Phase g{}; g.kind = PH_GEMM; g.g = D.gateup; g.first_tile = ft; g.next_gemm = nx(base + 4); prog.push_back(g);
    Phase w{}; w.kind = stream_down ? PH_GEMM_STREAM : PH_GEMM; w.g = D.down; w.first_tile = ft; w.next_gemm = nx(base + 5); prog.push_back(w);
  }
  Phase lm{}; lm.kind = PH_GEMM; lm.g = fast_lm_desc(ctx, 1, nullptr); lm.first_tile = ft; lm.next_gemm = -1; prog.push_back(lm);
  ctx->n_phases = (int)prog.size();
  // which workgroups produce head h's rows of q, k and v: QKV unit u (segment * d/16 + tile) runs on workgroup u % n_cu
  const int tph = d.head_dim / 16, T = d.d_model / 16;
  std::vector<int> prod((size_t)d.n_heads * 3 * tph);
  for (int h = 0; h < d.n_heads; ++h)
    for (int seg = 0; seg < 3; ++seg)
      for (int c = 0; c < tph; ++c) {
        int w = (seg * T + h * tph + c) % ctx->n_cu;
        if (ctx->qkv_xcd_heads) w = 8 * (8 * (h / 8) + c) + h % 8;          // the inverse of fast_xcd_tile
        prod[((size_t)h * 3 + seg) * tph + c] = w;
      }
  const hipError_t ep = hipMemcpy(ctx->attn_prod, prod.data(), prod.size() * sizeof(int), hipMemcpyHostToDevice);
  if (ep != hipSuccess) return ep;
  return hipMemcpy(ctx->prog, prog.data(), prog.size() * sizeof(Phase), hipMemcpyHostToDevice);
}

static void persist_launch(heisd_verify_ctx *ctx, const heisd_kv_desc *kv, const int32_t *draft_tokens, int K,
                           int batch, const uint8_t *skip_mask, float *logits, const AcceptArgs &accept, hipStream_t st) {
  const heisd_model_desc &d = ctx->d;
  PersistArgs p{};
  p.prog = ctx->prog; p.n_phases = ctx->n_phases;
  p.d = d.d_model; p.H = d.n_heads; p.vocab = d.vocab; p.cap = d.kv_capacity;
  p.tok_emb = static_cast<const uint16_t *>(d.tok_emb);
  p.scale = 1.0f / std::sqrt((float)d.head_dim);
  p.rope = ctx->rope;
  p.ids = draft_tokens;
  p.k_cache = static_cast<uint16_t *>(kv->k_cache); p.v_cache = static_cast<uint16_t *>(kv->v_cache);
  p.kv_layer_stride = (size_t)batch * d.n_heads * d.kv_capacity * d.head_dim;
  p.prefix_len = kv->prefix_len; p.skip = skip_mask; p.K = K; p.batch = batch; p.logits = logits;
  p.flags = ctx->flags; p.err = ctx->dev_err;
  p.trace = ctx->trace_on ? ctx->trace : nullptr;
  p.attn_prod = ctx->attn_prod; p.n_prod = 3 * d.head_dim / 16;
  p.spin_limit = ctx->wait_limit;
  p.flag_copies = 1;
  if (ctx->sflags) {
    p.flags = ctx->sflags;
    p.flag_copies = kFlagCopies;
  }
  p.acc = accept;
  p.epoch0 = ctx->epoch;
  ctx->epoch += persist_epochs(ctx->n_phases);
  const dim3 grid(ctx->n_cu), block(kFastThreads);
  const size_t lds = persist_lds(ctx);
  if (d.head_dim == 128) persist_forward<128><<<grid, block, lds, st>>>(p);
  else persist_forward<64><<<grid, block, lds, st>>>(p);
}

// ---- init / free ------------------------------------------------------------------------

extern "C" int heisd_verify_init(const heisd_model_desc *desc, heisd_verify_ctx **out) {
  if (!desc || !out) return fail(nullptr, HEISD_EINVAL, "init: NULL argument");
  *out = nullptr;
  if (!shape_ok(desc)) return fail(nullptr, HEISD_EINVAL, "init: inconsistent model shape");
  if (!desc->tok_emb || !desc->wq || !desc->wk || !desc->wv || !desc->wo || !desc->w_gate || !desc->w_up ||
      !desc->w_down || !desc->attn_norm || !desc->ffn_norm || !desc->final_norm || !desc->lm_head ||
      !desc->workspace)
    return fail(nullptr, HEISD_EINVAL, "init: NULL weight, table or workspace pointer");
  for (int l = 0; l < desc->n_layers; ++l)
    if (!desc->wq[l] || !desc->wk[l] || !desc->wv[l] || !desc->wo[l] || !desc->w_gate[l] || !desc->w_up[l] ||
        !desc->w_down[l] || !desc->attn_norm[l] || !desc->ffn_norm[l])
      return fail(nullptr, HEISD_EINVAL, "init: NULL weight pointer in layer %d", l);
  if (desc->head_dim != 64 && desc->head_dim != 128)
    return fail(nullptr, HEISD_EUNSUPPORTED, "init: head_dim %d (64 or 128 supported)", desc->head_dim);
  if (desc->d_model % 16 || desc->d_ffn % 16 || desc->n_bins % 16)
    return fail(nullptr, HEISD_EUNSUPPORTED, "init: d_model, d_ffn and n_bins must be multiples of 16");
  if (desc->max_k > 1024) return fail(nullptr, HEISD_EUNSUPPORTED, "init: max_k %d > 1024", desc->max_k);
  if (desc->kv_capacity > 4096)
    return fail(nullptr, HEISD_EUNSUPPORTED, "init: kv_capacity %d > 4096", desc->kv_capacity);
  if (((uintptr_t)desc->workspace & 255) != 0) return fail(nullptr, HEISD_EINVAL, "init: workspace not 256-byte aligned");
  const WsLayout w = ws_layout(desc);
  if (desc->workspace_bytes < w.total)
    return fail(nullptr, HEISD_ENOMEM, "init: workspace %zu bytes < %zu needed", desc->workspace_bytes, w.total);

  heisd_verify_ctx *c = new (std::nothrow) heisd_verify_ctx();
  if (!c) return fail(nullptr, HEISD_EHIP, "init: host allocation failed");
  c->d = *desc;
  c->err[0] = 0;
  const int L = desc->n_layers;
  c->wq.assign(desc->wq, desc->wq + L);
  c->wk.assign(desc->wk, desc->wk + L);
  c->wv.assign(desc->wv, desc->wv + L);
  c->wo.assign(desc->wo, desc->wo + L);
  c->w_gate.assign(desc->w_gate, desc->w_gate + L);
  c->w_up.assign(desc->w_up, desc->w_up + L);
  c->w_down.assign(desc->w_down, desc->w_down + L);
  c->attn_norm.assign(desc->attn_norm, desc->attn_norm + L);
  c->ffn_norm.assign(desc->ffn_norm, desc->ffn_norm + L);
  c->d.wq = c->d.wk = c->d.wv = c->d.wo = c->d.w_gate = c->d.w_up = c->d.w_down = nullptr;
  c->d.attn_norm = c->d.ffn_norm = nullptr;
  unsigned char *base = static_cast<unsigned char *>(desc->workspace);
  c->rope = reinterpret_cast<float2 *>(base + w.rope);
  c->x = reinterpret_cast<float *>(base + w.x);
  c->qkv = reinterpret_cast<float *>(base + w.qkv);
  c->attn_o = reinterpret_cast<float *>(base + w.attn_o);
  c->act = reinterpret_cast<float *>(base + w.act);
  c->logits = reinterpret_cast<float *>(base + w.logits);
  c->tbins = reinterpret_cast<int32_t *>(base + w.tbins);
  c->tree_depth = reinterpret_cast<int32_t *>(base + w.tree_depth);
  c->tree_path = reinterpret_cast<int32_t *>(base + w.tree_path);
  c->tree_anc = reinterpret_cast<unsigned long long *>(base + w.tree_anc);
  c->fscr = base + w.fscr;
  c->bscr = base + w.bscr;
  c->prog = reinterpret_cast<Phase *>(base + w.players);
  c->attn_prod = reinterpret_cast<int *>(base + w.attn_prod);
  c->flags = reinterpret_cast<unsigned *>(base + w.flags);
  c->dev_err = c->flags + 1024;
  c->lm_done = c->flags + 1024 + 16;
  c->trace = reinterpret_cast<unsigned long long *>(base + w.trace);
  c->fast_ok = desc->d_model <= kFastWaves * kKS * 32;
  c->path = HEISD_PATH_AUTO;

  // rotary table: angle = position * rope_base^(-2i/head_dim), computed in double on the host
  const int half = desc->head_dim / 2;
  std::vector<float2> tab((size_t)desc->kv_capacity * half);
  for (int p = 0; p < desc->kv_capacity; ++p)
    for (int i = 0; i < half; ++i) {
      const double ang = (double)p * std::pow((double)desc->rope_base, -2.0 * i / desc->head_dim);
      tab[(size_t)p * half + i] = make_float2((float)std::cos(ang), (float)std::sin(ang));
    }
  hipError_t e = hipMemcpy(c->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemset(base + w.fscr, 0, w.fscr_bytes);   // records start as zeros
  if (e == hipSuccess) e = hipMemset(base + w.bscr, 0, w.bscr_bytes);   // (the zero k-tiles stay zero)
  if (e == hipSuccess) {
    int dev = 0;
    hipDeviceProp_t prop;
    e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e == hipSuccess) c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  }
  c->qkv_xcd_heads = qkv_xcd_eligible(c) ? 1 : 0;
  if (e == hipSuccess) e = hipMemset(base + w.flags, 0, (size_t)(1024 + 64) * sizeof(unsigned));
  if (e == hipSuccess) e = pack_all(c, base + w.packed);
  if (e == hipSuccess) e = fast_prepare(desc->head_dim, desc->kv_capacity);
  if (e == hipSuccess) e = persist_prepare(c);
  if (e == hipSuccess && c->persist_ok) e = persist_build_program(c);
  if (e == hipSuccess && c->persist_ok && c->n_cu == 256) {
    int dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) {
      c->sflags = flag_slot_acquire(dev, &c->sflag_slot);
      c->sflag_dev = dev;
    }
  }
  if (e == hipSuccess) e = bat_prepare();
  if (e == hipSuccess) e = gemm_prepare_mc<1>();
  if (e == hipSuccess) e = gemm_prepare_mc<2>();
  if (e == hipSuccess) e = gemm_prepare_mc<4>();
  if (e == hipSuccess) e = gemm_prepare_mc<8>();
  if (e == hipSuccess) e = attn_prepare(desc->head_dim, desc->kv_capacity);
  if (e != hipSuccess) {
    const int rc = fail(nullptr, HEISD_EHIP, "init: %s", hipGetErrorString(e));
    if (c->sflags) flag_slot_release(c->sflag_dev, c->sflag_slot);
    delete c;
    return rc;
  }
  *out = c;
  g_init_err[0] = 0;
  return HEISD_OK;
}

extern "C" int heisd_verify_set_path(heisd_verify_ctx *ctx, int path) {
  if (!ctx) return HEISD_EINVAL;
  if (path != HEISD_PATH_AUTO && path != HEISD_PATH_GENERIC && path != HEISD_PATH_FAST && path != HEISD_PATH_PERSIST &&
      path != HEISD_PATH_BATCH)
    return fail(ctx, HEISD_EINVAL, "set_path: unknown path %d", path);
  if (path == HEISD_PATH_GENERIC && ctx->originals_gone)
    return fail(ctx, HEISD_EUNSUPPORTED, "set_path: the projection matrices were released (heisd_verify_release_projections)");
  if (path == HEISD_PATH_FAST && !ctx->fast_ok)
    return fail(ctx, HEISD_EUNSUPPORTED, "set_path: model shape outside the fast kernels");
  if (path == HEISD_PATH_PERSIST && !ctx->persist_ok)
    return fail(ctx, HEISD_EUNSUPPORTED, "set_path: the persistent kernel does not fit this device or shape");
  ctx->path = path;
  return HEISD_OK;
}

extern "C" int heisd_verify_release_projections(heisd_verify_ctx *ctx) {
  if (!ctx) return HEISD_EINVAL;
  if (ctx->path == HEISD_PATH_GENERIC)
    return fail(ctx, HEISD_EUNSUPPORTED, "release_projections: HEISD_PATH_GENERIC is selected and reads them");
  ctx->originals_gone = true;
  for (auto *v : {&ctx->wq, &ctx->wk, &ctx->wv, &ctx->wo, &ctx->w_gate, &ctx->w_up, &ctx->w_down}) v->assign(v->size(), nullptr);
  ctx->d.lm_head = nullptr;
  return HEISD_OK;
}

extern "C" int heisd_verify_set_activations(heisd_verify_ctx *ctx, int format) {
  if (!ctx) return HEISD_EINVAL;
  if (format != HEISD_ACT_SPLIT && format != HEISD_ACT_BF16) return fail(ctx, HEISD_EINVAL, "set_activations: unknown format %d", format);
  ctx->act_bf16 = format == HEISD_ACT_BF16;
  return HEISD_OK;
}

extern "C" int heisd_verify_set_handover(heisd_verify_ctx *ctx, int mode) {
  if (!ctx) return HEISD_EINVAL;
  if (mode < 0 || mode > 5) return fail(ctx, HEISD_EINVAL, "set_handover: unknown mode %d", mode);
  if (!ctx->persist_ok) return fail(ctx, HEISD_EUNSUPPORTED, "set_handover: the persistent kernel does not fit this device or shape");
  if (hipDeviceSynchronize() != hipSuccess) return fail(ctx, HEISD_EHIP, "set_handover: device error");
  ctx->handover_mode = mode;
  ctx->qkv_xcd_heads = qkv_xcd_eligible(ctx) && mode != 5 ? 1 : 0;
  const hipError_t e = persist_build_program(ctx);
  if (e != hipSuccess) return fail(ctx, HEISD_EHIP, "set_handover: %s", hipGetErrorString(e));
  return HEISD_OK;
}

// Measurement aid: timestamps (100 MHz counter) every workgroup of the persistent kernel takes in every
// phase of a step, [phase][workgroup][8].  enable != 0 switches recording on; out (HOST) may be NULL.
extern "C" int heisd_debug_trace(heisd_verify_ctx *ctx, int enable, unsigned long long *out, int max_entries) {
  if (!ctx) return HEISD_EINVAL;
  if (enable && !ctx->trace_on) {      // slots a workgroup does not write in a phase read 0
    if (hipDeviceSynchronize() != hipSuccess ||
        hipMemset(ctx->trace, 0, (size_t)ctx->n_phases * ctx->n_cu * 8 * sizeof(unsigned long long)) != hipSuccess)
      return HEISD_EHIP;
  }
  ctx->trace_on = enable != 0;
  if (out) {
    const long long all = (long long)ctx->n_phases * ctx->n_cu * 8;
    const int n = all < max_entries ? (int)all : max_entries;
    if (hipDeviceSynchronize() != hipSuccess ||
        hipMemcpy(out, ctx->trace, (size_t)n * sizeof(unsigned long long), hipMemcpyDeviceToHost) != hipSuccess)
      return HEISD_EHIP;
    return n;
  }
  return HEISD_OK;
}

extern "C" int heisd_verify_check(heisd_verify_ctx *ctx) {
  if (!ctx) return HEISD_EINVAL;
  unsigned w = 0;
  if (hipDeviceSynchronize() != hipSuccess ||
      hipMemcpy(&w, ctx->dev_err, sizeof(w), hipMemcpyDeviceToHost) != hipSuccess)
    return fail(ctx, HEISD_EHIP, "check: device error");
  if (w != 0) {
    (void)hipMemset(ctx->dev_err, 0, sizeof(w));
    if (w & kErrBarrier)
      return fail(ctx, HEISD_EHIP, "check: a bounded wait inside a launch gave up (a grid barrier of the persistent kernel, or a row scale "
                  "of the path for more than 8 rows)");
    return fail(ctx, HEISD_EINVAL, "check: an episode's new rows did not fit its cache (prefix_len + rows > kv_capacity, or "
                "a negative prefix_len): it was left unverified, its cache untouched, its accepted_len / next_bin -1");
  }
  return HEISD_OK;
}

// Test aid: the bounds of the waits inside the kernels, so that their give-up paths can be exercised with every
// kernel still running to its end.  grid_polls: polls of a grid barrier of the persistent kernel (<= 0: the
// default); scale_polls: polls for a row's 1/rms word (<= 0: the default); skip_scales != 0: the launches of the
// path for more than 8 rows do not produce those words, so every epilogue gives up after scale_polls polls.
extern "C" int heisd_debug_set_wait_limits(heisd_verify_ctx *ctx, int grid_polls, int scale_polls, int skip_scales) {
  if (!ctx) return HEISD_EINVAL;
  ctx->wait_limit = grid_polls > 0 ? grid_polls : kSpinLimit;
  ctx->scale_spin = scale_polls > 0 ? scale_polls : kScaleSpin;
  ctx->skip_scales = skip_scales != 0;
  return HEISD_OK;
}

extern "C" int heisd_verify_profile_enable(heisd_verify_ctx *ctx, int enable) {
  if (!ctx) return HEISD_EINVAL;
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  ctx->ev.clear();
  ctx->ev_class.clear();
  ctx->ev_used = 0;
  ctx->prof_steps = 0;
  ctx->prof_on = false;
  if (enable) {
    const size_t per_step = (size_t)ctx->d.n_layers * 5 * 8 + 17;   // launches of one step, row blocks included
    ctx->ev.resize(per_step * 2 * HEISD_PROFILE_MAX_STEPS);
    for (size_t i = 0; i < ctx->ev.size(); ++i)
      if (hipEventCreate(&ctx->ev[i]) != hipSuccess) {
        for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(ctx->ev[j]);
        ctx->ev.clear();
        return fail(ctx, HEISD_EHIP, "profile: hipEventCreate failed");
      }
    ctx->ev_class.reserve(ctx->ev.size() / 2);
    ctx->prof_on = true;
  }
  return HEISD_OK;
}

extern "C" int heisd_verify_profile_read(heisd_verify_ctx *ctx, double *ms, int64_t *launches) {
  if (!ctx || !ms || !launches) return HEISD_EINVAL;
  for (int i = 0; i < HEISD_N_KERNEL_CLASSES; ++i) { ms[i] = 0.0; launches[i] = 0; }
  const size_t pairs = ctx->ev_used / 2;
  if (pairs) {
    if (hipEventSynchronize(ctx->ev[ctx->ev_used - 1]) != hipSuccess)
      return fail(ctx, HEISD_EHIP, "profile: hipEventSynchronize failed");
    for (size_t p = 0; p < pairs; ++p) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, ctx->ev[2 * p], ctx->ev[2 * p + 1]) != hipSuccess)
        return fail(ctx, HEISD_EHIP, "profile: hipEventElapsedTime failed");
      ms[ctx->ev_class[p]] += t;
      launches[ctx->ev_class[p]] += 1;
    }
  }
  ctx->ev_used = 0;
  ctx->ev_class.clear();
  ctx->prof_steps = 0;
  return HEISD_OK;
}

extern "C" void heisd_free(heisd_verify_ctx *ctx) {
  if (!ctx) return;
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  if (ctx->sflags) {
    (void)hipDeviceSynchronize();      // the slot goes to another context only when nothing of this one runs any more
    flag_slot_release(ctx->sflag_dev, ctx->sflag_slot);
  }
  delete ctx;
}

extern "C" const char *heisd_last_error(const heisd_verify_ctx *ctx) { return ctx ? ctx->err : g_init_err; }

// The decoder forward for any M, one launch per phase (LDS-staged activations, 64-row blocks).
// ---- batched path (any M; the automatic choice for M > 8 rows) -------------------------------

template <int MC>
static hipError_t bat_prepare_mc() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&bat_gemm<MC, 3>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)bat_lds_bytes<MC>());
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void *>(&bat_gemm<MC, 2>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)bat_lds_bytes<MC>());
}

template <int MC>
static void bat_wide_variants(std::vector<const void *> &v) {
  v.push_back(reinterpret_cast<const void *>(&bat_gemm_wide<4, false, 2, MC>));
  v.push_back(reinterpret_cast<const void *>(&bat_gemm_wide<4, true, 2, MC>));
  v.push_back(reinterpret_cast<const void *>(&bat_gemm_wide<2, false, 2, MC>));
  v.push_back(reinterpret_cast<const void *>(&bat_gemm_wide<2, true, 2, MC>));
  v.push_back(reinterpret_cast<const void *>(&bat_gemm_wide<4, false, 1, MC>));
  v.push_back(reinterpret_cast<const void *>(&bat_gemm_wide<4, true, 1, MC>));
  v.push_back(reinterpret_cast<const void *>(&bat_gemm_wide<2, false, 1, MC>));
  v.push_back(reinterpret_cast<const void *>(&bat_gemm_wide<2, true, 1, MC>));
}

static hipError_t bat_prepare() {
  hipError_t e;
  if ((e = bat_prepare_mc<2>()) != hipSuccess) return e;
  if ((e = bat_prepare_mc<3>()) != hipSuccess) return e;
  if ((e = bat_prepare_mc<4>()) != hipSuccess) return e;
  if ((e = bat_prepare_mc<5>()) != hipSuccess) return e;
  if ((e = bat_prepare_mc<6>()) != hipSuccess) return e;
  if ((e = bat_prepare_mc<7>()) != hipSuccess) return e;
  if ((e = bat_prepare_mc<8>()) != hipSuccess) return e;
  std::vector<const void *> wide;
  bat_wide_variants<5>(wide);
  bat_wide_variants<6>(wide);
  bat_wide_variants<7>(wide);
  bat_wide_variants<8>(wide);
  for (const void *f : wide)
    if ((e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBatWideLds)) != hipSuccess) return e;
  return bat_ns_prepare();
}

template <int MC>
static void bat_launch_mc(const BatGemm &g, int grid, hipStream_t st) {
  if (g.epi == FEPI_SWIGLU)
    bat_gemm<MC, 2><<<dim3(grid), dim3(kBatThreads), bat_lds_bytes<MC>(), st>>>(g);
  else
    bat_gemm<MC, 3><<<dim3(grid), dim3(kBatThreads), bat_lds_bytes<MC>(), st>>>(g);
}

template <int MC, int NT, int KW>
static hipError_t bat_ns_prepare_one() {
  return hipFuncSetAttribute(reinterpret_cast<const void *>(&bat_gemm_ns<MC, NT, KW>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)bat_ns_lds_bytes<MC>());
}
static hipError_t bat_ns_prepare() {
  hipError_t e;
  if ((e = bat_ns_prepare_one<4, 2, 1>()) != hipSuccess) return e;
  if ((e = bat_ns_prepare_one<4, 2, 2>()) != hipSuccess) return e;
  if ((e = bat_ns_prepare_one<6, 2, 1>()) != hipSuccess) return e;
  if ((e = bat_ns_prepare_one<6, 2, 2>()) != hipSuccess) return e;
  if ((e = bat_ns_prepare_one<8, 2, 1>()) != hipSuccess) return e;
  return bat_ns_prepare_one<8, 2, 2>();
}

// Up to 64 rows, gate/up + SwiGLU: six waves split the (gate, up) pairs - 6 pairs, or 3 pairs x 2
// shares of the reduction - and share the activation fragments through LDS.  Fewer workgroups mean
// less record traffic but fewer compute units pulling weights: 6 pairs per workgroup only if that
// still gives three quarters of the compute units a workgroup.  (Tried for the plain projections
// too: with one tile per wave the LDS reads bound it, with two tiles per wave QKV gets only 128
// workgroups - 42 against 37 us at M = 56 - and O-proj and down have fewer tiles still.)
template <int MC>
static void bat_ns_launch_mc(BatGemm g, int n_cu, hipStream_t st) {
  const int wunits = g.n_units;
  const int kw = (wunits + kNsCompute - 1) / kNsCompute >= (3 * n_cu) / 4 ? 1 : 2;
  const int nw = kNsCompute / kw;
  g.NW = nw;
  const int groups = (wunits + nw - 1) / nw;
  const dim3 grid(groups < n_cu ? groups : n_cu), block(kBatThreads);
  if (kw == 1) bat_gemm_ns<MC, 2, 1><<<grid, block, bat_ns_lds_bytes<MC>(), st>>>(g);
  else bat_gemm_ns<MC, 2, 2><<<grid, block, bat_ns_lds_bytes<MC>(), st>>>(g);
}

// Column tiles (8 rows each) from which bat_gemm_wide takes over.  3 x 2 arrangement: from 65 rows for gate/up
// (the rows no longer fit bat_gemm_ns) and for every projection whose reduction may be split; without room
// for a split from 185 rows (measured at 76, 115, 162, 176, 224, 256, 360 and 448 rows).  6 x 1 arrangement
// with split reductions, up to 64 rows: from 33 rows, and from 17 rows for projections with no more weight
// tiles than compute units (measured at 22, 45 and 56 rows: QKV at 22 rows is the one case bat_gemm wins).
constexpr int kWideMinCT = 24, kWideMinCTGateUp = 9, kWideMinCTSplit = 9;
constexpr int kWide1MinCT = 5, kWide1MinCTFew = 3;

// Room for the sums of split reductions: part holds up to `units` units x `tiles` column tiles (runs x tiles in use).
constexpr int kActBf16MinRows = 33;

struct SplitRoom {
  float2 *part = nullptr;
  int units = 0, tiles = 0;
};

// bat_gemm_wide in the arrangement MW (2: blocks of 16 column tiles, 1: blocks of 8), nt weight tiles per
// wave and the reduction in ks runs.
template <int MW, int MC>
static void bat_wide_launch_t(const BatGemm &g, int nt, int ks, bool whole, int grid, int n_blk, float2 *part, hipStream_t st) {
  const dim3 gr(grid), bl(kBatThreads);
  if (nt == 4) {
    if (whole) bat_gemm_wide<4, true, MW, MC><<<gr, bl, kBatWideLds, st>>>(g, n_blk, ks, part);
    else bat_gemm_wide<4, false, MW, MC><<<gr, bl, kBatWideLds, st>>>(g, n_blk, ks, part);
  } else {
    if (whole) bat_gemm_wide<2, true, MW, MC><<<gr, bl, kBatWideLds, st>>>(g, n_blk, ks, part);
    else bat_gemm_wide<2, false, MW, MC><<<gr, bl, kBatWideLds, st>>>(g, n_blk, ks, part);
  }
}
template <int MW>
static void bat_wide_launch_mc(int mc, const BatGemm &g, int nt, int ks, bool whole, int grid, int n_blk, float2 *part, hipStream_t st) {
  switch (mc) {
    case 5: bat_wide_launch_t<MW, 5>(g, nt, ks, whole, grid, n_blk, part, st); break;
    case 6: bat_wide_launch_t<MW, 6>(g, nt, ks, whole, grid, n_blk, part, st); break;
    case 7: bat_wide_launch_t<MW, 7>(g, nt, ks, whole, grid, n_blk, part, st); break;
    default: bat_wide_launch_t<MW, 8>(g, nt, ks, whole, grid, n_blk, part, st); break;
  }
}

static void bat_wide_launch(const BatGemm &g, int mw, int n_cu, hipStream_t st, const SplitRoom &room) {
  const int CT = g.CT, nwv = kWdCompute / mw;
  // column tiles per wave: 8, or fewer (down to 5) if the blocks then hold fewer padding tiles and no more
  // tiles in all than blocks of 8 per wave would (the records are allocated for those)
  int mc = kWdMC;
  {
    const int pad8 = (CT + mw * kWdMC - 1) / (mw * kWdMC) * (mw * kWdMC);
    int best = pad8;
    for (int m = kWdMC - 1; m >= 5; --m) {
      const int padded = (CT + mw * m - 1) / (mw * m) * (mw * m);
      if (padded < best) { best = padded; mc = m; }
    }
  }
  const int cols = mw * mc;
  const int n_blk = (CT + cols - 1) / cols;
  const int per_unit = g.epi == FEPI_SWIGLU ? 2 : 1;        // weight tiles per unit
  const int total = (g.Kd + 31) / 32, n_chunks = (total + kWdS - 1) / kWdS;
  constexpr int CPR = kWdRA / kWdS;
  auto groups = [&](int nt) { const int upg = nwv * nt / per_unit; return (g.n_units + upg - 1) / upg; };
  // Estimated time in us of (nt weight tiles per wave, reduction in ks runs): whole rounds of workgroups
  // over the compute units (one workgroup fills a unit's LDS); per k-step 0.42 us with 2 tiles per wave
  // and 0.65 us with 4 in the 3 x 2 arrangement (measured on the 7B shapes at 224 and 448 rows), 0.27 and
  // 0.445 us in the 6 x 1 arrangement (fitted to 2..16 runs at 56 rows); a few us to start and end a
  // workgroup; a split reduction adds the launch that sums the runs and what it moves (at 2 TB/s).
  auto estimate = [&](int nt, int ks) {
    const long wgs = (long)((groups(nt) + 7) / 8 * 8) * n_blk * ks;     // as launched: the surplus ones come last
    const double rounds = (double)((wgs + n_cu - 1) / n_cu);
    const int per = (n_chunks + ks - 1) / ks;
    const double finish = ks > 1 ? 8.0 + 2.0 * ks * g.n_units * CT * 512.0 / 2.0e6 : 0.0;
    const double per_step = mw == 2 ? (nt == 4 ? 0.65 : 0.42) : (nt == 4 ? 0.445 : 0.27);
    return rounds * ((double)per * kWdS * per_step + (mw == 2 ? 4.0 : 8.0)) + finish;
  };
  const bool may_split = room.part && g.epi != FEPI_SWIGLU && g.n_units <= room.units;
  int nt = 4, ks = 1;
  double best = estimate(4, 1);
  for (int n : {4, 2})
    for (int k = 1; k <= kSplitMax; ++k) {
      if (k > 1 && (!may_split || k * CT * (g.single ? 2 : 1) > room.tiles)) break;
      if ((k - 1) * ((n_chunks + k - 1) / k) >= n_chunks) continue;      // the last run would be empty
      const double e = estimate(n, k);
      if (e < best) { best = e; nt = n; ks = k; }
    }
  const int per = (n_chunks + ks - 1) / ks;
  const bool whole = per % CPR == 0 && n_chunks % per == 0;   // every run a whole number of ring revolutions (see the kernel)
  const int grid = (groups(nt) + 7) / 8 * 8 * n_blk * ks;
  if (mw == 2) bat_wide_launch_mc<2>(mc, g, nt, ks, whole, grid, n_blk, room.part, st);
  else bat_wide_launch_mc<1>(mc, g, nt, ks, whole, grid, n_blk, room.part, st);
  if (ks > 1) bat_split_finish<<<dim3((g.n_units * CT + 3) / 4), dim3(256), 0, st>>>(g, ks, room.part);
}

// Wave arrangement for CT column tiles: MW groups of MC tiles (MC from the compiled set).
// (Gate/up at up to 64 rows stays on bat_gemm_ns: on the 6 x 1 wide kernel, which cannot split it,
// it measured 60 against 49 us at 56 rows.)
static void bat_launch(BatGemm g, int n_cu, hipStream_t st, const SplitRoom &room = SplitRoom()) {
  const int CT = g.CT;
  if (g.single) {                      // single-bf16 records: the wide kernels, and bat_gemm_ns for gate/up on few rows
    if (CT <= 4 && g.epi == FEPI_SWIGLU) bat_ns_launch_mc<4>(g, n_cu, st);
    else bat_wide_launch(g, CT <= 8 ? 1 : 2, n_cu, st, g.epi == FEPI_SWIGLU ? SplitRoom() : room);
    return;
  }
  if (CT <= 8 && g.epi == FEPI_SWIGLU) {
    // column tiles per wave: 4, 6 or 8 (45 rows: 42.7 us with 6 against 46.7 us with 8; 7 tiles per wave
    // measured slower than 8 at 56 rows, 48.2 against 47.1 us)
    if (CT <= 4) bat_ns_launch_mc<4>(g, n_cu, st);
    else if (CT <= 6) bat_ns_launch_mc<6>(g, n_cu, st);
    else bat_ns_launch_mc<8>(g, n_cu, st);
    return;
  }
  if (CT <= 8 && room.part && (CT >= kWide1MinCT || (CT >= kWide1MinCTFew && g.n_units <= n_cu))) {
    bat_wide_launch(g, 1, n_cu, st, room);                    // six waves across the weight tiles, 8 column tiles
    return;
  }
  if (CT >= (g.epi == FEPI_SWIGLU ? kWideMinCTGateUp : (room.part ? kWideMinCTSplit : kWideMinCT))) {
    bat_wide_launch(g, 2, n_cu, st, room);                    // 3 x 2 waves, 16 column tiles
    return;
  }
  const int MW = CT <= 8 ? 1 : (CT <= 16 ? 2 : (CT <= 32 ? 4 : 8));
  const int need = (CT + MW - 1) / MW < 8 ? (CT + MW - 1) / MW : 8;
  g.MW = MW;
  const int grid = g.n_units < n_cu ? g.n_units : n_cu;
  switch (need) {                      // a wave group holds exactly the column tiles it needs
    case 1: case 2: bat_launch_mc<2>(g, grid, st); break;
    case 3: bat_launch_mc<3>(g, grid, st); break;
    case 4: bat_launch_mc<4>(g, grid, st); break;
    case 5: bat_launch_mc<5>(g, grid, st); break;
    case 6: bat_launch_mc<6>(g, grid, st); break;
    case 7: bat_launch_mc<7>(g, grid, st); break;
    default: bat_launch_mc<8>(g, grid, st); break;
  }
}

static void batch_forward(heisd_verify_ctx *ctx, const heisd_kv_desc *kv, const int32_t *draft_tokens, int K,
                          int batch, const uint8_t *skip_mask, float *logits, hipStream_t st, bool prof,
                          const int32_t *depth = nullptr, const unsigned long long *anc = nullptr,
                          const float *x_rows = nullptr) {
  const heisd_model_desc &d = ctx->d;
  const int M = batch * K, dm = d.d_model, F = d.d_ffn, H = d.n_heads, HD = d.head_dim, cap = d.kv_capacity;
  const BatScratch bs(&d);
  const int CTS = bs.CTS;
  // One bf16 per activation (opt-in, heisd_verify_set_activations): from 33 rows, where every projection runs on
  // bat_gemm_wide or bat_gemm_ns, and only if the 16-row column tiles stay inside the buffers laid out for 8-row ones.
  const int single = ctx->act_bf16 && M >= kActBf16MinRows && (M + 15) / 16 * 16 <= CTS * 8 ? 1 : 0;
  const int RPT = single ? 16 : 8;                       // activation rows per column tile
  const int CT = (M + RPT - 1) / RPT;
  uint16_t *rec_x = reinterpret_cast<uint16_t *>(ctx->bscr + bs.rec_x);
  uint16_t *rec_o = reinterpret_cast<uint16_t *>(ctx->bscr + bs.rec_o);
  uint16_t *rec_act = reinterpret_cast<uint16_t *>(ctx->bscr + bs.rec_act);
  float *ssq = reinterpret_cast<float *>(ctx->bscr + bs.ssq);
  SplitRoom part;
  part.part = reinterpret_cast<float2 *>(ctx->bscr + bs.part);
  part.units = 3 * dm / 16;
  part.tiles = bs.part_tiles();
  // The projections of a normalised input take the rows' 1/rms from words their own launch computes (bat_scales_produce):
  // one epoch per such projection.
  auto normalised = [&](BatGemm &g) {
    g.ssq_in = ssq; g.ssq_tiles = dm / 16; g.eps = d.rms_eps;
    g.scale_tag = reinterpret_cast<unsigned long long *>(ctx->bscr + bs.inv_rms);
    if (++ctx->scale_epoch == 0u) ctx->scale_epoch = 1u;
    g.scale_epoch = ctx->scale_epoch; g.err = ctx->dev_err;
    g.scale_spin = ctx->scale_spin; g.scale_skip = ctx->skip_scales ? 1 : 0;
  };
  {
    ProfScope ps(ctx, HEISD_KC_EMBED, st, prof);
    bat_embed<<<dim3(dm / 16, (CT * (single ? 2 : 1) + 7) / 8), dim3(64), 0, st>>>(
        draft_tokens, x_rows, static_cast<const uint16_t *>(d.tok_emb), d.vocab, dm, M, CT, CTS, ctx->attn_norm[0], ctx->x, rec_x,
        ssq, single, reinterpret_cast<unsigned long long *>(ctx->bscr + bs.inv_rms));
  }
  const size_t layer_stride = (size_t)batch * H * cap * HD;
  BatGemm base{};
  base.CT = CT; base.CTS = CTS; base.M = M; base.single = single;
  for (int l = 0; l < d.n_layers; ++l) {
    // q, k, v = RMSNorm(x) . {Wq, Wk, Wv}^T  (fp32 rows for the attention kernel)
    BatGemm g = base;
    g.epi = FEPI_STORE_ROWS;
    g.w[0] = ctx->pq[l];
    g.w[1] = ctx->pk[l];
    g.w[2] = ctx->pv[l];
    g.seg_tiles = dm / 16; g.n_units = 3 * dm / 16; g.Kd = dm;
    g.b = rec_x; normalised(g); g.out = ctx->qkv; g.ldo = 3 * dm;
    { ProfScope ps(ctx, HEISD_KC_QKV, st, prof); bat_launch(g, ctx->n_cu, st, part); }
    // RoPE + KV-append + attention; the output goes straight into records
    AttnArgs a{};
    a.qkv = ctx->qkv;
    a.k_cache = static_cast<uint16_t *>(kv->k_cache) + (size_t)l * layer_stride;
    a.v_cache = static_cast<uint16_t *>(kv->v_cache) + (size_t)l * layer_stride;
    a.prefix_len = kv->prefix_len; a.skip = skip_mask; a.rope = ctx->rope; a.out = nullptr;
    a.o_planes = rec_o; a.CTS = CTS; a.single = single;
    a.K = K; a.H = H; a.cap = cap; a.d = dm; a.scale = 1.0f / std::sqrt((float)HD);
    a.depth = depth; a.anc = anc;
    {
      ProfScope ps(ctx, HEISD_KC_ATTN, st, prof);
      attn_launch(a, HD, H, batch, cap, ctx->n_cu, st);
    }
    // x += o . Wo^T; records of x * ffn gain, partial sums of squares
    g = base;
    g.epi = FEPI_RESID_NORM;
    g.w[0] = ctx->po[l];
    g.seg_tiles = dm / 16; g.n_units = dm / 16; g.Kd = dm;
    g.b = rec_o; g.out = ctx->x; g.ldo = dm;
    g.next_gain = ctx->ffn_norm[l]; g.o_planes = rec_x; g.ssq_out = ssq;
    {
      ProfScope ps(ctx, HEISD_KC_OPROJ, st, prof);
      bat_launch(g, ctx->n_cu, st, part);
    }
    // a = silu(RMSNorm(x) . Wg^T) * (RMSNorm(x) . Wu^T), as records
    g = base;
    g.epi = FEPI_SWIGLU;
    g.w[0] = ctx->pg[l];
    g.w[1] = ctx->pu[l];
    g.seg_tiles = F / 16; g.n_units = F / 16; g.Kd = dm;
    g.b = rec_x; normalised(g); g.o_planes = rec_act;
    { ProfScope ps(ctx, HEISD_KC_GATEUP, st, prof); bat_launch(g, ctx->n_cu, st); }
    // x += a . Wd^T; records of x * (next norm's gain), partial sums of squares
    g = base;
    g.epi = FEPI_RESID_NORM;
    g.w[0] = ctx->pd[l];
    g.seg_tiles = dm / 16; g.n_units = dm / 16; g.Kd = F;
    g.b = rec_act; g.out = ctx->x; g.ldo = dm;
    g.next_gain = (l + 1 < d.n_layers) ? ctx->attn_norm[l + 1] : d.final_norm;
    g.o_planes = rec_x; g.ssq_out = ssq;
    {
      ProfScope ps(ctx, HEISD_KC_DOWN, st, prof);
      bat_launch(g, ctx->n_cu, st, part);
    }
  }
  // logits over the action bins = RMSNorm(x; final) . W_lm[bin rows]^T
  BatGemm g = base;
  g.epi = FEPI_STORE_ROWS;
  g.w[0] = ctx->plm;
  g.seg_tiles = d.n_bins / 16; g.n_units = d.n_bins / 16; g.Kd = dm;
  g.b = rec_x; normalised(g); g.out = logits; g.ldo = d.n_bins;
  ProfScope ps(ctx, HEISD_KC_LMHEAD, st, prof);
  bat_launch(g, ctx->n_cu, st, part);
}

static void generic_forward(heisd_verify_ctx *ctx, const heisd_kv_desc *kv, const int32_t *draft_tokens, int K,
                            int batch, const uint8_t *skip_mask, float *logits, hipStream_t st, bool prof,
                            const int32_t *depth = nullptr, const unsigned long long *anc = nullptr,
                            const float *x_rows = nullptr) {
  const heisd_model_desc &d = ctx->d;
  const int M = batch * K, dm = d.d_model, F = d.d_ffn, H = d.n_heads, HD = d.head_dim, cap = d.kv_capacity;
  {
    ProfScope ps(ctx, HEISD_KC_EMBED, st, prof);
    if (x_rows && !draft_tokens)
      (void)hipMemcpyAsync(ctx->x, x_rows, (size_t)M * dm * sizeof(float), hipMemcpyDeviceToDevice, st);
    else
      embed_rows<<<dim3(M), dim3(256), 0, st>>>(draft_tokens, static_cast<const uint16_t *>(d.tok_emb), d.vocab, dm,
                                                ctx->x, x_rows);
  }
  const size_t layer_stride = (size_t)batch * H * cap * HD;
  for (int l = 0; l < d.n_layers; ++l) {
    GemmArgs g{};
    // q, k, v = RMSNorm(x) . {Wq, Wk, Wv}^T
    g.act = ctx->x; g.gain = ctx->attn_norm[l];
    g.w[0] = static_cast<const uint16_t *>(ctx->wq[l]);
    g.w[1] = static_cast<const uint16_t *>(ctx->wk[l]);
    g.w[2] = static_cast<const uint16_t *>(ctx->wv[l]);
    g.seg_tiles = dm / 16; g.n_units = 3 * dm / 16; g.Kd = dm; g.eps = d.rms_eps;
    g.out = ctx->qkv; g.ldo = 3 * dm; g.resid = nullptr;
    { ProfScope ps(ctx, HEISD_KC_QKV, st, prof); gemm_launch(g, M, EPI_STORE, st); }
    // RoPE + KV-append + attention
    AttnArgs a{};
    a.qkv = ctx->qkv;
    a.k_cache = static_cast<uint16_t *>(kv->k_cache) + (size_t)l * layer_stride;
    a.v_cache = static_cast<uint16_t *>(kv->v_cache) + (size_t)l * layer_stride;
    a.prefix_len = kv->prefix_len; a.skip = skip_mask; a.rope = ctx->rope; a.out = ctx->attn_o;
    a.K = K; a.H = H; a.cap = cap; a.d = dm; a.scale = 1.0f / std::sqrt((float)HD);
    a.depth = depth; a.anc = anc;
    {
      ProfScope ps(ctx, HEISD_KC_ATTN, st, prof);
      attn_launch(a, HD, H, batch, cap, ctx->n_cu, st);
    }
    // x += o . Wo^T
    g = GemmArgs{};
    g.act = ctx->attn_o; g.gain = nullptr; g.w[0] = static_cast<const uint16_t *>(ctx->wo[l]);
    g.seg_tiles = dm / 16; g.n_units = dm / 16; g.Kd = dm; g.eps = 0.f;
    g.out = ctx->x; g.ldo = dm; g.resid = ctx->x;
    { ProfScope ps(ctx, HEISD_KC_OPROJ, st, prof); gemm_launch(g, M, EPI_STORE, st); }
    // a = silu(RMSNorm(x) . Wg^T) * (RMSNorm(x) . Wu^T)
    g = GemmArgs{};
    g.act = ctx->x; g.gain = ctx->ffn_norm[l];
    g.w[0] = static_cast<const uint16_t *>(ctx->w_gate[l]);
    g.w[1] = static_cast<const uint16_t *>(ctx->w_up[l]);
    g.seg_tiles = F / 16; g.n_units = F / 16; g.Kd = dm; g.eps = d.rms_eps;
    g.out = ctx->act; g.ldo = F; g.resid = nullptr;
    { ProfScope ps(ctx, HEISD_KC_GATEUP, st, prof); gemm_launch(g, M, EPI_SWIGLU, st); }
    // x += a . Wd^T
    g = GemmArgs{};
    g.act = ctx->act; g.gain = nullptr; g.w[0] = static_cast<const uint16_t *>(ctx->w_down[l]);
    g.seg_tiles = dm / 16; g.n_units = dm / 16; g.Kd = F; g.eps = 0.f;
    g.out = ctx->x; g.ldo = dm; g.resid = ctx->x;
    { ProfScope ps(ctx, HEISD_KC_DOWN, st, prof); gemm_launch(g, M, EPI_STORE, st); }
  }
  // logits over the action bins = RMSNorm(x; final) . W_lm[bin rows]^T
  {
    GemmArgs g{};
    g.act = ctx->x; g.gain = d.final_norm;
    g.w[0] = static_cast<const uint16_t *>(d.lm_head) + (size_t)d.bin_token_base * dm;
    g.seg_tiles = d.n_bins / 16; g.n_units = d.n_bins / 16; g.Kd = dm; g.eps = d.rms_eps;
    g.out = logits; g.ldo = d.n_bins; g.resid = nullptr;
    ProfScope ps(ctx, HEISD_KC_LMHEAD, st, prof);
    gemm_launch(g, M, EPI_STORE, st);
  }
}

// ---- one verify step ----------------------------------------------------------------------

// The persistent kernel needs every compute unit of the device: two of them started at the same time from
// two streams could each hold half of the chip and wait for the other half (until their bounded spins give
// up).  The automatic path choice therefore takes the persistent kernel only when the last one launched
// through this library on the device went to the same stream or has finished, and never on a stream that is
// being captured (an event query is not allowed there); otherwise the step runs one launch per phase.
// A context switched to HEISD_PATH_PERSIST by its caller skips the test: the caller then owns the device.
constexpr int kMaxDevices = 64;
struct PersistGuard {
  std::mutex m;
  hipEvent_t done = nullptr;      // recorded behind the last persistent launch
  hipStream_t stream = nullptr;
  bool valid = false;
};
static PersistGuard g_persist_guard[kMaxDevices];

// Does the context's path selection ask for the persistent kernel (for a call of at most 8 rows)?  AUTO asks for
// it where it pays: measured at batch 1, K = 7 over model widths 512 .. 4096 (8 layers each), with its barrier flags
// in uncached memory it is 9 % faster than one launch per phase at 405 MB of projection weights per layer, 11 % at
// 227 MB, 6 % at 101 MB, 2 % at 57 MB, and 11 % slower at 26 MB (five barriers per layer cost about what five kernel
// boundaries cost; what is handed over across them has to pay); with the flags in the workspace (no slot of
// uncached memory) it wins only from about 320 MB.
static bool persist_wanted(const heisd_verify_ctx *ctx) {
  if (!ctx->persist_ok) return false;
  if (ctx->path == HEISD_PATH_PERSIST) return true;
  const double dm = ctx->d.d_model, F = ctx->d.d_ffn;
  return ctx->path == HEISD_PATH_AUTO && (4.0 * dm * dm + 3.0 * dm * F) * 2.0 >= (ctx->sflags ? 80e6 : 320e6);
}

// Launch the persistent kernel if it may run now (or unconditionally with force); returns whether it was launched.
static bool persist_try_launch(heisd_verify_ctx *ctx, bool force, const heisd_kv_desc *kv, const int32_t *draft_tokens,
                               int K, int batch, const uint8_t *skip_mask, float *logits, const AcceptArgs &aa,
                               hipStream_t st, bool prof) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    if (!force) return false;
    ProfScope ps(ctx, HEISD_KC_PERSIST, st, prof);
    persist_launch(ctx, kv, draft_tokens, K, batch, skip_mask, logits, aa, st);
    return true;
  }
  PersistGuard &g = g_persist_guard[dev];
  std::lock_guard<std::mutex> lock(g.m);
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  const bool capturing = hipStreamIsCapturing(st, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone;
  if (!force) {
    if (capturing) { (void)hipGetLastError(); return false; }
    if (g.valid && g.stream != st && hipEventQuery(g.done) != hipSuccess) { (void)hipGetLastError(); return false; }
    if (!g.done && hipEventCreateWithFlags(&g.done, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      g.done = nullptr;
      return false;
    }
  }
  {
    ProfScope ps(ctx, HEISD_KC_PERSIST, st, prof);
    persist_launch(ctx, kv, draft_tokens, K, batch, skip_mask, logits, aa, st);
  }
  if (!capturing && g.done && hipEventRecord(g.done, st) == hipSuccess) {
    g.stream = st;
    g.valid = true;
  }
  return true;
}

extern "C" int heisd_verify_step(heisd_verify_ctx *ctx, const heisd_kv_desc *kv, const int32_t *draft_tokens,
                                 int32_t K, int32_t batch, const heisd_accept_desc *accept,
                                 const uint8_t *skip_mask, int32_t *accepted_len, int32_t *next_token,
                                 int32_t *target_bins, float *bin_logits, void *stream) {
  if (!ctx) return HEISD_EINVAL;
  if (!kv || !kv->k_cache || !kv->v_cache || !kv->prefix_len || !kv->first_pred || !draft_tokens || !accept ||
      !accepted_len || !next_token)
    return fail(ctx, HEISD_EINVAL, "step: NULL required pointer");
  const heisd_model_desc &d = ctx->d;
  if (K < 1 || batch < 1 || K > d.max_k || batch > d.max_batch || K > d.kv_capacity)
    return fail(ctx, HEISD_EINVAL, "step: K=%d batch=%d outside [1,%d] x [1,%d] (kv_capacity %d)", K, batch,
                d.max_k, d.max_batch, d.kv_capacity);
  if (accept->n_groups < 1 || accept->n_groups > HEISD_MAX_GROUPS)
    return fail(ctx, HEISD_EINVAL, "step: n_groups=%d outside [1,%d]", accept->n_groups, HEISD_MAX_GROUPS);
  for (int g = 0; g < accept->n_groups; ++g)
    if (accept->group_sizes[g] < 1) return fail(ctx, HEISD_EINVAL, "step: group_sizes[%d] < 1", g);
  if (accept->tok_threshold < 0 || accept->seq_budget < 0)
    return fail(ctx, HEISD_EINVAL, "step: negative acceptance threshold");
  if (accept->mode != 0 && accept->mode != 1) return fail(ctx, HEISD_EINVAL, "step: mode %d", accept->mode);

  hipStream_t st = static_cast<hipStream_t>(stream);
  const int M = batch * K, dm = d.d_model, F = d.d_ffn, H = d.n_heads, HD = d.head_dim, cap = d.kv_capacity;
  float *logits = bin_logits ? bin_logits : ctx->logits;
  int32_t *tbins = target_bins ? target_bins : ctx->tbins;
  (void)hipGetLastError();

  const bool use_fast = ctx->fast_ok && M <= 8 && ctx->path != HEISD_PATH_GENERIC;
  if ((ctx->path == HEISD_PATH_FAST || ctx->path == HEISD_PATH_PERSIST) && !use_fast)
    return fail(ctx, HEISD_EUNSUPPORTED, "step: this path needs batch*K <= 8 (got %d)", M);
  const bool prof = ctx->prof_on && ctx->prof_steps < HEISD_PROFILE_MAX_STEPS;
  if (prof) ctx->prof_steps++;
  // AUTO takes the persistent kernel when it may run (see PersistGuard), else one launch per phase
  const bool want_persist = use_fast && persist_wanted(ctx);
  AcceptArgs aa{};
  aa.logits = logits; aa.logits_rw = logits; aa.draft = draft_tokens; aa.first_pred = kv->first_pred;
  aa.skip = skip_mask; aa.accepted_len = accepted_len; aa.next_token = next_token; aa.target_bins = tbins;
  aa.K = K; aa.n_bins = d.n_bins; aa.bin_base = d.bin_token_base;
  aa.tok_threshold = accept->tok_threshold; aa.seq_budget = accept->seq_budget;
  aa.n_groups = accept->n_groups; aa.mode = accept->mode; aa.exact_mask = accept->exact_group_mask;
  for (int i = 0; i < 8; ++i) aa.group_sizes[i] = i < accept->n_groups ? accept->group_sizes[i] : 1;
  aa.prefix_len = kv->prefix_len; aa.cap = cap; aa.err = ctx->dev_err;
  bool accept_done = false, persisted = false;
  if (want_persist) {
    persisted = persist_try_launch(ctx, ctx->path == HEISD_PATH_PERSIST, kv, draft_tokens, K, batch, skip_mask, logits, aa,
                                   st, prof);
    accept_done = persisted;                             // acceptance at the end of the same launch
  }
  if (persisted) {
  } else if (use_fast) {
    fast_forward(ctx, kv, draft_tokens, K, batch, skip_mask, logits, st, prof, &aa);   // acceptance inside the LM-head launch
    accept_done = true;
  } else if (ctx->path != HEISD_PATH_GENERIC) {          // BATCH, or AUTO when the M <= 8 kernels do not apply
    batch_forward(ctx, kv, draft_tokens, K, batch, skip_mask, logits, st, prof);
  } else {
    generic_forward(ctx, kv, draft_tokens, K, batch, skip_mask, logits, st, prof);
  }
  if (!accept_done) {
    ProfScope ps(ctx, HEISD_KC_ACCEPT, st, prof);
    argmax_accept<<<dim3(batch), dim3(256), 0, st>>>(aa);
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(ctx, HEISD_EHIP, "step: %s", hipGetErrorString(e));
  ctx->err[0] = 0;
  return HEISD_OK;
}

// ---- one tree verify step -------------------------------------------------------------------

static int check_accept_desc(heisd_verify_ctx *ctx, const heisd_accept_desc *accept, const char *who) {
  if (accept->n_groups < 1 || accept->n_groups > HEISD_MAX_GROUPS)
    return fail(ctx, HEISD_EINVAL, "%s: n_groups=%d outside [1,%d]", who, accept->n_groups, HEISD_MAX_GROUPS);
  for (int g = 0; g < accept->n_groups; ++g)
    if (accept->group_sizes[g] < 1) return fail(ctx, HEISD_EINVAL, "%s: group_sizes[%d] < 1", who, g);
  if (accept->tok_threshold < 0 || accept->seq_budget < 0)
    return fail(ctx, HEISD_EINVAL, "%s: negative acceptance threshold", who);
  if (accept->mode != 0 && accept->mode != 1) return fail(ctx, HEISD_EINVAL, "%s: mode %d", who, accept->mode);
  return HEISD_OK;
}

extern "C" int heisd_verify_tree_step(heisd_verify_ctx *ctx, const heisd_kv_desc *kv, const int32_t *tree_tokens,
                                      const int32_t *parent, int32_t T, int32_t batch,
                                      const heisd_accept_desc *accept, const uint8_t *skip_mask,
                                      int32_t *accepted_len, int32_t *next_token, int32_t *accepted_path,
                                      int32_t *target_bins, float *bin_logits, void *stream) {
  if (!ctx) return HEISD_EINVAL;
  if (!kv || !kv->k_cache || !kv->v_cache || !kv->prefix_len || !kv->first_pred || !tree_tokens || !parent ||
      !accept || !accepted_len || !next_token)
    return fail(ctx, HEISD_EINVAL, "tree_step: NULL required pointer");
  const heisd_model_desc &d = ctx->d;
  if (T < 1 || batch < 1 || T > d.max_k || T > kTreeMax || batch > d.max_batch || T > d.kv_capacity)
    return fail(ctx, HEISD_EINVAL, "tree_step: T=%d batch=%d outside [1,%d] x [1,%d] (kv_capacity %d)", T, batch,
                d.max_k < kTreeMax ? d.max_k : kTreeMax, d.max_batch, d.kv_capacity);
  const int rc = check_accept_desc(ctx, accept, "tree_step");
  if (rc != HEISD_OK) return rc;
  if (ctx->path == HEISD_PATH_FAST || ctx->path == HEISD_PATH_PERSIST)
    return fail(ctx, HEISD_EUNSUPPORTED, "tree_step: the selected path serves linear steps of at most 8 rows only");

  hipStream_t st = static_cast<hipStream_t>(stream);
  float *logits = bin_logits ? bin_logits : ctx->logits;
  int32_t *tbins = target_bins ? target_bins : ctx->tbins;
  int32_t *path = accepted_path ? accepted_path : ctx->tree_path;
  (void)hipGetLastError();
  const bool prof = ctx->prof_on && ctx->prof_steps < HEISD_PROFILE_MAX_STEPS;
  if (prof) ctx->prof_steps++;
  {
    ProfScope ps(ctx, HEISD_KC_EMBED, st, prof);
    tree_setup<<<dim3(batch), dim3(kTreeMax), 0, st>>>(parent, T, ctx->tree_depth, ctx->tree_anc);
  }
  if (ctx->path == HEISD_PATH_GENERIC)
    generic_forward(ctx, kv, tree_tokens, T, batch, skip_mask, logits, st, prof, ctx->tree_depth, ctx->tree_anc);
  else
    batch_forward(ctx, kv, tree_tokens, T, batch, skip_mask, logits, st, prof, ctx->tree_depth, ctx->tree_anc);
  TreeAcceptArgs aa{};
  aa.logits = logits; aa.logits_rw = logits; aa.tokens = tree_tokens; aa.parent = parent;
  aa.first_pred = kv->first_pred; aa.skip = skip_mask; aa.accepted_len = accepted_len; aa.next_token = next_token;
  aa.path = path; aa.target_bins = tbins;
  aa.T = T; aa.n_bins = d.n_bins; aa.bin_base = d.bin_token_base;
  aa.tok_threshold = accept->tok_threshold; aa.seq_budget = accept->seq_budget;
  aa.n_groups = accept->n_groups; aa.mode = accept->mode; aa.exact_mask = accept->exact_group_mask;
  for (int i = 0; i < 8; ++i) aa.group_sizes[i] = i < accept->n_groups ? accept->group_sizes[i] : 1;
  aa.prefix_len = kv->prefix_len; aa.cap = d.kv_capacity; aa.err = ctx->dev_err;
  TreeCompactArgs ca{};
  ca.k_cache = static_cast<uint16_t *>(kv->k_cache); ca.v_cache = static_cast<uint16_t *>(kv->v_cache);
  ca.prefix_len = kv->prefix_len; ca.skip = skip_mask; ca.accepted_len = accepted_len; ca.path = path;
  ca.T = T; ca.H = d.n_heads; ca.cap = d.kv_capacity; ca.HD = d.head_dim; ca.batch = batch;
  {
    ProfScope ps(ctx, HEISD_KC_ACCEPT, st, prof);
    tree_accept<<<dim3(batch), dim3(256), 0, st>>>(aa);
    tree_compact<<<dim3(d.n_heads, batch, d.n_layers), dim3(256), 0, st>>>(ca);
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(ctx, HEISD_EHIP, "tree_step: %s", hipGetErrorString(e));
  ctx->err[0] = 0;
  return HEISD_OK;
}

// ---- the draft tree from retrieved candidates (host code) -------------------------------------

namespace {
struct TreeBuilder {
  const int32_t *cand;
  int R, K, max_tokens;
  std::vector<int> lv_start, lv_end, lv_group;
  unsigned exact_mask;
  int32_t *tokens, *parent;
  int n = 0;

  bool same_seq(int a, int b, int s, int e) const {
    for (int j = s; j < e; ++j)
      if (cand[(size_t)a * K + j] != cand[(size_t)b * K + j]) return false;
    return true;
  }
  // Children of the node that ends at token `last` (-1: the prefix) and stands for candidates `carried`.
  void grow(int level, int last, uint64_t carried) {
    if (level == (int)lv_start.size()) return;
    const int s = lv_start[level], e = lv_end[level];
    const bool exact = (exact_mask >> lv_group[level]) & 1u;
    const uint64_t eligible = exact ? carried : (R == 64 ? ~0ull : ((1ull << R) - 1));
    uint64_t done = 0;
    for (int c = 0; c < R; ++c) {
      if (!((eligible >> c) & 1) || ((done >> c) & 1)) continue;
      uint64_t owners = 0;
      for (int o = c; o < R; ++o)
        if (((eligible >> o) & 1) && same_seq(c, o, s, e)) owners |= 1ull << o;
      done |= owners;
      if (n + (e - s) > max_tokens) continue;
      int prev = last;
      for (int j = s; j < e; ++j) {
        tokens[n] = cand[(size_t)c * K + j];
        parent[n] = prev;
        prev = n++;
      }
      grow(level + 1, prev, owners);
    }
  }
};
}  // namespace

extern "C" int heisd_build_sequence_tree(const int32_t *candidates, int32_t R, int32_t K,
                                         const heisd_accept_desc *accept, int32_t max_tokens, int32_t *tokens,
                                         int32_t *parent, int32_t *n_tokens) {
  if (!candidates || !accept || !tokens || !parent || !n_tokens)
    return fail(nullptr, HEISD_EINVAL, "build_tree: NULL pointer");
  if (R < 1 || R > 64 || K < 1 || max_tokens < 1)
    return fail(nullptr, HEISD_EINVAL, "build_tree: R=%d K=%d max_tokens=%d", R, K, max_tokens);
  if (accept->n_groups < 1 || accept->n_groups > HEISD_MAX_GROUPS)
    return fail(nullptr, HEISD_EINVAL, "build_tree: n_groups=%d", accept->n_groups);
  for (int g = 0; g < accept->n_groups; ++g)
    if (accept->group_sizes[g] < 1) return fail(nullptr, HEISD_EINVAL, "build_tree: group_sizes[%d] < 1", g);
  TreeBuilder tb;
  tb.cand = candidates; tb.R = R; tb.K = K; tb.max_tokens = max_tokens;
  tb.exact_mask = accept->exact_group_mask; tb.tokens = tokens; tb.parent = parent;
  for (int j = 0, g = 0; j < K; ++g) {
    const int gi = g % accept->n_groups, size = accept->group_sizes[gi];
    tb.lv_start.push_back(j);
    tb.lv_end.push_back(j + size < K ? j + size : K);
    tb.lv_group.push_back(gi);
    j += size;
  }
  tb.grow(0, -1, R == 64 ? ~0ull : ((1ull << R) - 1));
  *n_tokens = tb.n;
  g_init_err[0] = 0;
  return HEISD_OK;
}

// ---- prefix extension: chunked prefill and the autoregressive decode step -----------------------

extern "C" int heisd_prefill_chunk(heisd_verify_ctx *ctx, const heisd_kv_desc *kv, const int32_t *token_ids,
                                   const float *x_rows, int32_t n_rows, int32_t batch, int32_t *next_bin,
                                   float *last_logits, void *stream) {
  if (!ctx) return HEISD_EINVAL;
  if (!kv || !kv->k_cache || !kv->v_cache || !kv->prefix_len || !next_bin)
    return fail(ctx, HEISD_EINVAL, "prefill_chunk: NULL required pointer");
  if (!token_ids && !x_rows)
    return fail(ctx, HEISD_EINVAL, "prefill_chunk: token_ids, x_rows or both must be given");
  const heisd_model_desc &d = ctx->d;
  if (n_rows < 1 || batch < 1 || n_rows > d.max_k || batch > d.max_batch || n_rows > d.kv_capacity)
    return fail(ctx, HEISD_EINVAL, "prefill_chunk: n_rows=%d batch=%d outside [1,%d] x [1,%d] (kv_capacity %d)", n_rows,
                batch, d.max_k, d.max_batch, d.kv_capacity);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int M = batch * n_rows;
  (void)hipGetLastError();
  const bool use_fast = ctx->fast_ok && M <= 8 && token_ids && !x_rows && ctx->path != HEISD_PATH_GENERIC && ctx->path != HEISD_PATH_BATCH;
  if ((ctx->path == HEISD_PATH_FAST || ctx->path == HEISD_PATH_PERSIST) && !use_fast)
    return fail(ctx, HEISD_EUNSUPPORTED, "prefill_chunk: the selected path serves token rows with batch*n_rows <= 8 only");
  const bool prof = ctx->prof_on && ctx->prof_steps < HEISD_PROFILE_MAX_STEPS;
  if (prof) ctx->prof_steps++;
  bool persisted = false;
  if (use_fast && persist_wanted(ctx)) {
    const AcceptArgs none{};          // no drafts to judge: the greedy bin after the last row is taken below
    persisted = persist_try_launch(ctx, ctx->path == HEISD_PATH_PERSIST, kv, token_ids, n_rows, batch, nullptr, ctx->logits,
                                   none, st, prof);
  }
  if (persisted) {
  } else if (use_fast)
    fast_forward(ctx, kv, token_ids, n_rows, batch, nullptr, ctx->logits, st, prof);
  else if (ctx->path == HEISD_PATH_GENERIC)
    generic_forward(ctx, kv, token_ids, n_rows, batch, nullptr, ctx->logits, st, prof, nullptr, nullptr, x_rows);
  else
    batch_forward(ctx, kv, token_ids, n_rows, batch, nullptr, ctx->logits, st, prof, nullptr, nullptr, x_rows);
  {
    ProfScope ps(ctx, HEISD_KC_ACCEPT, st, prof);
    last_row_argmax<<<dim3(batch), dim3(64), 0, st>>>(ctx->logits, n_rows, d.n_bins, next_bin, last_logits, kv->prefix_len,
                                                      d.kv_capacity, ctx->dev_err);
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(ctx, HEISD_EHIP, "prefill_chunk: %s", hipGetErrorString(e));
  ctx->err[0] = 0;
  return HEISD_OK;
}

// ---- the verify-skip decision (Sec. 4.1, Alg. 1) ------------------------------------------------

static bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

extern "C" int heisd_export_features(heisd_verify_ctx *ctx, const int32_t *row, int32_t rows_per_episode,
                                     int32_t batch, float *feat, void *stream) {
  if (!ctx) return HEISD_EINVAL;
  if (!feat || !aligned16(feat)) return fail(ctx, HEISD_EINVAL, "export_features: NULL or misaligned output");
  const heisd_model_desc &d = ctx->d;
  if (rows_per_episode < 1 || batch < 1 || rows_per_episode > d.max_k || batch > d.max_batch)
    return fail(ctx, HEISD_EINVAL, "export_features: rows_per_episode=%d batch=%d outside the context", rows_per_episode, batch);
  if (d.d_model % 4) return fail(ctx, HEISD_EUNSUPPORTED, "export_features: d_model not a multiple of 4");
  (void)hipGetLastError();
  export_features<<<dim3(batch), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(ctx->x, row, rows_per_episode, d.d_model,
                                                                                   d.final_norm, d.rms_eps, feat);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(ctx, HEISD_EHIP, "export_features: %s", hipGetErrorString(e));
  ctx->err[0] = 0;
  return HEISD_OK;
}

static int similarity_launch(const float *a, const float *b, int n, int m, int d, float *S, float T,
                             unsigned long long *key, hipStream_t st, const char *who) {
  if (!a || !b || !aligned16(a) || !aligned16(b)) return fail(nullptr, HEISD_EINVAL, "%s: NULL or misaligned features", who);
  if (n < 1 || m < 1 || d < 4 || d % 4 || n > 65535 || m > 65535)
    return fail(nullptr, HEISD_EINVAL, "%s: n=%d m=%d d=%d (1..65535 points, d a multiple of 4)", who, n, m, d);
  const long long pairs = (long long)n * m;
  pair_similarity<<<dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, st>>>(a, b, n, m, d, S, T, key);
  return HEISD_OK;
}

extern "C" int heisd_feature_similarity(const float *a, const float *b, int32_t n, int32_t m, int32_t d, float *S,
                                        void *stream) {
  if (!S) return fail(nullptr, HEISD_EINVAL, "feature_similarity: NULL output");
  (void)hipGetLastError();
  const int rc = similarity_launch(a, b, n, m, d, S, 0.f, nullptr, static_cast<hipStream_t>(stream), "feature_similarity");
  if (rc != HEISD_OK) return rc;
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(nullptr, HEISD_EHIP, "feature_similarity: %s", hipGetErrorString(e));
  g_init_err[0] = 0;
  return HEISD_OK;
}

extern "C" int heisd_skip_offline(const float *feat, int32_t n, int32_t d, float T, float *S, uint64_t *work,
                                  float *min_s, int32_t *o_dist, void *stream) {
  if (!work || !min_s || !o_dist || ((uintptr_t)work & 7)) return fail(nullptr, HEISD_EINVAL, "skip_offline: NULL or misaligned pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  if (!feat || !aligned16(feat) || n < 1 || n > 65535 || d < 4 || d % 4)
    return fail(nullptr, HEISD_EINVAL, "skip_offline: n=%d d=%d (1..65535 points, d a multiple of 4) or bad pointer", n, d);
  unsigned long long *key = reinterpret_cast<unsigned long long *>(work);
  skip_key_init<<<dim3(1), dim3(1), 0, st>>>(key);
  const int rc = similarity_launch(feat, feat, n, n, d, S, T, key, st, "skip_offline");
  if (rc != HEISD_OK) return rc;
  skip_key_decode<<<dim3(1), dim3(1), 0, st>>>(key, min_s, o_dist);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(nullptr, HEISD_EHIP, "skip_offline: %s", hipGetErrorString(e));
  g_init_err[0] = 0;
  return HEISD_OK;
}

extern "C" int heisd_skip_decide(const float *feat_prev, const float *feat_last, const int32_t *dist, int32_t batch,
                                 int32_t d, const float *min_s, const int32_t *o_dist, uint8_t *skip_mask,
                                 float *similarity, void *stream) {
  if (!feat_prev || !feat_last || !dist || !min_s || !o_dist || !skip_mask || !aligned16(feat_prev) || !aligned16(feat_last))
    return fail(nullptr, HEISD_EINVAL, "skip_decide: NULL or misaligned pointer");
  if (batch < 1 || d < 4 || d % 4) return fail(nullptr, HEISD_EINVAL, "skip_decide: batch=%d d=%d", batch, d);
  (void)hipGetLastError();
  skip_decide<<<dim3(batch), dim3(64), 0, static_cast<hipStream_t>(stream)>>>(feat_prev, feat_last, dist, d, min_s, o_dist,
                                                                              skip_mask, similarity);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(nullptr, HEISD_EHIP, "skip_decide: %s", hipGetErrorString(e));
  g_init_err[0] = 0;
  return HEISD_OK;
}

// ---- retrieval: exact cosine Top-K over the embedding database (App. C) -------------------------

struct RetrieveLayout {
  size_t scores, cand_val, cand_idx, total;
  int n_chunks;
  long long ld_scores;
  RetrieveLayout(long long N, int batch, int K) {
    n_chunks = (int)((N + kTopChunk - 1) / kTopChunk);
    ld_scores = (N + 63) / 64 * 64;
    size_t off = 0;
    scores = off;   off += align256((size_t)batch * (size_t)ld_scores * sizeof(float));
    cand_val = off; off += align256((size_t)batch * n_chunks * K * sizeof(float));
    cand_idx = off; off += align256((size_t)batch * n_chunks * K * sizeof(int));
    total = off;
  }
};

static bool retrieve_args_ok(int64_t N, int32_t batch, int32_t K) {
  return N >= 1 && N <= 0x7FFFFFFFLL && batch >= 1 && batch <= 1024 && K >= 1 && K <= kTopMaxK;
}

extern "C" size_t heisd_retrieve_workspace_bytes(int64_t n_vectors, int32_t batch, int32_t K) {
  if (!retrieve_args_ok(n_vectors, batch, K)) return 0;
  return RetrieveLayout(n_vectors, batch, K).total;
}

// What the retrieval calls need to know about the current device, found once per device: the number of
// compute units, the scan kernels' LDS limit raised to the largest query block they may be given, and the
// address of this device's copy of the static scratch array (see heisd_retrieve_topk_static).
constexpr size_t kRetrieveStaticBytes = (size_t)8 << 20;
constexpr int kRetrieveMaxD = 8192;
constexpr int kRetrieveMaxDevices = 64;

// Scratch of heisd_retrieve_topk_static: scores and first-round winners, laid out by RetrieveLayout.  In
// host code this name is only a handle for hipGetSymbolAddress; the device address is kept per device.
static __device__ __align__(256) unsigned char retrieve_static_scratch[kRetrieveStaticBytes];

struct RetrieveDevice {
  bool ready = false;
  int n_cu = 256;
  unsigned char *scratch = nullptr;
};
static RetrieveDevice g_retrieve_dev[kRetrieveMaxDevices];
static std::mutex g_retrieve_mutex;

template <int NQ>
static hipError_t retrieve_scores_prepare() {
  return hipFuncSetAttribute(reinterpret_cast<const void *>(&retrieve_scores<NQ>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, NQ * kRetrieveMaxD * (int)sizeof(float));
}

// The current device's entry (set up on the first call made with that device current); nullptr + *err on failure.
static const RetrieveDevice *retrieve_device(hipError_t *err) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess && (dev < 0 || dev >= kRetrieveMaxDevices)) e = hipErrorInvalidDevice;
  if (e != hipSuccess) { *err = e; return nullptr; }
  std::lock_guard<std::mutex> lock(g_retrieve_mutex);
  RetrieveDevice &rd = g_retrieve_dev[dev];
  if (!rd.ready) {
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e == hipSuccess && prop.multiProcessorCount > 0) rd.n_cu = prop.multiProcessorCount;
    if (e == hipSuccess) e = retrieve_scores_prepare<1>();
    if (e == hipSuccess) e = retrieve_scores_prepare<2>();
    if (e == hipSuccess) e = retrieve_scores_prepare<3>();
    if (e == hipSuccess) e = retrieve_scores_prepare<4>();
    void *p = nullptr;
    if (e == hipSuccess) e = hipGetSymbolAddress(&p, HIP_SYMBOL(retrieve_static_scratch));
    if (e == hipSuccess && !p) e = hipErrorInvalidSymbol;
    if (e != hipSuccess) { *err = e; return nullptr; }
    rd.scratch = static_cast<unsigned char *>(p);
    rd.ready = true;
  }
  return &rd;
}

template <int NQ>
static hipError_t retrieve_scores_launch(const uint16_t *db, long long N, int d, const float *q, float *scores,
                                         long long ld, int n_cu, hipStream_t st) {
  const int lds = NQ * d * (int)sizeof(float);
  const long long pairs = (N + 1) / 2, want = (pairs + kScanThreads / 64 - 1) / (kScanThreads / 64);
  const long long resident = (NQ <= 2 ? 4LL : 2LL) * n_cu;      // workgroups a compute unit holds at this LDS size
  const int grid = (int)(want < resident ? want : resident);
  retrieve_scores<NQ><<<dim3(grid), dim3(kScanThreads), lds, st>>>(db, N, d, q, scores, ld);
  return hipGetLastError();
}

static int retrieve_check_args(const void *db, int64_t n_vectors, int32_t d, const float *queries, int32_t batch, int32_t K,
                               const int32_t *payload, int32_t payload_len, const int32_t *top_index, const float *top_score,
                               const int32_t *top_payload, const char *who) {
  if (!db || !queries || !top_index || !top_score) return fail(nullptr, HEISD_EINVAL, "%s: NULL required pointer", who);
  if (!retrieve_args_ok(n_vectors, batch, K) || d < 4 || d % 4 || d > kRetrieveMaxD)
    return fail(nullptr, HEISD_EINVAL, "%s: n_vectors=%lld batch=%d K=%d d=%d outside the supported range", who,
                (long long)n_vectors, batch, K, d);
  if ((payload != nullptr) != (top_payload != nullptr) || (payload && payload_len < 1))
    return fail(nullptr, HEISD_EINVAL, "%s: payload and top_payload go together, with payload_len >= 1", who);
  if (((uintptr_t)db & 7) || !aligned16(queries)) return fail(nullptr, HEISD_EINVAL, "%s: misaligned pointer", who);
  return HEISD_OK;
}

// The three launches of one search; `base` holds the buffers of `lay`.
static int retrieve_enqueue(const RetrieveDevice *rd, const RetrieveLayout &lay, unsigned char *base, const void *db,
                            int64_t n_vectors, int32_t d, const float *queries, int32_t batch, int32_t K,
                            const int32_t *payload, int32_t payload_len, int32_t *top_index, float *top_score,
                            int32_t *top_payload, hipStream_t st, const char *who) {
  float *scores = reinterpret_cast<float *>(base + lay.scores);
  float *cand_val = reinterpret_cast<float *>(base + lay.cand_val);
  int *cand_idx = reinterpret_cast<int *>(base + lay.cand_idx);
  (void)hipGetLastError();
  const uint16_t *dbp = static_cast<const uint16_t *>(db);
  hipError_t e = hipSuccess;
  for (int q0 = 0; q0 < batch && e == hipSuccess; q0 += 4) {       // the database is streamed once per four queries
    const int nq = batch - q0 < 4 ? batch - q0 : 4;
    const float *qp = queries + (size_t)q0 * d;
    float *sp = scores + (size_t)q0 * lay.ld_scores;
    if (nq == 1) e = retrieve_scores_launch<1>(dbp, n_vectors, d, qp, sp, lay.ld_scores, rd->n_cu, st);
    else if (nq == 2) e = retrieve_scores_launch<2>(dbp, n_vectors, d, qp, sp, lay.ld_scores, rd->n_cu, st);
    else if (nq == 3) e = retrieve_scores_launch<3>(dbp, n_vectors, d, qp, sp, lay.ld_scores, rd->n_cu, st);
    else e = retrieve_scores_launch<4>(dbp, n_vectors, d, qp, sp, lay.ld_scores, rd->n_cu, st);
  }
  if (e == hipSuccess) {
    retrieve_top_chunks<<<dim3(lay.n_chunks, batch), dim3(256), 0, st>>>(scores, lay.ld_scores, n_vectors, K, cand_val,
                                                                        cand_idx, lay.n_chunks);
    retrieve_top_merge<<<dim3(batch), dim3(256), 0, st>>>(cand_val, cand_idx, lay.n_chunks * K, K, top_score, top_index,
                                                         payload, payload_len, top_payload);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return fail(nullptr, HEISD_EHIP, "%s: %s", who, hipGetErrorString(e));
  g_init_err[0] = 0;
  return HEISD_OK;
}

extern "C" int heisd_retrieve_topk(const void *db, int64_t n_vectors, int32_t d, const float *queries, int32_t batch,
                                   int32_t K, const int32_t *payload, int32_t payload_len, int32_t *top_index,
                                   float *top_score, int32_t *top_payload, void *workspace, size_t workspace_bytes,
                                   void *stream) {
  const char *who = "retrieve_topk";
  const int rc = retrieve_check_args(db, n_vectors, d, queries, batch, K, payload, payload_len, top_index, top_score,
                                     top_payload, who);
  if (rc != HEISD_OK) return rc;
  if (!workspace || ((uintptr_t)workspace & 255)) return fail(nullptr, HEISD_EINVAL, "%s: NULL or misaligned workspace", who);
  const RetrieveLayout lay(n_vectors, batch, K);
  if (workspace_bytes < lay.total)
    return fail(nullptr, HEISD_ENOMEM, "%s: workspace %zu bytes < %zu needed", who, workspace_bytes, lay.total);
  hipError_t e = hipSuccess;
  const RetrieveDevice *rd = retrieve_device(&e);
  if (!rd) return fail(nullptr, HEISD_EHIP, "%s: %s", who, hipGetErrorString(e));
  return retrieve_enqueue(rd, lay, static_cast<unsigned char *>(workspace), db, n_vectors, d, queries, batch, K, payload,
                          payload_len, top_index, top_score, top_payload, static_cast<hipStream_t>(stream), who);
}

extern "C" size_t heisd_retrieve_static_bytes(void) { return kRetrieveStaticBytes; }

extern "C" int heisd_retrieve_topk_static(const void *db, int64_t n_vectors, int32_t d, const float *queries,
                                          int32_t batch, int32_t K, const int32_t *payload, int32_t payload_len,
                                          int32_t *top_index, float *top_score, int32_t *top_payload, void *stream) {
  const char *who = "retrieve_topk_static";
  const int rc = retrieve_check_args(db, n_vectors, d, queries, batch, K, payload, payload_len, top_index, top_score,
                                     top_payload, who);
  if (rc != HEISD_OK) return rc;
  const RetrieveLayout lay(n_vectors, batch, K);
  if (lay.total > kRetrieveStaticBytes)
    return fail(nullptr, HEISD_ENOMEM, "%s: this search needs %zu bytes of scratch, the static array holds %zu "
                "(use heisd_retrieve_topk with a workspace)", who, lay.total, kRetrieveStaticBytes);
  hipError_t e = hipSuccess;
  const RetrieveDevice *rd = retrieve_device(&e);
  if (!rd) return fail(nullptr, HEISD_EHIP, "%s: %s", who, hipGetErrorString(e));
  // rd->scratch is the device address of this GPU's copy of the array; every buffer in it is written
  // before it is read within one call (all scores below n_vectors, K winners per chunk), so nothing
  // of an earlier call's contents is ever seen and nothing has to be cleared.
  return retrieve_enqueue(rd, lay, rd->scratch, db, n_vectors, d, queries, batch, K, payload, payload_len, top_index,
                          top_score, top_payload, static_cast<hipStream_t>(stream), who);
}

// ---- reference measurements (not part of the method) ---------------------------------------------

extern "C" int heisd_measure_read(const void *buf, size_t bytes, int32_t pattern, int32_t ksteps, int32_t in_flight,
                                  int32_t workgroups, uint32_t *sink, void *stream) {
  if (!buf || !sink || ((uintptr_t)buf & 15)) return fail(nullptr, HEISD_EINVAL, "measure_read: NULL or misaligned pointer");
  if ((pattern != 0 && pattern != 1) || (in_flight != 8 && in_flight != 16) || workgroups < 1 || workgroups > 65535)
    return fail(nullptr, HEISD_EINVAL, "measure_read: pattern %d in_flight %d workgroups %d", pattern, in_flight, workgroups);
  hipStream_t st = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  const mu32x4 *p = static_cast<const mu32x4 *>(buf);
  if (pattern == 0) {
    const size_t n_vec = bytes / 16;
    if (n_vec < (size_t)workgroups * 8 * 64 * in_flight) return fail(nullptr, HEISD_EINVAL, "measure_read: buffer too small for this grid");
    if (in_flight == 8) measure_read_contiguous<8><<<dim3(workgroups), dim3(kMeasureThreads), 0, st>>>(p, n_vec, sink);
    else measure_read_contiguous<16><<<dim3(workgroups), dim3(kMeasureThreads), 0, st>>>(p, n_vec, sink);
  } else {
    if (ksteps < 8 || ksteps > 65536) return fail(nullptr, HEISD_EINVAL, "measure_read: ksteps %d", ksteps);
    const size_t n_tiles = bytes / ((size_t)ksteps * 1024);
    if (n_tiles < 1 || n_tiles > 0x7FFFFFFF) return fail(nullptr, HEISD_EINVAL, "measure_read: buffer holds no whole tile");
    if (in_flight == 8) measure_read_tiles<8><<<dim3(workgroups), dim3(kMeasureThreads), 0, st>>>(p, (int)n_tiles, ksteps, sink);
    else measure_read_tiles<16><<<dim3(workgroups), dim3(kMeasureThreads), 0, st>>>(p, (int)n_tiles, ksteps, sink);
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(nullptr, HEISD_EHIP, "measure_read: %s", hipGetErrorString(e));
  return HEISD_OK;
}

extern "C" int heisd_measure_empty_launch(int32_t workgroups, void *stream) {
  if (workgroups < 1 || workgroups > 65535) return fail(nullptr, HEISD_EINVAL, "measure_empty_launch: workgroups %d", workgroups);
  (void)hipGetLastError();
  measure_empty<<<dim3(workgroups), dim3(kMeasureThreads), 0, static_cast<hipStream_t>(stream)>>>();
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(nullptr, HEISD_EHIP, "measure_empty_launch: %s", hipGetErrorString(e));
  return HEISD_OK;
}
