/*
 * heisd_verify.h - C ABI of the target-model verify step of HeiSD's hybrid
 * speculative decoding, for one AMD MI355X (gfx950).
 *
 * What one call computes (paper Sec. 2.2, Eq. 2-2; Sec. 4.1; Sec. 4.2; App. A.1/A.2):
 * given the cached keys/values of a vision+text prefix, a block of K drafted
 * action tokens per episode (from the retrieval or the drafter branch), and the
 * target model's weights, run ONE teacher-forced decoder forward over the K
 * tokens, restrict the LM head to the 256 action bins, take the greedy bin per
 * position, and apply the sequence-wise relaxed acceptance rule.  Episodes whose
 * verify-skip flag is set bypass verification and keep their whole draft.
 *
 * Plain C99: no C++ types, no exceptions cross this boundary.  Every pointer is
 * marked HOST or DEVICE.  The library never allocates device memory, never
 * synchronises in heisd_verify_step, and keeps only what the opaque context holds.
 */
#ifndef HEISD_VERIFY_H
#define HEISD_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Return codes: 0 on success, negative on failure.  Argument errors (EINVAL, EUNSUPPORTED, ENOMEM)
 * are found before anything is enqueued.  EHIP means the HIP runtime refused a launch: launches
 * issued before the refused one stay enqueued, and the call's outputs are undefined. */
#define HEISD_OK 0
#define HEISD_EINVAL (-1)        /* NULL / out-of-range argument, inconsistent shapes        */
#define HEISD_EUNSUPPORTED (-2)  /* shape the compiled kernels do not cover                   */
#define HEISD_ENOMEM (-3)        /* workspace smaller than heisd_verify_workspace_bytes()     */
#define HEISD_EHIP (-4)          /* the HIP runtime reported an error                          */

#define HEISD_MAX_GROUPS 8

typedef struct heisd_verify_ctx heisd_verify_ctx; /* opaque */

/*
 * The target model M_V: a Llama-2-style decoder (App. A.1) whose action head reads
 * n_bins consecutive vocabulary ids (App. A.2: 256 bins per action dimension).
 * All matrices are DEVICE pointers to bf16, row-major [out, in], caller-owned,
 * read-only, and must outlive the context.  Gains are DEVICE fp32 vectors.
 * The pointer tables themselves (wq[l] ...) are HOST arrays of n_layers device
 * pointers; they are copied at init.
 */
typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
  int32_t n_bins;         /* number of action bins (256)                                  */
  int32_t bin_token_base; /* bin b <-> vocabulary id bin_token_base + b                   */
  float rms_eps;          /* RMSNorm epsilon                                               */
  float rope_base;        /* rotary base (rotate-half pairing, absolute positions)         */
  int32_t max_batch;      /* largest `batch` a step may pass                               */
  int32_t max_k;          /* largest `K` a step may pass (<= 1024; tree steps: <= 256)     */
  int32_t kv_capacity;    /* rows per (layer, episode, head) in the caller's KV cache      */
  const void *tok_emb;    /* DEVICE bf16 [vocab, d_model]                                  */
  const void *const *wq, *const *wk, *const *wv, *const *wo;    /* HOST tables of DEVICE bf16 [d_model, d_model] */
  const void *const *w_gate, *const *w_up;                       /* ... DEVICE bf16 [d_ffn, d_model]              */
  const void *const *w_down;                                     /* ... DEVICE bf16 [d_model, d_ffn]              */
  const float *const *attn_norm, *const *ffn_norm;               /* HOST tables of DEVICE fp32 [d_model]          */
  const float *final_norm;                                       /* DEVICE fp32 [d_model]                         */
  const void *lm_head;    /* DEVICE bf16 [vocab, d_model]; only rows bin_token_base .. +n_bins-1 are read */
  void *workspace;        /* DEVICE scratch, caller-allocated, 256-byte aligned, owned by the ctx until heisd_free */
  size_t workspace_bytes; /* at least heisd_verify_workspace_bytes(desc)                   */
} heisd_model_desc;

/*
 * The prefix (observations + prompt of Eq. 2-2) as cached keys and values.
 * Layout: bf16 [n_layers][batch][n_heads][kv_capacity][head_dim], keys already
 * rotated.  A step READS rows 0 .. prefix_len[b]-1 and WRITES rows prefix_len[b] ..
 * prefix_len[b]+K-1 of every non-skipped episode b (the drafts' keys/values), so
 * that the caller's next step can start at prefix_len[b] + accepted_len[b]; rows
 * past that are garbage to be overwritten.  prefix_len[b] + K <= kv_capacity is the
 * caller's duty; device data cannot be checked on the host without a sync, so an episode
 * that breaks it (or has a negative prefix_len) is left out of the step ON THE DEVICE:
 * nothing of its cache is read or written, its accepted_len and next_token (next_bin
 * of heisd_prefill_chunk) are -1, its target_bins -1, its logits NaN, the other episodes
 * are unaffected, and heisd_verify_check reports it.
 * first_pred[b] is the target's greedy bin after the last prefix position, i.e.
 * a_hat_0 of Eq. 2-2, which depends on the prefix alone and is produced by whoever
 * filled the cache.
 */
typedef struct {
  void *k_cache;             /* DEVICE bf16, see layout above */
  void *v_cache;             /* DEVICE bf16                   */
  const int32_t *prefix_len; /* DEVICE i32 [batch]            */
  const int32_t *first_pred; /* DEVICE i32 [batch], bin index in [0, n_bins) */
} heisd_kv_desc;

/*
 * Sequence-wise relaxed acceptance (Sec. 4.2).  Draft positions are cut into
 * consecutive groups following group_sizes, repeating every sum(group_sizes)
 * positions (one action slice: (X,Y,Z), (rX,rY,rZ), (G)).  bias_j = |draft bin -
 * target bin|.  A group is accepted iff every bias_j <= tok_threshold and the sum of
 * its biases <= seq_budget; a group whose bit is set in exact_group_mask (the
 * gripper) is accepted iff every bias is 0.  accepted_len is the total length of the
 * leading run of accepted groups.  Strict verification (Eq. 2-2) is thresholds 0/0.
 * The paper's values: tok_threshold 15, seq_budget 30, groups {3,3,1}, mask 1<<2.
 * mode 0 is that rule.  mode 1 is a token-granular variant that is NOT in the paper:
 * accept up to the first token whose bias exceeds tok_threshold, or whose running
 * sum of biases over the block exceeds seq_budget, or exact-group token with bias != 0.
 */
typedef struct {
  int32_t tok_threshold;
  int32_t seq_budget;
  int32_t n_groups;
  int32_t group_sizes[HEISD_MAX_GROUPS];
  uint32_t exact_group_mask;
  int32_t mode;
} heisd_accept_desc;

/* Bytes of device workspace heisd_verify_init needs for this model description
 * (depends only on the shape fields).  Returns 0 if the description is invalid.
 * The workspace holds, besides activations and exchange buffers, one copy of every projection
 * matrix (and of the n_bins LM-head rows) in the order the matrix cores consume them, so it is
 * a little larger than the decoder's weights (13.1 GB at the 7B shape). */
size_t heisd_verify_workspace_bytes(const heisd_model_desc *desc);

/*
 * Validate the description, copy the pointer tables, lay out the workspace, build the
 * rotary table, copy the projection matrices into the workspace in fragment order (the weights
 * must hold their final values when init is called; later changes to them are not seen by the
 * record kernels).  Synchronises the device.  *out receives a context to be released
 * with heisd_free.  Not thread-safe; one step in flight per context.
 * Everything the library keeps on the device lives in the caller's workspace, with one exception: the first
 * init on a device allocates 2 MB of uncached device memory (hipExtMallocWithFlags) that is never freed, a pool
 * of 32 slots for the grid-barrier flags of the persistent kernel; a context takes a slot here and returns it in
 * heisd_free, and one that finds no slot (or no such memory) keeps its flags in the workspace, which is slower
 * and no less correct.
 * Errors: EINVAL (NULL pointers, non-positive sizes, d_model != n_heads*head_dim,
 * bins outside the vocabulary), EUNSUPPORTED (head_dim not 64 or 128, d_model or d_ffn
 * or n_bins not a multiple of 16, max_k > 1024, kv_capacity > 4096), ENOMEM (workspace too
 * small), EHIP.
 */
int heisd_verify_init(const heisd_model_desc *desc, heisd_verify_ctx **out);

/*
 * Enqueue one verify step on `stream` (asynchronous; outputs are valid once the
 * caller has synchronised the stream).  Idempotent for unchanged inputs.
 *
 *   draft_tokens  DEVICE i32 [batch][K]   vocabulary ids of the drafts (an id outside the
 *                                         bin range is clamped for the embedding lookup and
 *                                         makes its group fail)
 *   skip_mask     DEVICE u8  [batch]      nonzero = bypass verification (Sec. 4.1, Sec. 6.2);
 *                                         NULL = verify every episode
 *   accepted_len  DEVICE i32 [batch] out  n in [0, K]; K for skipped episodes
 *   next_token    DEVICE i32 [batch] out  vocabulary id of the target's own token at position
 *                                         n (the correction after a rejection, or the bonus
 *                                         token when n = K); -1 for skipped episodes
 *   target_bins   DEVICE i32 [batch][K+1] out, optional (NULL ok): a_hat_0 .. a_hat_K as bins;
 *                                         -1 for skipped episodes
 *   bin_logits    DEVICE f32 [batch][K][n_bins] out, optional (NULL ok): logits of the action
 *                                         bins at every draft position; NaN for skipped episodes
 *   stream        hipStream_t passed as void*; NULL = the default stream
 *
 * Errors (nothing enqueued): EINVAL for NULL required pointers, K < 1, batch < 1,
 * K > max_k, batch > max_batch, K > kv_capacity, n_groups outside [1, HEISD_MAX_GROUPS],
 * a group size < 1, negative thresholds, mode not 0/1; EHIP if a launch fails.
 */
int heisd_verify_step(heisd_verify_ctx *ctx, const heisd_kv_desc *kv, const int32_t *draft_tokens,
                      int32_t K, int32_t batch, const heisd_accept_desc *accept,
                      const uint8_t *skip_mask, int32_t *accepted_len, int32_t *next_token,
                      int32_t *target_bins, float *bin_logits, void *stream);

/*
 * Sequence-wise TREE verification (Sec. 4.2: Top-K retrieval; the draft tree is built sequence by
 * sequence; every chain from the root is checked with the relaxed rule).  One decoder forward over
 * all T tree tokens of every episode: token t sits at position prefix_len + depth(t) and attends to
 * the prefix, its ancestors and itself, which gives every chain the numbers a forward of that chain
 * alone would give.  Then, per episode, the chain that the acceptance rule lets get furthest is
 * chosen (among equals: the one whose last accepted token has the lowest index), and the key/value
 * rows of its accepted tokens are moved to cache rows prefix_len .. prefix_len + n - 1, so that the
 * cache continues exactly as after a linear step over that chain.
 *
 *   tree_tokens   DEVICE i32 [batch][T]   vocabulary ids of the tree tokens
 *   parent        DEVICE i32 [batch][T]   index of the token before t in its chain; -1 = t follows
 *                                         the prefix.  A value outside [-1, t) marks padding: the
 *                                         token is in no chain (it still costs a row of the forward)
 *   T             tokens per episode, 1 .. min(max_k, 256); cache rows prefix_len .. prefix_len+T-1
 *                 of a verified episode are overwritten
 *   accepted_len  DEVICE i32 [batch] out  n = tokens of the chosen chain that are accepted; for a
 *                                         skipped episode the length of the first chain (token 0,
 *                                         then always the lowest-index child), executed unverified
 *   next_token    DEVICE i32 [batch] out  the target's own token after the accepted tokens (after
 *                                         the prefix when n = 0); -1 for skipped episodes
 *   accepted_path DEVICE i32 [batch][T] out  the n accepted token indices in chain order, then -1
 *   target_bins   DEVICE i32 [batch][T+1] out, optional: [0] = first_pred, [t+1] = the target's
 *                                         greedy bin after token t; -1 for skipped episodes
 *   bin_logits    DEVICE f32 [batch][T][n_bins] out, optional; NaN for skipped episodes
 *   accept        as in heisd_verify_step; the sequence a token belongs to follows from its depth
 *   other arguments as in heisd_verify_step.
 *
 * Runs on the record kernels (any T); asynchronous, allocates nothing, idempotent only if the
 * caller restores nothing: the prefix rows are never written, and the rows past prefix_len are
 * rewritten from the inputs by every call.
 * Errors (nothing enqueued): as heisd_verify_step, plus EINVAL for T > 256 and EUNSUPPORTED when the
 * context is pinned to a path that only serves batch*K <= 8 (HEISD_PATH_FAST / _PERSIST).
 */
int heisd_verify_tree_step(heisd_verify_ctx *ctx, const heisd_kv_desc *kv, const int32_t *tree_tokens,
                           const int32_t *parent, int32_t T, int32_t batch, const heisd_accept_desc *accept,
                           const uint8_t *skip_mask, int32_t *accepted_len, int32_t *next_token,
                           int32_t *accepted_path, int32_t *target_bins, float *bin_logits, void *stream);

/*
 * Host-side construction of the draft tree from R retrieved candidates of K tokens each
 * (Sec. 4.2: sequences of different retrieval results may follow each other, except the gripper).
 * Plain CPU code, no device access.  Under a node, the children for a sequence level that is not
 * exact are the distinct sequences of ALL candidates at that level; for an exact level (gripper)
 * only those of the candidates whose sequence the node carries.  Equal siblings are merged.  Layout:
 * depth-first preorder, candidates in the given order; a node that would exceed max_tokens is left
 * out with its subtree.
 *
 *   candidates    HOST i32 [R][K]          vocabulary ids
 *   accept        group sizes and exact mask (thresholds are not used)
 *   tokens,parent HOST i32 [max_tokens] out
 *   n_tokens      HOST out                 tokens written (<= max_tokens)
 * Errors: EINVAL for NULL pointers, R < 1, K < 1, max_tokens < 1, R > 64, a bad group description.
 */
int heisd_build_sequence_tree(const int32_t *candidates, int32_t R, int32_t K, const heisd_accept_desc *accept,
                              int32_t max_tokens, int32_t *tokens, int32_t *parent, int32_t *n_tokens);

/*
 * Extend every episode's cached prefix by n_rows rows: the decoder forward over the new rows against
 * the rows already cached, appending their keys and values, and the target's greedy action bin after
 * the LAST new row (Eq. 2-1).  Two uses, both on the same kernels as the verify step:
 *   - chunked prefill of the vision+text prefix (App. A.1: 256 visual tokens arrive as embeddings, the
 *     prompt as token ids): one call per chunk of at most max_k rows; after the last chunk `next_bin`
 *     is the `first_pred` the verify step expects;
 *   - the autoregressive decode step the method falls back to when every candidate is rejected
 *     (Sec. 4.2) and that speculative decoding replaces (Sec. 2.2, App. A.2): n_rows = 1, token_ids =
 *     the token just produced; `next_bin` is the next action token's bin.
 *
 *   token_ids    DEVICE i32 [batch][n_rows]            vocabulary ids, or NULL
 *   x_rows       DEVICE f32 [batch][n_rows][d_model]   input embeddings, or NULL.  One of the two, or both:
 *                with both, a row whose token id is negative takes its embedding from x_rows and every other
 *                row is looked up, so that visual and prompt rows can share a chunk (one pass over the
 *                weights instead of two)
 *   next_bin     DEVICE i32 [batch] out                greedy bin after the last new row
 *   last_logits  DEVICE f32 [batch][n_bins] out, optional (NULL ok)
 * Cache rows prefix_len[b] .. prefix_len[b]+n_rows-1 are written; the library does not advance
 * prefix_len (the caller adds n_rows).  kv->first_pred is not read.  Asynchronous, allocates nothing.
 * Errors (nothing enqueued): EINVAL for NULL required pointers, neither input given, n_rows or
 * batch outside [1, max_k] x [1, max_batch]; EUNSUPPORTED when the context is pinned to the <= 8-row
 * kernels and the call has more rows or embeddings as input; EHIP.
 */
int heisd_prefill_chunk(heisd_verify_ctx *ctx, const heisd_kv_desc *kv, const int32_t *token_ids,
                        const float *x_rows, int32_t n_rows, int32_t batch, int32_t *next_bin,
                        float *last_logits, void *stream);

/*
 * The verify-skip DECISION (Sec. 4.1, Alg. 1), which produces the skip mask heisd_verify_step consumes.
 * The paper captures the input features of the final (`lm_head`) layer while a draft is verified,
 * computes the feature similarity S of pairs of trajectory points, collects on historical trajectories
 * the minimum acceptable similarity min_S with its point distance O_dist (offline stage), and on a new
 * task skips the verification of points that are "excessively similar".  Similarity is the cosine; the
 * readings of what the paper leaves open are stated per call.  fp32 throughout; all calls asynchronous
 * on `stream`, none allocates.
 *
 * heisd_export_features: feat[b] = the final-norm hidden state (the LM head's input) of row row[b]
 *   (NULL: the last row) of episode b in the MOST RECENT step of this context (heisd_verify_step,
 *   heisd_verify_tree_step or heisd_prefill_chunk with the same rows_per_episode and batch).
 *     row   DEVICE i32 [batch] or NULL;  feat  DEVICE f32 [batch][d_model] out, 16-byte aligned
 * heisd_feature_similarity: S[i][j] = cosine(a[i], b[j]) (0 if a vector is all zero).
 *     a DEVICE f32 [n][d], b DEVICE f32 [m][d], S DEVICE f32 [n][m] out; d a multiple of 4, 16-byte aligned
 * heisd_skip_offline: offline stage of Alg. 1 over n trajectory points: the smallest S(feat[i], feat[i+dd])
 *   that exceeds T, and its distance dd; among equal similarities the pair found first with i ascending,
 *   then dd ascending.  No pair above T: min_s = +inf, o_dist = 0 (never skip).
 *     S     DEVICE f32 [n][n] out, optional (the whole similarity matrix)
 *     work  DEVICE, 8 bytes, 8-byte aligned (scratch);  min_s DEVICE f32 [1] out;  o_dist DEVICE i32 [1] out
 * heisd_skip_decide: skip_mask[b] = 1 iff dist[b] <= *o_dist and cosine(feat_prev[b], feat_last[b]) >= *min_s,
 *   where feat_last is the feature of the episode's last VERIFIED trajectory point, feat_prev that of the
 *   verified point before it, and dist[b] how many points the current one lies after the last verified
 *   one (features exist only for verified points, so the rule looks back).
 *     feat_prev, feat_last DEVICE f32 [batch][d]; dist DEVICE i32 [batch]; min_s, o_dist DEVICE scalars;
 *     skip_mask DEVICE u8 [batch] out; similarity DEVICE f32 [batch] out, optional
 * The adaptive update of min_S / O_dist from task feedback (online stage) is scalar host logic and not
 * part of this library.
 * Errors: EINVAL (NULL / misaligned pointers, sizes out of range: at most 65535 points), EHIP.
 */
int heisd_export_features(heisd_verify_ctx *ctx, const int32_t *row, int32_t rows_per_episode, int32_t batch,
                          float *feat, void *stream);
int heisd_feature_similarity(const float *a, const float *b, int32_t n, int32_t m, int32_t d, float *S, void *stream);
int heisd_skip_offline(const float *feat, int32_t n, int32_t d, float T, float *S, uint64_t *work, float *min_s,
                       int32_t *o_dist, void *stream);
int heisd_skip_decide(const float *feat_prev, const float *feat_last, const int32_t *dist, int32_t batch, int32_t d,
                      const float *min_s, const int32_t *o_dist, uint8_t *skip_mask, float *similarity, void *stream);

/*
 * The retrieval branch's search (App. C: C.1 database construction, C.2 performance; Sec. 4.2: Top-K
 * instead of Top-1): every stored timestep is an L2-normalised embedding (4352-dim in the paper) with a payload (the action tokens that followed); a query
 * embedding retrieves the K entries of highest cosine similarity, whose payloads become the draft
 * candidates (heisd_build_sequence_tree takes them).  The paper searches an HNSW graph on the CPU
 * (approximate); this call is the exact search, as one scan of the database in HBM.
 *
 *   db           DEVICE bf16 [n_vectors][d], row-major, rows L2-normalised by the caller (the similarity
 *                is the plain dot product of the stored values with the query)
 *   queries      DEVICE f32 [batch][d], 16-byte aligned
 *   K            1 .. 64
 *   payload      DEVICE i32 [n_vectors][payload_len], optional (then top_payload must be given too)
 *   top_index    DEVICE i32 [batch][K] out   higher similarity first, equal similarities by lower index;
 *                                            -1 past the end when n_vectors < K
 *   top_score    DEVICE f32 [batch][K] out   (-inf where top_index is -1)
 *   top_payload  DEVICE i32 [batch][K][payload_len] out, optional
 *   workspace    DEVICE, 256-byte aligned, at least heisd_retrieve_workspace_bytes(n_vectors, batch, K):
 *                all scores of every query, and the first selection round's winners
 * Asynchronous on `stream`, allocates nothing.  d a multiple of 4, at most 8192; n_vectors < 2^31;
 * batch at most 1024 (the database is streamed once per four queries).
 * Errors: EINVAL, ENOMEM (workspace too small), EHIP.
 */
size_t heisd_retrieve_workspace_bytes(int64_t n_vectors, int32_t batch, int32_t K);
int heisd_retrieve_topk(const void *db, int64_t n_vectors, int32_t d, const float *queries, int32_t batch, int32_t K,
                        const int32_t *payload, int32_t payload_len, int32_t *top_index, float *top_score,
                        int32_t *top_payload, void *workspace, size_t workspace_bytes, void *stream);

/*
 * heisd_retrieve_topk for callers that cannot allocate device memory and have no workspace to hand over:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * kernels and results, but the scores and the first selection round's winners live in a static array
 * inside the library, heisd_retrieve_static_bytes() = 8 MiB per GPU (every GPU the library runs on
 * holds its own copy until the process ends).  The call allocates and frees nothing.  A search that
 * needs more scratch than that - heisd_retrieve_workspace_bytes(n_vectors, batch, K) is the amount; the
 * paper-sized database fits with up to 7 queries - fails with ENOMEM and enqueues nothing: use
 * heisd_retrieve_topk then.
 * All calls on one GPU share that GPU's array: two calls that may overlap in time (different streams,
 * different host threads) race and both results are undefined; calls on one stream are safe.  Nothing
 * in the array has to start cleared: every call writes what it reads.  The first call on a device
 * looks up the array's address and the device's properties (no allocation); make it outside graph
 * capture.
 * Errors: EINVAL, ENOMEM (search larger than the static array), EHIP.
 */
size_t heisd_retrieve_static_bytes(void);
int heisd_retrieve_topk_static(const void *db, int64_t n_vectors, int32_t d, const float *queries, int32_t batch,
                               int32_t K, const int32_t *payload, int32_t payload_len, int32_t *top_index,
                               float *top_score, int32_t *top_payload, void *stream);

/*
 * Per-kernel timing for measurement runs (not part of the method).  With profiling enabled,
 * heisd_verify_step brackets every kernel launch with HIP events on the caller's stream;
 * heisd_verify_profile_read waits for the recorded events, adds the elapsed milliseconds
 * of each kernel class to ms[class] and the number of launches to launches[class] (HOST
 * arrays of HEISD_N_KERNEL_CLASSES entries, overwritten), and clears the record.
 * Enabling creates events (host objects); disabling destroys them.  At most
 * HEISD_PROFILE_MAX_STEPS steps are kept between two reads; later steps are not recorded.
 */
#define HEISD_N_KERNEL_CLASSES 9
#define HEISD_KC_EMBED 0
#define HEISD_KC_QKV 1      /* RMSNorm + QKV projection                 */
#define HEISD_KC_ATTN 2     /* RoPE + KV-append + verify attention      */
#define HEISD_KC_OPROJ 3    /* output projection + residual             */
#define HEISD_KC_GATEUP 4   /* RMSNorm + gate/up projection + SwiGLU    */
#define HEISD_KC_DOWN 5     /* down projection + residual               */
#define HEISD_KC_LMHEAD 6   /* final RMSNorm + 256-bin LM-head slice    */
#define HEISD_KC_ACCEPT 7   /* argmax + relaxed acceptance scan         */
#define HEISD_KC_PERSIST 8  /* whole decoder forward in one persistent kernel (embedding .. LM-head slice) */
#define HEISD_PROFILE_MAX_STEPS 64
int heisd_verify_profile_enable(heisd_verify_ctx *ctx, int enable);
int heisd_verify_profile_read(heisd_verify_ctx *ctx, double *ms, int64_t *launches);

/*
 * Kernel-path selection, for tests and measurement.  AUTO (default) picks the fastest path
 * that covers the call.  For batch*K <= 8 (when the model fits those kernels: d_model <= 4096) that
 * is PERSIST - if it fits the device, the model is large enough for it to pay (80 MB of projection
 * weights per layer or more; 320 MB if the context got no slot of uncached barrier flags), the stream is not being captured into a graph, and the last
 * persistent kernel launched through this library on the device went to the same stream or has
 * finished (two of them started together from two streams could each hold half of the compute units
 * and wait for the other half) - and FAST otherwise; for more rows it is BATCH.  GENERIC forces the first any-M path
 * (activations converted and staged through LDS by every workgroup, one launch per phase);
 * BATCH forces the any-M path that exchanges pre-split bf16 activation records (waves arranged
 * over rows and over the reduction according to batch*K); FAST forces the batch*K <= 8 kernels
 * with one launch per phase; PERSIST forces the batch*K <= 8 persistent kernel (the whole decoder
 * forward and the acceptance scan in one launch, one workgroup per compute unit, grid barriers inside)
 * without the test AUTO makes: the caller then sees to it that no two persistent kernels run at once.
 * FAST and PERSIST make a larger step fail with EUNSUPPORTED.  Results of the paths agree to fp32
 * rounding (FAST and PERSIST bit for bit).
 *
 * The persistent kernel spins at its grid barriers with a bound; if the bound expires (the
 * GPU was shared with work that kept some of its workgroups from running) it raises a bit of the
 * context's device error word and ends; its outputs are then undefined.  The path for more than 8 rows has
 * one bounded wait of the same kind: the epilogues of a projection of a normalised input take each row's
 * 1/rms from a word the first workgroups of the same launch compute, and a word that never arrives raises
 * the same bit (the row's outputs are then zero).  An episode whose new rows did
 * not fit its cache raises another bit (see heisd_kv_desc).  heisd_verify_check synchronises the
 * device, clears the word and returns EHIP for an expired wait, EINVAL for an episode that did
 * not fit, else OK (heisd_last_error says which).
 */
#define HEISD_PATH_AUTO 0
#define HEISD_PATH_GENERIC 1
#define HEISD_PATH_FAST 2
#define HEISD_PATH_PERSIST 3
#define HEISD_PATH_BATCH 4
int heisd_verify_check(heisd_verify_ctx *ctx);
int heisd_verify_set_path(heisd_verify_ctx *ctx, int path);

/*
 * How activations enter the matrix cores on the path for more than 8 rows (paper Sec. 5.1 runs its models in
 * bf16; Eq. 2-2 is the forward this affects).  HEISD_ACT_SPLIT (default): every fp32 activation is a bf16 head
 * plus a bf16 tail (about 16 mantissa bits), two matrix-core operands.  HEISD_ACT_BF16: one bf16 (round to
 * nearest even), half the matrix-core work; used by steps, tree steps and prefill chunks of 33 rows or more
 * (smaller ones keep the split form), everything else - residual stream, softmax, accumulators, the
 * acceptance rule - unchanged.  Logits then differ from the fp32-activation result by about 1e-2 of a row's
 * range instead of 3e-5.  Takes effect with the next call.  Errors: EINVAL (NULL ctx, unknown format).
 */
#define HEISD_ACT_SPLIT 0
#define HEISD_ACT_BF16 1
int heisd_verify_set_activations(heisd_verify_ctx *ctx, int format);

/*
 * Footprint (App. A.1: the 7B target model is 13 GB of projection weights).  heisd_verify_init copies the
 * seven projection matrices of every layer (wq, wk, wv, wo, w_gate, w_up, w_down) and the n_bins LM-head rows
 * into the workspace in the order the matrix cores consume them; after that only HEISD_PATH_GENERIC reads the
 * caller's originals.  A caller that keeps both holds the model twice.  This call records the caller's promise
 * that it will not select HEISD_PATH_GENERIC again: from then on the library never dereferences those eight
 * pointers, the caller may free that memory (tok_emb, attn_norm, ffn_norm and final_norm are still read in place
 * and must stay alive), and heisd_verify_set_path(ctx, HEISD_PATH_GENERIC) fails with EUNSUPPORTED.  Not
 * reversible for this context.  Host-side only; enqueues nothing.
 * Errors: EINVAL (NULL ctx), EUNSUPPORTED (HEISD_PATH_GENERIC is the selected path).
 */
int heisd_verify_release_projections(heisd_verify_ctx *ctx);

/*
 * Measurement aid for the persistent kernel (not part of the method): with enable != 0 every later
 * persistent step records device timestamps (100 MHz counter) of every workgroup in every phase of its
 * program, as [phase][workgroup][8]: [0] phase entered, [1] inputs seen (grid barrier passed),
 * [2] weights consumed, [3] outputs published, [4] and [5] epilogue begun and ended (GEMM phases),
 * [6] the barrier's polls have seen every flag ([1] minus [6] is the wait for weights handed over in LDS);
 * slot 7 is unused, and a slot a workgroup does not pass in a phase reads 0 (switching recording on
 * synchronises the device and clears the record).  One workgroup runs per compute unit.  With out != NULL (HOST array of
 * max_entries values) the call synchronises the device, copies the record of the last persistent step
 * and returns the number of values copied (phases * workgroups * 8 at most); otherwise it returns OK.
 * Errors: EINVAL (NULL ctx), EHIP.
 */
int heisd_debug_trace(heisd_verify_ctx *ctx, int enable, unsigned long long *out, int max_entries);

/*
 * Test aid: the bounds of the waits inside the kernels (see heisd_verify_check), so that a test can make them
 * give up while every kernel still runs to its end.  grid_polls: polls a workgroup of the persistent kernel makes at
 * a grid barrier before it raises the error word and leaves (<= 0: the default, about 4 million); scale_polls: polls an
 * epilogue of the path for more than 8 rows makes for a row's 1/rms word (<= 0: the default, about 1 million);
 * skip_scales != 0: those launches do not produce the words at all, so every such epilogue gives up.  After a step
 * that gave up, heisd_verify_check returns EHIP and the step's outputs are undefined; with the defaults restored the
 * next step is unaffected.  Host-side only.  Errors: EINVAL (NULL ctx).
 */
int heisd_debug_set_wait_limits(heisd_verify_ctx *ctx, int grid_polls, int scale_polls, int skip_scales);

/*
 * Measurement aid for the persistent kernel: what a phase requests across the grid barrier that ends it.
 *   0 (default)  the whole first weight tile of the next GEMM phase (16 k-steps of every wave: 128 KB per
 *                workgroup) is handed over through LDS, started as soon as the phase's own stores have been
 *                acknowledged (the O-projection's at the end of the attention phase); nothing else is
 *                requested before the wait
 *   1            as 0, but the O-projection's hand-over starts at the end of the QKV phase
 *   2            no LDS hand-over: the whole first tile is requested into registers before the wait
 *   3            nothing is requested before the wait
 *   4            as 0, and the second weight tile is requested into registers before the wait
 *   5            as 0, with the QKV tiles dealt to the workgroups in their plain order (in mode 0, at d_model
 *                4096 / head_dim 128 on a 256-unit device, a head's q, k and v rows are produced on the XCD
 *                whose workgroups run that head's attention units)
 * Synchronises the device and rewrites the phase program.  Results are identical in every mode.
 * Errors: EINVAL (NULL ctx, unknown mode), EUNSUPPORTED (no persistent kernel for this context), EHIP.
 */
int heisd_verify_set_handover(heisd_verify_ctx *ctx, int mode);

/*
 * Reference measurements behind the roofline accounting (not part of the method): one launch of a kernel
 * that only reads `bytes` of device memory, in the access pattern of the weight-streaming GEMMs, and an
 * empty launch.  The caller times them (events, or rocprofv3 around the process).
 *   pattern 0   every wave reads one contiguous span (bytes / waves), `in_flight` KB per wave requested ahead
 *   pattern 1   the fragment-ordered weight copy as the <= 8-row GEMMs walk it: tiles of `ksteps` KB
 *               (ksteps = reduction length / 32), dealt round-robin to the workgroups, the 8 waves of a
 *               workgroup an eighth of a tile's k-steps each, `in_flight` KB per wave requested ahead
 *   in_flight   8 or 16;  workgroups: grid size (512 threads each; 256 = one per compute unit)
 *   sink        DEVICE u32 [1], never written in practice (keeps the loads alive)
 * Asynchronous on `stream`, allocates nothing.  Errors: EINVAL, EHIP.
 */
int heisd_measure_read(const void *buf, size_t bytes, int32_t pattern, int32_t ksteps, int32_t in_flight,
                       int32_t workgroups, uint32_t *sink, void *stream);
int heisd_measure_empty_launch(int32_t workgroups, void *stream);

/* Release the context (not the workspace, weights or caches: those are the caller's). NULL ok. */
void heisd_free(heisd_verify_ctx *ctx);

/* HOST string describing the last error of this context ("" if none); for ctx == NULL, the
 * last error of a failed heisd_verify_init on this thread. */
const char *heisd_last_error(const heisd_verify_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* HEISD_VERIFY_H */
