/*
 * lkv.h -- C ABI of the MI355X (gfx950) implementation of LKV's inference-time
 * KV-cache eviction path: token scoring, head-wise budgeted top-k, compaction
 * into a padding-free ragged cache, and GQA decode attention over that cache
 * (lkv_score, lkv_select, lkv_compact, lkv_decode_attn); further down, the same
 * path one layer at a time during prefill, the growth of the packed cache
 * during decoding with re-eviction, attention with a multiplicative mask over
 * the uncompacted cache, the training-time attention kernel with that mask
 * (forward and backward), the LKV-H budget allocation with the forward
 * Soft-TopK operator and its backward pass, and the observation-window scorer that the paper's
 * ablation runs under the same budgets (lkv_score_window).
 *
 * General conventions
 * -------------------
 * Memory.   Every pointer is marked HOST or DEVICE.  All device buffers are
 *           allocated, owned and freed by the caller; no call allocates device
 *           memory.  The context owns only a
 *           small ring of pinned host staging buffers.  Device pointers must be
 *           16-byte aligned.
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = the default
 *           stream).  The hot calls only enqueue work on it; they do not
 *           synchronise the host with the device and results are valid once the
 *           caller has synchronised the stream.  Calls that only enqueue kernels
 *           can be recorded into a HIP graph.  The one exception is an upload
 *           of segment offsets computed from HOST budgets: lkv_plan_offsets,
 *           lkv_reevict, and lkv_select when it is given host budgets for 640
 *           or more segments (fewer travel in the kernel arguments).  Such an
 *           upload goes through a ring of 8 pinned buffers owned by the
 *           context, may wait on the host until the ring slot's previous
 *           upload has finished, and is refused with LKV_ERR_UNSUPPORTED while
 *           `stream` is capturing (a replay would copy whatever a later call
 *           left in the slot).  To stay free of both, call lkv_plan_offsets
 *           once, outside any capture, and pass budgets = NULL to lkv_select.
 * Layout.   Cache tensors are bf16, row-major [n_layers, n_kv_heads, T, 128]
 *           per sequence.  A "segment" is one (sequence, layer, kv head); the
 *           segments are numbered s = (seq * n_layers + layer) * n_kv_heads +
 *           head.  Within a segment kept tokens are in ascending token order.
 * Errors.   Every call returns an lkv_status and never throws.  All argument
 *           checks happen on the host before anything is launched; on failure
 *           nothing has been enqueued and lkv_last_error() describes the cause.
 *           LKV_ERR_HIP reports a failed HIP runtime call.
 * Threads.  A context must not be used from two host threads at once.
 */
#ifndef LKV_H_
#define LKV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lkv_ctx lkv_ctx;

typedef enum {
  LKV_OK = 0,
  LKV_ERR_INVALID_ARG = 1, /* null / misaligned pointer, inconsistent sizes, budget outside [0, T] */
  LKV_ERR_UNSUPPORTED = 2, /* head_dim != 128, hidden not a multiple of 16 in [16, 128], group > 16 */
  LKV_ERR_WORKSPACE = 3,   /* workspace missing or smaller than the *_workspace_bytes() figure */
  LKV_ERR_HIP = 4          /* a HIP runtime call failed */
} lkv_status;

typedef enum { LKV_SCORER_LINEAR = 0, LKV_SCORER_MLP = 1 } lkv_scorer_kind;
typedef enum { LKV_ACT_SILU = 0, LKV_ACT_GELU_ERF = 1 } lkv_act;
typedef enum { LKV_POOL_MAX = 0, LKV_POOL_AVG = 1 } lkv_pool;

/* Geometry of a prefilled KV cache (Sec. 3.1 of the paper: per layer and KV
 * head, K and V are t x d matrices).  The struct and the arrays it points to
 * are HOST memory and are read during the call only. */
typedef struct {
  int32_t n_seq;            /* number of sequences (>= 1) */
  int32_t n_layers;         /* L */
  int32_t n_kv_heads;       /* H */
  int32_t n_q_heads;        /* Hq, a multiple of H; query head hq reads KV head hq / (Hq / H) */
  int32_t head_dim;         /* d, must be 128 */
  const int32_t *seq_len;   /* HOST [n_seq]: T_s >= 1 */
  const void *const *k;     /* HOST [n_seq] of DEVICE pointers: bf16 [L, H, T_s, d] */
  const void *const *v;     /* HOST [n_seq] of DEVICE pointers: bf16 [L, H, T_s, d] */
} lkv_cache;

/* Parameters of the LKV-T token scorer (Sec. 3.4: u_i = MLP([k_i ; v_i]); the
 * input is the 256-vector made of the key row followed by the value row).
 * LINEAR : u = w1 . x + b1
 * MLP    : u = w2 . act(W1 x + b1) (+ b2); Table 5 of the paper uses
 *          256 -> 128 -> 1 with SiLU, a hidden bias and no output bias.
 * The struct is HOST memory; the arrays are DEVICE memory, caller-owned.
 * Hs = n_kv_heads when per_head != 0 (one scorer per head, as in the paper),
 * Hs = 1 otherwise (one scorer per layer shared by its heads). */
typedef struct {
  int32_t kind;      /* lkv_scorer_kind */
  int32_t act;       /* lkv_act, MLP only */
  int32_t hidden;    /* MLP only: multiple of 16 in [16, 128] */
  int32_t per_head;  /* 0 or 1 */
  const void *w1;    /* DEVICE bf16. LINEAR [L, Hs, 256]; MLP [L, Hs, hidden, 256] (one row per hidden unit) */
  const float *b1;   /* DEVICE fp32. LINEAR [L, Hs] (scalar bias); MLP [L, Hs, hidden] */
  const float *w2;   /* DEVICE fp32. MLP [L, Hs, hidden]; LINEAR: ignored */
  const float *b2;   /* DEVICE fp32. MLP [L, Hs], or NULL for no output bias; LINEAR: ignored */
} lkv_scorer;

/* Create / destroy a context bound to HIP device `device`.  lkv_create selects
 * that device for the calling thread. */
lkv_status lkv_create(lkv_ctx **out, int device);
void lkv_destroy(lkv_ctx *ctx);

/* Text of the last error recorded on `ctx` (valid until the next call on it). */
const char *lkv_last_error(const lkv_ctx *ctx);

/* Library version string. */
const char *lkv_version(void);

/* Token scoring (Sec. 3.4, "Head-Specific Intrinsic Scoring").
 * For every sequence s, layer l, head h and token i writes
 *   scores[s][(l*H + h)*T_s + i] = f_{l,h}([K[l,h,i,:] ; V[l,h,i,:]])
 * as fp32.  bf16 inputs, fp32 accumulation.  Each K/V row is read once.
 * scores : HOST [n_seq] of DEVICE pointers, each fp32 [L, H, T_s]. */
lkv_status lkv_score(lkv_ctx *ctx, const lkv_cache *cache, const lkv_scorer *scorer,
                     float *const *scores, void *stream);

/* Observation-window token scoring: the attention-based selection policy that
 * the ablation of Sec. 4.4 combines with the LKV-H budgets (complexity O(W T)
 * in the table of Sec. 4.5).  The paper names the policy and cites its
 * publication for the rule; the rule as implemented here, every parameter an
 * argument:
 *   the window is the last W = `window` positions of the prompt; its query row
 *   i stands at position T - W + i and sees keys 0 .. T - W + i;
 *   a[hq, i, :] = softmax over those keys of scale * q_win[l, hq, i, :] . K[l, h, j, :],
 *                 h = hq / (Hq / H);
 *   vote[l, h, j] = mean over the query heads of h's group of sum_i a[hq, i, j],
 *                 for the prefix tokens j < T - W;
 *   scores[l, h, j] = centred pooling of vote[l, h, :] of width `pool_width`
 *                 (stride 1, same length): LKV_POOL_MAX takes the largest vote
 *                 in the part of [j - c, j + c] inside the prefix, LKV_POOL_AVG
 *                 the sum over that part divided by pool_width, c = (pool_width - 1) / 2;
 *   scores[l, h, j] = +inf for the window tokens j >= T - W,
 * so that lkv_select with a budget b >= W keeps the window and the b - W prefix
 * tokens with the largest pooled votes.  bf16 inputs, fp32 accumulation and
 * fp32 softmax; each key row is read twice (once for the normalisers, once
 * for the weights), once if the caller supplies the normalisers; cache->v is not read and may be NULL.  Results are reproducible bit for bit
 * for the same call; the keys are split into blocks by the size of the whole call, so a layer
 * scored alone and the same layer scored inside a whole-cache call can differ in the last bits
 * (the order of the fp32 sums), never in more.
 * q_win     : HOST [n_seq] of DEVICE pointers, bf16 [L, Hq, W, 128]: the queries
 *             of the last W positions (as they met the keys in prefill, i.e.
 *             position-encoded like the cached keys)
 * lse_win   : NULL, or HOST [n_seq] of DEVICE pointers, fp32 [L, Hq, W]: the natural-log normalisers
 *             log sum_{j <= T - W + i} exp(scale * q . k_j) of the window rows, which the prefill's
 *             attention kernel has already computed for these queries.  With them the keys are
 *             read once instead of twice (the normaliser pass is skipped); the scores are then as
 *             accurate as the normalisers given.
 * window    : 1 <= W <= every T_s, and (Hq / H) * W <= 128 (else LKV_ERR_UNSUPPORTED)
 * pool_width: odd, 1 .. 63 (1 = no pooling); pool_kind: lkv_pool
 * scale     : positive, finite (1 / sqrt(d) in Eq. 1)
 * scores    : HOST [n_seq] of DEVICE pointers, each fp32 [L, H, T_s]
 * workspace : DEVICE, 256-byte aligned, at least lkv_score_window_workspace_bytes(cache)
 *             bytes (per-block normaliser pairs, about 8 bytes per cached key
 *             row and head); contents are scratch. */
size_t lkv_score_window_workspace_bytes(const lkv_cache *cache);
lkv_status lkv_score_window(lkv_ctx *ctx, const lkv_cache *cache, const void *const *q_win,
                            const float *const *lse_win, int32_t window, int32_t pool_width, int32_t pool_kind,
                            float scale, float *const *scores, void *workspace, size_t workspace_bytes,
                            void *stream);

/* Head-wise budgeted hard top-k (Sec. 3.4, inference: m = TopK(u, b); budgets
 * b = floor(r t) come from LKV-H, Sec. 3.3, and are an input here).
 * For segment s keeps the budgets[s] tokens with the largest score; equal
 * scores are resolved towards the lower token index; a NaN score ranks as
 * -inf; scores are compared by the total order of their fp32 bit patterns
 * (-0.0 below +0.0).  Writes
 *   offsets[s]              = sum of budgets of the segments before s (s = 0..n_segments),
 *   idx[offsets[s] + j]     = j-th kept token of segment s, ascending.
 * The result is unique, hence reproducible bit for bit.
 * scores  : HOST [n_seq] of DEVICE pointers, fp32 [L, H, T_s] (as written by lkv_score)
 * budgets : HOST int32 [n_seq * L * H], 0 <= budgets[s] <= T_seq(s); sum < 2^31.
 *           Or NULL: `offsets` already holds the prefix sums that lkv_plan_offsets
 *           wrote for the budgets (budgets are static, Sec. 3.3, so this is done once);
 *           it is then an input, nothing is copied and the host never waits, whatever
 *           the number of segments.  The budgets cannot be checked in that case: a
 *           planned budget above T_seq(s) keeps all T_seq(s) tokens and leaves the rest
 *           of that segment's idx range unwritten.
 * idx     : DEVICE int32 [sum of budgets]
 * offsets : DEVICE int32 [n_seq * L * H + 1]; written, or read when budgets is NULL */
lkv_status lkv_select(lkv_ctx *ctx, const lkv_cache *cache, const float *const *scores,
                      const int32_t *budgets, int32_t *idx, int32_t *offsets, void *stream);

/* ---- Scoring that counts for the top-k -------------------------------------------------------
 * The top-k finds its threshold by a radix descent over the score bits; the first level looks at
 * the top 11 bits of every score.  lkv_score_counted writes the same scores as lkv_score and, on
 * the way, counts those 11-bit digits per segment (inside the scoring kernel for the MLP scorers;
 * by one extra pass over the scores, 4 bytes per token, for the linear scorer).
 * lkv_select_counted then starts from the counts instead of from a pass over the scores: heads too
 * long for the top-k's on-chip key cache (more than 34304 tokens) are read twice instead of three
 * times, shorter ones skip the counting.  Same result as lkv_select, bit for bit.
 * counts : DEVICE uint32 [n_seq * L * H, 2048], 16-byte aligned, lkv_counts_bytes(n_segments) bytes.
 *          Must be all zero when lkv_score_counted is called; lkv_select_counted reads every
 *          segment's counters and leaves them zero again, so a buffer cleared once with
 *          lkv_clear_counts serves any number of score / select pairs.  The two calls must see the
 *          same cache geometry and the scores must not change in between. */
size_t lkv_counts_bytes(int64_t n_segments);
/* The same plus room for two bitmaps of max_seq_len bits per segment behind the counters (no need to clear them).
 * Given a buffer of this size, lkv_evict_layer splits the top-k pass over the scores of every head over several
 * workgroups when a call covers few heads that are too long for the on-chip key cache (one layer of a
 * 65536-token or longer prompt: 8 heads would otherwise keep 8 compute units busy). */
size_t lkv_counts_bytes_split(int64_t n_segments, int32_t max_seq_len);
lkv_status lkv_clear_counts(lkv_ctx *ctx, uint32_t *counts, int64_t n_segments, void *stream);
lkv_status lkv_score_counted(lkv_ctx *ctx, const lkv_cache *cache, const lkv_scorer *scorer,
                             float *const *scores, uint32_t *counts, void *stream);
lkv_status lkv_select_counted(lkv_ctx *ctx, const lkv_cache *cache, const float *const *scores,
                              const int32_t *budgets, uint32_t *counts, int32_t *idx, int32_t *offsets,
                              void *stream);

/* Compaction into the padding-free ragged cache (Sec. 4.5: the compressed
 * cache is flattened so that no padding is stored).
 *   kp[offsets[s] + j, :] = K[seq, l, h, idx[offsets[s] + j], :]   (same for vp / V)
 * Rows are copied bit for bit.
 * idx, offsets : DEVICE, as written by lkv_select
 * total_kept   : sum of the budgets (HOST scalar; equals offsets[n_segments])
 * kp, vp       : DEVICE bf16 [total_kept, d] */
lkv_status lkv_compact(lkv_ctx *ctx, const lkv_cache *cache, const int32_t *idx,
                       const int32_t *offsets, int64_t total_kept, void *kp, void *vp,
                       void *stream);

/* Bytes of DEVICE workspace lkv_decode_attn needs for this problem size. */
size_t lkv_decode_workspace_bytes(int32_t n_segments, int64_t total_kept, int32_t n_q_heads,
                                  int32_t n_kv_heads);

/* One decode step of grouped-query attention over the ragged cache (Eq. 1 of
 * the paper restricted to the kept tokens; the retention mask is per KV head,
 * so all query heads of a group read the same segment, Sec. 3.1).
 * For query row r = (seq*L + l)*Hq + hq, segment s = (seq*L + l)*H + hq/(Hq/H):
 *   p_j = softmax_j(scale * q[r,:] . kp[offsets[s] + j, :]),  out[r,:] = sum_j p_j vp[offsets[s] + j, :]
 *   lse[r] = log sum_j exp(scale * q . k_j)
 * An empty segment gives out = 0 and lse = -inf.  bf16 inputs, fp32 softmax
 * and accumulation, fp32 output.
 * q        : DEVICE bf16 [n_seq, L, Hq, d]
 * kp, vp   : DEVICE bf16 [total_kept, d]
 * offsets  : DEVICE int32 [n_seq*L*H + 1]
 * out      : DEVICE fp32 [n_seq, L, Hq, d]
 * lse      : DEVICE fp32 [n_seq, L, Hq], or NULL
 * workspace: DEVICE, at least lkv_decode_workspace_bytes(...) bytes, 256-byte aligned;
 *            contents are scratch and need not be initialised. */
lkv_status lkv_decode_attn(lkv_ctx *ctx, int32_t n_seq, int32_t n_layers, int32_t n_kv_heads,
                           int32_t n_q_heads, int32_t head_dim, const void *q, const void *kp,
                           const void *vp, const int32_t *offsets, int64_t total_kept,
                           float scale, float *out, float *lse, void *workspace,
                           size_t workspace_bytes, void *stream);

/* lkv_decode_attn for callers that cannot allocate device memory or carry a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results; the split-K partials go to a fixed array of
 * LKV_DECODE_STATIC_SCRATCH_BYTES in the library's device image instead of a caller-owned workspace
 * (each GPU the library is used on holds that array until the process ends).  The call allocates
 * nothing and frees nothing.  A problem whose lkv_decode_workspace_bytes(...) exceeds the array is
 * refused with LKV_ERR_WORKSPACE before anything is enqueued (the five benchmark workloads need 1.6
 * to 9.6 MB).  All calls on one GPU share the array, from whatever context or stream: two of them
 * that overlap in time race on it, so order them on one stream or with events.  The array keeps the
 * last call's partials; nothing needs clearing, because every slot that a call reads it has
 * written first. */
#define LKV_DECODE_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
lkv_status lkv_decode_attn_static(lkv_ctx *ctx, int32_t n_seq, int32_t n_layers, int32_t n_kv_heads,
                                  int32_t n_q_heads, int32_t head_dim, const void *q, const void *kp,
                                  const void *vp, const int32_t *offsets, int64_t total_kept,
                                  float scale, float *out, float *lse, void *stream);

/* ---- Layer-by-layer eviction during prefill (Sec. 1: each layer's cache is evicted as soon as
 * the prefill has produced it, so the full cache of all layers never exists) ---------------- */

/* The packed layout follows from the budgets alone (they are static, Sec. 3.3), so it can be
 * fixed before any layer exists: offsets[s] = sum of the budgets of the segments before s.
 * budgets    : HOST int32 [n_segments], each >= 0, sum < 2^31
 * offsets    : DEVICE int32 [n_segments + 1]
 * total_kept : HOST out, may be NULL
 * The upload is asynchronous on `stream` (pinned staging owned by the context). */
lkv_status lkv_plan_offsets(lkv_ctx *ctx, int64_t n_segments, const int32_t *budgets, int32_t *offsets,
                            int64_t *total_kept, void *stream);

/* Score, select and compact ONE layer (or a few consecutive ones) into its final rows of the packed cache;
 * the result is bit for bit what lkv_score + lkv_select + lkv_compact over the whole cache write for it.
 * All work is enqueued on `stream`, so it can overlap the prefill of the next layer on another
 * stream; the layer's K/V may be released once the stream has passed this call.
 * layer       : a cache description whose k[s], v[s] point at bf16 [m, H, T_s, d] of m = layer->n_layers
 *               consecutive layers starting at layer_index (m = 1: one layer at a time, the lowest peak
 *               memory; a larger m trades live layer buffers for fewer dependent launches per layer);
 *               at most 32 sequences
 * layer_index : which layer of the model the view starts at; layer_index + m <= n_layers
 * scorer      : the whole model's scorer (parameters of all layers), as for lkv_score; or NULL:
 *               `scores` already holds the view's scores (from any scorer, for example
 *               lkv_score_window on the same view) and only the top-k and the compaction run
 * budgets     : HOST int32 [n_seq, n_layers, H], the same table lkv_plan_offsets was given
 * offsets     : DEVICE int32 [n_seq * n_layers * H + 1] written by lkv_plan_offsets
 * scores      : HOST [n_seq] of DEVICE fp32 [m, H, T_s]: scratch, overwritten (an input when scorer is NULL)
 * idx         : DEVICE int32 [total_kept], the global index buffer (the view's part is written)
 * kp, vp      : DEVICE bf16 [total_kept, d], the global packed cache (the view's rows are written)
 * counts      : NULL, or DEVICE uint32 [n_seq * n_layers * H, 2048] as for lkv_score_counted (all zero
 *               on entry, left zero): the scoring then counts for the top-k.  Ignored when scorer is NULL.
 *               Calls that run at the same time on different streams touch different segments'
 *               counters, so they can share the buffer.
 * counts_bytes: size of that buffer: lkv_counts_bytes(n_segments), or lkv_counts_bytes_split(n_segments,
 *               longest sequence) to let the call split long heads over several workgroups; smaller:
 *               LKV_ERR_WORKSPACE */
lkv_status lkv_evict_layer(lkv_ctx *ctx, const lkv_cache *layer, int32_t layer_index, int32_t n_layers,
                           const lkv_scorer *scorer, const int32_t *budgets, const int32_t *offsets,
                           float *const *scores, int32_t *idx, void *kp, void *vp, uint32_t *counts,
                           size_t counts_bytes, void *stream);

/* ---- Decode-time growth of the packed cache -----------------------------------------------
 * The paper evicts during prefill (Sec. 1), lets step t attend every cached token up to t (Eq. 1)
 * and sets the budget of a head at step t to floor(r t) (Sec. 3.3), but does not say how the
 * compacted cache follows t.  The layout used here: every segment s owns the rows
 * cap_offsets[s] .. cap_offsets[s+1] of kp / vp / up, of which the first lengths[s] are in use;
 * `slack` spare rows per segment take the tokens generated after prefill, one per decode step.
 * When the slack is used up the caller re-evicts (lkv_reevict) with the budgets of the new
 * length.  `up` holds the LKV-T score of every row in use. */

/* lkv_compact into a cache with `slack` spare rows behind every segment.
 * Row j of segment s goes to row offsets[s] + slack * s + j; the score of that token goes to up.
 * Also writes cap_offsets[s] = offsets[s] + slack * s (s = 0..n_segments) and lengths[s] = budget.
 * scores      : HOST [n_seq] of DEVICE fp32 [L, H, T_s], the scores the selection used
 * idx, offsets: DEVICE, as written by lkv_select
 * kp, vp      : DEVICE bf16 [total_kept + n_segments * slack, d]
 * up          : DEVICE fp32 [total_kept + n_segments * slack]
 * cap_offsets : DEVICE int32 [n_segments + 1];  lengths : DEVICE int32 [n_segments]
 * Spare rows are left as they are (never read). */
lkv_status lkv_compact_grow(lkv_ctx *ctx, const lkv_cache *cache, const float *const *scores,
                            const int32_t *idx, const int32_t *offsets, int64_t total_kept, int32_t slack,
                            void *kp, void *vp, float *up, int32_t *cap_offsets, int32_t *lengths,
                            void *stream);

/* One generated token: its key, value and LKV-T score (Sec. 3.4, computed here from the token's
 * own key and value with the given scorer) are written to the first spare row of every segment
 * and lengths[s] grows by one.  A segment without a spare row is left untouched and *overflow is
 * set to 1 (the caller keeps count of the appends since the last eviction and re-evicts in time;
 * the flag is the safety net).
 * k_new, v_new : DEVICE bf16 [n_seq, L, H, d]
 * scorer       : as for lkv_score; the MLP hidden width may be any value in [1, 128] here
 * overflow     : DEVICE int32 [1] or NULL; never cleared by this call */
lkv_status lkv_append(lkv_ctx *ctx, int32_t n_seq, int32_t n_layers, int32_t n_kv_heads, int32_t head_dim,
                      const lkv_scorer *scorer, const void *k_new, const void *v_new, void *kp, void *vp,
                      float *up, const int32_t *cap_offsets, int32_t *lengths, int32_t *overflow,
                      void *stream);

/* lkv_decode_attn over the rows in use of a cache with slack: segment s is rows
 * cap_offsets[s] .. cap_offsets[s] + lengths[s].  total_rows = cap_offsets[n_segments]; the
 * workspace is sized by lkv_decode_workspace_bytes(n_segments, total_rows, ...).  Everything
 * else as for lkv_decode_attn. */
lkv_status lkv_decode_attn_grown(lkv_ctx *ctx, int32_t n_seq, int32_t n_layers, int32_t n_kv_heads,
                                 int32_t n_q_heads, int32_t head_dim, const void *q, const void *kp,
                                 const void *vp, const int32_t *cap_offsets, const int32_t *lengths,
                                 int64_t total_rows, float scale, float *out, float *lse,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* Re-eviction of a cache with slack (the budgets floor(r t') of a longer context t', Sec. 3.3):
 * every segment keeps the new_budgets[s] rows it holds with the largest stored scores (the hard
 * top-k and tie rule of lkv_select, position = row inside the segment, which is time order) and
 * the result is written, in that order, to a new cache with fresh slack.  Tokens evicted earlier
 * do not return.
 * kp, vp, up, cap_offsets, lengths : DEVICE, the cache to shrink (not modified)
 * lengths_host  : HOST int32 [n_segments], the caller's count of the rows in use (budget at the
 *                 last eviction + appends since); must equal the device array
 * new_budgets   : HOST int32 [n_segments], 0 <= new_budgets[s] <= lengths_host[s]
 * idx           : DEVICE int32 [sum of new_budgets]: scratch, receives the kept row positions
 * offsets       : DEVICE int32 [n_segments + 1]: scratch, receives the prefix sums of new_budgets
 * kp_new, vp_new: DEVICE bf16 [sum of new_budgets + n_segments * slack, d]; up_new fp32 of as many rows
 * cap_offsets_new, lengths_new : DEVICE int32 [n_segments + 1] / [n_segments]
 * total_kept    : HOST out (sum of new_budgets), may be NULL
 * The new buffers must not overlap the old ones. */
lkv_status lkv_reevict(lkv_ctx *ctx, int64_t n_segments, int32_t head_dim, const void *kp, const void *vp,
                       const float *up, const int32_t *cap_offsets, const int32_t *lengths,
                       const int32_t *lengths_host, const int32_t *new_budgets, int32_t slack,
                       int32_t *idx, int32_t *offsets, void *kp_new, void *vp_new, float *up_new,
                       int32_t *cap_offsets_new, int32_t *lengths_new, int64_t *total_kept, void *stream);

/* ---- Attention with a multiplicative retention mask over the UNCOMPACTED cache (App. B.2) ----
 * For one query per head: p_i = e^{s_i} m_i / sum_j e^{s_j} m_j, s_i = scale * q . K[l, h, i, :],
 * out = sum_i p_i V[l, h, i, :]; this equals softmax(s + log m).  With a 0/1 mask it is what
 * lkv_decode_attn computes on the compacted cache (the identity the eviction rests on); with
 * m = ST_k(u / tau) it is the relaxed forward the scorer is trained through (Sec. 3.4).
 * q    : DEVICE bf16 [n_seq, L, Hq, d]
 * mask : HOST [n_seq] of DEVICE fp32 [L, H, T_s], values in [0, 1]; a head whose mask is all zero
 *        gives out = 0 and lse = -inf
 * out  : DEVICE fp32 [n_seq, L, Hq, d];  lse : DEVICE fp32 [n_seq, L, Hq] or NULL
 *        (lse = log sum_i m_i e^{s_i})
 * workspace : DEVICE, at least lkv_masked_decode_workspace_bytes(cache) bytes, 256-byte aligned.
 * Sequences are processed one after the other on `stream`. */
size_t lkv_masked_decode_workspace_bytes(const lkv_cache *cache);
lkv_status lkv_masked_decode_attn(lkv_ctx *ctx, const lkv_cache *cache, const void *q,
                                  const float *const *mask, float scale, float *out, float *lse,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* ---- Training-time attention with the multiplicative soft mask (Sec. 3.5, App. B) ---------
 * Causal self-attention of one layer of one sequence, every token a query:
 *   p_ij = e^{s_ij} m_j / sum_{k <= i} e^{s_ik} m_k,  s_ij = scale * q_i . k_j,  o_i = sum_{j <= i} p_ij v_j.
 * The mask multiplies the exponentials inside the online softmax (App. B.2); no log m is taken,
 * so m_j = 0 is an ordinary value.  Query head hq reads KV head hq / (n_q_heads / n_kv_heads) and
 * that head's mask (Sec. 3.1).
 * q   : DEVICE bf16 [n_q_heads, seq_len, d]        k, v : DEVICE bf16 [n_kv_heads, seq_len, d]
 * m   : DEVICE fp32 [n_kv_heads, seq_len], values in [0, 1]
 * o   : DEVICE fp32 [n_q_heads, seq_len, d] (fp32 so that the backward pass forms D_i = d_o_i . o_i from
 *       unrounded outputs: with a bf16 o the rounding of D dominates the gradient error of short prefixes)
 * lse : DEVICE fp32 [n_q_heads, seq_len] = log sum_{k <= i} e^{s_ik} m_k (needed by the backward pass)
 * A query whose whole prefix has weight 0 gets o = 0 and lse = -inf.
 * q, k, v, o 16-byte aligned; head_dim must be 128; scale > 0;
 * seq_len < 2^24; n_q_heads * ceil(seq_len / 128) < 2^31.
 * Errors: LKV_ERR_INVALID_ARG / LKV_ERR_UNSUPPORTED before anything is enqueued. */
lkv_status lkv_masked_attn_forward(lkv_ctx *ctx, int32_t n_q_heads, int32_t n_kv_heads, int32_t seq_len,
                                   int32_t head_dim, const void *q, const void *k, const void *v,
                                   const float *m, float scale, float *o, float *lse, void *stream);

/* Backward pass of lkv_masked_attn_forward (App. B.3): gradients of a scalar loss given its
 * gradient d_o with respect to o.  With e_ij = e^{s_ij - lse_i}, p_ij = e_ij m_j, dP_ij = d_o_i . v_j,
 * D_i = d_o_i . o_i:
 *   dv_j = sum_i p_ij d_o_i        dm_j = sum_i e_ij (dP_ij - D_i)        dS_ij = p_ij (dP_ij - D_i)
 *   dq_i = scale sum_j dS_ij k_j   dk_j = scale sum_i dS_ij q_i
 * over the causal pairs j <= i; dk, dv and dm also sum over the query heads that share the KV head.
 * The factor towards the mask is e_ij, not 1 / m_j, so dm is finite where m_j = 0.  Queries with
 * lse = -inf contribute nothing.
 * q, k, v, m : as given to the forward call;  o, lse : as it returned them
 * d_o : DEVICE bf16 [n_q_heads, seq_len, d]
 * dq  : DEVICE fp32 [n_q_heads, seq_len, d];  dk, dv : DEVICE fp32 [n_kv_heads, seq_len, d]
 * dm  : DEVICE fp32 [n_kv_heads, seq_len]
 * workspace : DEVICE, at least lkv_masked_attn_backward_workspace_bytes(n_q_heads, n_kv_heads, seq_len)
 *             bytes, 16-byte aligned (holds D and, for short sequences with grouped heads, per-query-head
 *             partial sums of dk, dv and dm that a last pass adds up in a fixed order).
 * Every output element is written exactly once (no atomics: results are reproducible bit for bit).
 * Outputs and workspace must not overlap the inputs or each other.
 * Errors as for the forward call, plus LKV_ERR_WORKSPACE. */
size_t lkv_masked_attn_backward_workspace_bytes(int32_t n_q_heads, int32_t n_kv_heads, int32_t seq_len);
lkv_status lkv_masked_attn_backward(lkv_ctx *ctx, int32_t n_q_heads, int32_t n_kv_heads, int32_t seq_len,
                                    int32_t head_dim, const void *q, const void *k, const void *v,
                                    const float *m, const float *o, const float *lse, const void *d_o,
                                    float scale, float *dq, float *dk, float *dv, float *dm,
                                    void *workspace, size_t workspace_bytes, void *stream);

/* ---- LKV-H: global budget allocation, inference side (Sec. 3.3) ------------------------- */

/* Forward Soft-TopK operator ST_k of Sec. 3.2 (threshold in closed form, Eq. 2 and App. A.1):
 *   y_i = f(x_i / tau - lambda),  f(z) = (1 + sgn(z)(1 - e^{-|z|})) / 2,  sum_i y_i = k.
 * fp64 arithmetic, sums carried as logarithms (any tau > 0 is safe).  One workgroup sorts the
 * input in LDS when it fits (32768 fp32 or 16384 fp64 values); longer inputs, up to
 * lkv_soft_topk_max_n() = 2^22 values, take the same closed form after the split index has been
 * found by bracketing the threshold with passes over the input (about 50 of them).
 * x    : DEVICE fp32 [n] (x_is_f64 = 0) or fp64 [n] (x_is_f64 = 1); finite values
 * k    : target sum, in the open interval (0, n)
 * tau  : temperature, > 0
 * y    : DEVICE fp64 [n]; may be the same buffer as an fp64 x
 * info : DEVICE fp64 [2] or NULL: info[0] = lambda (in units of x / tau), info[1] = split index m
 * Errors: LKV_ERR_INVALID_ARG for k, tau or n out of range, LKV_ERR_UNSUPPORTED beyond the size limit. */
int32_t lkv_soft_topk_max_n(int32_t x_is_f64);
lkv_status lkv_soft_topk(lkv_ctx *ctx, const void *x, int32_t x_is_f64, int32_t n, double k, double tau,
                         double *y, double *info, void *stream);

/* Backward of the Soft-TopK operator (App. A.2).  The threshold is an implicit function of the
 * inputs; with z_i = x_i / tau - lambda and f'(z) = e^{-|z|} / 2,
 *   d lambda / d x_j = f'(z_j) / sum_i f'(z_i),   d lambda / d k = -1 / sum_i f'(z_i),
 * and for an upstream gradient g = dL/dy of y = ST_k(x / tau):
 *   dx_j = (f'(z_j) / tau) (g_j - gbar),   dk = gbar = sum_i g_i f'(z_i) / sum_i f'(z_i).
 * fp64 arithmetic, sums in a fixed order (reproducible); the ratios are formed relative to the
 * smallest |z|, so a temperature so cold that every f'(z_i) underflows gives dx = 0 and a finite dk.
 * x, x_is_f64, n, tau : as given to lkv_soft_topk
 * info : DEVICE fp64 [2] as written by that call (info[0] = lambda is read)
 * g    : DEVICE fp64 [n]
 * dx   : DEVICE fp64 [n]; may be the same buffer as g
 * dk   : DEVICE fp64 [1] or NULL */
lkv_status lkv_soft_topk_backward(lkv_ctx *ctx, const void *x, int32_t x_is_f64, int32_t n, double tau,
                                  const double *info, const double *g, double *dx, double *dk, void *stream);

/* The two calls above for n_vec vectors of n values at once, one workgroup per vector: what the
 * relaxed forward of Sec. 3.4 needs, one soft mask m = ST_b((u + g) / tau) per head of a layer.
 * x, y, g, dx : DEVICE [n_vec, n], row-major; info : DEVICE fp64 [n_vec, 2]; dk : DEVICE fp64 [n_vec] or NULL
 * k    : DEVICE fp64 [n_vec], the target sum of every vector (for example r_h * t from
 *        lkv_head_budgets' ratios); values are clamped into [1e-6, n - 1e-6], the open interval
 *        the paper keeps the budget in (App. A.1)
 * n    : >= 2 for the forward call (the interval above is empty otherwise) */
lkv_status lkv_soft_topk_batched(lkv_ctx *ctx, const void *x, int32_t x_is_f64, int32_t n_vec, int32_t n,
                                 const double *k, double tau, double *y, double *info, void *stream);
lkv_status lkv_soft_topk_backward_batched(lkv_ctx *ctx, const void *x, int32_t x_is_f64, int32_t n_vec, int32_t n,
                                          double tau, const double *info, const double *g, double *dx,
                                          double *dk, void *stream);

/* Shared head predictor of LKV-H (Sec. 3.3; Table 5: 128 -> 64 -> 1, SiLU, hidden bias, no
 * output bias).  All pointers DEVICE fp32; b2 may be NULL. */
typedef struct lkv_head_predictor {
  int32_t d_e;       /* embedding width */
  int32_t hidden;    /* hidden units, <= 4096 */
  const float *w1;   /* [hidden, d_e] */
  const float *b1;   /* [hidden] */
  const float *w2;   /* [hidden] */
  const float *b2;   /* [1] or NULL */
} lkv_head_predictor;

/* Retention ratios and integer budgets of all heads (Sec. 3.3):
 *   s_i = MLP_head(e_i),  r = ST_{R n}(s) at tau = 1,  b_i = floor(r_i * t).
 * fp64 arithmetic.  The ratios depend only on static parameters: compute once, keep.
 * emb : DEVICE fp32 [n_heads, d_e], heads flattened layer-major (l * H + h)
 * R   : global retention ratio in (0, 1)
 * t   : context length the budgets are for (ignored when b is NULL)
 * r   : DEVICE fp64 [n_heads], every value in (0, 1), sum = R * n_heads
 * b   : DEVICE int32 [n_heads] or NULL; sum <= floor(R * n_heads * t)
 * Budgets reach lkv_select through host memory: copy b back after the stream has finished. */
lkv_status lkv_head_budgets(lkv_ctx *ctx, const float *emb, const lkv_head_predictor *predictor,
                            int32_t n_heads, double R, int32_t t, double *r, int32_t *b, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LKV_H_ */
