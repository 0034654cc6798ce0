// Host side of the C ABI declared in include/lkv.h: argument checks, launch
// tables, the pinned staging ring for the offsets upload, and error reporting.
// Every check runs before anything is enqueued.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>

#include "../../include/lkv.h"
#include "lkv_kernels.h"

namespace {

constexpr int kStageSlots = 8;
constexpr size_t kStageBytes = 1u << 20;   // 1 MiB per slot: up to 262143 segments
constexpr int64_t kMaxSegments = (int64_t)(kStageBytes / sizeof(int32_t)) - 1;

}  // namespace

struct lkv_ctx {
  int device = 0;
  std::string err;
  void* stage[kStageSlots] = {};
  hipEvent_t stage_done[kStageSlots] = {};
  bool stage_used[kStageSlots] = {};
  int stage_next = 0;
};

namespace {

lkv_status fail(lkv_ctx* ctx, lkv_status st, const char* fmt, ...) {
  if (ctx != nullptr) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    ctx->err = buf;
  }
  return st;
}

lkv_status hip_fail(lkv_ctx* ctx, hipError_t e, const char* what) {
  return fail(ctx, LKV_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

lkv_status check_cache(lkv_ctx* ctx, const lkv_cache* c, bool need_kv) {
  if (c == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "cache is NULL");
  if (c->n_seq < 1 || c->n_layers < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1)
    return fail(ctx, LKV_ERR_INVALID_ARG, "n_seq, n_layers, n_kv_heads and n_q_heads must be >= 1");
  if (c->n_q_heads % c->n_kv_heads != 0)
    return fail(ctx, LKV_ERR_INVALID_ARG, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)", c->n_q_heads,
                c->n_kv_heads);
  if (c->head_dim != lkv::kHeadDim) return fail(ctx, LKV_ERR_UNSUPPORTED, "head_dim must be 128, got %d", c->head_dim);
  if (c->seq_len == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "seq_len is NULL");
  if (need_kv && (c->k == nullptr || c->v == nullptr)) return fail(ctx, LKV_ERR_INVALID_ARG, "k or v table is NULL");
  const int64_t heads = (int64_t)c->n_layers * c->n_kv_heads;
  if (heads * c->n_seq >= (int64_t)1 << 31) return fail(ctx, LKV_ERR_UNSUPPORTED, "too many segments");
  for (int s = 0; s < c->n_seq; ++s) {
    if (c->seq_len[s] < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "seq_len[%d] = %d must be >= 1", s, c->seq_len[s]);
    if (need_kv) {
      if (c->k[s] == nullptr || c->v[s] == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "k[%d] or v[%d] is NULL", s, s);
      if (!aligned16(c->k[s]) || !aligned16(c->v[s]))
        return fail(ctx, LKV_ERR_INVALID_ARG, "k[%d] or v[%d] is not 16-byte aligned", s, s);
    }
  }
  return LKV_OK;
}

// Scorer description: kinds, pointers, widths.  `mfma_widths`: the cache-wide scoring kernels take hidden widths
// that are multiples of 16 up to 128; the one-token path of lkv_append takes any width up to 128.
lkv_status check_scorer(lkv_ctx* ctx, const lkv_scorer* s, bool mfma_widths) {
  if (s == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "scorer is NULL");
  if (s->kind != LKV_SCORER_LINEAR && s->kind != LKV_SCORER_MLP)
    return fail(ctx, LKV_ERR_INVALID_ARG, "unknown scorer kind %d", s->kind);
  if (s->w1 == nullptr || s->b1 == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "scorer w1 or b1 is NULL");
  if (!aligned16(s->w1)) return fail(ctx, LKV_ERR_INVALID_ARG, "scorer w1 is not 16-byte aligned");
  if (s->per_head != 0 && s->per_head != 1) return fail(ctx, LKV_ERR_INVALID_ARG, "per_head must be 0 or 1");
  if (s->kind == LKV_SCORER_MLP) {
    if (s->act != LKV_ACT_SILU && s->act != LKV_ACT_GELU_ERF)
      return fail(ctx, LKV_ERR_INVALID_ARG, "unknown activation %d", s->act);
    if (s->w2 == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "scorer w2 is NULL");
    if (mfma_widths && (s->hidden < 16 || s->hidden > 128 || s->hidden % 16 != 0))
      return fail(ctx, LKV_ERR_UNSUPPORTED, "hidden = %d must be a multiple of 16 in [16, 128]", s->hidden);
    if (!mfma_widths && (s->hidden < 1 || s->hidden > 128))
      return fail(ctx, LKV_ERR_UNSUPPORTED, "hidden = %d must lie in [1, 128]", s->hidden);
  }
  return LKV_OK;
}

// A caller-owned workspace: present, large enough and aligned to `align` bytes (a power of two).
lkv_status check_workspace(lkv_ctx* ctx, const void* workspace, size_t bytes, size_t need, size_t align, const char* what) {
  if (workspace == nullptr || bytes < need)
    return fail(ctx, LKV_ERR_WORKSPACE, "%s workspace: need %zu bytes, got %zu", what, need, bytes);
  if ((reinterpret_cast<uintptr_t>(workspace) & (align - 1)) != 0)
    return fail(ctx, LKV_ERR_WORKSPACE, "%s workspace is not %zu-byte aligned", what, align);
  return LKV_OK;
}

// Geometry of a decode call over a packed cache: counts, the GQA group and the number of segments.
lkv_status check_decode_geometry(lkv_ctx* ctx, int32_t n_seq, int32_t n_layers, int32_t n_kv_heads, int32_t n_q_heads,
                                 int32_t head_dim, int* group, int64_t* n_segments) {
  if (n_seq < 1 || n_layers < 1 || n_kv_heads < 1 || n_q_heads < 1)
    return fail(ctx, LKV_ERR_INVALID_ARG, "n_seq, n_layers, n_kv_heads and n_q_heads must be >= 1");
  if (n_q_heads % n_kv_heads != 0) return fail(ctx, LKV_ERR_INVALID_ARG, "n_q_heads is not a multiple of n_kv_heads");
  if (head_dim != lkv::kHeadDim) return fail(ctx, LKV_ERR_UNSUPPORTED, "head_dim must be 128, got %d", head_dim);
  *group = n_q_heads / n_kv_heads;
  if (*group > lkv::kDecodeMaxGroup)
    return fail(ctx, LKV_ERR_UNSUPPORTED, "GQA group %d exceeds %d", *group, lkv::kDecodeMaxGroup);
  *n_segments = (int64_t)n_seq * n_layers * n_kv_heads;
  if (*n_segments > kMaxSegments) return fail(ctx, LKV_ERR_UNSUPPORTED, "too many segments");
  return LKV_OK;
}

// Geometry and scale of the training-time attention calls (one layer of one sequence).
lkv_status check_attention_geometry(lkv_ctx* ctx, int32_t n_q_heads, int32_t n_kv_heads, int32_t seq_len, int32_t head_dim,
                                    float scale) {
  if (n_q_heads < 1 || n_kv_heads < 1 || seq_len < 1)
    return fail(ctx, LKV_ERR_INVALID_ARG, "n_q_heads, n_kv_heads and seq_len must be >= 1");
  if (n_q_heads % n_kv_heads != 0) return fail(ctx, LKV_ERR_INVALID_ARG, "n_q_heads is not a multiple of n_kv_heads");
  if (head_dim != lkv::kHeadDim) return fail(ctx, LKV_ERR_UNSUPPORTED, "head_dim must be 128, got %d", head_dim);
  if (seq_len >= 1 << 24) return fail(ctx, LKV_ERR_UNSUPPORTED, "seq_len = %d must be below 2^24", seq_len);
  if (((int64_t)seq_len + 127) / 128 * n_q_heads >= (int64_t)1 << 31)
    return fail(ctx, LKV_ERR_UNSUPPORTED, "n_q_heads * seq_len is too large for one launch");
  if (!(scale > 0.f) || std::isinf(scale)) return fail(ctx, LKV_ERR_INVALID_ARG, "scale = %g must be positive and finite", (double)scale);
  return LKV_OK;
}

hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// lkv_score, optionally counting the first-level top-k digits of every segment on the way (counts zero on entry).
// The segment of (sequence s, view head j) is seg_base + s * seg_stride + j.
lkv_status score_impl(lkv_ctx* ctx, const lkv_cache* cache, const lkv_scorer* scorer, float* const* scores,
                      uint32_t* counts, int seg_base, int seg_stride, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (lkv_status st = check_cache(ctx, cache, true)) return st;
  if (scores == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "scores is NULL");
  if (lkv_status st = check_scorer(ctx, scorer, true)) return st;
  const int64_t heads = (int64_t)cache->n_layers * cache->n_kv_heads;
  for (int s = 0; s < cache->n_seq; ++s) {
    if (scores[s] == nullptr || !aligned16(scores[s]))
      return fail(ctx, LKV_ERR_INVALID_ARG, "scores[%d] is NULL or not 16-byte aligned", s);
  }
  const int heads_per_row = scorer->per_head ? 1 : cache->n_kv_heads;
  hipStream_t st = as_stream(stream);

  // launches of up to kMaxSeqPerLaunch sequences; MLP launches also need one tile size per launch
  int s = 0;
  while (s < cache->n_seq) {
    lkv::SeqTable tab;
    memset(&tab, 0, sizeof(tab));
    int64_t blocks = 0;
    const int s_first = s;
    const int rpb0 = scorer->kind == LKV_SCORER_MLP ? lkv::score_mlp_rows_per_block(cache->seq_len[s], (int)heads, scorer->hidden) : 0;
    int n = 0;
    while (s < cache->n_seq && n < lkv::kMaxSeqPerLaunch) {
      const int T = cache->seq_len[s];
      int64_t per_head;
      if (scorer->kind == LKV_SCORER_MLP) {
        if (lkv::score_mlp_rows_per_block(T, (int)heads, scorer->hidden) != rpb0) break;
        per_head = (T + rpb0 - 1) / rpb0;
      } else {
        per_head = lkv::score_linear_blocks_per_head(T);
      }
      if (blocks + per_head * heads >= ((int64_t)1 << 31) - 1) {
        if (n == 0) return fail(ctx, LKV_ERR_UNSUPPORTED, "sequence %d is too long for one launch", s);
        break;
      }
      tab.k[n] = static_cast<const uint16_t*>(cache->k[s]);
      tab.v[n] = static_cast<const uint16_t*>(cache->v[s]);
      tab.scores[n] = scores[s];
      tab.T[n] = T;
      tab.first[n] = (int32_t)blocks;
      blocks += per_head * heads;
      ++n;
      ++s;
    }
    tab.first[n] = (int32_t)blocks;
    tab.n = n;
    const int launch_seg_base = seg_base + s_first * seg_stride;
    if (scorer->kind == LKV_SCORER_LINEAR) {
      lkv::launch_score_linear(tab, static_cast<const uint16_t*>(scorer->w1), scorer->b1, heads_per_row, st);
      if (counts != nullptr) {
        // the linear kernel's blocks are too small to carry a histogram: a pass over the scores counts instead
        if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_score launch");
        int64_t cblocks = 0;
        for (int i = 0; i < n; ++i) {
          tab.first[i] = (int32_t)cblocks;
          cblocks += heads * lkv::count_level0_blocks_per_head(tab.T[i]);
        }
        tab.first[n] = (int32_t)cblocks;
        lkv::launch_count_level0(tab, counts, launch_seg_base, seg_stride, st);
      }
    } else {
      lkv::launch_score_mlp(tab, static_cast<const uint16_t*>(scorer->w1), scorer->b1, scorer->w2, scorer->b2,
                            scorer->hidden, scorer->act == LKV_ACT_SILU ? 0 : 1, heads_per_row, rpb0, st, counts,
                            launch_seg_base, seg_stride);
    }
    if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_score launch");
  }
  return LKV_OK;
}

}  // namespace

extern "C" {

const char* lkv_version(void) { return "lkv-mi355x 0.1 (gfx950)"; }

lkv_status lkv_create(lkv_ctx** out, int device) {
  if (out == nullptr) return LKV_ERR_INVALID_ARG;
  *out = nullptr;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) return LKV_ERR_HIP;
  if (hipSetDevice(device) != hipSuccess) return LKV_ERR_HIP;
  lkv_ctx* ctx = new (std::nothrow) lkv_ctx();
  if (ctx == nullptr) return LKV_ERR_HIP;
  ctx->device = device;
  for (int i = 0; i < kStageSlots; ++i) {
    if (hipHostMalloc(&ctx->stage[i], kStageBytes, hipHostMallocDefault) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->stage_done[i], hipEventDisableTiming) != hipSuccess) {
      lkv_destroy(ctx);
      return LKV_ERR_HIP;
    }
  }
  if (lkv::select_prepare() != hipSuccess || lkv::decode_prepare(device) != hipSuccess ||
      lkv::score_mlp_prepare() != hipSuccess || lkv::lkv_h_prepare() != hipSuccess ||
      lkv::masked_attn_prepare() != hipSuccess || lkv::masked_attn_bwd_prepare() != hipSuccess) {
    lkv_destroy(ctx);
    return LKV_ERR_HIP;
  }
  *out = ctx;
  return LKV_OK;
}

void lkv_destroy(lkv_ctx* ctx) {
  if (ctx == nullptr) return;
  for (int i = 0; i < kStageSlots; ++i) {
    if (ctx->stage_done[i] != nullptr) {
      if (ctx->stage_used[i]) (void)hipEventSynchronize(ctx->stage_done[i]);
      (void)hipEventDestroy(ctx->stage_done[i]);
    }
    if (ctx->stage[i] != nullptr) (void)hipHostFree(ctx->stage[i]);
  }

  delete ctx;
}

const char* lkv_last_error(const lkv_ctx* ctx) { return ctx != nullptr ? ctx->err.c_str() : "context is NULL"; }

lkv_status lkv_score(lkv_ctx* ctx, const lkv_cache* cache, const lkv_scorer* scorer, float* const* scores,
                     void* stream) {
  return score_impl(ctx, cache, scorer, scores, nullptr, 0, 0, stream);
}

lkv_status lkv_score_counted(lkv_ctx* ctx, const lkv_cache* cache, const lkv_scorer* scorer, float* const* scores,
                             uint32_t* counts, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (counts == nullptr || !aligned16(counts)) return fail(ctx, LKV_ERR_INVALID_ARG, "counts is NULL or not 16-byte aligned");
  if (cache == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "cache is NULL");
  return score_impl(ctx, cache, scorer, scores, counts, 0, cache->n_layers * cache->n_kv_heads, stream);
}

size_t lkv_counts_bytes(int64_t n_segments) {
  return n_segments > 0 ? (size_t)n_segments * lkv::kLevel0Bins * sizeof(uint32_t) : 0;
}

size_t lkv_counts_bytes_split(int64_t n_segments, int32_t max_seq_len) {
  if (n_segments <= 0 || max_seq_len <= 0) return 0;
  const size_t words = ((size_t)max_seq_len + 31) / 32;
  return lkv_counts_bytes(n_segments) + (size_t)n_segments * 2 * words * sizeof(uint32_t);
}

lkv_status lkv_clear_counts(lkv_ctx* ctx, uint32_t* counts, int64_t n_segments, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (counts == nullptr || !aligned16(counts)) return fail(ctx, LKV_ERR_INVALID_ARG, "counts is NULL or not 16-byte aligned");
  if (n_segments < 1 || n_segments > kMaxSegments) return fail(ctx, LKV_ERR_INVALID_ARG, "n_segments = %lld is out of range", (long long)n_segments);
  lkv::launch_clear_counts(counts, n_segments, as_stream(stream));
  if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_clear_counts launch");
  return LKV_OK;
}

size_t lkv_score_window_workspace_bytes(const lkv_cache* cache) {
  if (cache == nullptr || cache->seq_len == nullptr || cache->n_seq < 1 || cache->n_layers < 1 || cache->n_kv_heads < 1)
    return 0;
  const int64_t heads = (int64_t)cache->n_layers * cache->n_kv_heads;
  size_t need = 0;
  for (int s = 0; s < cache->n_seq; ++s) {
    if (cache->seq_len[s] < 1) return 0;
    need += lkv::score_window_pairs_bytes(heads, cache->seq_len[s]);
  }
  return need;
}

lkv_status lkv_score_window(lkv_ctx* ctx, const lkv_cache* cache, const void* const* q_win,
                            const float* const* lse_win, int32_t window, int32_t pool_width, int32_t pool_kind,
                            float scale, float* const* scores, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (lkv_status st = check_cache(ctx, cache, false)) return st;   // only the keys are read
  if (cache->k == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "k table is NULL");
  if (q_win == nullptr || scores == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "q_win or scores is NULL");
  if (window < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "window = %d must be >= 1", window);
  if (pool_width < 1 || pool_width % 2 == 0 || pool_width > 63)
    return fail(ctx, LKV_ERR_INVALID_ARG, "pool_width = %d must be odd and lie in [1, 63]", pool_width);
  if (pool_kind != LKV_POOL_MAX && pool_kind != LKV_POOL_AVG)
    return fail(ctx, LKV_ERR_INVALID_ARG, "unknown pooling kind %d", pool_kind);
  if (!(scale > 0.f) || !std::isfinite(scale)) return fail(ctx, LKV_ERR_INVALID_ARG, "scale must be positive and finite");
  const int G = cache->n_q_heads / cache->n_kv_heads;
  const int64_t heads = (int64_t)cache->n_layers * cache->n_kv_heads;
  int64_t cells = 0;
  for (int s = 0; s < cache->n_seq; ++s) {
    if (window > cache->seq_len[s])
      return fail(ctx, LKV_ERR_INVALID_ARG, "window = %d exceeds seq_len[%d] = %d", window, s, cache->seq_len[s]);
    if (cache->k[s] == nullptr || !aligned16(cache->k[s]))
      return fail(ctx, LKV_ERR_INVALID_ARG, "k[%d] is NULL or not 16-byte aligned", s);
    if (q_win[s] == nullptr || !aligned16(q_win[s]))
      return fail(ctx, LKV_ERR_INVALID_ARG, "q_win[%d] is NULL or not 16-byte aligned", s);
    if (scores[s] == nullptr || !aligned16(scores[s]))
      return fail(ctx, LKV_ERR_INVALID_ARG, "scores[%d] is NULL or not 16-byte aligned", s);
    if (lse_win != nullptr && lse_win[s] == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "lse_win[%d] is NULL", s);
    cells += heads * cache->seq_len[s];
  }
  if ((int64_t)G * window > lkv::score_window_max_rows())
    return fail(ctx, LKV_ERR_UNSUPPORTED, "group %d x window %d exceeds %d query rows per KV head", G, window,
                lkv::score_window_max_rows());
  const size_t need = lkv_score_window_workspace_bytes(cache);
  if (lkv_status st = check_workspace(ctx, workspace, workspace_bytes, need, 256, "window scoring")) return st;
  const int rpb = lkv::score_window_rows_per_block(cells);
  hipStream_t st = as_stream(stream);

  // every sequence's blocks must fit one grid before anything is launched
  for (int s = 0; s < cache->n_seq; ++s)
    if (heads * ((cache->seq_len[s] + 127) / 128) >= ((int64_t)1 << 31) - 1)
      return fail(ctx, LKV_ERR_UNSUPPORTED, "sequence %d is too long for one launch", s);

  unsigned char* ws = static_cast<unsigned char*>(workspace);
  int s = 0;
  while (s < cache->n_seq) {
    lkv::WinTable tab;
    memset(&tab, 0, sizeof(tab));
    int64_t blocks = 0;
    int n = 0;
    while (s < cache->n_seq && n < lkv::kMaxSeqPerLaunch) {
      const int T = cache->seq_len[s];
      const int64_t mine = heads * ((T + rpb - 1) / rpb);
      if (n > 0 && blocks + mine >= ((int64_t)1 << 31) - 1) break;
      tab.k[n] = static_cast<const uint16_t*>(cache->k[s]);
      tab.q[n] = static_cast<const uint16_t*>(q_win[s]);
      tab.scores[n] = scores[s];
      tab.lse[n] = lse_win != nullptr ? lse_win[s] : nullptr;
      tab.partial[n] = reinterpret_cast<float*>(ws);
      ws += lkv::score_window_pairs_bytes(heads, T);
      tab.T[n] = T;
      tab.first[n] = (int32_t)blocks;
      blocks += mine;
      ++n;
      ++s;
    }
    tab.first[n] = (int32_t)blocks;
    tab.n = n;
    lkv::launch_score_window(tab, (int)heads, window, G, pool_width, pool_kind, rpb, scale, st);
    if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_score_window launch");
  }
  return LKV_OK;
}

}  // extern "C"

namespace {

// A pinned staging slot for an offsets upload on `st`.  The upload path cannot be recorded into a HIP
// graph (a replay would copy whatever a later call has left in the slot) and may wait on the host for
// the slot's previous upload, so it is refused while `st` is capturing.
lkv_status take_stage_slot(lkv_ctx* ctx, hipStream_t st, const char* who, int* slot_out) {
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipError_t e = hipStreamIsCapturing(st, &cap)) return hip_fail(ctx, e, "capture status query");
  if (cap != hipStreamCaptureStatusNone)
    return fail(ctx, LKV_ERR_UNSUPPORTED,
                "%s would upload offsets from host memory, which cannot be captured into a HIP graph: call "
                "lkv_plan_offsets before the capture and pass budgets = NULL inside it", who);
  const int slot = ctx->stage_next;
  ctx->stage_next = (slot + 1) % kStageSlots;
  if (ctx->stage_used[slot]) {
    if (hipError_t e = hipEventSynchronize(ctx->stage_done[slot])) return hip_fail(ctx, e, "staging slot wait");
  }
  *slot_out = slot;
  return LKV_OK;
}

lkv_status select_impl(lkv_ctx* ctx, const lkv_cache* cache, const float* const* scores, const int32_t* budgets,
                       uint32_t* counts, int32_t* idx, int32_t* offsets, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (lkv_status st = check_cache(ctx, cache, false)) return st;
  if (scores == nullptr || offsets == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "scores or offsets is NULL");
  const int heads = cache->n_layers * cache->n_kv_heads;
  const int64_t n_seg = (int64_t)heads * cache->n_seq;
  if ((size_t)(n_seg + 1) * sizeof(int32_t) > kStageBytes)
    return fail(ctx, LKV_ERR_UNSUPPORTED, "%lld segments exceed the staging capacity", (long long)n_seg);
  for (int s = 0; s < cache->n_seq; ++s)
    if (scores[s] == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "scores[%d] is NULL", s);
  hipStream_t st = as_stream(stream);

  // Offsets.  budgets == NULL: the device array already holds them (lkv_plan_offsets), nothing is
  // computed or copied here.  Otherwise they are computed on the host; few segments ride in the kernel
  // arguments and the kernel publishes them, many are uploaded through a pinned slot of the ring.
  const bool planned = budgets == nullptr;
  const bool inline_offsets = !planned && n_seg < lkv::select_inline_capacity() && cache->n_seq <= lkv::kMaxSeqPerLaunch;
  int32_t inline_buf[1024];
  int32_t* host_off = inline_buf;
  if (planned) {
    if (idx == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "idx is NULL");
  } else {
    int64_t total = 0;
    for (int s = 0; s < cache->n_seq; ++s) {
      const int T = cache->seq_len[s];
      for (int h = 0; h < heads; ++h) {
        const int32_t b = budgets[(size_t)s * heads + h];
        if (b < 0 || b > T)
          return fail(ctx, LKV_ERR_INVALID_ARG, "budget %d of segment %lld is outside [0, %d]", b,
                      (long long)s * heads + h, T);
        total += b;
      }
    }
    if (total >= (int64_t)1 << 31) return fail(ctx, LKV_ERR_UNSUPPORTED, "sum of budgets %lld >= 2^31", (long long)total);
    if (total > 0 && idx == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "idx is NULL");
    int slot = -1;
    if (!inline_offsets) {
      if (lkv_status e = take_stage_slot(ctx, st, "lkv_select with host budgets for 640 or more segments", &slot)) return e;
      host_off = static_cast<int32_t*>(ctx->stage[slot]);
    }
    int32_t run = 0;
    for (int64_t i = 0; i < n_seg; ++i) {
      host_off[i] = run;
      run += budgets[i];
    }
    host_off[n_seg] = run;
    if (!inline_offsets) {
      if (hipError_t e = hipMemcpyAsync(offsets, host_off, (size_t)(n_seg + 1) * sizeof(int32_t), hipMemcpyHostToDevice, st))
        return hip_fail(ctx, e, "offsets upload");
      if (hipError_t e = hipEventRecord(ctx->stage_done[slot], st)) return hip_fail(ctx, e, "staging event");
      ctx->stage_used[slot] = true;
    }
  }

  for (int s0 = 0; s0 < cache->n_seq; s0 += lkv::kMaxSeqPerLaunch) {
    lkv::SeqTable tab;
    memset(&tab, 0, sizeof(tab));
    const int n = cache->n_seq - s0 < lkv::kMaxSeqPerLaunch ? cache->n_seq - s0 : lkv::kMaxSeqPerLaunch;
    for (int i = 0; i < n; ++i) {
      tab.scores[i] = const_cast<float*>(scores[s0 + i]);
      tab.T[i] = cache->seq_len[s0 + i];
      tab.first[i] = i * heads;
    }
    tab.first[n] = n * heads;
    tab.n = n;
    lkv::launch_select(tab, inline_offsets ? host_off : nullptr, (int)n_seg, offsets, idx, s0 * heads, heads, st, nullptr,
                       nullptr, nullptr, counts);
    if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_select launch");
  }
  return LKV_OK;
}

}  // namespace

extern "C" {

lkv_status lkv_select(lkv_ctx* ctx, const lkv_cache* cache, const float* const* scores, const int32_t* budgets,
                      int32_t* idx, int32_t* offsets, void* stream) {
  return select_impl(ctx, cache, scores, budgets, nullptr, idx, offsets, stream);
}

lkv_status lkv_select_counted(lkv_ctx* ctx, const lkv_cache* cache, const float* const* scores, const int32_t* budgets,
                              uint32_t* counts, int32_t* idx, int32_t* offsets, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (counts == nullptr || !aligned16(counts)) return fail(ctx, LKV_ERR_INVALID_ARG, "counts is NULL or not 16-byte aligned");
  return select_impl(ctx, cache, scores, budgets, counts, idx, offsets, stream);
}

lkv_status lkv_compact(lkv_ctx* ctx, const lkv_cache* cache, const int32_t* idx, const int32_t* offsets,
                       int64_t total_kept, void* kp, void* vp, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (lkv_status st = check_cache(ctx, cache, true)) return st;
  if (offsets == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "offsets is NULL");
  if (total_kept < 0 || total_kept >= (int64_t)1 << 31)
    return fail(ctx, LKV_ERR_INVALID_ARG, "total_kept = %lld is outside [0, 2^31)", (long long)total_kept);
  if (total_kept == 0) return LKV_OK;
  if (idx == nullptr || kp == nullptr || vp == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "idx, kp or vp is NULL");
  if (!aligned16(kp) || !aligned16(vp)) return fail(ctx, LKV_ERR_INVALID_ARG, "kp or vp is not 16-byte aligned");
  const int heads = cache->n_layers * cache->n_kv_heads;
  const int n_seg = heads * cache->n_seq;
  hipStream_t st = as_stream(stream);
  for (int s0 = 0; s0 < cache->n_seq; s0 += lkv::kMaxSeqPerLaunch) {
    lkv::SeqTable tab;
    memset(&tab, 0, sizeof(tab));
    const int n = cache->n_seq - s0 < lkv::kMaxSeqPerLaunch ? cache->n_seq - s0 : lkv::kMaxSeqPerLaunch;
    for (int i = 0; i < n; ++i) {
      tab.k[i] = static_cast<const uint16_t*>(cache->k[s0 + i]);
      tab.v[i] = static_cast<const uint16_t*>(cache->v[s0 + i]);
      tab.T[i] = cache->seq_len[s0 + i];
    }
    tab.n = n;
    lkv::launch_compact(tab, idx, offsets, n_seg, heads, s0, 0, heads, 0, total_kept, kp, vp, st,
                        cache->n_seq > lkv::kMaxSeqPerLaunch);
    if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_compact launch");
  }
  return LKV_OK;
}

size_t lkv_decode_workspace_bytes(int32_t n_segments, int64_t total_kept, int32_t n_q_heads, int32_t n_kv_heads) {
  if (n_segments < 0 || total_kept < 0 || n_kv_heads < 1 || n_q_heads < n_kv_heads) return 0;
  return lkv::decode_workspace_bytes(n_segments, total_kept, n_q_heads / n_kv_heads);
}

lkv_status lkv_decode_attn(lkv_ctx* ctx, int32_t n_seq, int32_t n_layers, int32_t n_kv_heads, int32_t n_q_heads,
                           int32_t head_dim, const void* q, const void* kp, const void* vp, const int32_t* offsets,
                           int64_t total_kept, float scale, float* out, float* lse, void* workspace,
                           size_t workspace_bytes, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  int G = 0;
  int64_t n_seg = 0;
  if (lkv_status st = check_decode_geometry(ctx, n_seq, n_layers, n_kv_heads, n_q_heads, head_dim, &G, &n_seg)) return st;
  if (total_kept < 0 || total_kept >= (int64_t)1 << 31)
    return fail(ctx, LKV_ERR_INVALID_ARG, "total_kept = %lld is outside [0, 2^31)", (long long)total_kept);
  if (q == nullptr || offsets == nullptr || out == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "q, offsets or out is NULL");
  if (total_kept > 0 && (kp == nullptr || vp == nullptr)) return fail(ctx, LKV_ERR_INVALID_ARG, "kp or vp is NULL");
  if (!aligned16(q) || !aligned16(kp) || !aligned16(vp) || !aligned16(out))
    return fail(ctx, LKV_ERR_INVALID_ARG, "q, kp, vp or out is not 16-byte aligned");
  const size_t need = lkv::decode_workspace_bytes((int)n_seg, total_kept, G);
  if (lkv_status st = check_workspace(ctx, workspace, workspace_bytes, need, 256, "decode")) return st;
  if (hipError_t e = lkv::launch_decode(G, q, kp, vp, offsets, nullptr, (int)n_seg, total_kept, scale, out, lse,
                                        static_cast<float*>(workspace), as_stream(stream)))
    return hip_fail(ctx, e, "lkv_decode_attn launch");
  return LKV_OK;
}

lkv_status lkv_decode_attn_static(lkv_ctx* ctx, int32_t n_seq, int32_t n_layers, int32_t n_kv_heads, int32_t n_q_heads,
                                  int32_t head_dim, const void* q, const void* kp, const void* vp, const int32_t* offsets,
                                  int64_t total_kept, float scale, float* out, float* lse, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  int G = 0;
  int64_t n_seg = 0;
  if (lkv_status st = check_decode_geometry(ctx, n_seq, n_layers, n_kv_heads, n_q_heads, head_dim, &G, &n_seg)) return st;
  if (total_kept < 0 || total_kept >= (int64_t)1 << 31)
    return fail(ctx, LKV_ERR_INVALID_ARG, "total_kept = %lld is outside [0, 2^31)", (long long)total_kept);
  if (q == nullptr || offsets == nullptr || out == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "q, offsets or out is NULL");
  if (total_kept > 0 && (kp == nullptr || vp == nullptr)) return fail(ctx, LKV_ERR_INVALID_ARG, "kp or vp is NULL");
  if (!aligned16(q) || !aligned16(kp) || !aligned16(vp) || !aligned16(out))
    return fail(ctx, LKV_ERR_INVALID_ARG, "q, kp, vp or out is not 16-byte aligned");
  const size_t need = lkv::decode_workspace_bytes((int)n_seg, total_kept, G);
  if (need > lkv::decode_static_scratch_bytes())
    return fail(ctx, LKV_ERR_WORKSPACE,
                "this problem needs %zu bytes of split-K scratch, the static array holds %zu: use lkv_decode_attn with a "
                "caller-owned workspace", need, lkv::decode_static_scratch_bytes());
  // the device address of the static array on this context's GPU (looked up by lkv_create), never the symbol itself
  float* ws = static_cast<float*>(lkv::decode_static_scratch(ctx->device));
  if (ws == nullptr) return fail(ctx, LKV_ERR_HIP, "the static scratch array of device %d has no address", ctx->device);
  if (hipError_t e = lkv::launch_decode(G, q, kp, vp, offsets, nullptr, (int)n_seg, total_kept, scale, out, lse, ws,
                                        as_stream(stream)))
    return hip_fail(ctx, e, "lkv_decode_attn_static launch");
  return LKV_OK;
}

lkv_status lkv_plan_offsets(lkv_ctx* ctx, int64_t n_segments, const int32_t* budgets, int32_t* offsets,
                            int64_t* total_kept, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (budgets == nullptr || offsets == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "budgets or offsets is NULL");
  if (n_segments < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "n_segments = %lld must be >= 1", (long long)n_segments);
  if (n_segments > kMaxSegments) return fail(ctx, LKV_ERR_UNSUPPORTED, "%lld segments exceed the staging capacity", (long long)n_segments);
  int64_t total = 0;
  for (int64_t i = 0; i < n_segments; ++i) {
    if (budgets[i] < 0) return fail(ctx, LKV_ERR_INVALID_ARG, "budget %d of segment %lld is negative", budgets[i], (long long)i);
    total += budgets[i];
  }
  if (total >= (int64_t)1 << 31) return fail(ctx, LKV_ERR_UNSUPPORTED, "sum of budgets %lld >= 2^31", (long long)total);
  hipStream_t st = as_stream(stream);
  int slot = -1;
  if (lkv_status e = take_stage_slot(ctx, st, "lkv_plan_offsets", &slot)) return e;
  int32_t* host_off = static_cast<int32_t*>(ctx->stage[slot]);
  int32_t run = 0;
  for (int64_t i = 0; i < n_segments; ++i) {
    host_off[i] = run;
    run += budgets[i];
  }
  host_off[n_segments] = run;
  if (hipError_t e = hipMemcpyAsync(offsets, host_off, (size_t)(n_segments + 1) * sizeof(int32_t), hipMemcpyHostToDevice, st))
    return hip_fail(ctx, e, "offsets upload");
  if (hipError_t e = hipEventRecord(ctx->stage_done[slot], st)) return hip_fail(ctx, e, "staging event");
  ctx->stage_used[slot] = true;
  if (total_kept != nullptr) *total_kept = total;
  return LKV_OK;
}

lkv_status lkv_evict_layer(lkv_ctx* ctx, const lkv_cache* layer, int32_t layer_index, int32_t n_layers,
                           const lkv_scorer* scorer, const int32_t* budgets, const int32_t* offsets,
                           float* const* scores, int32_t* idx, void* kp, void* vp, uint32_t* counts, size_t counts_bytes,
                           void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (lkv_status st = check_cache(ctx, layer, true)) return st;
  if (counts != nullptr && !aligned16(counts)) return fail(ctx, LKV_ERR_INVALID_ARG, "counts is not 16-byte aligned");
  const int m = layer->n_layers;   // consecutive layers in the view
  if (n_layers < 1 || layer_index < 0 || layer_index > n_layers - m)
    return fail(ctx, LKV_ERR_INVALID_ARG, "layers %d .. %d of the view are outside [0, %d)", layer_index, layer_index + m - 1,
                n_layers);
  if (budgets == nullptr || offsets == nullptr || scores == nullptr)
    return fail(ctx, LKV_ERR_INVALID_ARG, "budgets, offsets or scores is NULL");
  for (int s = 0; s < layer->n_seq; ++s)
    if (scores[s] == nullptr || !aligned16(scores[s]))
      return fail(ctx, LKV_ERR_INVALID_ARG, "scores[%d] is NULL or not 16-byte aligned", s);
  const int H = layer->n_kv_heads;
  const int heads_all = n_layers * H;
  const int64_t n_seg = (int64_t)heads_all * layer->n_seq;
  if (n_seg > kMaxSegments) return fail(ctx, LKV_ERR_UNSUPPORTED, "too many segments");

  // row ranges of this layer's segments in the packed cache, from the same prefix sums the plan uploaded
  int64_t run = 0, layer_rows = 0;
  int64_t row_lo[lkv::kMaxSeqPerLaunch], row_hi[lkv::kMaxSeqPerLaunch];
  if (layer->n_seq > lkv::kMaxSeqPerLaunch)
    return fail(ctx, LKV_ERR_UNSUPPORTED, "a layer view holds at most %d sequences, got %d", lkv::kMaxSeqPerLaunch, layer->n_seq);
  for (int s = 0; s < layer->n_seq; ++s) {
    const int T = layer->seq_len[s];
    for (int j = 0; j < heads_all; ++j) {
      const int32_t b = budgets[(size_t)s * heads_all + j];
      if (b < 0 || b > T)
        return fail(ctx, LKV_ERR_INVALID_ARG, "budget %d of segment %lld is outside [0, %d]", b, (long long)s * heads_all + j, T);
      if (j == layer_index * H) row_lo[s] = run;
      run += b;
      if (j == (layer_index + m) * H - 1) row_hi[s] = run;
    }
    layer_rows += row_hi[s] - row_lo[s];
  }
  if (run >= (int64_t)1 << 31) return fail(ctx, LKV_ERR_UNSUPPORTED, "sum of budgets %lld >= 2^31", (long long)run);
  if (layer_rows > 0 && (idx == nullptr || kp == nullptr || vp == nullptr)) return fail(ctx, LKV_ERR_INVALID_ARG, "idx, kp or vp is NULL");
  if (!aligned16(kp) || !aligned16(vp)) return fail(ctx, LKV_ERR_INVALID_ARG, "kp or vp is not 16-byte aligned");

  // score with the scorer parameters of the view's layers, unless the caller has already scored them
  if (scorer != nullptr) {
    if (lkv_status st = check_scorer(ctx, scorer, true)) return st;
    lkv_scorer sl = *scorer;
    const size_t rows = (size_t)layer_index * (scorer->per_head ? H : 1);   // scorer rows ahead of this layer
    if (scorer->kind == LKV_SCORER_LINEAR) {
      sl.w1 = static_cast<const uint16_t*>(scorer->w1) + rows * 2 * lkv::kHeadDim;
      sl.b1 = scorer->b1 + rows;
    } else {
      sl.w1 = static_cast<const uint16_t*>(scorer->w1) + rows * (size_t)scorer->hidden * 2 * lkv::kHeadDim;
      sl.b1 = scorer->b1 + rows * scorer->hidden;
      sl.w2 = scorer->w2 + rows * scorer->hidden;
      sl.b2 = scorer->b2 != nullptr ? scorer->b2 + rows : nullptr;
    }
    if (lkv_status st = score_impl(ctx, layer, &sl, scores, counts, layer_index * H, heads_all, stream)) return st;
  } else {
    counts = nullptr;   // the scores came from elsewhere: nothing has counted them
  }
  // room behind the counters for two bitmaps per segment lets a launch over few long heads split each head's pass over
  // the scores over several workgroups
  uint32_t* pre_maps = nullptr;
  int pre_words = 0;
  if (counts != nullptr) {
    if (counts_bytes < lkv_counts_bytes(n_seg))
      return fail(ctx, LKV_ERR_WORKSPACE, "counts: need %zu bytes, got %zu", lkv_counts_bytes(n_seg), counts_bytes);
    const size_t words = (counts_bytes - lkv_counts_bytes(n_seg)) / ((size_t)n_seg * 2 * sizeof(uint32_t));
    int max_T = 0;
    for (int s = 0; s < layer->n_seq; ++s) max_T = layer->seq_len[s] > max_T ? layer->seq_len[s] : max_T;
    if (words >= ((size_t)max_T + 31) / 32) {
      pre_maps = counts + (size_t)n_seg * lkv::kLevel0Bins;
      pre_words = (int)(words < ((size_t)lkv::select_max_bitmap_tokens() / 32) ? words : (size_t)lkv::select_max_bitmap_tokens() / 32);
    }
  }

  hipStream_t st = as_stream(stream);
  lkv::SeqTable tab;
  memset(&tab, 0, sizeof(tab));
  for (int i = 0; i < layer->n_seq; ++i) {
    tab.k[i] = static_cast<const uint16_t*>(layer->k[i]);
    tab.v[i] = static_cast<const uint16_t*>(layer->v[i]);
    tab.scores[i] = scores[i];
    tab.T[i] = layer->seq_len[i];
    tab.first[i] = i * m * H;
  }
  tab.first[layer->n_seq] = layer->n_seq * m * H;
  tab.n = layer->n_seq;
  // select: segment of (sequence i, view head j) is i * n_layers * H + layer_index * H + j, offsets already on the device
  lkv::launch_select(tab, nullptr, (int)n_seg, const_cast<int32_t*>(offsets), idx, layer_index * H, heads_all, st, nullptr,
                     nullptr, nullptr, counts, pre_maps, pre_words);
  if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_evict_layer select launch");
  // compact: one contiguous row range per sequence
  for (int i = 0; i < layer->n_seq; ++i) {
    lkv::SeqTable one;
    memset(&one, 0, sizeof(one));
    one.k[0] = tab.k[i];
    one.v[0] = tab.v[i];
    one.T[0] = tab.T[i];
    one.n = 1;
    lkv::launch_compact(one, idx, offsets, (int)n_seg, heads_all, i, layer_index * H, m * H, row_lo[i], row_hi[i], kp, vp, st);
    if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_evict_layer compact launch");
  }
  return LKV_OK;
}

lkv_status lkv_compact_grow(lkv_ctx* ctx, const lkv_cache* cache, const float* const* scores, const int32_t* idx,
                            const int32_t* offsets, int64_t total_kept, int32_t slack, void* kp, void* vp, float* up,
                            int32_t* cap_offsets, int32_t* lengths, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (lkv_status st = check_cache(ctx, cache, true)) return st;
  if (scores == nullptr || offsets == nullptr || cap_offsets == nullptr || lengths == nullptr)
    return fail(ctx, LKV_ERR_INVALID_ARG, "scores, offsets, cap_offsets or lengths is NULL");
  if (slack < 0) return fail(ctx, LKV_ERR_INVALID_ARG, "slack = %d must be >= 0", slack);
  const int heads = cache->n_layers * cache->n_kv_heads;
  const int64_t n_seg = (int64_t)heads * cache->n_seq;
  if (total_kept < 0 || total_kept + n_seg * slack >= (int64_t)1 << 31)
    return fail(ctx, LKV_ERR_INVALID_ARG, "total_kept + n_segments * slack = %lld is outside [0, 2^31)",
                (long long)(total_kept + n_seg * slack));
  if (total_kept > 0 && (idx == nullptr || kp == nullptr || vp == nullptr || up == nullptr))
    return fail(ctx, LKV_ERR_INVALID_ARG, "idx, kp, vp or up is NULL");
  if (!aligned16(kp) || !aligned16(vp)) return fail(ctx, LKV_ERR_INVALID_ARG, "kp or vp is not 16-byte aligned");
  for (int s = 0; s < cache->n_seq; ++s)
    if (scores[s] == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "scores[%d] is NULL", s);
  hipStream_t st = as_stream(stream);
  lkv::launch_grown_layout(offsets, (int)n_seg, slack, cap_offsets, lengths, st);
  if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_compact_grow layout launch");
  for (int s0 = 0; s0 < cache->n_seq; s0 += lkv::kMaxSeqPerLaunch) {
    lkv::SeqTable tab;
    memset(&tab, 0, sizeof(tab));
    const int n = cache->n_seq - s0 < lkv::kMaxSeqPerLaunch ? cache->n_seq - s0 : lkv::kMaxSeqPerLaunch;
    for (int i = 0; i < n; ++i) {
      tab.k[i] = static_cast<const uint16_t*>(cache->k[s0 + i]);
      tab.v[i] = static_cast<const uint16_t*>(cache->v[s0 + i]);
      tab.scores[i] = const_cast<float*>(scores[s0 + i]);
      tab.T[i] = cache->seq_len[s0 + i];
    }
    tab.n = n;
    lkv::launch_compact_grow(tab, idx, offsets, (int)n_seg, heads, s0, total_kept, slack, kp, vp, up, st,
                             cache->n_seq > lkv::kMaxSeqPerLaunch);
    if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_compact_grow launch");
  }
  return LKV_OK;
}

lkv_status lkv_append(lkv_ctx* ctx, int32_t n_seq, int32_t n_layers, int32_t n_kv_heads, int32_t head_dim,
                      const lkv_scorer* scorer, const void* k_new, const void* v_new, void* kp, void* vp, float* up,
                      const int32_t* cap_offsets, int32_t* lengths, int32_t* overflow, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (n_seq < 1 || n_layers < 1 || n_kv_heads < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "n_seq, n_layers and n_kv_heads must be >= 1");
  if (head_dim != lkv::kHeadDim) return fail(ctx, LKV_ERR_UNSUPPORTED, "head_dim must be 128, got %d", head_dim);
  const int64_t n_seg = (int64_t)n_seq * n_layers * n_kv_heads;
  if (n_seg > kMaxSegments) return fail(ctx, LKV_ERR_UNSUPPORTED, "too many segments");
  if (scorer == nullptr || k_new == nullptr || v_new == nullptr || kp == nullptr || vp == nullptr || up == nullptr ||
      cap_offsets == nullptr || lengths == nullptr)
    return fail(ctx, LKV_ERR_INVALID_ARG, "a required pointer is NULL");
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(kp) || !aligned16(vp))
    return fail(ctx, LKV_ERR_INVALID_ARG, "k_new, v_new, kp or vp is not 16-byte aligned");
  if (lkv_status st = check_scorer(ctx, scorer, false)) return st;
  lkv::launch_append((int)n_seg, n_layers * n_kv_heads, n_kv_heads, scorer->kind == LKV_SCORER_LINEAR ? 0 : 1,
                     scorer->act == LKV_ACT_SILU ? 0 : 1, scorer->hidden, scorer->per_head,
                     static_cast<const uint16_t*>(scorer->w1), scorer->b1, scorer->w2, scorer->b2, k_new, v_new, kp, vp,
                     up, cap_offsets, lengths, overflow, as_stream(stream));
  if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_append launch");
  return LKV_OK;
}

lkv_status lkv_decode_attn_grown(lkv_ctx* ctx, int32_t n_seq, int32_t n_layers, int32_t n_kv_heads,
                                 int32_t n_q_heads, int32_t head_dim, const void* q, const void* kp, const void* vp,
                                 const int32_t* cap_offsets, const int32_t* lengths, int64_t total_rows, float scale,
                                 float* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  int G = 0;
  int64_t n_seg = 0;
  if (lkv_status st = check_decode_geometry(ctx, n_seq, n_layers, n_kv_heads, n_q_heads, head_dim, &G, &n_seg)) return st;
  if (total_rows < 0 || total_rows >= (int64_t)1 << 31)
    return fail(ctx, LKV_ERR_INVALID_ARG, "total_rows = %lld is outside [0, 2^31)", (long long)total_rows);
  if (q == nullptr || cap_offsets == nullptr || lengths == nullptr || out == nullptr)
    return fail(ctx, LKV_ERR_INVALID_ARG, "q, cap_offsets, lengths or out is NULL");
  if (total_rows > 0 && (kp == nullptr || vp == nullptr)) return fail(ctx, LKV_ERR_INVALID_ARG, "kp or vp is NULL");
  if (!aligned16(q) || !aligned16(kp) || !aligned16(vp) || !aligned16(out))
    return fail(ctx, LKV_ERR_INVALID_ARG, "q, kp, vp or out is not 16-byte aligned");
  const size_t need = lkv::decode_workspace_bytes((int)n_seg, total_rows, G);
  if (lkv_status st = check_workspace(ctx, workspace, workspace_bytes, need, 256, "decode")) return st;
  if (hipError_t e = lkv::launch_decode(G, q, kp, vp, cap_offsets, lengths, (int)n_seg, total_rows, scale, out, lse,
                                        static_cast<float*>(workspace), as_stream(stream)))
    return hip_fail(ctx, e, "lkv_decode_attn_grown launch");
  return LKV_OK;
}

lkv_status lkv_reevict(lkv_ctx* ctx, int64_t n_segments, int32_t head_dim, const void* kp, const void* vp,
                       const float* up, const int32_t* cap_offsets, const int32_t* lengths,
                       const int32_t* lengths_host, const int32_t* new_budgets, int32_t slack, int32_t* idx,
                       int32_t* offsets, void* kp_new, void* vp_new, float* up_new, int32_t* cap_offsets_new,
                       int32_t* lengths_new, int64_t* total_kept, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (head_dim != lkv::kHeadDim) return fail(ctx, LKV_ERR_UNSUPPORTED, "head_dim must be 128, got %d", head_dim);
  if (n_segments < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "n_segments = %lld must be >= 1", (long long)n_segments);
  if (n_segments > kMaxSegments) return fail(ctx, LKV_ERR_UNSUPPORTED, "too many segments");
  if (cap_offsets == nullptr || lengths == nullptr || lengths_host == nullptr || new_budgets == nullptr ||
      offsets == nullptr || cap_offsets_new == nullptr || lengths_new == nullptr)
    return fail(ctx, LKV_ERR_INVALID_ARG, "a required pointer is NULL");
  if (slack < 0) return fail(ctx, LKV_ERR_INVALID_ARG, "slack = %d must be >= 0", slack);
  int64_t total = 0;
  int max_len = 1;
  for (int64_t i = 0; i < n_segments; ++i) {
    if (lengths_host[i] < 0) return fail(ctx, LKV_ERR_INVALID_ARG, "length %d of segment %lld is negative", lengths_host[i], (long long)i);
    if (new_budgets[i] < 0 || new_budgets[i] > lengths_host[i])
      return fail(ctx, LKV_ERR_INVALID_ARG, "new budget %d of segment %lld is outside [0, %d]", new_budgets[i],
                  (long long)i, lengths_host[i]);
    total += new_budgets[i];
    if (lengths_host[i] > max_len) max_len = lengths_host[i];
  }
  if (total + n_segments * slack >= (int64_t)1 << 31)
    return fail(ctx, LKV_ERR_UNSUPPORTED, "new cache of %lld rows >= 2^31", (long long)(total + n_segments * slack));
  if (total > 0 && (kp == nullptr || vp == nullptr || up == nullptr || idx == nullptr || kp_new == nullptr ||
                    vp_new == nullptr || up_new == nullptr))
    return fail(ctx, LKV_ERR_INVALID_ARG, "a cache, score or index buffer is NULL");
  if (!aligned16(kp) || !aligned16(vp) || !aligned16(kp_new) || !aligned16(vp_new))
    return fail(ctx, LKV_ERR_INVALID_ARG, "kp, vp, kp_new or vp_new is not 16-byte aligned");
  // tight offsets of the new budgets, the layout the selection writes its indices in
  if (lkv_status st = lkv_plan_offsets(ctx, n_segments, new_budgets, offsets, nullptr, stream)) return st;
  hipStream_t st = as_stream(stream);
  lkv::SeqTable tab;
  memset(&tab, 0, sizeof(tab));
  tab.T[0] = max_len;          // upper bound of every segment's length: sizes the LDS region
  tab.first[0] = 0;
  tab.first[1] = (int32_t)n_segments;
  tab.n = 1;
  lkv::launch_select(tab, nullptr, (int)n_segments, offsets, idx, 0, 0, st, up, cap_offsets, lengths);
  if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_reevict select launch");
  lkv::launch_compact_regrow(idx, offsets, (int)n_segments, total, slack, kp, vp, up, cap_offsets, lengths, kp_new, vp_new,
                             up_new, st);
  if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_reevict compact launch");
  lkv::launch_grown_layout(offsets, (int)n_segments, slack, cap_offsets_new, lengths_new, st);
  if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_reevict layout launch");
  if (total_kept != nullptr) *total_kept = total;
  return LKV_OK;
}

size_t lkv_masked_decode_workspace_bytes(const lkv_cache* cache) {
  if (cache == nullptr || cache->seq_len == nullptr || cache->n_seq < 1 || cache->n_layers < 1 ||
      cache->n_kv_heads < 1 || cache->n_q_heads < cache->n_kv_heads)
    return 0;
  const int heads = cache->n_layers * cache->n_kv_heads;
  size_t need = 0;
  for (int s = 0; s < cache->n_seq; ++s) {
    const size_t b = lkv::decode_workspace_bytes(heads, (int64_t)heads * cache->seq_len[s], cache->n_q_heads / cache->n_kv_heads);
    if (b > need) need = b;
  }
  return need + (((size_t)heads + 1) * sizeof(int32_t) + 255) / 256 * 256;
}

lkv_status lkv_masked_decode_attn(lkv_ctx* ctx, const lkv_cache* cache, const void* q, const float* const* mask,
                                  float scale, float* out, float* lse, void* workspace, size_t workspace_bytes,
                                  void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (lkv_status st = check_cache(ctx, cache, true)) return st;
  if (q == nullptr || mask == nullptr || out == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "q, mask or out is NULL");
  if (!aligned16(q) || !aligned16(out)) return fail(ctx, LKV_ERR_INVALID_ARG, "q or out is not 16-byte aligned");
  const int G = cache->n_q_heads / cache->n_kv_heads;
  if (G > lkv::kDecodeMaxGroup) return fail(ctx, LKV_ERR_UNSUPPORTED, "GQA group %d exceeds %d", G, lkv::kDecodeMaxGroup);
  const int heads = cache->n_layers * cache->n_kv_heads;
  for (int s = 0; s < cache->n_seq; ++s) {
    if (mask[s] == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "mask[%d] is NULL", s);
    if ((int64_t)heads * cache->seq_len[s] >= (int64_t)1 << 31)
      return fail(ctx, LKV_ERR_UNSUPPORTED, "sequence %d has 2^31 or more cache rows", s);
  }
  const size_t need = lkv_masked_decode_workspace_bytes(cache);
  if (lkv_status st = check_workspace(ctx, workspace, workspace_bytes, need, 256, "masked decode")) return st;
  const size_t off_bytes = (((size_t)heads + 1) * sizeof(int32_t) + 255) / 256 * 256;
  int32_t* offsets = static_cast<int32_t*>(workspace);
  float* ws = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + off_bytes);
  hipStream_t st = as_stream(stream);
  // the uncompacted cache of one sequence is a packed cache whose segments all have T rows
  for (int s = 0; s < cache->n_seq; ++s) {
    const int T = cache->seq_len[s];
    lkv::launch_uniform_offsets(heads, T, offsets, st);
    if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_masked_decode_attn offsets launch");
    const size_t qrow = (size_t)s * cache->n_layers * cache->n_q_heads;
    if (hipError_t e = lkv::launch_decode(G, static_cast<const uint16_t*>(q) + qrow * lkv::kHeadDim, cache->k[s],
                                          cache->v[s], offsets, nullptr, heads, (int64_t)heads * T, scale,
                                          out + qrow * lkv::kHeadDim, lse != nullptr ? lse + qrow : nullptr, ws, st,
                                          mask[s]))
      return hip_fail(ctx, e, "lkv_masked_decode_attn launch");
  }
  return LKV_OK;
}

lkv_status lkv_masked_attn_forward(lkv_ctx* ctx, int32_t n_q_heads, int32_t n_kv_heads, int32_t seq_len,
                                   int32_t head_dim, const void* q, const void* k, const void* v, const float* m,
                                   float scale, float* o, float* lse, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (lkv_status st = check_attention_geometry(ctx, n_q_heads, n_kv_heads, seq_len, head_dim, scale)) return st;
  if (q == nullptr || k == nullptr || v == nullptr || m == nullptr || o == nullptr || lse == nullptr)
    return fail(ctx, LKV_ERR_INVALID_ARG, "q, k, v, m, o or lse is NULL");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o))
    return fail(ctx, LKV_ERR_INVALID_ARG, "q, k, v or o is not 16-byte aligned");
  lkv::launch_masked_attn_fwd(q, k, v, m, n_q_heads, n_kv_heads, seq_len, scale, o, lse, as_stream(stream));
  if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_masked_attn_forward launch");
  return LKV_OK;
}

size_t lkv_masked_attn_backward_workspace_bytes(int32_t n_q_heads, int32_t n_kv_heads, int32_t seq_len) {
  if (n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads != 0 || seq_len < 1) return 0;
  return lkv::masked_attn_bwd_workspace_bytes(n_q_heads, n_kv_heads, seq_len);
}

lkv_status lkv_masked_attn_backward(lkv_ctx* ctx, int32_t n_q_heads, int32_t n_kv_heads, int32_t seq_len,
                                    int32_t head_dim, const void* q, const void* k, const void* v, const float* m,
                                    const float* o, const float* lse, const void* d_o, float scale, float* dq, float* dk,
                                    float* dv, float* dm, void* workspace, size_t workspace_bytes, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (lkv_status st = check_attention_geometry(ctx, n_q_heads, n_kv_heads, seq_len, head_dim, scale)) return st;
  if ((int64_t)n_q_heads * seq_len >= ((int64_t)1 << 31) * 16)
    return fail(ctx, LKV_ERR_UNSUPPORTED, "n_q_heads * seq_len is too large for one launch");
  if (q == nullptr || k == nullptr || v == nullptr || m == nullptr || o == nullptr || lse == nullptr || d_o == nullptr ||
      dq == nullptr || dk == nullptr || dv == nullptr || dm == nullptr)
    return fail(ctx, LKV_ERR_INVALID_ARG, "an input or output pointer is NULL");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o))
    return fail(ctx, LKV_ERR_INVALID_ARG, "q, k, v, o or d_o is not 16-byte aligned");
  const size_t need = lkv::masked_attn_bwd_workspace_bytes(n_q_heads, n_kv_heads, seq_len);
  if (lkv_status st = check_workspace(ctx, workspace, workspace_bytes, need, 16, "masked attention backward")) return st;
  lkv::launch_masked_attn_bwd(q, k, v, m, o, lse, d_o, n_q_heads, n_kv_heads, seq_len, scale, dq, dk, dv, dm,
                              static_cast<float*>(workspace), as_stream(stream));
  if (hipError_t e = hipGetLastError()) return hip_fail(ctx, e, "lkv_masked_attn_backward launch");
  return LKV_OK;
}

int32_t lkv_soft_topk_max_n(int32_t x_is_f64) { return lkv::soft_topk_max_n(x_is_f64 != 0); }

lkv_status lkv_soft_topk(lkv_ctx* ctx, const void* x, int32_t x_is_f64, int32_t n, double k, double tau, double* y,
                         double* info, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (x == nullptr || y == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "x or y is NULL");
  if (n < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "n = %d must be >= 1", n);
  if (!(k > 0.0) || !(k < (double)n)) return fail(ctx, LKV_ERR_INVALID_ARG, "k = %g must lie in the open interval (0, %d)", k, n);
  if (!(tau > 0.0) || std::isinf(tau)) return fail(ctx, LKV_ERR_INVALID_ARG, "tau = %g must be positive and finite", tau);
  if (n > lkv::soft_topk_max_n(x_is_f64 != 0))
    return fail(ctx, LKV_ERR_UNSUPPORTED, "n = %d exceeds the single-workgroup limit %d for this input type", n,
                lkv::soft_topk_max_n(x_is_f64 != 0));
  if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, LKV_ERR_HIP, "hipSetDevice failed");
  lkv::launch_soft_topk(x, x_is_f64 != 0, n, k, tau, y, info, nullptr, 0.0, as_stream(stream));
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e, "soft top-k launch");
  return LKV_OK;
}

lkv_status lkv_soft_topk_backward(lkv_ctx* ctx, const void* x, int32_t x_is_f64, int32_t n, double tau,
                                  const double* info, const double* g, double* dx, double* dk, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (x == nullptr || info == nullptr || g == nullptr || dx == nullptr)
    return fail(ctx, LKV_ERR_INVALID_ARG, "x, info, g or dx is NULL");
  if (n < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "n = %d must be >= 1", n);
  if (!(tau > 0.0) || std::isinf(tau)) return fail(ctx, LKV_ERR_INVALID_ARG, "tau = %g must be positive and finite", tau);
  if (n > lkv::soft_topk_max_n(x_is_f64 != 0))
    return fail(ctx, LKV_ERR_UNSUPPORTED, "n = %d exceeds the limit %d", n, lkv::soft_topk_max_n(x_is_f64 != 0));
  if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, LKV_ERR_HIP, "hipSetDevice failed");
  lkv::launch_soft_topk_backward(x, x_is_f64 != 0, n, tau, info, g, dx, dk, as_stream(stream));
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e, "soft top-k backward launch");
  return LKV_OK;
}

lkv_status lkv_soft_topk_batched(lkv_ctx* ctx, const void* x, int32_t x_is_f64, int32_t n_vec, int32_t n, const double* k,
                                 double tau, double* y, double* info, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (x == nullptr || y == nullptr || k == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "x, y or k is NULL");
  if (n < 2) return fail(ctx, LKV_ERR_INVALID_ARG, "n = %d must be >= 2", n);
  if (n_vec < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "n_vec = %d must be >= 1", n_vec);
  if (!(tau > 0.0) || std::isinf(tau)) return fail(ctx, LKV_ERR_INVALID_ARG, "tau = %g must be positive and finite", tau);
  if (n > lkv::soft_topk_max_n(x_is_f64 != 0))
    return fail(ctx, LKV_ERR_UNSUPPORTED, "n = %d exceeds the limit %d", n, lkv::soft_topk_max_n(x_is_f64 != 0));
  if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, LKV_ERR_HIP, "hipSetDevice failed");
  lkv::launch_soft_topk(x, x_is_f64 != 0, n, 0.0, tau, y, info, nullptr, 0.0, as_stream(stream), n_vec, k);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e, "batched soft top-k launch");
  return LKV_OK;
}

lkv_status lkv_soft_topk_backward_batched(lkv_ctx* ctx, const void* x, int32_t x_is_f64, int32_t n_vec, int32_t n,
                                          double tau, const double* info, const double* g, double* dx, double* dk,
                                          void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (x == nullptr || info == nullptr || g == nullptr || dx == nullptr)
    return fail(ctx, LKV_ERR_INVALID_ARG, "x, info, g or dx is NULL");
  if (n < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "n = %d must be >= 1", n);
  if (n_vec < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "n_vec = %d must be >= 1", n_vec);
  if (!(tau > 0.0) || std::isinf(tau)) return fail(ctx, LKV_ERR_INVALID_ARG, "tau = %g must be positive and finite", tau);
  if (n > lkv::soft_topk_max_n(x_is_f64 != 0))
    return fail(ctx, LKV_ERR_UNSUPPORTED, "n = %d exceeds the limit %d", n, lkv::soft_topk_max_n(x_is_f64 != 0));
  if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, LKV_ERR_HIP, "hipSetDevice failed");
  lkv::launch_soft_topk_backward(x, x_is_f64 != 0, n, tau, info, g, dx, dk, as_stream(stream), n_vec);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e, "batched soft top-k backward launch");
  return LKV_OK;
}

lkv_status lkv_head_budgets(lkv_ctx* ctx, const float* emb, const lkv_head_predictor* p, int32_t n_heads, double R,
                            int32_t t, double* r, int32_t* b, void* stream) {
  if (ctx == nullptr) return LKV_ERR_INVALID_ARG;
  if (emb == nullptr || p == nullptr || r == nullptr) return fail(ctx, LKV_ERR_INVALID_ARG, "emb, predictor or r is NULL");
  if (p->w1 == nullptr || p->b1 == nullptr || p->w2 == nullptr)
    return fail(ctx, LKV_ERR_INVALID_ARG, "predictor w1, b1 or w2 is NULL");
  if (n_heads < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "n_heads = %d must be >= 1", n_heads);
  if (p->d_e < 1 || p->hidden < 1) return fail(ctx, LKV_ERR_INVALID_ARG, "d_e and hidden must be >= 1");
  if (p->hidden > lkv::head_scores_max_hidden())
    return fail(ctx, LKV_ERR_UNSUPPORTED, "hidden = %d exceeds %d", p->hidden, lkv::head_scores_max_hidden());
  if (n_heads > lkv::soft_topk_max_n(true))
    return fail(ctx, LKV_ERR_UNSUPPORTED, "n_heads = %d exceeds %d", n_heads, lkv::soft_topk_max_n(true));
  // k = R L H must stay inside (0, n): the operator is undefined at the ends (App. A.1)
  const double k = R * (double)n_heads;
  if (!(k > 0.0) || !(k < (double)n_heads)) return fail(ctx, LKV_ERR_INVALID_ARG, "R = %g must lie in the open interval (0, 1)", R);
  if (b != nullptr && t < 0) return fail(ctx, LKV_ERR_INVALID_ARG, "t = %d must be >= 0", t);
  if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, LKV_ERR_HIP, "hipSetDevice failed");
  lkv::launch_head_scores(emb, p->w1, p->b1, p->w2, p->b2, n_heads, p->d_e, p->hidden, r, as_stream(stream));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e, "head score launch");
  lkv::launch_soft_topk(r, true, n_heads, k, 1.0, r, nullptr, b, (double)t, as_stream(stream));
  e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e, "soft top-k launch");
  return LKV_OK;
}

}  // extern "C"
