// Head-wise budgeted hard top-k: m = TopK(u, b) per KV head (Sec. 3.4 of the
// paper, inference), with the budget b an input (LKV-H, Sec. 3.3).
//
// One workgroup of 1024 threads per segment (sequence, layer, head).
//   1. Scores are mapped to order-preserving uint32 keys (NaN -> -inf first).
//   2. The key of the b-th largest score is found by a radix descent over the
//      key bits in three levels of 11, 11 and 10 bits: an LDS histogram of the
//      keys that still match the prefix, then a block-wide scan from the top
//      bin down.  This yields the threshold key `thr` and `need`, the number of
//      tokens equal to `thr` that are kept.
//   3. Emission in ascending token order: a token is kept if key > thr, or if
//      key == thr and fewer than `need` tokens with that key precede it.  Each
//      wave owns a contiguous range of tokens; per-wave counts are scanned once
//      across the block, then every wave writes its range using prefix counts.
//      The lower-index tie rule and the ascending output order both fall out of
//      this ordered scan; no atomic decides a position, so the result is unique
//      and reproducible bit for bit.
// Where the keys live depends on the head length T:
//   * T <= 34304: the keys are cached in LDS by one batched read of the scores (the first
//     level's histogram is counted on the way in); the later passes and the classification
//     read LDS, eight keys at a time.
//   * longer heads do not fit.  The first level reads the scores from memory (they sit in L2 /
//     the memory-side cache right after scoring).  A second read settles every token outside
//     the one undecided bin and lists the tokens inside it (up to 16384 indices, in the LDS the
//     emission stages through later); the last two levels and the final comparison touch the
//     listed tokens only.  If more tokens than that share the bin, all three levels and the
//     classification re-read the scores instead.
//   In every case each token is classified against `thr` into two LDS bitmaps (greater / equal)
//   and the ordered emission runs on the bitmaps, 1024 tokens per wave step: every lane expands
//   its 16 bits into the wave's LDS staging buffer at the position given by a prefix count, then
//   the wave copies the staged indices out with fully coalesced stores.
//   * T <= 327680 is the limit for the bitmaps; longer heads re-read the scores in order during
//     emission, 64 tokens a step.
// All global reads are issued eight at a time per thread before any is used: the kernel is
// latency-bound, not bandwidth-bound, so what counts is how few dependent round trips each pass
// makes.  A launch can also rank ragged pieces of one flat score array (the re-eviction of a
// packed cache) instead of the heads of a [L, H, T] tensor.
#include "lkv_common.h"

namespace lkv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelBins = 2048;
constexpr int kSelRegionBytes = 144 * 1024;                 // LDS after the histogram: key cache and/or bitmaps
constexpr int kSelMaxCachedKeys = 34304;                    // 134 KB of keys + 8.4 KB of bitmaps fit the region
constexpr int kSelStageWords = 1024;                        // staged indices per wave and step (one per token of the step)
constexpr int kSelStageBytes = kSelWaves * kSelStageWords * 4;   // 64 KB
constexpr int kSelCandCap = kSelStageBytes / 4;             // candidate tokens of a long head (they overlay the staging buffer)
constexpr int kSelMaxBitmapT = (kSelRegionBytes - kSelStageBytes) / 8 * 32;   // 327680 tokens: two bitmaps + staging
static_assert(kSelMaxCachedKeys * 4 + 2 * ((kSelMaxCachedKeys + 31) / 32) * 4 <= kSelRegionBytes, "key cache + bitmaps");
constexpr int kSelBatch = 8;                                // loads in flight per thread
constexpr int kSelInlineOffsets = 640;                      // offsets that fit the kernel arguments next to the launch table
constexpr int kSelSplitMaxHeads = 64;                       // launches with at most this many (long) heads split each head's pass
constexpr int kSelSplitTargetBlocks = 256;                  // over about this many workgroups in all,
constexpr int kSelSplitMax = 32;                            // at most this many per head

struct InlineOffsets {
  int32_t v[kSelInlineOffsets];
};

struct SelShared {
  uint32_t hist[kSelBins];
  uint32_t wave_tot[kSelWaves];
  uint32_t wave_gt[kSelWaves];
  uint32_t wave_eq[kSelWaves];
  uint32_t found_bin;
  uint32_t found_above;
  uint32_t found_count;
  uint32_t cand_count;
};

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t y = __shfl_up(x, d, 64);
    if (lane >= d) x += y;
  }
  return x;
}

// Sum of x over the 64 lanes of a wave, in every lane.
__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
  return x;
}

// Sum of the per-wave totals of the waves ahead of `wave`: one LDS read per lane and a wave
// reduction instead of a chain of dependent reads.
__device__ __forceinline__ uint32_t waves_before(const uint32_t* totals, int wave, int lane) {
  return wave_sum(lane < wave ? totals[lane] : 0u);
}

// Calls f(key, token) for every token of the head, in no particular order, reading the fp32
// scores from global memory with kSelBatch loads in flight per thread (16-byte loads when the
// head is 16-byte aligned and its length a multiple of four).
template <typename F>
__device__ __forceinline__ void for_each_global_key(const float* __restrict__ u, int T, F f) {
  const int tid = threadIdx.x;
  if ((T & 3) == 0 && (reinterpret_cast<uintptr_t>(u) & 15u) == 0) {
    const float4* u4 = reinterpret_cast<const float4*>(u);
    const int n4 = T >> 2;
    for (int base = tid; base < n4; base += kSelThreads * kSelBatch) {
      float4 v[kSelBatch];
#pragma unroll
      for (int k = 0; k < kSelBatch; ++k) {
        const int i = base + k * kSelThreads;
        v[k] = u4[i < n4 ? i : base];
      }
#pragma unroll
      for (int k = 0; k < kSelBatch; ++k) {
        const int i = base + k * kSelThreads;
        if (i < n4) {
          f(order_key(v[k].x), 4 * i);
          f(order_key(v[k].y), 4 * i + 1);
          f(order_key(v[k].z), 4 * i + 2);
          f(order_key(v[k].w), 4 * i + 3);
        }
      }
    }
  } else {
    for (int base = tid; base < T; base += kSelThreads * kSelBatch) {
      float v[kSelBatch];
#pragma unroll
      for (int k = 0; k < kSelBatch; ++k) {
        const int i = base + k * kSelThreads;
        v[k] = u[i < T ? i : base];
      }
#pragma unroll
      for (int k = 0; k < kSelBatch; ++k) {
        const int i = base + k * kSelThreads;
        if (i < T) f(order_key(v[k]), i);
      }
    }
  }
}

// One level of the radix descent.  `count(fn)` must call fn(key) for every key of the head.
// On return prefix / prefix_mask / need are advanced by this level's digit.  Returns the number of
// keys in the bin the descent entered (the same value in every thread: it is published by the one
// thread that found the bin and read between two block barriers, so a branch on it is uniform).
// `counted`: the histogram of this level has already been filled (and a barrier passed).
template <typename Count>
__device__ __forceinline__ uint32_t descend_level(SelShared& sh, int level, uint32_t& prefix, uint32_t& prefix_mask,
                                              uint32_t& need, Count count, bool counted = false) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int shift = level == 0 ? 21 : (level == 1 ? 10 : 0);
  const int nbins = level == 2 ? 1024 : 2048;
  if (!counted) {
    for (int i = tid; i < kSelBins; i += kSelThreads) sh.hist[i] = 0;
    __syncthreads();   // also orders an LDS key cache fill before its first use
    const uint32_t pfx = prefix, msk = prefix_mask;
    count([&](uint32_t key) {
      if ((key & msk) == pfx) atomicAdd(&sh.hist[(key >> shift) & (nbins - 1)], 1u);
    });
    __syncthreads();
  }
  // scan the bins from the top: thread t owns bins nbins-1-2t and nbins-2-2t
  uint32_t c0 = 0, c1 = 0;
  const int top = nbins - 1 - 2 * tid;
  if (top >= 0) c0 = sh.hist[top];
  if (top - 1 >= 0) c1 = sh.hist[top - 1];
  const uint32_t incl = wave_inclusive_scan(c0 + c1, lane);
  if (lane == 63) sh.wave_tot[wave] = incl;
  __syncthreads();
  const uint32_t before = waves_before(sh.wave_tot, wave, lane);
  const uint32_t excl = before + incl - (c0 + c1);   // keys in bins above this thread's pair
  // exactly one bin satisfies: above < need <= above + count
  if (c0 && excl < need && need <= excl + c0) { sh.found_bin = (uint32_t)top; sh.found_above = excl; sh.found_count = c0; }
  if (c1 && excl + c0 < need && need <= excl + c0 + c1) {
    sh.found_bin = (uint32_t)(top - 1);
    sh.found_above = excl + c0;
    sh.found_count = c1;
  }
  __syncthreads();
  prefix |= sh.found_bin << shift;
  prefix_mask |= (uint32_t)(nbins - 1) << shift;
  need -= sh.found_above;
  const uint32_t in_bin = sh.found_count;
  __syncthreads();   // found_* and hist are rewritten at the next level
  return in_bin;
}

// Ordered emission from a per-token key source `key_of(i)` (LDS key cache, or global scores).
template <typename KeyOf>
__device__ __forceinline__ void emit_from_keys(SelShared& sh, int T, uint32_t thr, uint32_t need,
                                               int32_t* __restrict__ out, KeyOf key_of) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  // wave w owns tokens [w*per, (w+1)*per), per a multiple of 64
  const int per = ((T + kSelWaves - 1) / kSelWaves + 63) & ~63;
  const int lo = wave * per;
  const int hi = min(T, lo + per);
  uint32_t n_gt = 0, n_eq = 0;
  for (int base = lo; base < hi; base += 64) {
    const int i = base + lane;
    const bool in = i < hi;
    const uint32_t key = in ? key_of(i) : 0u;
    n_gt += __popcll(__ballot(in && key > thr));
    n_eq += __popcll(__ballot(in && key == thr));
  }
  if (lane == 0) { sh.wave_gt[wave] = n_gt; sh.wave_eq[wave] = n_eq; }
  __syncthreads();
  const uint32_t gt_before = waves_before(sh.wave_gt, wave, lane);
  const uint32_t eq_before = waves_before(sh.wave_eq, wave, lane);
  uint32_t eq_seen = eq_before;                                  // copies of thr before the current 64 tokens
  uint32_t pos = gt_before + min(eq_before, need);               // kept tokens before the current 64 tokens
  for (int base = lo; base < hi; base += 64) {
    const int i = base + lane;
    const bool in = i < hi;
    const uint32_t key = in ? key_of(i) : 0u;
    const bool is_eq = in && key == thr;
    const unsigned long long eq_mask = __ballot(is_eq);
    const unsigned long long below = (1ull << lane) - 1ull;
    const uint32_t eq_rank = eq_seen + __popcll(eq_mask & below);
    const bool keep = in && (key > thr || (is_eq && eq_rank < need));
    const unsigned long long keep_mask = __ballot(keep);
    if (keep) out[pos + __popcll(keep_mask & below)] = i;
    pos += __popcll(keep_mask);
    eq_seen += __popcll(eq_mask);
  }
}

// The `k` lowest set bits of x (k <= popcount(x)); a fixed five-step search, no lane divergence.
__device__ __forceinline__ uint32_t lowest_set_bits(uint32_t x, uint32_t k) {
  if (k >= (uint32_t)__popc(x)) return x;
  // smallest m in [0, 31] with popcount(x & ((1 << m) - 1)) >= k  (m = 0 when k = 0)
  int lo = -1, hi = 31;   // invariant: the prefix of length hi holds >= k bits, that of length lo (if >= 0) fewer
#pragma unroll
  for (int it = 0; it < 5; ++it) {
    const int mid = (lo + hi + 1) >> 1;
    if ((uint32_t)__popc(x & ((1u << mid) - 1u)) >= k) hi = mid; else lo = mid;
  }
  return x & ((1u << hi) - 1u);
}

__device__ __forceinline__ void wave_lds_sync() {
  // orders this wave's LDS writes and reads of its private staging; no block barrier needed
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Ordered emission from the two LDS bitmaps (bit i of gt: key_i > thr; of eq: key_i == thr).
// Each wave owns a contiguous range of bitmap words and handles 32 words (1024 tokens) per step,
// one 16-bit half word per lane.  Loops whose trip count could differ between lanes are avoided
// (the expansion loop runs a fixed 16 times), and every cross-lane exchange of a step comes
// before the staging traffic.
__device__ __forceinline__ void emit_from_bitmaps(SelShared& sh, int T, uint32_t need, int32_t* __restrict__ out,
                                                  const uint32_t* gt_map, const uint32_t* eq_map, uint32_t* stage_all) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  uint32_t* stage = stage_all + wave * kSelStageWords;
  const int n_words = (T + 31) >> 5;
  const int per = ((n_words + kSelWaves - 1) / kSelWaves + 31) & ~31;   // words per wave, a multiple of 32
  const int lo = wave * per;
  const int hi = min(n_words, lo + per);
  uint32_t n_gt = 0, n_eq = 0;
  for (int w = lo + lane; w < hi; w += 64) { n_gt += __popc(gt_map[w]); n_eq += __popc(eq_map[w]); }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) { n_gt += __shfl_xor(n_gt, d, 64); n_eq += __shfl_xor(n_eq, d, 64); }
  if (lane == 0) { sh.wave_gt[wave] = n_gt; sh.wave_eq[wave] = n_eq; }
  __syncthreads();
  const uint32_t gt_before = waves_before(sh.wave_gt, wave, lane);
  const uint32_t eq_before = waves_before(sh.wave_eq, wave, lane);
  uint32_t eq_seen = eq_before;
  uint32_t pos = gt_before + min(eq_before, need);
  const int half = lane & 1;
  for (int base = lo; base < hi; base += 32) {
    const int w = base + (lane >> 1);
    const bool in = w < hi;
    const uint32_t gth = in ? (gt_map[w] >> (16 * half)) & 0xffffu : 0u;
    const uint32_t eqh = in ? (eq_map[w] >> (16 * half)) & 0xffffu : 0u;
    // copies of thr before this lane's half word, and how many of its own copies are still kept
    const uint32_t eq_cnt = __popc(eqh);
    const uint32_t eq_incl = wave_inclusive_scan(eq_cnt, lane);
    const uint32_t eq_rank = eq_seen + eq_incl - eq_cnt;
    const uint32_t take = eq_rank < need ? min(eq_cnt, need - eq_rank) : 0u;
    uint32_t bits = gth | lowest_set_bits(eqh, take);
    const uint32_t cnt = __popc(bits);
    const uint32_t incl = wave_inclusive_scan(cnt, lane);
    const uint32_t total = (uint32_t)__builtin_amdgcn_readfirstlane((int)__shfl(incl, 63, 64));
    eq_seen += __shfl(eq_incl, 63, 64);
    uint32_t p = incl - cnt;
    const uint32_t tok0 = ((uint32_t)w << 5) + 16u * half;
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      if (bits) {
        stage[p++] = tok0 + __builtin_ctz(bits);
        bits &= bits - 1;
      }
    }
    wave_lds_sync();
    for (uint32_t j0 = 0; j0 < total; j0 += 64) {   // uniform trip count
      const uint32_t j = j0 + lane;
      if (j < total) out[pos + j] = stage[j];
    }
    pos += total;
    wave_lds_sync();   // the staging buffer is rewritten by the next step
  }
}

// Up to kSelInlineOffsets segment offsets travel in the kernel arguments instead of through a
// host-to-device copy (which costs an extra dependent transfer before the kernel can start);
// the blocks then also publish them to the device array that the later calls read.
// Segments that are not heads of a [L, H, T] score tensor but ragged pieces of one flat array
// (re-eviction of a packed cache): segment s has len[s] scores starting at flat[start[s]].
struct SelRagged {
  const float* flat;      // null: the launch table describes the scores
  const int32_t* start;
  const int32_t* len;
};

// kCounted: the first-level digits of every segment's scores have already been counted by the scoring launch
// (`counts`: uint32 [segments][kLevel0Bins]); the block takes its histogram from there instead of from a pass over
// the scores, and leaves the counters zero for the next scoring launch.
template <bool kInline, bool kCounted>
__global__ void __launch_bounds__(kSelThreads)
select_kernel(SeqTable tab, InlineOffsets inl, SelRagged ragged, int32_t* __restrict__ offsets, int32_t* __restrict__ idx,
              uint32_t* __restrict__ counts,
              const uint32_t* __restrict__ pre_maps /* per segment [2][pre_words]: written by select_classify_kernel, or null */,
              int pre_words,
              int seg_base, int seg_stride /* global segment = seg_base + sequence * seg_stride + head */,
              int cached_limit /* heads of at most this many tokens use the LDS key cache */,
              int bitmap_limit /* longer heads up to this many tokens use the LDS bitmaps */,
              int cached_stage_off, int bitmap_stage_off /* word offsets of the staging buffer in the region */) {
  extern __shared__ __align__(16) unsigned char smem[];
  SelShared& sh = *reinterpret_cast<SelShared*>(smem);
  uint32_t* region = reinterpret_cast<uint32_t*>(smem + sizeof(SelShared));

  const int tid = threadIdx.x;
  const int local_seg = blockIdx.x;
  const int seq = seq_of_unit(tab, local_seg);
  const int lh = local_seg - tab.first[seq];
  const int seg = seg_base + seq * seg_stride + lh;
  // a ragged segment can be no longer than the launch table says (the LDS region is sized by it)
  const int T = ragged.flat != nullptr ? min(ragged.len[seg], tab.T[seq]) : tab.T[seq];
  const float* u = ragged.flat != nullptr ? ragged.flat + ragged.start[seg] : tab.scores[seq] + (size_t)lh * (size_t)T;
  const int off = kInline ? inl.v[seg] : offsets[seg];
  const int budget = (kInline ? inl.v[seg + 1] : offsets[seg + 1]) - off;
  if (kInline && tid == 0) {
    offsets[seg] = off;
    if (local_seg == (int)gridDim.x - 1) offsets[seg + 1] = off + budget;   // the total, by the launch's last block
  }
  int32_t* out = idx + off;
  uint32_t* my_counts = kCounted ? counts + (size_t)seg * kLevel0Bins : nullptr;
  if (budget <= 0 || budget >= T) {   // nothing or everything is kept
    if (kCounted)
      for (int i = tid; i < kLevel0Bins; i += kSelThreads) my_counts[i] = 0;
    if (budget > 0)
      for (int i = tid; i < T; i += kSelThreads) out[i] = i;
    return;
  }
  if (kCounted) {
    for (int i = tid; i < kSelBins; i += kSelThreads) {
      sh.hist[i] = my_counts[i];
      my_counts[i] = 0;
    }
    __syncthreads();
  }

  uint32_t prefix = 0;        // bits of the threshold key decided so far
  uint32_t prefix_mask = 0;   // which bits those are
  uint32_t need = (uint32_t)budget;   // rank of the threshold among keys that match the prefix (1-based)

  if (T <= cached_limit) {
    uint32_t* keys = region;
    const int n_words = (T + 31) >> 5;
    uint32_t* gt_map = region + cached_limit;   // after the key cache of the launch's longest cached head
    uint32_t* eq_map = gt_map + n_words;
    // the first level's histogram is counted while the keys pass through registers on their way to LDS
    // (unless the scoring launch has counted it already)
    if (kCounted) {
      for_each_global_key(u, T, [&](uint32_t key, int i) { keys[i] = key; });
    } else {
      for (int i = tid; i < kSelBins; i += kSelThreads) sh.hist[i] = 0;
      __syncthreads();
      for_each_global_key(u, T, [&](uint32_t key, int i) {
        keys[i] = key;
        atomicAdd(&sh.hist[key >> 21], 1u);
      });
    }
    __syncthreads();
    // later levels read the cached keys eight at a time so that the LDS latency is paid once per batch
    auto count = [&](auto fn) {
      for (int base = tid; base < T; base += kSelThreads * kSelBatch) {
        uint32_t kb[kSelBatch];
#pragma unroll
        for (int k = 0; k < kSelBatch; ++k) {
          const int i = base + k * kSelThreads;
          kb[k] = keys[i < T ? i : base];
        }
#pragma unroll
        for (int k = 0; k < kSelBatch; ++k)
          if (base + k * kSelThreads < T) fn(kb[k]);
      }
    };
    descend_level(sh, 0, prefix, prefix_mask, need, count, true);
#pragma unroll 1
    for (int level = 1; level < 3; ++level) descend_level(sh, level, prefix, prefix_mask, need, count);
    const uint32_t thr = prefix;
    // classification: a wave covers 64 consecutive tokens, so a ballot is two finished bitmap
    // words.  The words of 32 rounds are collected in registers (lane 2k + j keeps half j of round
    // k) and written with one LDS store per lane and map.
    const int lane = tid & 63;
    const int wave = tid >> 6;
    constexpr int kClsBatch = 4;
    for (int chunk0 = 0; chunk0 < T; chunk0 += 32 * kSelThreads) {   // one pass for every length the cache holds up to 32768
      uint32_t my_gt = 0, my_eq = 0;
      const int rounds = min(32, (T - chunk0 + kSelThreads - 1) / kSelThreads);   // short heads need fewer
#pragma unroll 1
      for (int kk = 0; kk < rounds; kk += kClsBatch) {
        uint32_t kb[kClsBatch];
#pragma unroll
        for (int k = 0; k < kClsBatch; ++k) {
          const int i = chunk0 + (kk + k) * kSelThreads + wave * 64 + lane;
          kb[k] = i < T ? keys[i] : 0u;
        }
#pragma unroll
        for (int k = 0; k < kClsBatch; ++k) {
          const int i = chunk0 + (kk + k) * kSelThreads + wave * 64 + lane;
          const unsigned long long m_gt = __ballot(i < T && kb[k] > thr);
          const unsigned long long m_eq = __ballot(i < T && kb[k] == thr);
          const int slot = 2 * (kk + k);
          if (lane == slot) { my_gt = (uint32_t)m_gt; my_eq = (uint32_t)m_eq; }
          if (lane == slot + 1) { my_gt = (uint32_t)(m_gt >> 32); my_eq = (uint32_t)(m_eq >> 32); }
        }
      }
      const int w = ((chunk0 + (lane >> 1) * kSelThreads + wave * 64) >> 5) + (lane & 1);
      if (w < n_words) { gt_map[w] = my_gt; eq_map[w] = my_eq; }
    }
    __syncthreads();
    emit_from_bitmaps(sh, T, need, out, gt_map, eq_map, region + cached_stage_off);   // the key cache is dead by now
    return;
  }

  auto count = [&](auto fn) { for_each_global_key(u, T, [&](uint32_t key, int) { fn(key); }); };
  const uint32_t n_cand = descend_level(sh, 0, prefix, prefix_mask, need, count, kCounted);   // keys left in the undecided bin
  // Heads too long for the key cache: the first level leaves one bin of 2048 undecided.  When its
  // keys are few enough to list (their token indices, in the space the emission stages through
  // later), one more pass over the scores settles everything above that bin and collects the
  // list; the remaining two levels and the final comparison then touch the listed tokens only.
  const uint32_t bin0 = prefix >> 21;
  if (T <= bitmap_limit && n_cand <= (uint32_t)kSelCandCap) {
    const int n_words = (T + 31) >> 5;
    uint32_t* gt_map = region;
    uint32_t* eq_map = region + n_words;
    uint32_t* cand = region + bitmap_stage_off;
    if (kCounted && pre_maps != nullptr) {
      // the pass over the scores has been done by the blocks of select_classify_kernel: take its two bitmaps
      // (above the undecided bin / inside it) and list the tokens inside
      const uint32_t* pre_gt = pre_maps + (size_t)seg * 2 * pre_words;
      const uint32_t* pre_in = pre_gt + pre_words;
      for (int i = tid; i < n_words; i += kSelThreads) { gt_map[i] = pre_gt[i]; eq_map[i] = 0; }
      if (tid == 0) sh.cand_count = 0;
      __syncthreads();
      for (int w0 = 0; w0 < n_words; w0 += kSelThreads) {   // uniform trip counts, here and in the inner loop
        const int w = w0 + tid;
        uint32_t bits = w < n_words ? pre_in[w] : 0u;
        while (__ballot(bits != 0u) != 0ull) {
          if (bits) {
            const uint32_t slot = atomicAdd(&sh.cand_count, 1u);
            if (slot < (uint32_t)kSelCandCap) cand[slot] = ((uint32_t)w << 5) + (uint32_t)__builtin_ctz(bits);
            bits &= bits - 1;
          }
        }
      }
      __syncthreads();
    } else {
      for (int i = tid; i < 2 * n_words; i += kSelThreads) region[i] = 0;
      if (tid == 0) sh.cand_count = 0;
      __syncthreads();
      for_each_global_key(u, T, [&](uint32_t key, int i) {
        const uint32_t top = key >> 21;
        if (top > bin0) {
          atomicOr(&gt_map[i >> 5], 1u << (i & 31));
        } else if (top == bin0) {
          // (handing out slots per wave with a ballot was measured slower than the plain atomic)
          const uint32_t slot = atomicAdd(&sh.cand_count, 1u);
          if (slot < (uint32_t)kSelCandCap) cand[slot] = (uint32_t)i;
        }
      });
      __syncthreads();
    }
    auto count_listed = [&](auto fn) {
      for (uint32_t j = tid; j < n_cand; j += kSelThreads) fn(order_key(u[cand[j]]));
    };
#pragma unroll 1
    for (int level = 1; level < 3; ++level) descend_level(sh, level, prefix, prefix_mask, need, count_listed);
    const uint32_t thr_listed = prefix;
    for (uint32_t j = tid; j < n_cand; j += kSelThreads) {
      const uint32_t i = cand[j];
      const uint32_t key = order_key(u[i]);
      if (key > thr_listed) atomicOr(&gt_map[i >> 5], 1u << (i & 31));
      else if (key == thr_listed) atomicOr(&eq_map[i >> 5], 1u << (i & 31));
    }
    __syncthreads();   // the list is dead: its space becomes the staging buffer
    emit_from_bitmaps(sh, T, need, out, gt_map, eq_map, region + bitmap_stage_off);
    return;
  }
#pragma unroll 1
  for (int level = 1; level < 3; ++level) descend_level(sh, level, prefix, prefix_mask, need, count);
  const uint32_t thr = prefix;   // full 32-bit key of the budget-th largest score; keep `need` of its copies

  if (T <= bitmap_limit) {
    const int n_words = (T + 31) >> 5;
    uint32_t* gt_map = region;
    uint32_t* eq_map = region + n_words;
    for (int i = tid; i < 2 * n_words; i += kSelThreads) region[i] = 0;
    __syncthreads();
    for_each_global_key(u, T, [&](uint32_t key, int i) {
      if (key > thr) atomicOr(&gt_map[i >> 5], 1u << (i & 31));
      else if (key == thr) atomicOr(&eq_map[i >> 5], 1u << (i & 31));
    });
    __syncthreads();
    emit_from_bitmaps(sh, T, need, out, gt_map, eq_map, region + bitmap_stage_off);
  } else {
    emit_from_keys(sh, T, thr, need, out, [&](int i) { return order_key(u[i]); });
  }
}


// First half of a top-k whose heads are split over several workgroups (launches over few, long heads: one layer at
// a time).  Needs the first-level counts of the scoring launch.  Every block finds the undecided first-level bin of
// its head from the counts (a 2048-bin scan, repeated in each block rather than communicated) and classifies its
// slice of the scores against it into two global bitmaps: above the bin (kept for certain), and inside it (the
// candidates the remaining two levels choose from).  select_kernel then starts from the bitmaps instead of passing
// over the scores.  The counters are left as they are (select_kernel reads them again and zeroes them).  A head
// whose undecided bin holds more tokens than select_kernel can list is skipped here and takes the unsplit route there.
__global__ void __launch_bounds__(kSelThreads)
select_classify_kernel(SeqTable tab, const int32_t* __restrict__ offsets, const uint32_t* __restrict__ counts,
                       uint32_t* __restrict__ pre_maps, int pre_words, int seg_base, int seg_stride, int split) {
  __shared__ SelShared sh;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int local_seg = blockIdx.x / split;
  const int part = blockIdx.x - local_seg * split;
  const int seq = seq_of_unit(tab, local_seg);
  const int lh = local_seg - tab.first[seq];
  const int seg = seg_base + seq * seg_stride + lh;
  const int T = tab.T[seq];
  const float* u = tab.scores[seq] + (size_t)lh * (size_t)T;
  const int budget = offsets[seg + 1] - offsets[seg];
  if (budget <= 0 || budget >= T) return;
  const uint32_t* my_counts = counts + (size_t)seg * kLevel0Bins;
  for (int i = tid; i < kSelBins; i += kSelThreads) sh.hist[i] = my_counts[i];
  __syncthreads();
  uint32_t prefix = 0, prefix_mask = 0, need = (uint32_t)budget;
  const uint32_t n_cand = descend_level(sh, 0, prefix, prefix_mask, need, [](auto) {}, true);
  if (n_cand > (uint32_t)kSelCandCap) return;
  const uint32_t bin0 = prefix >> 21;
  uint32_t* out_gt = pre_maps + (size_t)seg * 2 * pre_words;
  uint32_t* out_in = out_gt + pre_words;
  // slices of whole 64-token groups (two bitmap words per wave step)
  const int groups = (T + 63) >> 6;
  const int per = (groups + split - 1) / split;
  const int g_lo = part * per, g_hi = min(groups, g_lo + per);
  constexpr int kU = 4;
  for (int g0 = g_lo + wave; g0 < g_hi; g0 += kSelWaves * kU) {
    float v[kU];
#pragma unroll
    for (int k = 0; k < kU; ++k) {
      const int i = (g0 + k * kSelWaves) * 64 + lane;
      v[k] = u[i < T ? i : T - 1];
    }
#pragma unroll
    for (int k = 0; k < kU; ++k) {
      const int g = g0 + k * kSelWaves;
      const int i = g * 64 + lane;
      const uint32_t top = order_key(v[k]) >> 21;
      const bool in = g < g_hi && i < T;
      const unsigned long long m_gt = __ballot(in && top > bin0);
      const unsigned long long m_in = __ballot(in && top == bin0);
      if (g < g_hi && lane < 2) {
        const int w = 2 * g + lane;
        if (w < pre_words) {
          out_gt[w] = (uint32_t)(m_gt >> (32 * lane));
          out_in[w] = (uint32_t)(m_in >> (32 * lane));
        }
      }
    }
  }
}

hipError_t select_prepare() {
  const int lds = (int)(sizeof(SelShared) + (size_t)kSelRegionBytes);
  const void* kernels[] = {reinterpret_cast<const void*>(select_kernel<false, false>),
                           reinterpret_cast<const void*>(select_kernel<true, false>),
                           reinterpret_cast<const void*>(select_kernel<false, true>),
                           reinterpret_cast<const void*>(select_kernel<true, true>)};
  for (const void* k : kernels)
    if (hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds)) return e;
  return hipSuccess;
}

int select_inline_capacity() { return kSelInlineOffsets; }
int select_max_bitmap_tokens() { return kSelMaxBitmapT; }

// `host_offsets` non-null: all n_total_segments + 1 offsets are passed in the kernel arguments
// (n_total_segments < kSelInlineOffsets) and the kernel writes the device array; null: the
// device array has already been filled.
void launch_select(const SeqTable& tab, const int32_t* host_offsets, int n_total_segments, int32_t* offsets,
                   int32_t* idx, int seg_base, int seg_stride, hipStream_t stream, const float* ragged_scores,
                   const int32_t* ragged_start, const int32_t* ragged_len, uint32_t* counts, uint32_t* pre_maps,
                   int pre_words) {
  const int segs = tab.first[tab.n];
  if (segs <= 0) return;
  // the LDS region is sized for the longest sequence of this launch that can use it
  int cached_limit = 0, bitmap_limit = 0;
  for (int i = 0; i < tab.n; ++i) {
    const int T = tab.T[i];
    if (T <= kSelMaxCachedKeys) { if (T > cached_limit) cached_limit = T; }
    else if (T <= kSelMaxBitmapT) { if (T > bitmap_limit) bitmap_limit = T; }
  }
  // Region layout.  Cached heads: key cache of the longest one, then two bitmaps; the staging
  // buffer of the emission overlays the (by then dead) key cache when that is large enough,
  // else it follows the bitmaps.  Longer heads: two bitmaps, then the staging buffer.
  const size_t cached_words = cached_limit > 0 ? (size_t)cached_limit + 2 * (size_t)((cached_limit + 31) / 32) : 0;
  const bool overlay = (size_t)cached_limit * 4 >= (size_t)kSelStageBytes;
  const size_t cached_stage_off = overlay ? 0 : cached_words;
  size_t region = cached_limit > 0 ? (overlay ? cached_words * 4 : cached_words * 4 + kSelStageBytes) : 0;
  const size_t bitmap_stage_off = 2 * (size_t)((bitmap_limit + 31) / 32);
  if (bitmap_limit > 0 && bitmap_stage_off * 4 + kSelStageBytes > region) region = bitmap_stage_off * 4 + kSelStageBytes;
  const SelRagged ragged = {ragged_scores, ragged_start, ragged_len};
  InlineOffsets inl = {};
  if (host_offsets != nullptr)
    for (int i = 0; i <= n_total_segments; ++i) inl.v[i] = host_offsets[i];
  const dim3 grid(segs), block(kSelThreads);
  const size_t lds = sizeof(SelShared) + region;
  // Few long heads (a layer at a time): split the pass over the scores of every head over several workgroups first.
  // Needs the first-level counts, room for the two bitmaps, heads too long for the key cache and offsets on the device.
  bool split_heads = counts != nullptr && pre_maps != nullptr && host_offsets == nullptr && ragged_scores == nullptr &&
                     cached_limit == 0 && bitmap_limit > 0 && segs <= kSelSplitMaxHeads;
  for (int i = 0; i < tab.n && split_heads; ++i)
    if (tab.T[i] > kSelMaxBitmapT || (tab.T[i] + 31) / 32 > pre_words) split_heads = false;
  if (split_heads) {
    int split = kSelSplitTargetBlocks / segs;
    split = split > kSelSplitMax ? kSelSplitMax : split;
    hipLaunchKernelGGL(select_classify_kernel, dim3(segs * split), block, 0, stream, tab, offsets, counts, pre_maps,
                       pre_words, seg_base, seg_stride, split);
  } else {
    pre_maps = nullptr;
  }
#define LKV_SELECT_LAUNCH(kInline, kCounted)                                                                          \
  hipLaunchKernelGGL((select_kernel<kInline, kCounted>), grid, block, lds, stream, tab, inl, ragged, offsets, idx,     \
                     counts, pre_maps, pre_words, seg_base, seg_stride, cached_limit, bitmap_limit,                    \
                     (int)cached_stage_off, (int)bitmap_stage_off)
  if (host_offsets != nullptr) {
    if (counts != nullptr) LKV_SELECT_LAUNCH(true, true); else LKV_SELECT_LAUNCH(true, false);
  } else {
    if (counts != nullptr) LKV_SELECT_LAUNCH(false, true); else LKV_SELECT_LAUNCH(false, false);
  }
#undef LKV_SELECT_LAUNCH
}

}  // namespace lkv
