// Head-wise budgeted hard top-k: m = TopK(u, b) per KV head (Sec. 3.4 of the
// paper, inference), with the budget b an input (LKV-H, Sec. 3.3).
//
// One workgroup of 1024 threads per segment (sequence, layer, head).
//   1. Scores are mapped to order-preserving uint32 keys (NaN -> -inf first).
//      If the head fits, the keys are cached in LDS and every later pass reads
//      LDS; otherwise the passes re-read the fp32 scores from L2 / memory.
//   2. The key of the b-th largest score is found by a radix descent over the
//      key bits in three levels of 11, 11 and 10 bits: an LDS histogram of the
//      keys that still match the prefix, then a block-wide scan from the top
//      bin down.  This yields the threshold key `thr` and `need`, the number of
//      tokens equal to `thr` that are kept.
//   3. Emission in ascending token order: a token is kept if key > thr, or if
//      key == thr and fewer than `need` tokens with that key precede it.  Each
//      wave owns a contiguous range of tokens; per-wave counts are scanned once
//      across the block, then every wave writes its range using ballot prefix
//      counts.  The lower-index tie rule and the ascending output order both
//      fall out of this ordered scan; no atomics decide placement, so the
//      result is unique and reproducible bit for bit.
#include "lkv_common.h"

namespace lkv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelBins = 2048;
constexpr int kSelMaxCachedKeys = 36864;   // 144 KB of keys; with histogram and scan scratch < 160 KB LDS

__device__ __forceinline__ uint32_t order_key(float u) {
  uint32_t bits = __float_as_uint(u);
  if ((bits & 0x7fffffffu) > 0x7f800000u) bits = 0xff800000u;   // NaN ranks as -inf
  return (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
}

struct SelShared {
  uint32_t hist[kSelBins];
  uint32_t wave_tot[kSelWaves];
  uint32_t wave_gt[kSelWaves];
  uint32_t wave_eq[kSelWaves];
  uint32_t found_bin;
  uint32_t found_above;
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

template <bool kCached>
__device__ __forceinline__ uint32_t key_at(const uint32_t* keys_lds, const float* u, int i) {
  if (kCached) return keys_lds[i];
  return order_key(u[i]);
}

template <bool kCached>
__device__ void select_body(const float* __restrict__ u, int T, int budget, int32_t* __restrict__ out,
                            SelShared& sh, uint32_t* keys_lds) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;

  if (kCached) {
    for (int i = tid; i < T; i += kSelThreads) keys_lds[i] = order_key(u[i]);
  }

  // ---- radix descent for the threshold key ---------------------------------
  uint32_t prefix = 0;        // bits of the threshold key decided so far
  uint32_t prefix_mask = 0;   // which bits those are
  uint32_t need = (uint32_t)budget;   // rank of the threshold among keys that match the prefix (1-based)
#pragma unroll 1
  for (int level = 0; level < 3; ++level) {
    const int shift = level == 0 ? 21 : (level == 1 ? 10 : 0);
    const int nbins = level == 2 ? 1024 : 2048;
    for (int i = tid; i < kSelBins; i += kSelThreads) sh.hist[i] = 0;
    __syncthreads();   // also orders the key cache fill before its first use
    for (int i = tid; i < T; i += kSelThreads) {
      const uint32_t key = key_at<kCached>(keys_lds, u, i);
      if ((key & prefix_mask) == prefix) atomicAdd(&sh.hist[(key >> shift) & (nbins - 1)], 1u);
    }
    __syncthreads();
    // scan the bins from the top: thread t owns bins nbins-1-2t and nbins-2-2t
    uint32_t c0 = 0, c1 = 0;
    const int top = nbins - 1 - 2 * tid;
    if (top >= 0) c0 = sh.hist[top];
    if (top - 1 >= 0) c1 = sh.hist[top - 1];
    const uint32_t incl = wave_inclusive_scan(c0 + c1, lane);
    if (lane == 63) sh.wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < wave; ++w) before += sh.wave_tot[w];
    const uint32_t excl = before + incl - (c0 + c1);   // keys in bins above this thread's pair
    // exactly one bin satisfies: above < need <= above + count
    if (c0 && excl < need && need <= excl + c0) { sh.found_bin = (uint32_t)top; sh.found_above = excl; }
    if (c1 && excl + c0 < need && need <= excl + c0 + c1) { sh.found_bin = (uint32_t)(top - 1); sh.found_above = excl + c0; }
    __syncthreads();
    prefix |= sh.found_bin << shift;
    prefix_mask |= (uint32_t)(nbins - 1) << shift;
    need -= sh.found_above;
    __syncthreads();   // found_* and hist are rewritten at the next level
  }
  const uint32_t thr = prefix;   // full 32-bit key of the budget-th largest score; keep `need` of its copies

  // ---- ordered emission ------------------------------------------------------
  // wave w owns tokens [w*per, (w+1)*per), per a multiple of 64
  const int per = ((T + kSelWaves - 1) / kSelWaves + 63) & ~63;
  const int lo = wave * per;
  const int hi = min(T, lo + per);
  uint32_t n_gt = 0, n_eq = 0;
  for (int base = lo; base < hi; base += 64) {
    const int i = base + lane;
    const bool in = i < hi;
    const uint32_t key = in ? key_at<kCached>(keys_lds, u, i) : 0u;
    n_gt += __popcll(__ballot(in && key > thr));
    n_eq += __popcll(__ballot(in && key == thr));
  }
  if (lane == 0) { sh.wave_gt[wave] = n_gt; sh.wave_eq[wave] = n_eq; }
  __syncthreads();
  uint32_t gt_before = 0, eq_before = 0;
  for (int w = 0; w < wave; ++w) { gt_before += sh.wave_gt[w]; eq_before += sh.wave_eq[w]; }
  uint32_t eq_seen = eq_before;                                  // copies of thr before the current 64 tokens
  uint32_t pos = gt_before + min(eq_before, need);               // kept tokens before the current 64 tokens
  for (int base = lo; base < hi; base += 64) {
    const int i = base + lane;
    const bool in = i < hi;
    const uint32_t key = in ? key_at<kCached>(keys_lds, u, i) : 0u;
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

__global__ void __launch_bounds__(kSelThreads)
select_kernel(SeqTable tab, const int32_t* __restrict__ offsets, int32_t* __restrict__ idx,
              int seg_base, int cached_limit /* heads of at most this many tokens use the LDS key cache */) {
  extern __shared__ __align__(16) unsigned char smem[];
  SelShared& sh = *reinterpret_cast<SelShared*>(smem);
  uint32_t* keys_lds = reinterpret_cast<uint32_t*>(smem + sizeof(SelShared));

  const int local_seg = blockIdx.x;
  const int seq = seq_of_unit(tab, local_seg);
  const int lh = local_seg - tab.first[seq];
  const int T = tab.T[seq];
  const float* u = tab.scores[seq] + (size_t)lh * (size_t)T;
  const int seg = seg_base + local_seg;
  const int off = offsets[seg];
  const int budget = offsets[seg + 1] - off;
  int32_t* out = idx + off;
  if (budget <= 0) return;
  if (budget >= T) {   // everything is kept
    for (int i = threadIdx.x; i < T; i += kSelThreads) out[i] = i;
    return;
  }
  if (T <= cached_limit) select_body<true>(u, T, budget, out, sh, keys_lds);
  else select_body<false>(u, T, budget, out, sh, keys_lds);
}

hipError_t select_prepare() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)(sizeof(SelShared) + (size_t)kSelMaxCachedKeys * 4));
}

void launch_select(const SeqTable& tab, const int32_t* offsets, int32_t* idx, int seg_base,
                   hipStream_t stream) {
  const int segs = tab.first[tab.n];
  if (segs <= 0) return;
  // the LDS key cache is sized for the longest sequence of this launch that fits it
  int cached_limit = 0;
  for (int i = 0; i < tab.n; ++i)
    if (tab.T[i] <= kSelMaxCachedKeys && tab.T[i] > cached_limit) cached_limit = tab.T[i];
  const size_t lds = sizeof(SelShared) + (size_t)cached_limit * sizeof(uint32_t);
  hipLaunchKernelGGL(select_kernel, dim3(segs), dim3(kSelThreads), lds, stream, tab, offsets, idx, seg_base,
                     cached_limit);
}

}  // namespace lkv
