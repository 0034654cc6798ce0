// Compaction of the kept K/V rows into the padding-free ragged cache (Sec. 4.5
// of the paper: the compressed cache is flattened so that no padding is kept).
//
// A pure gather: packed row p of segment s copies row idx[p] of that segment's
// head, 256 bytes of K and 256 bytes of V, bit for bit.  The grid is flat over
// packed rows, so skewed budgets do not unbalance it.  Sixteen lanes move one
// row with one 16-byte load and store each; a block of 256 threads owns 64
// consecutive packed rows.  The segment of the block's first row is found by a
// wave-uniform binary search over the offsets; later rows walk forward from it.
#include <cstring>

#include "lkv_common.h"

namespace lkv {

constexpr int kCompactThreads = 256;
constexpr int kCompactRowsPerBlock = 64;    // one pass: every thread moves 4 rows' pieces (8 loads in flight, then 8 stores).
                                            // Blocks of 256 rows (four such passes in a loop) were 11 % slower.
constexpr int kCompactUnroll = 4;

__device__ __forceinline__ int len_or_one(const int32_t* len, int s) { return len != nullptr ? len[s] : 1; }

// What a launch gathers from and where it puts the rows.
//   kCompactPlain      : from the prefilled cache to packed row p.
//   kCompactGrowCache  : from the prefilled cache to row p + slack * s (every segment s is followed by
//                        `slack` spare rows for tokens generated later); the kept scores go along.
//   kCompactGrowPacked : the same destination, gathered from an older packed cache with slack
//                        (re-eviction): idx counts rows inside the old segment.
constexpr int kCompactPlain = 0;
constexpr int kCompactGrowCache = 1;
constexpr int kCompactGrowPacked = 2;

struct CompactGrow {
  int slack;
  float* up;               // destination scores, one per packed row
  const uint4* kp_old;     // kCompactGrowPacked: the source packed cache
  const uint4* vp_old;
  const float* up_old;
  const int32_t* cap_old;  // [n_segments + 1] first row of every old segment
  const int32_t* len_old;  // [n_segments] rows in use of every old segment
};

template <int kMode>
__global__ void __launch_bounds__(kCompactThreads)
compact_kernel(SeqTable tab, const int32_t* __restrict__ idx, const int32_t* __restrict__ offsets,
               int n_segments, int heads_per_seq, int seq_lo, int head_lo, int n_heads_view, int64_t row_lo,
               int64_t row_hi, int rows_of_own_sequences, uint4* __restrict__ kp, uint4* __restrict__ vp,
               CompactGrow grow) {
  // packed rows [row_lo, row_hi) are this launch's; the source tensors hold heads head_lo .. of each
  // sequence (all of them for a whole cache, one layer's for a layer view)
  if (rows_of_own_sequences) {
    // one of several launches over a cache of many sequences: the rows of the sequences this launch
    // describes are one contiguous range, read from the table (the host does not know the budgets
    // here); the grid was sized for all rows and the blocks past the range leave at once
    row_lo = offsets[min(seq_lo * heads_per_seq, n_segments)];
    row_hi = offsets[min((seq_lo + tab.n) * heads_per_seq, n_segments)];
  }
  const int64_t p0 = row_lo + (int64_t)blockIdx.x * kCompactRowsPerBlock;
  if (p0 >= row_hi) return;
  // the segment that contains row p0: the last one with offsets[s] <= p0
  const int s0 = wave_upper_segment(offsets, n_segments, p0, threadIdx.x & 63);

  const int rslot = threadIdx.x >> 4;   // 16 rows per pass over the block
  const int c = threadIdx.x & 15;
#pragma unroll 1
  for (int it = 0; it < kCompactRowsPerBlock / 16; it += kCompactUnroll) {
    // Loads are unconditional (a row past the end re-reads the last packed row) so that the
    // staged rows stay in registers; only the stores are predicated.
    uint4 kk[kCompactUnroll], vv[kCompactUnroll];
    float uu[kCompactUnroll];
    int64_t dst[kCompactUnroll];
    bool live[kCompactUnroll];
#pragma unroll
    for (int u = 0; u < kCompactUnroll; ++u) {
      int64_t p = p0 + (it + u) * 16 + rslot;
      live[u] = p < row_hi;
      p = live[u] ? p : row_hi - 1;
      int s = s0;
      // skips empty segments too; p < offsets[n_segments] when total_kept matches the table, and the
      // walk stops at the last segment when it does not
      while (s + 1 < n_segments && (int64_t)offsets[s + 1] <= p) ++s;
      dst[u] = kMode == kCompactPlain ? p : p + (int64_t)grow.slack * s;
      if (kMode == kCompactGrowPacked) {
        // a row index outside the old segment cannot come from the selection; clamped, never followed
        const int len = max(len_or_one(grow.len_old, s), 1);
        const int tok = min(max(idx[p], 0), len - 1);
        const size_t row = (size_t)grow.cap_old[s] + (size_t)tok;
        kk[u] = load_stream16(grow.kp_old + row * kChunksPerRow + c);
        vv[u] = load_stream16(grow.vp_old + row * kChunksPerRow + c);
        uu[u] = grow.up_old[row];
      } else {
        const int seq = s / heads_per_seq;
        int lh = s - seq * heads_per_seq - head_lo;
        int sl = seq - seq_lo;                        // this launch describes sequences seq_lo .. seq_lo + tab.n - 1
        live[u] = live[u] && sl >= 0 && sl < tab.n && lh >= 0 && lh < n_heads_view;
        sl = min(max(sl, 0), tab.n - 1);
        lh = min(max(lh, 0), n_heads_view - 1);       // rows of other heads are not this launch's: never followed
        // a token index outside [0, T) cannot come from lkv_select; it is clamped, never followed
        const int T = tab.T[sl];
        const int tok = min(max(idx[p], 0), T - 1);
        const size_t src = ((size_t)lh * (size_t)T + (size_t)tok) * kChunksPerRow + c;
        kk[u] = load_stream16(reinterpret_cast<const uint4*>(tab.k[sl]) + src);
        vv[u] = load_stream16(reinterpret_cast<const uint4*>(tab.v[sl]) + src);
        if (kMode == kCompactGrowCache) uu[u] = tab.scores[sl][(size_t)lh * (size_t)T + (size_t)tok];
      }
    }
#pragma unroll
    for (int u = 0; u < kCompactUnroll; ++u) {
      if (live[u]) {
        store_stream16(kp + dst[u] * kChunksPerRow + c, kk[u]);
        store_stream16(vp + dst[u] * kChunksPerRow + c, vv[u]);
        if (kMode != kCompactPlain && c == 0) grow.up[dst[u]] = uu[u];
      }
    }
  }
}

void launch_compact(const SeqTable& tab, const int32_t* idx, const int32_t* offsets, int n_segments,
                    int heads_per_seq, int seq_lo, int head_lo, int n_heads_view, int64_t row_lo, int64_t row_hi,
                    void* kp, void* vp, hipStream_t stream, bool rows_of_own_sequences) {
  if (row_hi <= row_lo) return;
  const int blocks = (int)((row_hi - row_lo + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock);
  CompactGrow none = {};
  hipLaunchKernelGGL(compact_kernel<kCompactPlain>, dim3(blocks), dim3(kCompactThreads), 0, stream, tab, idx,
                     offsets, n_segments, heads_per_seq, seq_lo, head_lo, n_heads_view, row_lo, row_hi,
                     rows_of_own_sequences ? 1 : 0, reinterpret_cast<uint4*>(kp), reinterpret_cast<uint4*>(vp), none);
}

// Compaction into a cache with `slack` spare rows behind every segment, from the prefilled cache
// (tab.scores holds the scores the selection used).
void launch_compact_grow(const SeqTable& tab, const int32_t* idx, const int32_t* offsets, int n_segments,
                         int heads_per_seq, int seq_lo, int64_t total_kept, int slack, void* kp, void* vp, float* up,
                         hipStream_t stream, bool rows_of_own_sequences) {
  if (total_kept <= 0) return;
  const int blocks = (int)((total_kept + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock);
  CompactGrow g = {};
  g.slack = slack;
  g.up = up;
  hipLaunchKernelGGL(compact_kernel<kCompactGrowCache>, dim3(blocks), dim3(kCompactThreads), 0, stream, tab, idx,
                     offsets, n_segments, heads_per_seq, seq_lo, 0, heads_per_seq, (int64_t)0, total_kept,
                     rows_of_own_sequences ? 1 : 0, reinterpret_cast<uint4*>(kp), reinterpret_cast<uint4*>(vp), g);
}

// The same from an older packed cache with slack: idx[p] is a row position inside the old segment.
void launch_compact_regrow(const int32_t* idx, const int32_t* offsets, int n_segments, int64_t total_kept, int slack,
                           const void* kp_old, const void* vp_old, const float* up_old, const int32_t* cap_old,
                           const int32_t* len_old, void* kp, void* vp, float* up, hipStream_t stream) {
  if (total_kept <= 0) return;
  const int blocks = (int)((total_kept + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock);
  SeqTable tab;
  memset(&tab, 0, sizeof(tab));
  CompactGrow g = {slack, up, reinterpret_cast<const uint4*>(kp_old), reinterpret_cast<const uint4*>(vp_old), up_old,
                   cap_old, len_old};
  hipLaunchKernelGGL(compact_kernel<kCompactGrowPacked>, dim3(blocks), dim3(kCompactThreads), 0, stream, tab, idx,
                     offsets, n_segments, 1, 0, 0, 1, (int64_t)0, total_kept, 0, reinterpret_cast<uint4*>(kp),
                     reinterpret_cast<uint4*>(vp), g);
}

// cap[s] = offsets[s] + slack * s (s = 0..n_segments), len[s] = offsets[s + 1] - offsets[s]
__global__ void grown_layout_kernel(const int32_t* __restrict__ offsets, int n_segments, int slack,
                                    int32_t* __restrict__ cap, int32_t* __restrict__ len) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s > n_segments) return;
  const int32_t o = offsets[s];
  cap[s] = o + slack * s;
  if (s < n_segments) len[s] = offsets[s + 1] - o;
}

void launch_grown_layout(const int32_t* offsets, int n_segments, int slack, int32_t* cap, int32_t* len,
                         hipStream_t stream) {
  hipLaunchKernelGGL(grown_layout_kernel, dim3((n_segments + 256) / 256), dim3(256), 0, stream, offsets, n_segments,
                     slack, cap, len);
}

}  // namespace lkv
