// Compaction of the kept K/V rows into the padding-free ragged cache (Sec. 4.5
// of the paper: the compressed cache is flattened so that no padding is kept).
//
// A pure gather: packed row p of segment s copies row idx[p] of that segment's
// head, 256 bytes of K and 256 bytes of V, bit for bit.  The grid is flat over
// packed rows, so skewed budgets do not unbalance it.  Sixteen lanes move one
// row with one 16-byte load and store each; a block of 256 threads owns 256
// consecutive packed rows.  The segment of the block's first row is found by a
// wave-uniform binary search over the offsets; later rows walk forward from it.
#include "lkv_common.h"

namespace lkv {

constexpr int kCompactThreads = 256;
constexpr int kCompactRowsPerBlock = 256;
constexpr int kCompactUnroll = 4;

__global__ void __launch_bounds__(kCompactThreads)
compact_kernel(SeqTable tab, const int32_t* __restrict__ idx, const int32_t* __restrict__ offsets,
               int n_segments, int heads_per_seq, int seq_lo, int head_lo, int n_heads_view, int64_t row_lo,
               int64_t row_hi, uint4* __restrict__ kp, uint4* __restrict__ vp) {
  // packed rows [row_lo, row_hi) are this launch's; the source tensors hold heads head_lo .. of each
  // sequence (all of them for a whole cache, one layer's for a layer view)
  const int64_t p0 = row_lo + (int64_t)blockIdx.x * kCompactRowsPerBlock;
  // the segment that contains row p0: the last one with offsets[s] <= p0
  const int s0 = wave_upper_segment(offsets, n_segments, p0, threadIdx.x & 63);

  const int rslot = threadIdx.x >> 4;   // 16 rows per pass over the block
  const int c = threadIdx.x & 15;
#pragma unroll 1
  for (int it = 0; it < kCompactRowsPerBlock / 16; it += kCompactUnroll) {
    // Loads are unconditional (a row past the end re-reads the last packed row) so that the
    // staged rows stay in registers; only the stores are predicated.
    uint4 kk[kCompactUnroll], vv[kCompactUnroll];
    bool live[kCompactUnroll];
#pragma unroll
    for (int u = 0; u < kCompactUnroll; ++u) {
      int64_t p = p0 + (it + u) * 16 + rslot;
      live[u] = p < row_hi;
      p = live[u] ? p : row_hi - 1;
      int s = s0;
      while ((int64_t)offsets[s + 1] <= p) ++s;     // skips empty segments too; p < offsets[n_segments]
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
    }
#pragma unroll
    for (int u = 0; u < kCompactUnroll; ++u) {
      const int64_t p = p0 + (it + u) * 16 + rslot;
      if (live[u]) {
        store_stream16(kp + p * kChunksPerRow + c, kk[u]);
        store_stream16(vp + p * kChunksPerRow + c, vv[u]);
      }
    }
  }
}

void launch_compact(const SeqTable& tab, const int32_t* idx, const int32_t* offsets, int n_segments,
                    int heads_per_seq, int seq_lo, int head_lo, int n_heads_view, int64_t row_lo, int64_t row_hi,
                    void* kp, void* vp, hipStream_t stream) {
  if (row_hi <= row_lo) return;
  const int blocks = (int)((row_hi - row_lo + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock);
  hipLaunchKernelGGL(compact_kernel, dim3(blocks), dim3(kCompactThreads), 0, stream, tab, idx, offsets,
                     n_segments, heads_per_seq, seq_lo, head_lo, n_heads_view, row_lo, row_hi,
                     reinterpret_cast<uint4*>(kp),
                     reinterpret_cast<uint4*>(vp));
}

}  // namespace lkv
