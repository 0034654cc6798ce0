// First-level digit counts of the top-k (the top 11 bits of the order-preserving key of every score) as a
// by-product of scoring.  The MLP scoring kernels count on their way out; for the linear scorer, whose blocks are
// too small to amortise a 2048-bin histogram, this file has a pass over the scores (4 bytes per token, under 1 % of
// the cache bytes).  Also the fill kernel that zeroes the counters (a kernel, not a memset, so that it can be
// recorded into a HIP graph).
#include "lkv_common.h"

namespace lkv {

constexpr int kCountThreads = 256;
constexpr int kCountSlice = 8192;   // tokens per block

__global__ void __launch_bounds__(kCountThreads) clear_counts_kernel(uint4* __restrict__ counts, size_t n_vec) {
  for (size_t i = (size_t)blockIdx.x * kCountThreads + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * kCountThreads)
    counts[i] = make_uint4(0, 0, 0, 0);
}

void launch_clear_counts(uint32_t* counts, int64_t n_segments, hipStream_t stream) {
  const size_t n_vec = (size_t)n_segments * kLevel0Bins / 4;
  if (n_vec == 0) return;
  const size_t want = (n_vec + kCountThreads - 1) / kCountThreads;
  const int blocks = (int)(want < 2048 ? want : 2048);
  hipLaunchKernelGGL(clear_counts_kernel, dim3(blocks), dim3(kCountThreads), 0, stream, reinterpret_cast<uint4*>(counts),
                     n_vec);
}

// tab.first[i]: blocks before sequence i; a sequence takes heads * ceil(T / kCountSlice) blocks.
__global__ void __launch_bounds__(kCountThreads)
count_level0_kernel(SeqTable tab, uint32_t* __restrict__ counts, int seg_base, int seg_stride) {
  __shared__ uint32_t hist[kLevel0Bins];
  const int seq = seq_of_unit(tab, blockIdx.x);
  const int local = blockIdx.x - tab.first[seq];
  const int T = tab.T[seq];
  const int slices = (T + kCountSlice - 1) / kCountSlice;
  const int lh = local / slices;
  const int t0 = (local - lh * slices) * kCountSlice;
  const int t1 = min(T, t0 + kCountSlice);
  for (int i = threadIdx.x; i < kLevel0Bins; i += kCountThreads) hist[i] = 0;
  __syncthreads();
  const float* u = tab.scores[seq] + (size_t)lh * (size_t)T;
  for (int i = t0 + threadIdx.x; i < t1; i += kCountThreads) atomicAdd(&hist[order_key(u[i]) >> kLevel0Shift], 1u);
  __syncthreads();
  flush_level0_counts(hist, counts, (size_t)(seg_base + seq * seg_stride + lh), kCountThreads);
}

int count_level0_blocks_per_head(int T) { return (T + kCountSlice - 1) / kCountSlice; }

void launch_count_level0(const SeqTable& tab, uint32_t* counts, int seg_base, int seg_stride, hipStream_t stream) {
  const int blocks = tab.first[tab.n];
  if (blocks <= 0) return;
  hipLaunchKernelGGL(count_level0_kernel, dim3(blocks), dim3(kCountThreads), 0, stream, tab, counts, seg_base, seg_stride);
}

}  // namespace lkv
