// LKV-T token scoring with a single linear layer: u = w . [k ; v] + b.
// (Sec. 3.4 of the paper defines the scorer on the concatenated key and value
// rows; the linear form is the simplest instance used by the workloads.)
//
// HBM-bound: 512 bytes in and 4 bytes out per token.  Each row of 256 bytes is
// read by the 16 lanes of one DPP row with one 16-byte load per lane, so a
// wave covers four full rows per load instruction.  The 16 partial dot
// products of a row are summed with four DPP adds.  A wave owns 64 consecutive
// tokens and lane (r, c) ends up holding the score of token 4c + r, which makes
// the result store one fully used 256-byte line per wave.
//
// A block's 256 rows are cut at 64 KB boundaries of the key array rather than at the head's first row, so that
// blocks read aligned runs whatever T is: with windows that start at each head's first row, a T that is not a
// multiple of 32 cost 2 to 5 % of the bandwidth.
#include "lkv_common.h"

namespace lkv {

constexpr int kScoreBlockThreads = 256;
constexpr int kScoreRowsPerWave = 64;
constexpr int kScoreRowsPerBlock = kScoreRowsPerWave * (kScoreBlockThreads / 64);   // 256
constexpr int kScoreUnroll = 4;   // row groups whose loads are in flight together (8 loads per lane)

// Blocks are 64 KB windows of the key array's address space (256 rows).  A head's first row can lie anywhere inside
// a window, so a head needs up to one block more than its rows fill; a block with no row of the head exits at once.
__host__ __device__ inline int score_linear_blocks_per_head_impl(int T) {
  return (T + 2 * kScoreRowsPerBlock - 2) / kScoreRowsPerBlock;
}
int score_linear_blocks_per_head(int T) { return score_linear_blocks_per_head_impl(T); }

__global__ void __launch_bounds__(kScoreBlockThreads)
score_linear_kernel(SeqTable tab, const uint16_t* __restrict__ w1, const float* __restrict__ b1,
                    int heads_per_scorer_row /* H if per-layer scorer, 1 if per-head */) {
  const int seq = seq_of_unit(tab, blockIdx.x);
  const int local = blockIdx.x - tab.first[seq];
  const int T = tab.T[seq];
  const int tiles = score_linear_blocks_per_head_impl(T);
  const int lh = local / tiles;                 // flattened (layer, head)
  const int tile = local - lh * tiles;
  const int scorer = lh / heads_per_scorer_row; // per-layer: lh / H = layer; per-head: lh

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int r = lane >> 4;       // row slot inside a group of four rows
  const int c = lane & 15;       // 16-byte piece of the row

  // this lane's slice of the weight vector: key channels 8c..8c+7 and value channels 8c..8c+7
  float wk[8], wv[8];
  {
    const uint4* wrow = reinterpret_cast<const uint4*>(w1 + (size_t)scorer * (2 * kHeadDim));
    unpack8(wrow[c], wk);
    unpack8(wrow[kChunksPerRow + c], wv);
  }
  const float bias = b1[scorer];

  const size_t head_row0 = (size_t)lh * (size_t)T;
  const uint4* Kh = reinterpret_cast<const uint4*>(tab.k[seq]) + head_row0 * kChunksPerRow;
  const uint4* Vh = reinterpret_cast<const uint4*>(tab.v[seq]) + head_row0 * kChunksPerRow;
  // Blocks are cut at 64 KB boundaries of the key array's addresses, not at multiples of 256 rows of the head: a
  // head whose first row does not sit on such a boundary gets a short first block, and every other block reads
  // 64 KB-aligned runs of K (and, when V and the scores are allocated alike, of V; 1 KB-aligned runs of scores)
  // whatever T is and wherever the tensor, or a layer view of it, starts.
  const int lead = (int)((reinterpret_cast<uintptr_t>(Kh) >> 8) & (uintptr_t)(kScoreRowsPerBlock - 1));
  const int row_base = tile * kScoreRowsPerBlock - lead + wave * kScoreRowsPerWave;
  if (row_base >= T || row_base + kScoreRowsPerWave <= 0) return;     // whole wave outside the head (wave-uniform)

  float mine = 0.f;
#pragma unroll
  for (int j0 = 0; j0 < kScoreRowsPerWave / 4; j0 += kScoreUnroll) {
    uint4 kk[kScoreUnroll], vv[kScoreUnroll];
#pragma unroll
    for (int u = 0; u < kScoreUnroll; ++u) {
      int row = row_base + 4 * (j0 + u) + r;
      row = row < T ? row : T - 1;             // rows outside the head: re-read its first or last row, result unused
      row = row < 0 ? 0 : row;
      kk[u] = load_stream16(Kh + (size_t)row * kChunksPerRow + c);
      vv[u] = load_stream16(Vh + (size_t)row * kChunksPerRow + c);
    }
#pragma unroll
    for (int u = 0; u < kScoreUnroll; ++u) {
      float fk[8], fv[8];
      unpack8(kk[u], fk);
      unpack8(vv[u], fv);
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc = fmaf(fk[e], wk[e], acc);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc = fmaf(fv[e], wv[e], acc);
      acc = row16_allreduce_sum(acc);
      mine = (c == j0 + u) ? acc : mine;
    }
  }
  const int out_row = row_base + 4 * c + r;
  if (out_row >= 0 && out_row < T) tab.scores[seq][head_row0 + out_row] = mine + bias;
}

void launch_score_linear(const SeqTable& tab, const uint16_t* w1, const float* b1, int heads_per_scorer_row,
                         hipStream_t stream) {
  const int blocks = tab.first[tab.n];
  if (blocks <= 0) return;
  hipLaunchKernelGGL(score_linear_kernel, dim3(blocks), dim3(kScoreBlockThreads), 0, stream, tab, w1,
                     b1, heads_per_scorer_row);
}



}  // namespace lkv
