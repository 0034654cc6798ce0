// Observation-window token scoring (the attention-based selection policy that the ablation of
// Sec. 4.4 runs under the LKV-H budgets; O(W T) in the complexity table of Sec. 4.5): a prefix
// token's score is the attention mass it receives from the last W queries of the prompt, summed
// over the window, averaged over the query heads of its GQA group and smoothed by a short 1-D
// pooling; the window tokens themselves score +inf.
//
// The work is one [G W x 128] x [128 x T] product per (layer, KV head) followed by a softmax over
// T, so the keys stream past the matrix cores exactly as they do for the MLP scorer: the G W
// window queries sit on the M side of v_mfma_f32_16x16x32_bf16 as register-resident A fragments,
// 16 keys at a time form the B operand, read once from HBM with coalesced 16-byte loads and
// staged in LDS.  A softmax needs its normaliser before any weight can be summed over the rows,
// so the keys are read twice:
//   pass 1  per window row, the log-sum-exp of its logits over one block's keys (causal inside
//           the window), written as a (reference, sum) pair per block;
//   pass 2  merges the pairs of all blocks of the head into the row's log-normaliser, recomputes
//           the logits and adds exp(logit - normaliser) over the rows: the token's vote;
//   pool    smooths the votes and writes the scores.
// Keeping the logits instead would cost as many bytes as reading the keys again (G W = 128
// logits per 128-element key).
//
// Pass 1 keeps a running reference per (row, lane) instead of a running maximum: the sum is
// taken relative to a reference that is only moved when a logit exceeds it by more than 64
// binary orders of magnitude, which costs one exponential per logit instead of two.  Any
// reference within that distance of the true maximum gives the same sum to fp32 rounding.
//
// A block is a pair of waves that share each staged tile of 16 keys; the window rows are split
// between the two (at most 64 rows, 64 fragment registers, per wave).
#include "lkv_common.h"

namespace lkv {

constexpr int kWinThreads = 128;
constexpr int kWinTokTile = 16;                  // keys per MFMA N tile
constexpr int kWinRowStride = 256 + 32;          // bytes per staged key row in LDS
constexpr int kWinTileLds = kWinTokTile * kWinRowStride;
constexpr int kWinMaxRowsPerBlock = 1024;
constexpr float kWinRebase = 64.f;               // log2 distance at which pass 1 moves a reference
constexpr float kWinNoRef = -1e30f;              // reference of a row that has seen no key yet

__device__ __forceinline__ int win_seq_of_unit(const WinTable& tab, int unit) {
  int s = 0;
  while (s + 1 < tab.n && unit >= tab.first[s + 1]) ++s;
  return s;
}

__device__ __forceinline__ float row16_allreduce_max(float x) {
  x = fmaxf(x, dpp_f32<kDppQuadXor1>(x));
  x = fmaxf(x, dpp_f32<kDppQuadXor2>(x));
  x = fmaxf(x, dpp_f32<kDppRowHalfMirror>(x));
  x = fmaxf(x, dpp_f32<kDppRowMirror>(x));
  return x;
}

// kPass 1: partial log-sum-exp pairs.  kPass 2: votes.  MTW: 16-row M tiles per wave; the rows past
// n_rows = G W are padding (zero queries, never counted).
template <int MTW, int kPass>
__global__ void __launch_bounds__(kWinThreads, 2)
score_window_kernel(WinTable tab, int window, int n_rows, int rows_per_block, float log2_scale, float inv_group) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int RP = 32 * MTW;                      // padded rows of the block

  const int seq = win_seq_of_unit(tab, blockIdx.x);
  const int local = blockIdx.x - tab.first[seq];
  const int T = tab.T[seq];
  const int chunks = (T + rows_per_block - 1) / rows_per_block;
  const int lh = local / chunks;
  const int chunk = local - lh * chunks;
  const int prefix = T - window;                    // tokens that are scored

  const int block_row0 = chunk * rows_per_block;
  const int block_end = kPass == 1 ? T : prefix;    // pass 2 has nothing to do inside the window
  if (block_row0 >= block_end) return;
  const int block_rows = min(block_end - block_row0, rows_per_block);
  const int n_tiles = (block_rows + 15) >> 4;

  const int lane = threadIdx.x & 63;
  const int half = threadIdx.x >> 6;
  const int r = lane >> 4;
  const int c = lane & 15;
  // LDS: two staged tiles, then (pass 2) the block's votes of either wave, then the rows' log-normalisers
  unsigned char* x_lds = smem;
  float* vote_lds = reinterpret_cast<float*>(smem + 2 * kWinTileLds);   // [2][rows_per_block]
  float* lse_lds = vote_lds + 2 * rows_per_block;                        // [RP]

  // A fragments: window row 16 (half MTW + mw) + c, features 32 ks + 8 r .. +7
  bf16x8_t qfrag[MTW][4];
  {
    const uint4* qb = reinterpret_cast<const uint4*>(tab.q[seq]) + (size_t)lh * n_rows * kChunksPerRow;
#pragma unroll
    for (int mw = 0; mw < MTW; ++mw) {
      const int row = 16 * (half * MTW + mw) + c;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row < n_rows) v = qb[(size_t)row * kChunksPerRow + ks * 4 + r];
        qfrag[mw][ks] = __builtin_bit_cast(bf16x8_t, v);
      }
    }
  }

  // per lane: rows 16 (half MTW + mw) + 4 r + e of token c of the current tile
  float ref[MTW][4], sum[MTW][4];   // pass 1: running reference (log2 units) and sum; pass 2: ref = log-normaliser
#pragma unroll
  for (int mw = 0; mw < MTW; ++mw)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int row = 16 * (half * MTW + mw) + 4 * r + e;
      ref[mw][e] = row < n_rows ? kWinNoRef : -kWinNoRef;   // a padding row never asks for a new reference
      sum[mw][e] = 0.f;
    }

  const size_t part_row0 = ((size_t)lh * chunks) * RP;
  if (kPass == 2) {
    // log-normaliser of every row: merge the pairs that pass 1 left for each block of this head
    const float* part = tab.partial[seq] + part_row0 * 2;
    for (int row = threadIdx.x; row < RP; row += kWinThreads) {
      float lse = INFINITY;                          // padding rows: weight exp2(-inf) = 0
      if (row < n_rows) {
        float m = kWinNoRef;
        for (int ch = 0; ch < chunks; ++ch) m = fmaxf(m, part[((size_t)ch * RP + row) * 2]);
        float l = 0.f;
        for (int ch = 0; ch < chunks; ++ch) {
          const float* p = part + ((size_t)ch * RP + row) * 2;
          l += p[1] * __builtin_amdgcn_exp2f(p[0] - m);
        }
        lse = m + __log2f(l);
      }
      lse_lds[row] = lse;
    }
    __syncthreads();
#pragma unroll
    for (int mw = 0; mw < MTW; ++mw) {
      const f32x4_t v = *reinterpret_cast<const f32x4_t*>(lse_lds + 16 * (half * MTW + mw) + 4 * r);
#pragma unroll
      for (int e = 0; e < 4; ++e) ref[mw][e] = v[e];
    }
  }

  const uint4* Kh = reinterpret_cast<const uint4*>(tab.k[seq]) + (size_t)lh * (size_t)T * kChunksPerRow;

  // Staging: thread (half, r, c) brings piece c of rows 8 half + r and 8 half + 4 + r of each tile.
  uint4 xa[2], xb[2];
  auto load_tile = [&](uint4 (&xx)[2], int i) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int row = block_row0 + 16 * i + 8 * half + 4 * j + r;
      row = row < T ? row : T - 1;   // ragged tail: re-read the last row, masked below
      xx[j] = load_stream16(Kh + (size_t)row * kChunksPerRow + c);
    }
  };
  auto stage_tile = [&](const uint4 (&xx)[2], int buf) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
      *reinterpret_cast<uint4*>(x_lds + buf * kWinTileLds + (8 * half + 4 * j + r) * kWinRowStride + c * 16) = xx[j];
  };
  auto products = [&](f32x4_t (&acc)[MTW], int buf) {
#pragma unroll
    for (int mw = 0; mw < MTW; ++mw) acc[mw] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const unsigned char* xt = x_lds + buf * kWinTileLds;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const uint4 x = *reinterpret_cast<const uint4*>(xt + c * kWinRowStride + ks * 64 + r * 16);
      const bf16x8_t xv = __builtin_bit_cast(bf16x8_t, x);
#pragma unroll
      for (int mw = 0; mw < MTW; ++mw)
        acc[mw] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qfrag[mw][ks], xv, acc[mw], 0, 0, 0);
    }
  };
  auto finish = [&](const f32x4_t (&acc)[MTW], int i) {
    const int row0 = block_row0 + 16 * i;
    if (kPass == 1) {
      float x[MTW][4];
      float top = -INFINITY;
#pragma unroll
      for (int mw = 0; mw < MTW; ++mw)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          x[mw][e] = fmaf(acc[mw][e], log2_scale, -ref[mw][e]);
          top = fmaxf(top, x[mw][e]);
        }
      // tiles that touch the window (causal limits) or the ragged tail, and tiles in which some logit
      // runs away from its reference, take the careful path
      const bool careful = row0 + 16 > prefix || __ballot(top > kWinRebase) != 0;
      if (!careful) {
#pragma unroll
        for (int mw = 0; mw < MTW; ++mw)
#pragma unroll
          for (int e = 0; e < 4; ++e) sum[mw][e] += __builtin_amdgcn_exp2f(x[mw][e]);
      } else {
        const int j = row0 + c;
#pragma unroll
        for (int mw = 0; mw < MTW; ++mw)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int row = 16 * (half * MTW + mw) + 4 * r + e;
            const int in_window = row % window;                       // this row's query stands at prefix + in_window
            const bool seen = row < n_rows && j <= prefix + in_window;
            const float s = acc[mw][e] * log2_scale;
            const float moved = fmaxf(ref[mw][e], s);
            const float kept = sum[mw][e] * __builtin_amdgcn_exp2f(ref[mw][e] - moved) + __builtin_amdgcn_exp2f(s - moved);
            sum[mw][e] = seen ? kept : sum[mw][e];
            ref[mw][e] = seen ? moved : ref[mw][e];
          }
      }
    } else {
      float part = 0.f;
#pragma unroll
      for (int mw = 0; mw < MTW; ++mw)
#pragma unroll
        for (int e = 0; e < 4; ++e) part += __builtin_amdgcn_exp2f(fmaf(acc[mw][e], log2_scale, -ref[mw][e]));
      part += __shfl_xor(part, 16, 64);
      part += __shfl_xor(part, 32, 64);
      if (r == 0) vote_lds[half * rows_per_block + 16 * i + c] = part;   // 16 i + c < rows_per_block
    }
  };

  // Barrier i makes tile i visible and means both waves have finished reading tile i - 1.
  // One step: products and arithmetic of tile i, staging of tile i + 1 (fetching tile i + 3 behind it).
  f32x4_t acc[MTW];
  auto step = [&](uint4 (&x_next)[2], int i) {
    products(acc, i & 1);
    if (i + 1 < n_tiles) {
      stage_tile(x_next, (i + 1) & 1);
      if (i + 3 < n_tiles) load_tile(x_next, i + 3);
    }
    finish(acc, i);
    __syncthreads();
  };
  load_tile(xa, 0);
  if (1 < n_tiles) load_tile(xb, 1);
  stage_tile(xa, 0);
  if (2 < n_tiles) load_tile(xa, 2);
  __syncthreads();
#pragma unroll 1
  for (int i = 0; i < n_tiles; i += 2) {
    step(xb, i);                                   // stages the odd tile i + 1
    if (i + 1 < n_tiles) step(xa, i + 1);          // uniform condition around the barrier
  }

  if (kPass == 1) {
    // one (reference, sum) pair per row: merge the 16 token lanes
    float* part = tab.partial[seq] + (part_row0 + (size_t)chunk * RP) * 2;
#pragma unroll
    for (int mw = 0; mw < MTW; ++mw)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int row = 16 * (half * MTW + mw) + 4 * r + e;
        const float mine = row < n_rows ? ref[mw][e] : kWinNoRef;
        const float m = row16_allreduce_max(mine);
        const float l = row16_allreduce_sum(sum[mw][e] * __builtin_amdgcn_exp2f(mine - m));
        if (c == 0) {
          part[row * 2] = m;
          part[row * 2 + 1] = l;
        }
      }
  } else {
    // the last barrier of the loop ordered the votes; mean over the group's query heads
    float* votes = tab.votes[seq] + (size_t)lh * T + block_row0;
    for (int t = threadIdx.x; t < block_rows; t += kWinThreads)
      votes[t] = (vote_lds[t] + vote_lds[rows_per_block + t]) * inv_group;
  }
}

// Scores from votes: centred pooling of width 2 c + 1 over the prefix, +inf on the window tokens.
// kind 0: maximum over the part of the span inside the prefix; kind 1: sum over it divided by the width.
__global__ void __launch_bounds__(256)
score_window_pool_kernel(WinTable tab, int window, int reach, int kind) {
  const int seq = win_seq_of_unit(tab, blockIdx.x);
  const int local = blockIdx.x - tab.first[seq];
  const int T = tab.T[seq];
  const int tiles = (T + 1023) >> 10;
  const int lh = local / tiles;
  const int tile = local - lh * tiles;
  const int prefix = T - window;
  const float* votes = tab.votes[seq] + (size_t)lh * T;
  float* out = tab.scores[seq] + (size_t)lh * T;
  const float inv_width = 1.f / (float)(2 * reach + 1);
  for (int j = tile * 1024 + threadIdx.x; j < min(T, tile * 1024 + 1024); j += 256) {
    float s = INFINITY;
    if (j < prefix) {
      const int lo = max(0, j - reach), hi = min(prefix - 1, j + reach);
      if (kind == 0) {
        s = votes[lo];
        for (int t = lo + 1; t <= hi; ++t) s = fmaxf(s, votes[t]);
      } else {
        s = 0.f;
        for (int t = lo; t <= hi; ++t) s += votes[t];
        s *= inv_width;
      }
    }
    out[j] = s;
  }
}

int score_window_max_rows() { return 128; }

int score_window_rows_per_block(int64_t tokens_times_heads) {
  // large blocks amortise the query fragments each wave loads; small problems take smaller blocks so
  // that the grid still covers the chip
  int rows = kWinMaxRowsPerBlock;
  while (rows > 128 && tokens_times_heads / rows < 2048) rows >>= 1;
  return rows;
}

// Workspace of one sequence: votes [heads, T] then pairs [heads, ceil(T / 128), 128, 2] (the largest the
// pairs can get: the smallest block and the most padded rows), each 256-byte aligned.
size_t score_window_votes_bytes(int64_t heads, int T) { return ((size_t)heads * T * sizeof(float) + 255) & ~(size_t)255; }
size_t score_window_pairs_bytes(int64_t heads, int T) {
  return ((size_t)heads * ((T + 127) / 128) * 128 * 2 * sizeof(float) + 255) & ~(size_t)255;
}

template <int MTW>
static void launch_passes(const WinTable& tab, int window, int n_rows, int rows_per_block, float log2_scale,
                          float inv_group, hipStream_t stream) {
  const int blocks = tab.first[tab.n];
  const size_t lds1 = 2 * kWinTileLds;
  const size_t lds2 = 2 * kWinTileLds + (2 * (size_t)rows_per_block + 32 * MTW) * sizeof(float);
  hipLaunchKernelGGL((score_window_kernel<MTW, 1>), dim3(blocks), dim3(kWinThreads), lds1, stream, tab, window,
                     n_rows, rows_per_block, log2_scale, inv_group);
  hipLaunchKernelGGL((score_window_kernel<MTW, 2>), dim3(blocks), dim3(kWinThreads), lds2, stream, tab, window,
                     n_rows, rows_per_block, log2_scale, inv_group);
}

// `tab.first` counts the blocks of the two passes; the pooling kernel derives its own grid.
void launch_score_window(const WinTable& tab, int heads, int window, int group, int pool_width, int pool_kind,
                         int rows_per_block, float scale, hipStream_t stream) {
  if (tab.n <= 0) return;
  const int n_rows = group * window;
  const float log2_scale = scale * 1.44269504088896340736f;
  const float inv_group = 1.f / (float)group;
  switch ((n_rows + 31) / 32) {
    case 1: launch_passes<1>(tab, window, n_rows, rows_per_block, log2_scale, inv_group, stream); break;
    case 2: launch_passes<2>(tab, window, n_rows, rows_per_block, log2_scale, inv_group, stream); break;
    case 3: launch_passes<3>(tab, window, n_rows, rows_per_block, log2_scale, inv_group, stream); break;
    case 4: launch_passes<4>(tab, window, n_rows, rows_per_block, log2_scale, inv_group, stream); break;
    default: return;
  }
  WinTable pool = tab;
  int64_t blocks = 0;
  for (int i = 0; i < tab.n; ++i) {
    pool.first[i] = (int32_t)blocks;
    blocks += (int64_t)heads * ((tab.T[i] + 1023) >> 10);
  }
  pool.first[tab.n] = (int32_t)blocks;
  hipLaunchKernelGGL(score_window_pool_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, pool, window,
                     (pool_width - 1) / 2, pool_kind);
}

}  // namespace lkv
