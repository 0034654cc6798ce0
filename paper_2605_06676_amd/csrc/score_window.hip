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
//   merge   the pairs of all blocks of a head into each row's log-normaliser (a small kernel);
//   pass 2  recomputes the logits and adds exp(logit - normaliser) over the rows: the token's vote,
//           the two waves of a block adding their rows' shares in LDS; then the block takes the
//           group mean, smooths and writes the scores of its keys.  The pooling reaches into the
//           neighbouring blocks' keys, so a block also computes the votes of up to two tiles on
//           either side of its own (3 to 6 % more work, less than a pooling launch costs).
// Keeping the logits instead would cost as many bytes as reading the keys again (G W = 128
// logits per 128-element key).  A caller that still has the log-normalisers of the window rows
// (the prefill's attention kernel computes them for every query) passes them in: pass 1 and the
// merge are skipped and the keys are read once.
//
// Pass 1 keeps a running reference per (row, lane) instead of a running maximum: the sum is
// taken relative to a reference that is only moved when a logit exceeds it by more than 64
// binary orders of magnitude, which costs one exponential per logit instead of two.  Any
// reference within that distance of the true maximum gives the same sum to fp32 rounding.
//
// A block is a pair of waves that share the staged keys (two tiles of 16 between barriers); the
// window rows are split between the two (at most 64 rows, 64 fragment registers, per wave).
// Both passes are bound by instruction issue rather than by HBM: per key and row one exponential
// (quarter rate) next to the matrix work, which the hardware overlaps only in part.
#include "lkv_common.h"

namespace lkv {

constexpr int kWinThreads = 128;
constexpr int kWinTokTile = 16;                  // keys per MFMA N tile
constexpr int kWinRowStride = 256 + 32;          // bytes per staged key row in LDS
constexpr int kWinTileLds = kWinTokTile * kWinRowStride;
constexpr int kWinTilesPerStep = 2;     // tiles staged, multiplied and finished between two barriers
constexpr int kWinStepLds = kWinTilesPerStep * kWinTileLds;
constexpr int kWinMaxRowsPerBlock = 1024;
constexpr int kWinMaxReach = 31;                // pooling widths up to 63
constexpr int kWinVoteSlots = kWinMaxRowsPerBlock + 32 + kWinMaxReach + 17;   // pass 2: a block's keys, two tiles before, the reach after, rounded up to a tile
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

// kPass 1: partial log-sum-exp pairs.  kPass 2: votes (the merged normalisers are read from the
// workspace).  MTW: 16-row M tiles per wave; the rows past n_rows = G W are padding (zero queries,
// never counted).
template <int MTW, int kPass>
__global__ void __launch_bounds__(kWinThreads, 2)
score_window_kernel(WinTable tab, int heads, int window, int n_rows, int rows_per_block, float log2_scale,
                    int reach /* pass 2: pooling reach c, width 2 c + 1 */, int pool_kind, float inv_group) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int RP = 32 * MTW;                      // padded rows of the block

  const int seq = win_seq_of_unit(tab, blockIdx.x);
  const int local = blockIdx.x - tab.first[seq];
  const int T = tab.T[seq];
  const int chunks = (T + rows_per_block - 1) / rows_per_block;
  const int lh = local / chunks;
  const int chunk = local - lh * chunks;
  const int prefix = T - window;                    // tokens that are scored

  // The block's own keys, and the keys it multiplies: in pass 2 also those within the pooling's reach on either
  // side (whole tiles before, single keys after), as far as they lie inside the prefix.
  const int own_row0 = chunk * rows_per_block;
  const int own_end = min(T, own_row0 + rows_per_block);
  const int block_end_all = kPass == 1 ? T : prefix;    // pass 2 has no votes to compute inside the window
  float* out = tab.scores[seq] + (size_t)lh * T;
  if (own_row0 >= block_end_all) {
    if (kPass == 2)   // a block of window tokens
      for (int j = own_row0 + (int)threadIdx.x; j < own_end; j += kWinThreads) out[j] = INFINITY;
    return;
  }
  const int halo = kPass == 2 ? ((reach + 15) >> 4) << 4 : 0;
  const int block_row0 = max(0, own_row0 - halo);
  const int block_end = kPass == 1 ? own_end : min(prefix, own_end + reach);
  const int block_rows = block_end - block_row0;
  const int n_tiles = (block_rows + 15) >> 4;

  const int lane = threadIdx.x & 63;
  const int half = threadIdx.x >> 6;
  const int r = lane >> 4;
  const int c = lane & 15;
  unsigned char* x_lds = smem;   // the staged keys of two steps
  // pass 2: the votes of the keys the block multiplies; both waves add the shares of their rows
  float* v_lds = reinterpret_cast<float*>(smem + 2 * kWinStepLds);
  if (kPass == 2)
    for (int i = threadIdx.x; i < kWinVoteSlots; i += kWinThreads) v_lds[i] = 0.f;   // ordered by the barrier below

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
    if (tab.lse[seq] != nullptr) {
      // the caller's log-normalisers (natural logarithm, one per window row of the group: what the prefill's
      // attention kernel already returns for these queries); padding rows get +inf, i.e. weight zero
      const float* lse = tab.lse[seq] + (size_t)lh * n_rows;
#pragma unroll
      for (int mw = 0; mw < MTW; ++mw)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int row = 16 * (half * MTW + mw) + 4 * r + e;
          ref[mw][e] = row < n_rows ? lse[row] * 1.44269504088896340736f : INFINITY;
        }
    } else {
      // log-normaliser of every row, merged from the pairs of pass 1 by the kernel in between
      const float* lse = tab.partial[seq] + (size_t)heads * chunks * RP * 2 + (size_t)lh * RP;
#pragma unroll
      for (int mw = 0; mw < MTW; ++mw) {
        const f32x4_t v = *reinterpret_cast<const f32x4_t*>(lse + 16 * (half * MTW + mw) + 4 * r);
#pragma unroll
        for (int e = 0; e < 4; ++e) ref[mw][e] = v[e];
      }
    }
  }

  const uint4* Kh = reinterpret_cast<const uint4*>(tab.k[seq]) + (size_t)lh * (size_t)T * kChunksPerRow;

  // Staging: thread (half, r, c) brings piece c of rows 16 nt + 8 half + r and 16 nt + 8 half + 4 + r of each step.
  constexpr int NT = kWinTilesPerStep;
  uint4 xa[2 * NT], xb[2 * NT];
  // No branch encloses a load between its issue and the staging that waits for it: the compiler counts the loads
  // still in flight at a wait from the path on which the fewest were issued, so a conditional load makes every wait
  // drain the whole queue.  Steps past the block's rows are clamped instead of skipped.
  const int last_row = block_row0 + block_rows - 1;
  auto load_step = [&](uint4 (&xx)[2 * NT], int i) {
#pragma unroll
    for (int j = 0; j < 2 * NT; ++j) {
      int row = block_row0 + 16 * NT * i + 16 * (j >> 1) + 8 * half + 4 * (j & 1) + r;
      row = row < last_row ? row : last_row;   // past the block's rows: re-read its last row, masked below
      xx[j] = load_stream16(Kh + (size_t)row * kChunksPerRow + c);
    }
  };
  auto stage_step = [&](const uint4 (&xx)[2 * NT], int buf) {
#pragma unroll
    for (int j = 0; j < 2 * NT; ++j)
      *reinterpret_cast<uint4*>(x_lds + buf * kWinStepLds + (16 * (j >> 1) + 8 * half + 4 * (j & 1) + r) * kWinRowStride + c * 16) = xx[j];
  };
  auto products = [&](f32x4_t (&acc)[MTW], const unsigned char* xt) {
#pragma unroll
    for (int mw = 0; mw < MTW; ++mw) acc[mw] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const uint4 x = *reinterpret_cast<const uint4*>(xt + c * kWinRowStride + ks * 64 + r * 16);
      const bf16x8_t xv = __builtin_bit_cast(bf16x8_t, x);
#pragma unroll
      for (int mw = 0; mw < MTW; ++mw)
        acc[mw] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qfrag[mw][ks], xv, acc[mw], 0, 0, 0);
    }
  };
  auto finish = [&](const f32x4_t (&acc)[MTW], int tile) {   // tile: 16-key tile of the block
    const int row0 = block_row0 + 16 * tile;
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
      part = sum_over_row_blocks(part);
      // two additions to a zero: the same sum whichever wave comes first
      if (r == 0 && row0 + c < block_end) atomicAdd(&v_lds[row0 + c - block_row0], part);
    }
  };

  // Barrier i makes the keys of step i visible and means both waves have finished reading those of step i - 1.
  const int n_steps = (n_tiles + NT - 1) / NT;
  // One step: products and arithmetic of its NT tiles, staging of step i + 1 (fetching step i + 3 behind it).
  f32x4_t acc[NT][MTW];
  auto step = [&](uint4 (&x_next)[2 * NT], int i) {
    const unsigned char* xt = x_lds + (i & 1) * kWinStepLds;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) products(acc[nt], xt + nt * kWinTileLds);
    stage_step(x_next, (i + 1) & 1);               // past the last step: rows nobody reads
    load_step(x_next, i + 3);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) finish(acc[nt], NT * i + nt);
    __syncthreads();
  };
  load_step(xa, 0);
  load_step(xb, 1);
  stage_step(xa, 0);
  load_step(xa, 2);
  __syncthreads();
  int i = 0;
#pragma unroll 1
  for (; i + 1 < n_steps; i += 2) {
    step(xb, i);                                   // stages the odd step i + 1
    step(xa, i + 1);
  }
  if (i < n_steps) step(xb, i);

  if (kPass == 2) {
    // Scores of the block's own keys: centred pooling over the votes inside the prefix (votes are non-negative and
    // the slots outside hold zeros, which change neither rule), group mean, +inf on window tokens.  The last
    // barrier of the loop has made all votes visible.
    const float inv_width = 1.f / (float)(2 * reach + 1);
    for (int j = own_row0 + (int)threadIdx.x; j < own_end; j += kWinThreads) {
      float sc = INFINITY;
      if (j < prefix) {
        const int lo = j - reach - block_row0;   // may be negative at the start of the head
        sc = 0.f;
        if (pool_kind == 0) {
          for (int u = 0; u <= 2 * reach; ++u) {
            const int t = lo + u;
            sc = fmaxf(sc, t >= 0 && t < block_rows ? v_lds[t] : 0.f);
          }
          sc *= inv_group;
        } else {
          for (int u = 0; u <= 2 * reach; ++u) {
            const int t = lo + u;
            sc += t >= 0 && t < block_rows ? v_lds[t] : 0.f;
          }
          sc *= inv_width * inv_group;
        }
      }
      out[j] = sc;
    }
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
  }
}

// Between the passes: the log-normaliser (log2 units) of every window row of every head, from the pairs
// the blocks of pass 1 left; +inf for the padding rows, whose weights then vanish.  One block per head.
__global__ void __launch_bounds__(128)
score_window_merge_kernel(WinTable tab, int heads, int n_rows, int rows_per_block, int padded_rows) {
  const int seq = blockIdx.x / heads;
  const int lh = blockIdx.x - seq * heads;
  const int chunks = (tab.T[seq] + rows_per_block - 1) / rows_per_block;
  const float* part = tab.partial[seq] + (size_t)lh * chunks * padded_rows * 2;
  float* lse = tab.partial[seq] + (size_t)heads * chunks * padded_rows * 2 + (size_t)lh * padded_rows;
  const int row = threadIdx.x;
  if (row >= padded_rows) return;
  float out = INFINITY;
  if (row < n_rows) {
    const float2* pairs = reinterpret_cast<const float2*>(part) + row;
    float m = kWinNoRef;
#pragma unroll 8
    for (int ch = 0; ch < chunks; ++ch) m = fmaxf(m, pairs[(size_t)ch * padded_rows].x);
    float l = 0.f;
#pragma unroll 8
    for (int ch = 0; ch < chunks; ++ch) {
      const float2 p = pairs[(size_t)ch * padded_rows];
      l += p.y * __builtin_amdgcn_exp2f(p.x - m);
    }
    out = m + __log2f(l);
  }
  lse[row] = out;
}

int score_window_max_rows() { return 128; }

int score_window_rows_per_block(int64_t tokens_times_heads) {
  // large blocks amortise the query fragments each wave loads; small problems take smaller blocks so
  // that the grid still covers the chip
  int rows = kWinMaxRowsPerBlock;
  while (rows > 128 && tokens_times_heads / rows < 2048) rows >>= 1;
  return rows;
}

// Workspace of one sequence: pairs [heads, ceil(T / 128), 128, 2] (the largest the pairs can get: the smallest
// block and the most padded rows) followed by the merged normalisers [heads, 128]; 256-byte aligned.
size_t score_window_pairs_bytes(int64_t heads, int T) {
  return ((size_t)heads * (((T + 127) / 128) * 2 + 1) * 128 * sizeof(float) + 255) & ~(size_t)255;
}

template <int MTW>
static void launch_passes(const WinTable& tab, int heads, int window, int n_rows, int rows_per_block, float log2_scale,
                          int reach, int pool_kind, float inv_group, hipStream_t stream) {
  const int blocks = tab.first[tab.n];
  const size_t lds1 = 2 * kWinStepLds;
  const size_t lds2 = lds1 + kWinVoteSlots * sizeof(float);
  if (tab.lse[0] == nullptr) {   // all sequences of a call come with normalisers, or none does
    hipLaunchKernelGGL((score_window_kernel<MTW, 1>), dim3(blocks), dim3(kWinThreads), lds1, stream, tab, heads, window,
                       n_rows, rows_per_block, log2_scale, 0, 0, 0.f);
    hipLaunchKernelGGL(score_window_merge_kernel, dim3(tab.n * heads), dim3(128), 0, stream, tab, heads, n_rows,
                       rows_per_block, 32 * MTW);
  }
  hipLaunchKernelGGL((score_window_kernel<MTW, 2>), dim3(blocks), dim3(kWinThreads), lds2, stream, tab, heads, window,
                     n_rows, rows_per_block, log2_scale, reach, pool_kind, inv_group);
}

// `tab.first` counts the blocks of the passes (the same grid for both).
void launch_score_window(const WinTable& tab, int heads, int window, int group, int pool_width, int pool_kind,
                         int rows_per_block, float scale, hipStream_t stream) {
  if (tab.n <= 0) return;
  const int n_rows = group * window;
  const float log2_scale = scale * 1.44269504088896340736f;
  const float inv_group = 1.f / (float)group;
  const int reach = (pool_width - 1) / 2;
  if (reach > kWinMaxReach) return;   // the host checks the width before
  switch ((n_rows + 31) / 32) {
    case 1: launch_passes<1>(tab, heads, window, n_rows, rows_per_block, log2_scale, reach, pool_kind, inv_group, stream); break;
    case 2: launch_passes<2>(tab, heads, window, n_rows, rows_per_block, log2_scale, reach, pool_kind, inv_group, stream); break;
    case 3: launch_passes<3>(tab, heads, window, n_rows, rows_per_block, log2_scale, reach, pool_kind, inv_group, stream); break;
    case 4: launch_passes<4>(tab, heads, window, n_rows, rows_per_block, log2_scale, reach, pool_kind, inv_group, stream); break;
    default: return;
  }
}

}  // namespace lkv
