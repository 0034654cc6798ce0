// LKV-T token scoring with the two-layer MLP of Sec. 3.4 / Table 5 of the
// paper: u = w2 . act(W1 [k ; v] + b1) (+ b2), hidden width 16..128.
//
// The hidden layer is the one dense contraction of the eviction path
// ([tokens x 256] x [256 x hidden], about 64 flop per byte streamed for
// hidden = 64), so it runs on the matrix cores: v_mfma_f32_16x16x32_bf16 with
// the hidden units on the M side and 16 tokens on the N side,
//     D[hidden, token] = W1[hidden, 0:256] . X[token, 0:256]^T + b1.
//  * W1 fragments (A operand) stay in registers for the whole block:
//    lane (i, kb) holds W1[16 mt + i][32 ks + 8 kb .. +7].
//  * Token rows are read from HBM once, coalesced (16 lanes x 16 bytes per
//    row), staged in a wave-private LDS tile whose row stride of 544 bytes
//    makes the fragment reads conflict free, and read back as B fragments:
//    lane (n, kb) holds X[token n][32 ks + 8 kb .. +7].
//  * The accumulator layout leaves each lane with 4 hidden units of one token
//    per M tile, so bias (as the initial accumulator), activation and the dot
//    with w2 are per-lane work, finished by two cross-lane adds.
// The next two 16-token tiles are prefetched into registers while the current
// one is multiplied; b1 and w2 are read from LDS.
#include <type_traits>
#include "lkv_act.h"
#include "lkv_common.h"

namespace lkv {

constexpr int kMlpThreads = 256;
constexpr int kMlpWaves = kMlpThreads / 64;
constexpr int kMlpTokTile = 16;                       // tokens per MFMA N tile
constexpr int kMlpRowStride = 2 * 256 + 32;           // bytes per staged [k ; v] row in LDS
constexpr int kMlpWaveLds = kMlpTokTile * kMlpRowStride;
constexpr int kMlpKSteps = 8;                         // 256 features / 32 per MFMA

__device__ __forceinline__ bf16x8_t as_bf16x8(const uint4& p) {
  return __builtin_bit_cast(bf16x8_t, p);
}

// Hidden widths up to 64: one wave multiplies a tile by the whole W1 (128 registers), two waves per SIMD.
// kCount: the block also counts the first-level top-k digits of the scores it writes (LDS histogram, added to the
// segment's global counters at the end); segment = seg_base + sequence * seg_stride + head of the view.
template <int MT, int kAct, bool kCount>
__global__ void __launch_bounds__(kMlpThreads, 2)
score_mlp_kernel(SeqTable tab, const uint16_t* __restrict__ w1, const float* __restrict__ b1,
                 const float* __restrict__ w2, const float* __restrict__ b2, int heads_per_scorer_row,
                 int rows_per_block, uint32_t* __restrict__ counts, int seg_base, int seg_stride) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int HID = MT * 16;

  const int seq = seq_of_unit(tab, blockIdx.x);
  const int local = blockIdx.x - tab.first[seq];
  const int T = tab.T[seq];
  const int tiles = (T + rows_per_block - 1) / rows_per_block;
  const int lh = local / tiles;
  const int tile = local - lh * tiles;
  const int scorer = lh / heads_per_scorer_row;

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int r = lane >> 4;        // coalesced-load view: row slot; fragment view: feature block kb
  const int c = lane & 15;        // coalesced-load view: 16-byte piece; fragment view: token n / hidden unit i
  unsigned char* tile_lds = smem + wave * kMlpWaveLds;

  // A fragments: W1[16 mt + c][32 ks + 8 r .. +7]
  bf16x8_t wfrag[MT][kMlpKSteps];
  {
    const uint4* wbase = reinterpret_cast<const uint4*>(w1 + (size_t)scorer * HID * 256);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int ks = 0; ks < kMlpKSteps; ++ks)
        wfrag[mt][ks] = as_bf16x8(wbase[(size_t)(mt * 16 + c) * 32 + ks * 4 + r]);
  }
  // b1 and w2 live in LDS (block-shared): lane (r, c) needs hidden units 16 mt + 4 r + e, which
  // are 16-byte groups, so each is one broadcast LDS read per M tile.  Keeping them out of the
  // register file leaves room for a second prefetch buffer.
  float* par_lds = reinterpret_cast<float*>(smem + kMlpWaves * kMlpWaveLds);   // b1[HID] then w2[HID]
  uint32_t* hist_lds = reinterpret_cast<uint32_t*>(par_lds + 2 * HID);          // [kLevel0Bins] when counting
  for (int i = threadIdx.x; i < 2 * HID; i += kMlpThreads)
    par_lds[i] = i < HID ? b1[(size_t)scorer * HID + i] : w2[(size_t)scorer * HID + i - HID];
  if (kCount)
    for (int i = threadIdx.x; i < kLevel0Bins; i += kMlpThreads) hist_lds[i] = 0;
  const float bias2 = b2 != nullptr ? b2[scorer] : 0.f;
  __syncthreads();

  const size_t head_row0 = (size_t)lh * (size_t)T;
  const uint4* Kh = reinterpret_cast<const uint4*>(tab.k[seq]) + head_row0 * kChunksPerRow;
  const uint4* Vh = reinterpret_cast<const uint4*>(tab.v[seq]) + head_row0 * kChunksPerRow;
  float* out = tab.scores[seq] + head_row0;

  // The four waves of a block interleave 16-row tiles: tile i of wave w covers rows
  // block_row0 + 64 i + 16 w, so that the block as a whole reads 16 KB of K and 16 KB of V
  // contiguously at a time (DRAM pages are used better than with four distant 4 KB streams).
  constexpr int kStep = kMlpWaves * kMlpTokTile;                 // 64 rows between a wave's tiles
  const int wave_row0 = tile * rows_per_block + wave * kMlpTokTile;
  const int wave_row1 = min(T, tile * rows_per_block + rows_per_block);
  if (!kCount && wave_row0 >= wave_row1) return;   // after the only block barrier (a counting block has one more)

  // Two register buffers of 16 rows each: while one tile is multiplied, the loads of the next
  // two are in flight (16 KB per wave), which is what it takes to keep HBM busy at two waves
  // per SIMD.
  uint4 ka[4], va[4], kb[4], vb[4];
  auto load_tile = [&](uint4 (&kk)[4], uint4 (&vv)[4], int row0) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int row = row0 + 4 * j + r;
      row = row < wave_row1 ? row : wave_row1 - 1;   // past the block's rows: re-read its last row, result unused
      kk[j] = load_stream16(Kh + (size_t)row * kChunksPerRow + c);
      vv[j] = load_stream16(Vh + (size_t)row * kChunksPerRow + c);
    }
  };
  auto stage_tile = [&](const uint4 (&kk)[4], const uint4 (&vv)[4]) {
    // row 4j + r, key piece c at byte 16c, value piece c at byte 256 + 16c
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      unsigned char* rowp = tile_lds + (4 * j + r) * kMlpRowStride + c * 16;
      *reinterpret_cast<uint4*>(rowp) = kk[j];
      *reinterpret_cast<uint4*>(rowp + 256) = vv[j];
    }
  };
  auto wave_lds_sync = [&]() {   // the tile is private to this wave: order its LDS accesses, no barrier
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  auto multiply_tile = [&](int row0) {
    wave_lds_sync();
    f32x4_t acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = *reinterpret_cast<const f32x4_t*>(par_lds + mt * 16 + 4 * r);   // bias
#pragma unroll
    for (int ks = 0; ks < kMlpKSteps; ++ks) {
      // B fragment: token c, features 32 ks + 8 r .. +7  = bytes 64 ks + 16 r of the staged row
      const uint4 x = *reinterpret_cast<const uint4*>(tile_lds + c * kMlpRowStride + ks * 64 + r * 16);
      const bf16x8_t xb = as_bf16x8(x);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfrag[mt][ks], xb, acc[mt], 0, 0, 0);
    }
    float part = 0.f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const f32x4_t wo = *reinterpret_cast<const f32x4_t*>(par_lds + HID + mt * 16 + 4 * r);
#pragma unroll
      for (int e = 0; e < 4; ++e) part = fmaf(wo[e], activation<kAct>(acc[mt][e]), part);
    }
    // sum the four feature-block lanes of each token: lanes c, c+16, c+32, c+48
    part = sum_over_row_blocks(part);
    const int row = row0 + c;
    if (r == 0 && row < T) {
      const float u = part + bias2;
      out[row] = u;
      if (kCount) atomicAdd(&hist_lds[order_key(u) >> kLevel0Shift], 1u);
    }
    wave_lds_sync();   // the next staging overwrites the tile
  };

  if (wave_row0 < wave_row1) {
    // No branch encloses a load between its issue and the staging that waits for it: the compiler counts the
    // loads still in flight at a wait from the path on which the fewest were issued, so a conditional load makes
    // every wait drain the whole queue.  Loads past the block's rows are clamped instead of skipped.
    load_tile(ka, va, wave_row0);
    load_tile(kb, vb, wave_row0 + kStep);
    int row0 = wave_row0;
#pragma unroll 1
    for (; row0 + kStep < wave_row1; row0 += 2 * kStep) {
      stage_tile(ka, va);
      load_tile(ka, va, row0 + 2 * kStep);
      multiply_tile(row0);
      stage_tile(kb, vb);
      load_tile(kb, vb, row0 + 3 * kStep);
      multiply_tile(row0 + kStep);
    }
    if (row0 < wave_row1) {
      stage_tile(ka, va);
      multiply_tile(row0);
    }
  }
  if (kCount) {
    __syncthreads();
    flush_level0_counts(hist_lds, counts, (size_t)(seg_base + seq * seg_stride + lh), kMlpThreads);
  }
}

// Hidden widths 80..128 (the paper's network is 256 -> 128 -> 1): W1 no longer fits the registers of
// one wave at two waves per SIMD, so the hidden units are split over a pair of waves, and a block is
// one pair.  Wave `half` keeps the fragments of M tiles [half * MTW, half * MTW + MTW) and both
// multiply the same staged 16-token tile; the two partial sums of a token meet in LDS.  Staging is
// split evenly: wave 0 brings the key halves of the rows, wave 1 the value halves, each two tiles
// ahead in registers.  The tile and the partial-sum slots are double buffered and one barrier per
// tile orders everything: a wave that stages tile i + 1 has passed barrier i, so its partner has
// finished reading tile i - 1.
// A wave issues in order, so every LDS round trip inside a step is time in which it issues nothing,
// and with two waves per SIMD there is little else to run: the output-layer weights therefore stay in
// registers, the bias is read at the top of the step together with the operand fragments, and the
// four-lane sums use row swaps instead of LDS shuffles (together 7 % faster than with all three in
// LDS).  A third register set for rows in flight, or no barrier at all, changed nothing measurable.
constexpr int kWideThreads = 128;

template <int MTW, int kAct, bool kCount>
__global__ void __launch_bounds__(kWideThreads, 2)
score_mlp_wide_kernel(SeqTable tab, const uint16_t* __restrict__ w1, const float* __restrict__ b1,
                      const float* __restrict__ w2, const float* __restrict__ b2, int hidden,
                      int heads_per_scorer_row, int rows_per_block, uint32_t* __restrict__ counts, int seg_base,
                      int seg_stride) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int HW = MTW * 16;                      // hidden units per wave (zero padded past `hidden`)
  const int MT = hidden / 16;

  const int seq = seq_of_unit(tab, blockIdx.x);
  const int local = blockIdx.x - tab.first[seq];
  const int T = tab.T[seq];
  const int tiles = (T + rows_per_block - 1) / rows_per_block;
  const int lh = local / tiles;
  const int tile = local - lh * tiles;
  const int scorer = lh / heads_per_scorer_row;

  const int lane = threadIdx.x & 63;
  const int half = threadIdx.x >> 6;
  const int r = lane >> 4;
  const int c = lane & 15;
  // LDS: two staged tiles, then [buffer][16] partial sums, then b1 / w2 (zero padded)
  unsigned char* x_lds = smem;
  float* sum_lds = reinterpret_cast<float*>(smem + 2 * kMlpWaveLds);
  float* par_lds = sum_lds + 32;   // b1[2 HW] then w2[2 HW]
  uint32_t* hist_lds = reinterpret_cast<uint32_t*>(par_lds + 4 * HW);   // [kLevel0Bins] when counting
  if (kCount)
    for (int i = threadIdx.x; i < kLevel0Bins; i += kWideThreads) hist_lds[i] = 0;

  bf16x8_t wfrag[MTW][kMlpKSteps];
  {
    const uint4* wbase = reinterpret_cast<const uint4*>(w1 + (size_t)scorer * hidden * 256);
#pragma unroll
    for (int mw = 0; mw < MTW; ++mw) {
      const int mt = half * MTW + mw;
#pragma unroll
      for (int ks = 0; ks < kMlpKSteps; ++ks) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (mt < MT) v = wbase[(size_t)(mt * 16 + c) * 32 + ks * 4 + r];
        wfrag[mw][ks] = as_bf16x8(v);
      }
    }
  }
  for (int i = threadIdx.x; i < 4 * HW; i += kWideThreads) {
    const int j = i < 2 * HW ? i : i - 2 * HW;
    const float* src = i < 2 * HW ? b1 : w2;
    par_lds[i] = j < hidden ? src[(size_t)scorer * hidden + j] : 0.f;
  }
  const float bias2 = b2 != nullptr ? b2[scorer] : 0.f;
  __syncthreads();
  // lane (r, c) owns hidden units 16 mw + 4 r + e of its wave's share: their bias and output weight
  f32x4_t b1r[MTW], w2r[MTW];
#pragma unroll
  for (int mw = 0; mw < MTW; ++mw) {
    b1r[mw] = *reinterpret_cast<const f32x4_t*>(par_lds + half * HW + mw * 16 + 4 * r);
    w2r[mw] = *reinterpret_cast<const f32x4_t*>(par_lds + 2 * HW + half * HW + mw * 16 + 4 * r);
  }

  const size_t head_row0 = (size_t)lh * (size_t)T;
  // this wave's half of the rows: keys for wave 0, values for wave 1
  const uint4* Xh = reinterpret_cast<const uint4*>(half == 0 ? tab.k[seq] : tab.v[seq]) + head_row0 * kChunksPerRow;
  float* out = tab.scores[seq] + head_row0;

  // tile i covers rows block_row0 + 16 i; rows past the end are clamped on load and not stored
  const int block_row0 = tile * rows_per_block;
  const int block_rows = min(T - block_row0, rows_per_block);
  const int n_tiles = (block_rows + 15) >> 4;

  uint4 xa[4], xb[4];   // this wave's halves of an even and of an odd tile on their way to LDS
  // Rows of a tile that lies wholly inside the head are addressed as a wave-uniform base (scalar arithmetic) plus a
  // per-lane constant, so a load costs no vector instruction for its address (the kernel is short of vector issue
  // slots, not of anything else); only a tile that reaches past the end of the head clamps its rows one by one.
  const uint4* Xb = Xh + (size_t)block_row0 * kChunksPerRow;            // uniform
  const int lane_off = r * kChunksPerRow + c;                           // in 16-byte pieces; + 64 per group of four rows
  const int full_tiles = (T - block_row0) >> 4;                         // tiles of this block with all 16 rows inside the head
  // No branch encloses a load between its issue and the staging that waits for it (the compiler counts the loads
  // still in flight at a wait from the path on which the fewest were issued, so a conditional load makes every
  // wait drain the whole queue): tiles past the block's rows are clamped, not skipped.
  const int last_row = block_row0 + block_rows - 1;
  auto load_half_fast = [&](uint4 (&xx)[4], int i) {   // tile i lies wholly inside the block's rows
    const uint4* tb = Xb + (size_t)i * (16 * kChunksPerRow);
#pragma unroll
    for (int j = 0; j < 4; ++j) xx[j] = load_stream16(tb + lane_off + j * (4 * kChunksPerRow));
  };
  auto load_half = [&](uint4 (&xx)[4], int i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int row = block_row0 + 16 * i + 4 * j + r;
      row = row < last_row ? row : last_row;
      xx[j] = load_stream16(Xh + (size_t)row * kChunksPerRow + c);
    }
  };
  auto stage_half = [&](const uint4 (&xx)[4], int buf) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      *reinterpret_cast<uint4*>(x_lds + buf * kMlpWaveLds + (4 * j + r) * kMlpRowStride + half * 256 + c * 16) = xx[j];
  };
  float prev = 0.f;   // wave 0: its own partial sums of the tile before this one
  auto products = [&](f32x4_t (&acc)[MTW], int i) {   // W1 times the staged tile i, bias as the initial value
#pragma unroll
    for (int mw = 0; mw < MTW; ++mw) acc[mw] = b1r[mw];
    const unsigned char* xt = x_lds + (i & 1) * kMlpWaveLds;
#pragma unroll
    for (int ks = 0; ks < kMlpKSteps; ++ks) {
      const uint4 x = *reinterpret_cast<const uint4*>(xt + c * kMlpRowStride + ks * 64 + r * 16);
      const bf16x8_t xv = as_bf16x8(x);
#pragma unroll
      for (int mw = 0; mw < MTW; ++mw)
        acc[mw] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfrag[mw][ks], xv, acc[mw], 0, 0, 0);
    }
  };
  auto store_before = [&](int i) {   // scores of tile i - 1: wave 0 adds the partner's partial sums, visible since barrier i - 1
    if (half == 0 && i >= 1) {
      const int row = block_row0 + 16 * (i - 1) + c;
      if (r == 0 && row < T) {
        const float u = prev + sum_lds[((i - 1) & 1) * 16 + c] + bias2;
        out[row] = u;
        if (kCount) atomicAdd(&hist_lds[order_key(u) >> kLevel0Shift], 1u);
      }
    }
  };
  auto finish = [&](const f32x4_t (&acc)[MTW], int i) {   // activation and output layer of tile i, partial sums exchanged
    float part = 0.f;
#pragma unroll
    for (int mw = 0; mw < MTW; ++mw)
#pragma unroll
      for (int e = 0; e < 4; ++e) part = fmaf(w2r[mw][e], activation<kAct>(acc[mw][e]), part);
    part = sum_over_row_blocks(part);
    if (half == 1) {
      if (r == 0) sum_lds[(i & 1) * 16 + c] = part;
    } else {
      prev = part;
    }
  };
  auto advance = [&](uint4 (&x_next)[4], int stage_tile, int load_tile, auto fast) {   // then the step's barrier
    stage_half(x_next, stage_tile & 1);   // past the last tile: rows nobody reads
    if (decltype(fast)::value) load_half_fast(x_next, load_tile); else load_half(x_next, load_tile);
    __syncthreads();
  };
  const int fast_tiles = min(n_tiles, full_tiles);   // tiles with all 16 rows inside the block and the head
  int i = 0;
  load_half(xa, 0);
  load_half(xb, 1);
  stage_half(xa, 0);
  load_half(xa, 2);
  __syncthreads();   // tile 0 is in LDS
  if (!kCount) {
    // Pipelined in the wave: the products of tile i + 1 sit in one scheduling region with the activations of tile i
    // (a second accumulator set), so that matrix and vector instructions alternate; tiles are staged one step
    // earlier for it.  1 % faster than the plain order below; with the histogram's registers on top it spills.
    f32x4_t acc0[MTW], acc1[MTW];
    auto step = [&](const f32x4_t (&acc_cur)[MTW], f32x4_t (&acc_next)[MTW], uint4 (&x_next)[4], int i, auto fast) {
      store_before(i);
      products(acc_next, i + 1);   // after the last tile: a stale buffer, result dropped
      finish(acc_cur, i);
      advance(x_next, i + 2, i + 4, fast);
    };
    products(acc0, 0);
    stage_half(xb, 1);
    load_half(xb, 3);
    __syncthreads();   // tile 1 is in LDS, the fragments of tile 0 have been read
#pragma unroll 1
    for (; i + 5 < fast_tiles; i += 2) {           // both steps fetch whole tiles: tiles i + 4 and i + 5
      step(acc0, acc1, xa, i, std::true_type{});
      step(acc1, acc0, xb, i + 1, std::true_type{});
    }
#pragma unroll 1
    for (; i + 1 < n_tiles; i += 2) {
      step(acc0, acc1, xa, i, std::false_type{});
      step(acc1, acc0, xb, i + 1, std::false_type{});
    }
    if (i < n_tiles) step(acc0, acc1, xa, i, std::false_type{});
  } else {
    // One step: products, activation and output layer of tile i; store of tile i - 1; staging of tile i + 1, whose
    // registers then fetch tile i + 3; barrier i.
    auto step = [&](uint4 (&x_next)[4], int i, auto fast) {
      f32x4_t acc[MTW];
      products(acc, i);
      store_before(i);
      finish(acc, i);
      advance(x_next, i + 1, i + 3, fast);
    };
#pragma unroll 1
    for (; i + 4 < fast_tiles; i += 2) {           // both steps fetch whole tiles: tiles i + 3 and i + 4
      step(xb, i, std::true_type{});               // stages the odd tile i + 1
      step(xa, i + 1, std::true_type{});
    }
#pragma unroll 1
    for (; i + 1 < n_tiles; i += 2) {
      step(xb, i, std::false_type{});
      step(xa, i + 1, std::false_type{});
    }
    if (i < n_tiles) step(xb, i, std::false_type{});
  }

  if (half == 0) {
    const int row = block_row0 + 16 * (n_tiles - 1) + c;
    if (r == 0 && row < T) {
      const float u = prev + sum_lds[((n_tiles - 1) & 1) * 16 + c] + bias2;
      out[row] = u;
      if (kCount) atomicAdd(&hist_lds[order_key(u) >> kLevel0Shift], 1u);
    }
  }
  if (kCount) {
    __syncthreads();
    flush_level0_counts(hist_lds, counts, (size_t)(seg_base + seq * seg_stride + lh), kWideThreads);
  }
}

int score_mlp_rows_per_block(int T, int heads, int hidden) {
  // large tiles amortise the W1 fragments each wave loads; short heads, and launches over few
  // heads (one layer at a time), take smaller tiles so that the grid still covers the chip.
  // The wave-pair kernel has twice as many resident blocks, so half the rows give it as many rounds.
  const int longest = hidden > 64 ? 2048 : 4096;
  int rows = T >= 16384 ? longest : (T >= 4096 ? 1024 : 256);
  while (rows > 256 && (int64_t)heads * ((T + rows - 1) / rows) < 1024) rows >>= 1;
  return rows;
}

hipError_t score_mlp_prepare() { return hipSuccess; }

template <int MT, bool kCount>
static void launch_mt(const SeqTable& tab, const uint16_t* w1, const float* b1, const float* w2,
                      const float* b2, int act, int heads_per_scorer_row, int rows_per_block,
                      uint32_t* counts, int seg_base, int seg_stride, hipStream_t stream) {
  const int blocks = tab.first[tab.n];
  const size_t lds = (size_t)kMlpWaves * kMlpWaveLds + 2 * MT * 16 * sizeof(float) + (kCount ? kLevel0Bins * 4 : 0);
  if (act == kActSilu)
    hipLaunchKernelGGL((score_mlp_kernel<MT, kActSilu, kCount>), dim3(blocks), dim3(kMlpThreads), lds, stream, tab,
                       w1, b1, w2, b2, heads_per_scorer_row, rows_per_block, counts, seg_base, seg_stride);
  else
    hipLaunchKernelGGL((score_mlp_kernel<MT, kActGelu, kCount>), dim3(blocks), dim3(kMlpThreads), lds, stream, tab,
                       w1, b1, w2, b2, heads_per_scorer_row, rows_per_block, counts, seg_base, seg_stride);
}

template <int MTW, bool kCount>
static void launch_wide(const SeqTable& tab, const uint16_t* w1, const float* b1, const float* w2,
                        const float* b2, int hidden, int act, int heads_per_scorer_row, int rows_per_block,
                        uint32_t* counts, int seg_base, int seg_stride, hipStream_t stream) {
  const int blocks = tab.first[tab.n];
  const size_t lds = (size_t)2 * kMlpWaveLds + 32 * sizeof(float) + 4 * MTW * 16 * sizeof(float) + (kCount ? kLevel0Bins * 4 : 0);
  if (act == kActSilu)
    hipLaunchKernelGGL((score_mlp_wide_kernel<MTW, kActSilu, kCount>), dim3(blocks), dim3(kWideThreads), lds, stream, tab,
                       w1, b1, w2, b2, hidden, heads_per_scorer_row, rows_per_block, counts, seg_base, seg_stride);
  else
    hipLaunchKernelGGL((score_mlp_wide_kernel<MTW, kActGelu, kCount>), dim3(blocks), dim3(kWideThreads), lds, stream, tab,
                       w1, b1, w2, b2, hidden, heads_per_scorer_row, rows_per_block, counts, seg_base, seg_stride);
}

template <bool kCount>
static void launch_score_mlp_impl(const SeqTable& tab, const uint16_t* w1, const float* b1, const float* w2,
                                  const float* b2, int hidden, int act, int heads_per_scorer_row, int rows_per_block,
                                  uint32_t* counts, int seg_base, int seg_stride, hipStream_t stream) {
#define LKV_MLP_ARGS act, heads_per_scorer_row, rows_per_block, counts, seg_base, seg_stride, stream
  switch (hidden / 16) {
    case 1: launch_mt<1, kCount>(tab, w1, b1, w2, b2, LKV_MLP_ARGS); break;
    case 2: launch_mt<2, kCount>(tab, w1, b1, w2, b2, LKV_MLP_ARGS); break;
    case 3: launch_mt<3, kCount>(tab, w1, b1, w2, b2, LKV_MLP_ARGS); break;
    case 4: launch_mt<4, kCount>(tab, w1, b1, w2, b2, LKV_MLP_ARGS); break;
    case 5: case 6: launch_wide<3, kCount>(tab, w1, b1, w2, b2, hidden, LKV_MLP_ARGS); break;
    case 7: case 8: launch_wide<4, kCount>(tab, w1, b1, w2, b2, hidden, LKV_MLP_ARGS); break;
    default: break;
  }
#undef LKV_MLP_ARGS
}

// All sequences of one launch must share rows_per_block (the host groups them so).  `counts` non-null: the launch
// also counts the first-level top-k digits of every segment (counts zero on entry).
void launch_score_mlp(const SeqTable& tab, const uint16_t* w1, const float* b1, const float* w2,
                      const float* b2, int hidden, int act, int heads_per_scorer_row, int rows_per_block,
                      hipStream_t stream, uint32_t* counts, int seg_base, int seg_stride) {
  if (tab.first[tab.n] <= 0) return;
  if (counts != nullptr)
    launch_score_mlp_impl<true>(tab, w1, b1, w2, b2, hidden, act, heads_per_scorer_row, rows_per_block, counts, seg_base,
                                seg_stride, stream);
  else
    launch_score_mlp_impl<false>(tab, w1, b1, w2, b2, hidden, act, heads_per_scorer_row, rows_per_block, nullptr, 0, 0,
                                 stream);
}

}  // namespace lkv
