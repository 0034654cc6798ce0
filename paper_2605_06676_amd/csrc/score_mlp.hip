// LKV-T token scoring with the two-layer MLP of Sec. 3.4 / Table 5 of the
// paper: u = w2 . act(W1 [k ; v] + b1) (+ b2), hidden width up to 64 here.
//
// The hidden layer is the one dense contraction of the eviction path
// ([tokens x 256] x [256 x hidden], about 64 flop per byte streamed for
// hidden = 64), so it runs on the matrix cores: v_mfma_f32_16x16x32_bf16 with
// the hidden units on the M side and 16 tokens on the N side,
//     D[hidden, token] = W1[hidden, 0:256] . X[token, 0:256]^T + b1.
//  * W1 fragments (A operand) stay in registers for the whole block:
//    lane (i, kb) holds W1[16 mt + i][32 ks + 8 kb .. +7].
//  * Token rows are read from HBM once, coalesced (16 lanes x 16 bytes per
//    row), staged in a wave-private LDS tile whose row stride of 528 bytes
//    makes the fragment reads conflict free, and read back as B fragments:
//    lane (n, kb) holds X[token n][32 ks + 8 kb .. +7].
//  * The accumulator layout leaves each lane with 4 hidden units of one token
//    per M tile, so bias (as the initial accumulator), activation and the dot
//    with w2 are per-lane work, finished by two cross-lane adds.
// The next 16 tokens are prefetched into registers while the current 16 are
// multiplied.
#include "lkv_common.h"

namespace lkv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

constexpr int kMlpThreads = 256;
constexpr int kMlpWaves = kMlpThreads / 64;
constexpr int kMlpTokTile = 16;                       // tokens per MFMA N tile
constexpr int kMlpRowStride = 2 * 256 + 16;           // bytes per staged [k ; v] row in LDS
constexpr int kMlpWaveLds = kMlpTokTile * kMlpRowStride;
constexpr int kMlpKSteps = 8;                         // 256 features / 32 per MFMA

constexpr int kActSilu = 0;
constexpr int kActGelu = 1;

template <int kAct>
__device__ __forceinline__ float activation(float z) {
  if (kAct == kActSilu) {
    // z * sigmoid(z); exp2 overflow for very negative z gives rcp(inf) = 0
    return z * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
  } else {
    return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
  }
}

__device__ __forceinline__ bf16x8_t as_bf16x8(const uint4& p) {
  return __builtin_bit_cast(bf16x8_t, p);
}

template <int MT, int kAct>
__global__ void __launch_bounds__(kMlpThreads, 2)
score_mlp_kernel(SeqTable tab, const uint16_t* __restrict__ w1, const float* __restrict__ b1,
                 const float* __restrict__ w2, const float* __restrict__ b2, int heads_per_scorer_row,
                 int rows_per_block) {
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
  // accumulator rows of this lane: hidden units 16 mt + 4 r + e
  float bias1[MT][4], wout[MT][4];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      bias1[mt][e] = b1[(size_t)scorer * HID + mt * 16 + 4 * r + e];
      wout[mt][e] = w2[(size_t)scorer * HID + mt * 16 + 4 * r + e];
    }
  const float bias2 = b2 != nullptr ? b2[scorer] : 0.f;

  const size_t head_row0 = (size_t)lh * (size_t)T;
  const uint4* Kh = reinterpret_cast<const uint4*>(tab.k[seq]) + head_row0 * kChunksPerRow;
  const uint4* Vh = reinterpret_cast<const uint4*>(tab.v[seq]) + head_row0 * kChunksPerRow;
  float* out = tab.scores[seq] + head_row0;

  const int rows_per_wave = rows_per_block / kMlpWaves;          // a multiple of 16
  const int wave_row0 = tile * rows_per_block + wave * rows_per_wave;
  const int wave_row1 = min(T, wave_row0 + rows_per_wave);
  if (wave_row0 >= wave_row1) return;

  uint4 kk[4], vv[4];
  auto load_tile = [&](int row0) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int row = row0 + 4 * j + r;
      row = row < T ? row : T - 1;
      kk[j] = load_stream16(Kh + (size_t)row * kChunksPerRow + c);
      vv[j] = load_stream16(Vh + (size_t)row * kChunksPerRow + c);
    }
  };
  load_tile(wave_row0);

#pragma unroll 1
  for (int row0 = wave_row0; row0 < wave_row1; row0 += kMlpTokTile) {
    // stage the 16 rows: row 4j + r, key piece c at byte 16c, value piece c at byte 256 + 16c
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      unsigned char* rowp = tile_lds + (4 * j + r) * kMlpRowStride + c * 16;
      *reinterpret_cast<uint4*>(rowp) = kk[j];
      *reinterpret_cast<uint4*>(rowp + 256) = vv[j];
    }
    if (row0 + kMlpTokTile < wave_row1) load_tile(row0 + kMlpTokTile);   // prefetch
    // the tile is private to this wave: order the LDS writes before the reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    f32x4_t acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4_t{bias1[mt][0], bias1[mt][1], bias1[mt][2], bias1[mt][3]};
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
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int e = 0; e < 4; ++e) part = fmaf(wout[mt][e], activation<kAct>(acc[mt][e]), part);
    // sum the four feature-block lanes of each token: lanes c, c+16, c+32, c+48
    part += __shfl_xor(part, 16, 64);
    part += __shfl_xor(part, 32, 64);
    const int row = row0 + c;
    if (r == 0 && row < T) out[row] = part + bias2;
    // the next iteration overwrites the tile: order these reads before those writes
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

int score_mlp_rows_per_block(int T) {
  // large tiles amortise the 32 KB of W1 each wave loads; small heads keep more blocks
  if (T >= 16384) return 2048;
  if (T >= 4096) return 1024;
  return 256;
}

hipError_t score_mlp_prepare() { return hipSuccess; }

template <int MT>
static void launch_mt(const SeqTable& tab, const uint16_t* w1, const float* b1, const float* w2,
                      const float* b2, int act, int heads_per_scorer_row, int rows_per_block,
                      hipStream_t stream) {
  const int blocks = tab.first[tab.n];
  const size_t lds = (size_t)kMlpWaves * kMlpWaveLds;
  if (act == kActSilu)
    hipLaunchKernelGGL((score_mlp_kernel<MT, kActSilu>), dim3(blocks), dim3(kMlpThreads), lds, stream, tab,
                       w1, b1, w2, b2, heads_per_scorer_row, rows_per_block);
  else
    hipLaunchKernelGGL((score_mlp_kernel<MT, kActGelu>), dim3(blocks), dim3(kMlpThreads), lds, stream, tab,
                       w1, b1, w2, b2, heads_per_scorer_row, rows_per_block);
}

// All sequences of one launch must share rows_per_block (the host groups them so).
void launch_score_mlp(const SeqTable& tab, const uint16_t* w1, const float* b1, const float* w2,
                      const float* b2, int hidden, int act, int heads_per_scorer_row, int rows_per_block,
                      hipStream_t stream) {
  if (tab.first[tab.n] <= 0) return;
  switch (hidden / 16) {
    case 1: launch_mt<1>(tab, w1, b1, w2, b2, act, heads_per_scorer_row, rows_per_block, stream); break;
    case 2: launch_mt<2>(tab, w1, b1, w2, b2, act, heads_per_scorer_row, rows_per_block, stream); break;
    case 3: launch_mt<3>(tab, w1, b1, w2, b2, act, heads_per_scorer_row, rows_per_block, stream); break;
    case 4: launch_mt<4>(tab, w1, b1, w2, b2, act, heads_per_scorer_row, rows_per_block, stream); break;
    default: break;
  }
}

}  // namespace lkv
