// One generated token joins the packed cache: its key and value row go to the first spare row of
// every segment and its LKV-T score (Sec. 3.4: a function of that token's own key and value) is
// stored beside them, so that a later re-eviction can rank it against the rows already held.
//
// One wave per segment; the work is a few hundred bytes and, for the MLP scorer, hidden x 256
// multiply-adds per segment, so the kernel is launch-latency sized and kept simple: the token's
// 256 features are unpacked to fp32 in LDS, lane j evaluates hidden units j and j + 64 with fp32
// FMAs, a wave reduction forms the output layer.
#include "lkv_act.h"
#include "lkv_common.h"

namespace lkv {

constexpr int kAppendThreads = 256;
constexpr int kAppendWaves = kAppendThreads / 64;

__global__ void __launch_bounds__(kAppendThreads)
append_kernel(int n_segments, int heads_per_seq, int n_kv_heads, int scorer_kind, int act, int hidden, int per_head,
              const uint16_t* __restrict__ w1, const float* __restrict__ b1, const float* __restrict__ w2,
              const float* __restrict__ b2, const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
              uint4* __restrict__ kp, uint4* __restrict__ vp, float* __restrict__ up,
              const int32_t* __restrict__ cap, int32_t* __restrict__ len, int32_t* __restrict__ overflow) {
  __shared__ float x_lds[kAppendWaves][2 * kHeadDim];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int seg = blockIdx.x * kAppendWaves + wave;
  if (seg >= n_segments) return;   // wave-uniform
  float* x = x_lds[wave];

  // lanes 0..15 hold the key row, 16..31 the value row, one 16-byte piece each
  uint4 piece = make_uint4(0, 0, 0, 0);
  if (lane < 16) piece = k_new[(size_t)seg * kChunksPerRow + lane];
  else if (lane < 32) piece = v_new[(size_t)seg * kChunksPerRow + (lane - 16)];
  if (lane < 32) {
    float f[8];
    unpack8(piece, f);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[lane * 8 + i] = f[i];
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  const int lh = seg % heads_per_seq;
  const size_t srow = per_head ? (size_t)lh : (size_t)(lh / n_kv_heads);
  float part = 0.f;
  if (scorer_kind == 0) {   // linear: w . [k ; v] + b
    const int pc = lane & 31;   // lanes 32..63 repeat a piece and are weighted out
    const uint4 wv = reinterpret_cast<const uint4*>(w1 + srow * 2 * kHeadDim)[pc];
    float wf[8];
    unpack8(wv, wf);
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) dot = fmaf(wf[i], x[pc * 8 + i], dot);
    part = lane < 32 ? dot : 0.f;
  } else {
    // every lane runs the same number of rounds (the reduction below needs the wave converged);
    // lanes past the last hidden unit repeat unit 0 and are weighted out
    for (int j0 = 0; j0 < hidden; j0 += 64) {
      const bool on = j0 + lane < hidden;
      const int j = on ? j0 + lane : 0;
      const uint4* wrow = reinterpret_cast<const uint4*>(w1 + (srow * hidden + j) * 2 * kHeadDim);
      float z = b1[srow * hidden + j];
      for (int q = 0; q < 2 * kHeadDim / 8; ++q) {
        float wf[8];
        unpack8(wrow[q], wf);
#pragma unroll
        for (int i = 0; i < 8; ++i) z = fmaf(wf[i], x[q * 8 + i], z);
      }
      const float a = act == kActSilu ? activation<kActSilu>(z) : activation<kActGelu>(z);
      part += on ? w2[srow * hidden + j] * a : 0.f;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off, 64);
  float u = part;
  if (scorer_kind == 0) u += b1[srow];
  else if (b2 != nullptr) u += b2[srow];

  const int used = len[seg];
  const int64_t row = (int64_t)cap[seg] + used;
  if (row < (int64_t)cap[seg + 1]) {
    if (lane < 16) kp[row * kChunksPerRow + lane] = piece;
    else if (lane < 32) vp[row * kChunksPerRow + (lane - 16)] = piece;
    if (lane == 0) {
      up[row] = u;
      len[seg] = used + 1;
    }
  } else if (lane == 0 && overflow != nullptr) {
    *overflow = 1;   // the segment is full: nothing is written, the caller must re-evict first
  }
}

void launch_append(int n_segments, int heads_per_seq, int n_kv_heads, int scorer_kind, int act, int hidden,
                   int per_head, const uint16_t* w1, const float* b1, const float* w2, const float* b2,
                   const void* k_new, const void* v_new, void* kp, void* vp, float* up, const int32_t* cap,
                   int32_t* len, int32_t* overflow, hipStream_t stream) {
  if (n_segments <= 0) return;
  hipLaunchKernelGGL(append_kernel, dim3((n_segments + kAppendWaves - 1) / kAppendWaves), dim3(kAppendThreads), 0,
                     stream, n_segments, heads_per_seq, n_kv_heads, scorer_kind, act, hidden, per_head, w1, b1, w2, b2,
                     reinterpret_cast<const uint4*>(k_new), reinterpret_cast<const uint4*>(v_new),
                     reinterpret_cast<uint4*>(kp), reinterpret_cast<uint4*>(vp), up, cap, len, overflow);
}

}  // namespace lkv
