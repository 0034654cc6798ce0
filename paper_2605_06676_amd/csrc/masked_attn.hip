// Training-time causal attention with the multiplicative soft mask of App. B of the paper,
// forward pass, at prefill shape (every token of a sequence is a query):
//
//   p_ij = e^{s_ij} m_j / sum_{k <= i} e^{s_ik} m_k,   s_ij = scale q_i . k_j,   o_i = sum_j p_ij v_j
//
// m is one weight in [0, 1] per KV head and key; the heads of a GQA group share their KV head's
// weights (Sec. 3.1).  As App. B.2 describes, the mask multiplies the exponentials inside the
// online softmax (the running maximum is that of the raw scores), so no logarithm of m is ever
// taken.  Next to the output the kernel returns log sum_k e^{s_ik} m_k per query, which the
// backward pass uses to rebuild p from s.
//
// Tiling (flash-attention style, for 64-wide waves and the 16x16x32 bf16 matrix instruction).  A block of four
// waves owns one query head and 64 * kQB consecutive queries, 16 * kQB per wave; it walks the keys up to its
// diagonal in tiles of 32 * kSteps.  A tile's K and V rows and its mask weights are staged once per block in
// LDS, double buffered with one barrier per tile, and read back as operands by all four waves.  Per wave and
// 32-key step:
//   S^T[key, query] = K[key, :] . Q[query, :]^T      (A = K rows from LDS, B = Q^T held in registers)
//   O[query, ch]   += P[query, key] V[key, ch]       (A = P, B = V rows by the transposing LDS read)
// The accumulator layout of S^T (lane (rb, query) holds keys 4 rb .. 4 rb + 3 of a 16-key half) is the
// A-operand layout of P for one K-step over the 32 keys, so probabilities go from the first product to the
// second without leaving their lanes.  Each K and V operand read is shared by the kQB query blocks of the wave.
// The online softmax is updated once per tile.  The denominator that divides the output is one more output
// column of the second product (P times a column of ones), see acc_l below.
#include <type_traits>

#include "lkv_common.h"
#include "lkv_kernels.h"

namespace lkv {

namespace {

constexpr int kMaThreads = 256;
constexpr int kMaWaves = kMaThreads / 64;
constexpr int kMaKeys = 32;                   // keys per tile: one K-step of the P.V product
constexpr int kMaKStride = 288;               // LDS bytes per staged K row (measured conflict free; 272 was not)
constexpr int kMaVStride = 288;               // LDS bytes per staged V row (conflict-free transposing reads)
constexpr int kMaTileLds = kMaKeys * (kMaKStride + kMaVStride) + kMaKeys * 4;   // K, V and the mask weights
constexpr float kMaLog2e = 1.4426950408889634f;
constexpr float kMaLn2 = 0.6931471805599453f;

__device__ __forceinline__ float ma_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ s16x4_t ma_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(p));
}

}  // namespace

template <int kQB, int kSteps>
__global__ void __launch_bounds__(kMaThreads, 2)
masked_attn_fwd_kernel(const uint16_t* __restrict__ q, const uint4* __restrict__ k, const uint4* __restrict__ v,
                       const float* __restrict__ m, int T, int n_heads, int G, float scale, float* __restrict__ o,
                       float* __restrict__ lse) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int kWaveQ = 16 * kQB;
  constexpr int kBlockQ = kMaWaves * kWaveQ;
  constexpr int kTileKeys = kMaKeys * kSteps;          // keys staged per barrier
  constexpr int kTileLds = kSteps * kMaTileLds;
  constexpr int kStage = kTileKeys / 16;               // staged rows per thread and tensor
  const int n_qtiles = (T + kBlockQ - 1) / kBlockQ;
  // blocks in order of decreasing work: the query tile is the slow index, the head the fast one,
  // so that the longest rows of the causal triangle of every head start first
  const int qtile = n_qtiles - 1 - (int)blockIdx.x / n_heads;
  const int hq = (int)blockIdx.x % n_heads;
  const int h = hq / G;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r = lane >> 4;
  const int c = lane & 15;
  const int q0 = qtile * kBlockQ;
  const int qw0 = q0 + wave * kWaveQ;                  // first query of this wave
  const int n_tiles = (min(q0 + kBlockQ, T) + kTileKeys - 1) / kTileKeys;
  const float qscale = scale * kMaLog2e;
  bf16x8_t ones;
#pragma unroll
  for (int i = 0; i < 8; ++i) ones[i] = (__bf16)1.0f;

  // B operand of the first product: Q^T, lane (query c of block qb, K-block r) holds q[query][32 ks + 8 r .. +7]
  bf16x8_t qfrag[kQB][4];
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    const int query = min(qw0 + 16 * qb + c, T - 1);   // queries past the end repeat the last one; never stored
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      qfrag[qb][ks] = __builtin_bit_cast(
          bf16x8_t, reinterpret_cast<const uint4*>(q + ((size_t)hq * T + query) * kHeadDim)[ks * 4 + r]);
  }
  float m_run[kQB], l_run[kQB];     // per query c of block qb: running maximum (log2 domain), this lane's share of the
                                    // unrounded denominator (for the log-normaliser that is returned)
  f32x4_t acc_o[kQB][8];            // O[query 4 r + e of block qb][channel 16 ct + c]
  // Denominator the output is divided by, for query 4 r + e, the same in all 16 lanes of a row block: it is
  // accumulated by the matrix cores as one more output column, P times a column of ones, hence from the same
  // bf16-rounded weights as the output.  The output is then an exact convex combination of value rows, which keeps o (and the
  // D_i = dO_i . o_i of the backward pass) accurate where one key holds nearly all the weight.
  f32x4_t acc_l[kQB];
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
    acc_l[qb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) acc_o[qb][ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }

  // staging: thread (row slot tid / 16, piece tid % 16) moves rows slot, slot + 16, ... of the tile.
  // The registers are loaded unconditionally (an array assigned under a condition ends up in scratch memory).
  const uint4* kh = k + (size_t)h * T * kChunksPerRow;
  const uint4* vh = v + (size_t)h * T * kChunksPerRow;
  const float* mh = m + (size_t)h * T;
  const int srow = tid >> 4, spiece = tid & 15;
  // Named registers: as arrays these ended up in scratch memory, which also serialised the loads.
  static_assert(kStage == 4, "the staging registers below are written out for 64-key tiles");
  uint4 k_s0, k_s1, k_s2, k_s3, v_s0, v_s1, v_s2, v_s3;
  float mk;
#define LKV_MA_LOAD_ROW(j_, kreg_, vreg_, t_)                                                                 \
  {                                                                                                           \
    const int key = min((t_) * kTileKeys + srow + 16 * (j_), T - 1); /* past the end: the last row, unused */ \
    const uint32_t off = (uint32_t)key * 256u + (uint32_t)spiece * 16u; /* a 32-bit offset from a uniform base */ \
    kreg_ = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(kh) + off);                \
    vreg_ = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(vh) + off);                \
  }
#define LKV_MA_LOAD_TILE(t_)                                            \
  {                                                                     \
    LKV_MA_LOAD_ROW(0, k_s0, v_s0, t_)                                  \
    LKV_MA_LOAD_ROW(1, k_s1, v_s1, t_)                                  \
    LKV_MA_LOAD_ROW(2, k_s2, v_s2, t_)                                  \
    LKV_MA_LOAD_ROW(3, k_s3, v_s3, t_)                                  \
    mk = mh[min((t_) * kTileKeys + (tid & (kTileKeys - 1)), T - 1)];    \
  }
#define LKV_MA_STORE_ROW(j_, kreg_, vreg_)                                                                     \
  {                                                                                                            \
    unsigned char* step_buf = buf + ((j_) >> 1) * kMaTileLds;                                                  \
    const int row = srow + 16 * ((j_) & 1);                                                                    \
    *reinterpret_cast<uint4*>(step_buf + row * kMaKStride + spiece * 16) = kreg_;                              \
    *reinterpret_cast<uint4*>(step_buf + kMaKeys * kMaKStride + row * kMaVStride + spiece * 16) = vreg_;       \
  }
  LKV_MA_LOAD_TILE(0)

#pragma unroll 1
  for (int t = 0; t < n_tiles; ++t) {
    // row 32 s + i of the tile lives in step buffer s: K rows, V rows, then the 32 mask weights
    unsigned char* buf = smem + (t & 1) * kTileLds;
    LKV_MA_STORE_ROW(0, k_s0, v_s0)
    LKV_MA_STORE_ROW(1, k_s1, v_s1)
    LKV_MA_STORE_ROW(2, k_s2, v_s2)
    LKV_MA_STORE_ROW(3, k_s3, v_s3)
    if (tid < kTileKeys)
      reinterpret_cast<float*>(buf + (tid >> 5) * kMaTileLds + kMaKeys * (kMaKStride + kMaVStride))[tid & 31] = mk;
    LKV_MA_LOAD_TILE(min(t + 1, n_tiles - 1))   // the last iteration re-reads its own tile: no branch around the loads
    // One barrier per tile is enough with two buffers: a wave that runs ahead writes the other
    // buffer, and it cannot come back to this one before every wave has passed the next barrier.
    __syncthreads();
    const int key0 = t * kTileKeys;
    // wave-uniform: nothing to do when the tile lies wholly above this wave's diagonal
    if (key0 <= qw0 + kWaveQ - 1 && qw0 < T) {

    // S^T for the 16-key pieces of the tile: lane (rb = r, query c) gets keys 16 sub + 4 r + e
    f32x4_t sacc[kQB][2 * kSteps];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
      for (int sub = 0; sub < 2 * kSteps; ++sub) sacc[qb][sub] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int sub = 0; sub < 2 * kSteps; ++sub) {
      const unsigned char* k_lds = buf + (sub >> 1) * kMaTileLds;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const uint4 kx = *reinterpret_cast<const uint4*>(k_lds + ((sub & 1) * 16 + c) * kMaKStride + ks * 64 + r * 16);
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb)
          sacc[qb][sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kx), qfrag[qb][ks],
                                                                  sacc[qb][sub], 0, 0, 0);
      }
    }

    bf16x8_t pfrag[kQB][kSteps];
    // online softmax of one query block over the tile; kDiag: some key of the tile lies above some query's diagonal
    auto softmax = [&](auto diag_tag) {
      constexpr bool kDiag = decltype(diag_tag)::value;
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb) {
        const int query = qw0 + 16 * qb + c;
        float sv[8 * kSteps];
        float mx = -INFINITY;
#pragma unroll
        for (int sub = 0; sub < 2 * kSteps; ++sub)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float s = sacc[qb][sub][e];
            sv[4 * sub + e] = kDiag && key0 + 16 * sub + 4 * r + e > query ? -INFINITY : s;
            mx = fmaxf(mx, sv[4 * sub + e]);
          }
        mx = max_over_row_blocks(mx);
        mx = fmaxf(m_run[qb], mx * qscale);              // qscale > 0: scaling commutes with the maximum
        const float ref = mx == -INFINITY ? 0.f : mx;
        const float alpha = ma_exp2(m_run[qb] - ref);    // exp2(-inf) = 0 on the first tile
        m_run[qb] = mx;
        float psum = 0.f;
#pragma unroll
        for (int st = 0; st < kSteps; ++st) {
          const float* m_lds = reinterpret_cast<const float*>(buf + st * kMaTileLds + kMaKeys * (kMaKStride + kMaVStride));
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) {
            const float4 mw4 = *reinterpret_cast<const float4*>(m_lds + 16 * tt + 4 * r);
            const float mw[4] = {mw4.x, mw4.y, mw4.z, mw4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              // the mask multiplies the exponential (App. B.2)
              const float p = ma_exp2(fmaf(sv[8 * st + 4 * tt + e], qscale, -ref)) * mw[e];
              psum += p;
              pfrag[qb][st][tt * 4 + e] = (__bf16)p;
            }
          }
        }
        l_run[qb] = l_run[qb] * alpha + psum;
        // rescale the output rows (queries 4 r + e) when any running maximum of the block moved
        if (__ballot(alpha != 1.f) != 0ull) {
          float al[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) al[e] = __shfl(alpha, 4 * r + e, 64);
#pragma unroll
          for (int ct = 0; ct < 8; ++ct)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc_o[qb][ct][e] *= al[e];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc_l[qb][e] *= al[e];
        }
      }
    };
    if (key0 + kTileKeys - 1 > qw0) softmax(std::true_type{});   // wave-uniform
    else softmax(std::false_type{});

    // O += P V: B operand lane (channel c of tile ct, K-block r) holds V[keys 4r..4r+3 and 16+4r..16+4r+3][channel]
#pragma unroll
    for (int st = 0; st < kSteps; ++st) {
      const unsigned char* v_lds = buf + st * kMaTileLds + kMaKeys * kMaKStride;
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb)
        acc_l[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pfrag[qb][st], ones, acc_l[qb], 0, 0, 0);
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const unsigned char* base = v_lds + (4 * r + (c >> 2)) * kMaVStride + ct * 32 + (c & 3) * 8;
        const s16x4_t v0 = ma_read_tr16(base);
        const s16x4_t v1 = ma_read_tr16(base + 16 * kMaVStride);
        const s16x8_t vb = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb)
          acc_o[qb][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pfrag[qb][st], __builtin_bit_cast(bf16x8_t, vb),
                                                                  acc_o[qb][ct], 0, 0, 0);
      }
    }
    }
  }
#undef LKV_MA_LOAD_TILE
#undef LKV_MA_LOAD_ROW
#undef LKV_MA_STORE_ROW

  // normalise and store: lane (r, c) holds O[query 4 r + e][channels 16 ct + c] and the (rounded) denominators of
  // those queries; the log-normaliser comes from the unrounded sum, held per query c
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    float l = l_run[qb];
    l = sum_over_row_blocks(l);
    const int query = qw0 + 16 * qb + c;
    if (r == 0 && query < T) lse[(size_t)hq * T + query] = l > 0.f ? m_run[qb] * kMaLn2 + __logf(l) : -INFINITY;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float lr = acc_l[qb][e];
      const float li = lr > 0.f ? 1.f / lr : 0.f;          // no weight in the whole prefix: zero output
      const int qrow = qw0 + 16 * qb + 4 * r + e;
      if (qrow < T) {
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) o[((size_t)hq * T + qrow) * kHeadDim + 16 * ct + c] = acc_o[qb][ct][e] * li;
      }
    }
  }
}

constexpr int kMaFwdSteps = 2;   // 64 keys per staged tile
constexpr int kMaFwdLds = 2 * kMaFwdSteps * kMaTileLds;

hipError_t masked_attn_prepare() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(masked_attn_fwd_kernel<2, kMaFwdSteps>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, kMaFwdLds);
}

void launch_masked_attn_fwd(const void* q, const void* k, const void* v, const float* m, int n_q_heads, int n_kv_heads,
                            int T, float scale, float* o, float* lse, hipStream_t stream) {
  const int G = n_q_heads / n_kv_heads;
  hipLaunchKernelGGL((masked_attn_fwd_kernel<2, kMaFwdSteps>), dim3((T + 127) / 128 * n_q_heads), dim3(kMaThreads),
                     kMaFwdLds, stream, static_cast<const uint16_t*>(q), static_cast<const uint4*>(k),
                     static_cast<const uint4*>(v), m, T, n_q_heads, G, scale, o, lse);
}

}  // namespace lkv
