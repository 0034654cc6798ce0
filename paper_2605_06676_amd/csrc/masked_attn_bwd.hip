// Backward pass of the training-time causal attention with the multiplicative soft mask
// (App. B.3 of the paper).  With s_ij = scale q_i . k_j, L_i = log sum_{k <= i} e^{s_ik} m_k (kept by
// the forward pass) and the upstream gradient dO:
//
//   e_ij  = e^{s_ij - L_i}                 the weight before the mask (a raw softmax up to its normaliser)
//   p_ij  = e_ij m_j                       the attention weight
//   dP_ij = dO_i . v_j,   D_i = dO_i . o_i = sum_j p_ij dP_ij
//   dV_j  = sum_i p_ij dO_i
//   dm_j  = sum_i e_ij (dP_ij - D_i)       the factor towards the mask is e_ij, never 1 / m_j: finite at m_j = 0
//   dS_ij = p_ij (dP_ij - D_i),   dQ_i = scale sum_j dS_ij k_j,   dK_j = scale sum_i dS_ij q_i
//
// sums over the causal pairs j <= i, and for K, V and m also over the query heads of the GQA group.
// Queries whose prefix carries no weight (L_i = -inf) contribute nothing.
//
// Three kernels (four for short sequences), no atomics, every output element written once:
//   masked_attn_bwd_prep_kernel   D_i for every query row.
//   masked_attn_bwd_dkv_kernel    one block (eight waves, 16 keys each) per KV head and 128 keys: K and V rows of
//                                 the block stay in registers as matrix operands, the Q and dO rows of all later queries
//                                 (and of every query head of the group) stream through LDS; yields
//                                 dK, dV and dm of its keys.
//                                 For short sequences a block takes one query head only and a reduce kernel adds
//                                 the per-query-head partial results in a fixed order.
//   masked_attn_bwd_dq_kernel     one block per query head and 128 queries: Q and dO rows in registers,
//                                 K and V rows of all earlier keys stream through LDS; yields dQ.
// Both recompute s and dP with the 16x16x32 bf16 matrix instruction.  As in the forward kernel the
// products whose result feeds another product are computed transposed, so that the accumulator
// layout of the first (lane (rb, col) holds rows 4 rb .. 4 rb + 3 of two 16-row halves) is the
// A-operand layout of the second over a K-step of 32, and the streamed tile is read once straight
// (A operand of the first products) and once through the transposing LDS read (B operand of the
// second ones).
#include <type_traits>

#include "lkv_common.h"
#include "lkv_kernels.h"

namespace lkv {

namespace {

constexpr int kMbThreads = 256;
constexpr int kMbWaves = kMbThreads / 64;
constexpr int kMbStep = 32;                    // streamed rows per K-step of the second products
constexpr int kMbSteps = 2;                    // steps staged per barrier (64 rows)
constexpr int kMbTile = kMbStep * kMbSteps;
constexpr int kMbStride = 288;                 // LDS bytes per staged row: measured conflict free for the straight 16-byte
                                               // reads and for the transposing reads (272 was not, for the straight ones)
constexpr float kMbLog2e = 1.4426950408889634f;

constexpr int kMbSplitBelowBlocks = 512;       // fewer dkv blocks than this: one block per query head instead of per KV head

__device__ __forceinline__ float mb_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bf16x8_t mb_read_straight(const unsigned char* p) {
  return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(p));
}

// B operand of a product whose K dimension runs over the 32 staged rows of a step: lane (r, c) gets,
// for output column c of column tile ct, rows 4r..4r+3 and 16+4r..16+4r+3 (the K-slot order in which
// the first products leave their results)
__device__ __forceinline__ bf16x8_t mb_read_transposed(const unsigned char* rows, int stride, int r, int c, int ct) {
  const unsigned char* base = rows + (4 * r + (c >> 2)) * stride + ct * 32 + (c & 3) * 8;
  const s16x4_t v0 =
      __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(base));
  const s16x4_t v1 =
      __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(base + 16 * stride));
  return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
}

}  // namespace

// D_i = dO_i . o_i: sixteen lanes per row, eight channels of each tensor per lane
__global__ void __launch_bounds__(256)
masked_attn_bwd_prep_kernel(const float4* __restrict__ o, const uint4* __restrict__ d_o, int64_t n_rows,
                            float* __restrict__ dvec) {
  const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int c = threadIdx.x & 15;
  const int64_t src = min(row, n_rows - 1);
  const float4 a0 = o[(src * kChunksPerRow + c) * 2], a1 = o[(src * kChunksPerRow + c) * 2 + 1];
  float b[8];
  unpack8(d_o[src * kChunksPerRow + c], b);
  float acc = a0.x * b[0];
  acc = fmaf(a0.y, b[1], acc);
  acc = fmaf(a0.z, b[2], acc);
  acc = fmaf(a0.w, b[3], acc);
  acc = fmaf(a1.x, b[4], acc);
  acc = fmaf(a1.y, b[5], acc);
  acc = fmaf(a1.z, b[6], acc);
  acc = fmaf(a1.w, b[7], acc);
  acc = row16_allreduce_sum(acc);
  if (c == 0 && row < n_rows) dvec[row] = acc;
}

// ---- dQ ------------------------------------------------------------------------------------------
// per 32-key step buffer: K rows (also read transposed), V rows, the 32 mask weights
constexpr int kDqStepLds = kMbStep * 2 * kMbStride + kMbStep * 4;
constexpr int kDqLds = 2 * kMbSteps * kDqStepLds;

template <int kQB>
__global__ void __launch_bounds__(kMbThreads, 2)
masked_attn_bwd_dq_kernel(const uint16_t* __restrict__ q, const uint4* __restrict__ k, const uint4* __restrict__ v,
                          const float* __restrict__ m, const float* __restrict__ lse, const float* __restrict__ dvec,
                          const uint16_t* __restrict__ d_o, int T, int n_heads, int G, float scale, float* __restrict__ dq) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int kWaveQ = 16 * kQB;
  constexpr int kBlockQ = kMbWaves * kWaveQ;
  constexpr int kTileLds = kMbSteps * kDqStepLds;
  const int n_qtiles = (T + kBlockQ - 1) / kBlockQ;
  // blocks in order of decreasing work: query tile slow, head fast
  const int qtile = n_qtiles - 1 - (int)blockIdx.x / n_heads;
  const int hq = (int)blockIdx.x % n_heads;
  const int h = hq / G;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r = lane >> 4;
  const int c = lane & 15;
  const int q0 = qtile * kBlockQ;
  const int qw0 = q0 + wave * kWaveQ;
  const int n_tiles = (min(q0 + kBlockQ, T) + kMbTile - 1) / kMbTile;
  const float qscale = scale * kMbLog2e;

  // B operands of the first products: lane (query c of block qb, K-block r) holds 8 channels of q and of dO
  bf16x8_t qfrag[kQB][4], gfrag[kQB][4];
  float lse2[kQB], dsum[kQB];
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    const int query = min(qw0 + 16 * qb + c, T - 1);   // queries past the end repeat the last one; never stored
    const size_t row = (size_t)hq * T + query;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      qfrag[qb][ks] = __builtin_bit_cast(bf16x8_t, reinterpret_cast<const uint4*>(q + row * kHeadDim)[ks * 4 + r]);
      gfrag[qb][ks] = __builtin_bit_cast(bf16x8_t, reinterpret_cast<const uint4*>(d_o + row * kHeadDim)[ks * 4 + r]);
    }
    const float l = lse[row];
    lse2[qb] = l == -INFINITY ? INFINITY : l * kMbLog2e;   // no weight in the prefix: every e_ij becomes 0
    dsum[qb] = dvec[row];
  }
  f32x4_t acc[kQB][8];              // dQ[query 4 r + e of block qb][channel 16 ct + c], before the scale
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) acc[qb][ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const uint4* kh = k + (size_t)h * T * kChunksPerRow;
  const uint4* vh = v + (size_t)h * T * kChunksPerRow;
  const float* mh = m + (size_t)h * T;
  const int srow = tid >> 4, spiece = tid & 15;
  // named staging registers (arrays of them ended up in scratch memory)
  uint4 k_s0, k_s1, k_s2, k_s3, v_s0, v_s1, v_s2, v_s3;
  float mk;
#define LKV_MB_LOAD_ROW(j_, kreg_, vreg_, t_)                                                             \
  {                                                                                                       \
    const int key = min((t_) * kMbTile + srow + 16 * (j_), T - 1); /* past the end: the last row, unused */ \
    const uint32_t off = (uint32_t)key * 256u + (uint32_t)spiece * 16u; /* 32-bit offset, uniform base */ \
    kreg_ = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(kh) + off);            \
    vreg_ = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(vh) + off);            \
  }
#define LKV_MB_LOAD_TILE(t_)                                      \
  {                                                               \
    LKV_MB_LOAD_ROW(0, k_s0, v_s0, t_)                            \
    LKV_MB_LOAD_ROW(1, k_s1, v_s1, t_)                            \
    LKV_MB_LOAD_ROW(2, k_s2, v_s2, t_)                            \
    LKV_MB_LOAD_ROW(3, k_s3, v_s3, t_)                            \
    mk = mh[min((t_) * kMbTile + (tid & (kMbTile - 1)), T - 1)];  \
  }
#define LKV_MB_STORE_ROW(j_, kreg_, vreg_)                                                                   \
  {                                                                                                          \
    unsigned char* step_buf = buf + ((j_) >> 1) * kDqStepLds;                                                \
    const int row = srow + 16 * ((j_) & 1);                                                                  \
    *reinterpret_cast<uint4*>(step_buf + row * kMbStride + spiece * 16) = kreg_;                            \
    *reinterpret_cast<uint4*>(step_buf + kMbStep * kMbStride + row * kMbStride + spiece * 16) = vreg_;     \
  }
  LKV_MB_LOAD_TILE(0)

#pragma unroll 1
  for (int t = 0; t < n_tiles; ++t) {
    unsigned char* buf = smem + (t & 1) * kTileLds;
    LKV_MB_STORE_ROW(0, k_s0, v_s0)
    LKV_MB_STORE_ROW(1, k_s1, v_s1)
    LKV_MB_STORE_ROW(2, k_s2, v_s2)
    LKV_MB_STORE_ROW(3, k_s3, v_s3)
    if (tid < kMbTile)
      reinterpret_cast<float*>(buf + (tid >> 5) * kDqStepLds + kMbStep * 2 * kMbStride)[tid & 31] = mk;
    LKV_MB_LOAD_TILE(min(t + 1, n_tiles - 1))   // the last iteration re-reads its own tile: no branch around the loads
    __syncthreads();                            // two buffers: one barrier per tile is enough
    const int key0 = t * kMbTile;
    if (key0 <= qw0 + kWaveQ - 1 && qw0 < T) {  // wave-uniform: otherwise the tile lies above this wave's diagonal
      const bool diagonal = key0 + kMbTile - 1 > qw0;   // some key of the tile lies above some query's diagonal
#pragma unroll
      for (int st = 0; st < kMbSteps; ++st) {
        const unsigned char* k_lds = buf + st * kDqStepLds;
        const unsigned char* v_lds = k_lds + kMbStep * kMbStride;
        const float* m_lds = reinterpret_cast<const float*>(v_lds + kMbStep * kMbStride);
        // S^T and dP^T for the two 16-key halves of the step: lane (rb = r, query c) gets keys 16 tt + 4 r + e
        f32x4_t sacc[kQB][2], pacc[kQB][2];
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) {
            sacc[qb][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            pacc[qb][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
          }
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            const bf16x8_t kx = mb_read_straight(k_lds + (tt * 16 + c) * kMbStride + ks * 64 + r * 16);
            const bf16x8_t vx = mb_read_straight(v_lds + (tt * 16 + c) * kMbStride + ks * 64 + r * 16);
#pragma unroll
            for (int qb = 0; qb < kQB; ++qb) {
              sacc[qb][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kx, qfrag[qb][ks], sacc[qb][tt], 0, 0, 0);
              pacc[qb][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vx, gfrag[qb][ks], pacc[qb][tt], 0, 0, 0);
            }
          }
        bf16x8_t dsfrag[kQB];
        auto pointwise = [&](auto diag_tag) {
          constexpr bool kDiag = decltype(diag_tag)::value;
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) {
            const float4 mw4 = *reinterpret_cast<const float4*>(m_lds + 16 * tt + 4 * r);
            const float mw[4] = {mw4.x, mw4.y, mw4.z, mw4.w};
#pragma unroll
            for (int qb = 0; qb < kQB; ++qb) {
              const int query = qw0 + 16 * qb + c;
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                float ev = mb_exp2(fmaf(sacc[qb][tt][e], qscale, -lse2[qb]));
                if (kDiag) ev = key0 + 32 * st + 16 * tt + 4 * r + e > query ? 0.f : ev;
                const float ds = ev * mw[e] * (pacc[qb][tt][e] - dsum[qb]);
                dsfrag[qb][tt * 4 + e] = (__bf16)ds;
              }
            }
          }
        };
        if (diagonal) pointwise(std::true_type{});   // wave-uniform
        else pointwise(std::false_type{});
        // dQ += dS K: B operand from the K rows by the transposing read
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) {
          const bf16x8_t kb = mb_read_transposed(k_lds, kMbStride, r, c, ct);
#pragma unroll
          for (int qb = 0; qb < kQB; ++qb)
            acc[qb][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dsfrag[qb], kb, acc[qb][ct], 0, 0, 0);
        }
      }
    }
  }
#undef LKV_MB_LOAD_ROW
#undef LKV_MB_LOAD_TILE
#undef LKV_MB_STORE_ROW

#pragma unroll
  for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int qrow = qw0 + 16 * qb + 4 * r + e;
      if (qrow < T) {
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) dq[((size_t)hq * T + qrow) * kHeadDim + 16 * ct + c] = acc[qb][ct][e] * scale;
      }
    }
}

// ---- dK, dV, dm ----------------------------------------------------------------------------------
// per 32-query step buffer: Q rows, dO rows (both also read transposed), 32 x lse (log2 domain), 32 x D
constexpr int kDkvStepLds = kMbStep * 2 * kMbStride + 2 * kMbStep * 4;
constexpr int kDkvLds = 2 * kMbSteps * kDkvStepLds;

constexpr int kDkvWaves = 8;                   // two per SIMD
constexpr int kDkvThreads = 64 * kDkvWaves;

template <int kKB>
__global__ void __launch_bounds__(kDkvThreads, 2)
masked_attn_bwd_dkv_kernel(const uint4* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                           const float* __restrict__ m, const float* __restrict__ lse, const float* __restrict__ dvec,
                           const uint4* __restrict__ d_o, int T, int n_kv_heads, int G, int split, float scale,
                           float* __restrict__ dk, float* __restrict__ dv, float* __restrict__ dm) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int kWaveK = 16 * kKB;
  constexpr int kBlockK = kDkvWaves * kWaveK;
  constexpr int kTileLds = kMbSteps * kDkvStepLds;
  constexpr int kRowSlots = 4 * kDkvWaves;               // staged rows covered by one pass of the block: 32, half a tile
  // A block owns 128 keys of one KV head and the query heads g_lo .. g_lo + g_cnt - 1 of its group: all of them
  // (split = 1, results go straight to dk, dv, dm) or one each (split = G: results are per-query-head partial sums,
  // row `unit` of buffers the host passes in place of the outputs, added up by the reduce kernel).  Blocks in order
  // of decreasing work: early keys have the most queries after them; key tile slow, unit fast.
  const int n_units = n_kv_heads * split;
  const int unit = (int)blockIdx.x % n_units;
  const int h = unit / split;
  const int g_cnt = G / split;
  const int g_lo = (unit - h * split) * g_cnt;
  const int k0 = (int)blockIdx.x / n_units * kBlockK;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r = lane >> 4;
  const int c = lane & 15;
  const int kw0 = k0 + wave * kWaveK;
  const float qscale = scale * kMbLog2e;

  // B operands of the first products: lane (key c of block kb, K-block r) holds 8 channels of k and of v
  bf16x8_t kfrag[kKB][4], vfrag[kKB][4];
  float mkey[kKB], dm_acc[kKB];
#pragma unroll
  for (int kb = 0; kb < kKB; ++kb) {
    const int key = min(kw0 + 16 * kb + c, T - 1);      // keys past the end repeat the last one; never stored
    const size_t row = (size_t)h * T + key;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      kfrag[kb][ks] = __builtin_bit_cast(bf16x8_t, reinterpret_cast<const uint4*>(k + row * kHeadDim)[ks * 4 + r]);
      vfrag[kb][ks] = __builtin_bit_cast(bf16x8_t, reinterpret_cast<const uint4*>(v + row * kHeadDim)[ks * 4 + r]);
    }
    mkey[kb] = m[row];
    dm_acc[kb] = 0.f;
  }
  f32x4_t acc_v[kKB][8], acc_k[kKB][8];   // dV, dK[key 4 r + e of block kb][channel 16 ct + c]
#pragma unroll
  for (int kb = 0; kb < kKB; ++kb)
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) {
      acc_v[kb][ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      acc_k[kb][ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

  // streamed items: for every query head of the group, the 64-query tiles from the one that holds query k0 on
  const int q_first = k0 / kMbTile * kMbTile;
  const int tiles_per_head = (T - q_first + kMbTile - 1) / kMbTile;
  const int n_items = g_cnt * tiles_per_head;
  const int srow = tid >> 4, spiece = tid & 15;
  uint4 q_s0, q_s1, g_s0, g_s1;   // thread (row slot tid / 16 in 0..31, piece tid % 16) moves rows slot and slot + 32
  float aux;   // threads 0..63: lse of query tid; threads 64..127: D of query tid - 64
#define LKV_MB_LOAD_ROW(j_, qreg_, greg_, base_, q0_)                                                       \
  {                                                                                                         \
    const int query = min((q0_) + srow + kRowSlots * (j_), T - 1); /* past the end: the last row, masked later */ \
    const uint32_t off = (uint32_t)query * 256u + (uint32_t)spiece * 16u; /* 32-bit offset, uniform base */ \
    qreg_ = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(q + (base_) * kChunksPerRow) + off);   \
    greg_ = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(d_o + (base_) * kChunksPerRow) + off); \
  }
#define LKV_MB_LOAD_ITEM(it_)                                                       \
  {                                                                                 \
    const int g_ = (it_) / tiles_per_head;                                          \
    const int q0_ = q_first + ((it_) - g_ * tiles_per_head) * kMbTile;              \
    const size_t base_ = ((size_t)h * G + g_lo + g_) * T;                           \
    LKV_MB_LOAD_ROW(0, q_s0, g_s0, base_, q0_)                                      \
    LKV_MB_LOAD_ROW(1, q_s1, g_s1, base_, q0_)                                      \
    const int query_ = min(q0_ + (tid & (kMbTile - 1)), T - 1);                     \
    aux = (tid & kMbTile) ? dvec[base_ + query_] : lse[base_ + query_];             \
  }
  /* staged row srow + kRowSlots * j of the 64-row tile: step (row / 32), row-in-step (row % 32) */
#define LKV_MB_STORE_ROW(j_, qreg_, greg_)                                                                   \
  {                                                                                                          \
    const int trow = srow + kRowSlots * (j_);                                                                \
    unsigned char* step_buf = buf + (trow >> 5) * kDkvStepLds;                                               \
    const int row = trow & 31;                                                                               \
    *reinterpret_cast<uint4*>(step_buf + row * kMbStride + spiece * 16) = qreg_;                            \
    *reinterpret_cast<uint4*>(step_buf + kMbStep * kMbStride + row * kMbStride + spiece * 16) = greg_;     \
  }
  LKV_MB_LOAD_ITEM(0)

#pragma unroll 1
  for (int it = 0; it < n_items; ++it) {
    unsigned char* buf = smem + (it & 1) * kTileLds;
    LKV_MB_STORE_ROW(0, q_s0, g_s0)
    LKV_MB_STORE_ROW(1, q_s1, g_s1)
    if (tid < 2 * kMbTile) {
      // lse goes to the log2 domain; -inf (no weight in the prefix) becomes +inf so that every e_ij is 0
      const float val = (tid & kMbTile) ? aux : (aux == -INFINITY ? INFINITY : aux * kMbLog2e);
      float* aux_lds = reinterpret_cast<float*>(buf + ((tid >> 5) & 1) * kDkvStepLds + 2 * kMbStep * kMbStride);
      aux_lds[(tid & kMbTile ? kMbStep : 0) + (tid & 31)] = val;
    }
    const int g_cur = it / tiles_per_head;
    const int qt0 = q_first + (it - g_cur * tiles_per_head) * kMbTile;   // first query of the staged tile
    LKV_MB_LOAD_ITEM(min(it + 1, n_items - 1))   // the last iteration re-reads its own item: no branch around the loads
    __syncthreads();                             // two buffers: one barrier per item is enough
#pragma unroll
    for (int st = 0; st < kMbSteps; ++st) {
      const int qs0 = qt0 + st * kMbStep;
      // wave-uniform: nothing to do when all 32 queries come before this wave's keys, or lie past the end
      if (qs0 + kMbStep - 1 < kw0 || qs0 >= T || kw0 >= T) continue;
      const unsigned char* q_lds = buf + st * kDkvStepLds;
      const unsigned char* g_lds = q_lds + kMbStep * kMbStride;
      const float* aux_lds = reinterpret_cast<const float*>(g_lds + kMbStep * kMbStride);
      // S and dP: lane (rb = r, key c) gets queries 16 tt + 4 r + e
      f32x4_t sacc[kKB][2], pacc[kKB][2];
#pragma unroll
      for (int kb = 0; kb < kKB; ++kb)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          sacc[kb][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
          pacc[kb][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const bf16x8_t qx = mb_read_straight(q_lds + (tt * 16 + c) * kMbStride + ks * 64 + r * 16);
          const bf16x8_t gx = mb_read_straight(g_lds + (tt * 16 + c) * kMbStride + ks * 64 + r * 16);
#pragma unroll
          for (int kb = 0; kb < kKB; ++kb) {
            sacc[kb][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qx, kfrag[kb][ks], sacc[kb][tt], 0, 0, 0);
            pacc[kb][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gx, vfrag[kb][ks], pacc[kb][tt], 0, 0, 0);
          }
        }
      bf16x8_t pfrag[kKB], dsfrag[kKB];
      auto pointwise = [&](auto edge_tag) {
        constexpr bool kEdge = decltype(edge_tag)::value;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const float4 l4 = *reinterpret_cast<const float4*>(aux_lds + 16 * tt + 4 * r);
          const float4 d4 = *reinterpret_cast<const float4*>(aux_lds + kMbStep + 16 * tt + 4 * r);
          const float lq[4] = {l4.x, l4.y, l4.z, l4.w};
          const float dq_[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int kb = 0; kb < kKB; ++kb) {
            const int key = kw0 + 16 * kb + c;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int query = qs0 + 16 * tt + 4 * r + e;
              float ev = mb_exp2(fmaf(sacc[kb][tt][e], qscale, -lq[e]));
              if (kEdge) ev = (key > query || query >= T) ? 0.f : ev;
              const float diff = pacc[kb][tt][e] - dq_[e];
              dm_acc[kb] = fmaf(ev, diff, dm_acc[kb]);
              const float p = ev * mkey[kb];
              pfrag[kb][tt * 4 + e] = (__bf16)p;
              dsfrag[kb][tt * 4 + e] = (__bf16)(p * diff);
            }
          }
        }
      };
      // wave-uniform: the plain path needs every query of the step at or after every key of the wave, and inside T
      if (qs0 < kw0 + kWaveK - 1 || qs0 + kMbStep > T) pointwise(std::true_type{});
      else pointwise(std::false_type{});
      // dV += P^T dO and dK += dS^T Q: B operands from the dO and Q rows by the transposing read
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const bf16x8_t gb = mb_read_transposed(g_lds, kMbStride, r, c, ct);
        const bf16x8_t qb = mb_read_transposed(q_lds, kMbStride, r, c, ct);
#pragma unroll
        for (int kb = 0; kb < kKB; ++kb) {
          acc_v[kb][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pfrag[kb], gb, acc_v[kb][ct], 0, 0, 0);
          acc_k[kb][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dsfrag[kb], qb, acc_k[kb][ct], 0, 0, 0);
        }
      }
    }
  }
#undef LKV_MB_LOAD_ROW
#undef LKV_MB_LOAD_ITEM
#undef LKV_MB_STORE_ROW

#pragma unroll
  for (int kb = 0; kb < kKB; ++kb) {
    float s = dm_acc[kb];
    s = sum_over_row_blocks(s);
    const int key = kw0 + 16 * kb + c;
    if (r == 0 && key < T) dm[(size_t)unit * T + key] = s;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int krow = kw0 + 16 * kb + 4 * r + e;
      if (krow < T) {
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) {
          dv[((size_t)unit * T + krow) * kHeadDim + 16 * ct + c] = acc_v[kb][ct][e];
          dk[((size_t)unit * T + krow) * kHeadDim + 16 * ct + c] = acc_k[kb][ct][e] * scale;
        }
      }
    }
  }
}

// out[h][i] = sum over the G query heads of the group of part[h * G + g][i]; `per_head` elements per head, in
// units of float4 when kVec4 (dK and dV) and of floats otherwise (dm).  Fixed order: reproducible.
template <typename Vec>
__global__ void __launch_bounds__(256)
masked_attn_bwd_reduce_kernel(const Vec* __restrict__ part, Vec* __restrict__ out, int64_t per_head, int G) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int h = blockIdx.y;
  if (i >= per_head) return;
  const Vec* src = part + (size_t)h * G * per_head + i;
  Vec acc = src[0];
  for (int g = 1; g < G; ++g) {
    const Vec x = src[(size_t)g * per_head];
    if constexpr (sizeof(Vec) == 16) {
      acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
    } else {
      acc += x;
    }
  }
  out[(size_t)h * per_head + i] = acc;
}

hipError_t masked_attn_bwd_prepare() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(masked_attn_bwd_dq_kernel<2>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kDqLds);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(masked_attn_bwd_dkv_kernel<1>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, kDkvLds);
}

// One block per query head (partial sums + a reduce pass) pays when the blocks of a KV head's whole group would be
// few and long: the longest of them walks G * T / 64 staged tiles one after the other.
static bool dkv_split_by_query_head(int n_kv_heads, int G, int T) {
  return G > 1 && (int64_t)((T + 127) / 128) * n_kv_heads < kMbSplitBelowBlocks;
}

static size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

// workspace: D (one float per query row), then, when the dK/dV kernel is split by query head, the partial
// dK, dV [n_q_heads, T, 128] and dm [n_q_heads, T]
size_t masked_attn_bwd_workspace_bytes(int n_q_heads, int n_kv_heads, int T) {
  size_t bytes = align256((size_t)n_q_heads * (size_t)T * sizeof(float));
  if (n_kv_heads >= 1 && n_q_heads % n_kv_heads == 0 && dkv_split_by_query_head(n_kv_heads, n_q_heads / n_kv_heads, T))
    bytes += 2 * align256((size_t)n_q_heads * T * kHeadDim * sizeof(float)) + align256((size_t)n_q_heads * T * sizeof(float));
  return bytes;
}

void launch_masked_attn_bwd(const void* q, const void* k, const void* v, const float* m, const float* o,
                            const float* lse, const void* d_o, int n_q_heads, int n_kv_heads, int T, float scale,
                            float* dq, float* dk, float* dv, float* dm, float* workspace, hipStream_t stream) {
  const int G = n_q_heads / n_kv_heads;
  const int64_t n_rows = (int64_t)n_q_heads * T;
  hipLaunchKernelGGL(masked_attn_bwd_prep_kernel, dim3((unsigned)((n_rows + 15) / 16)), dim3(256), 0, stream,
                     reinterpret_cast<const float4*>(o), static_cast<const uint4*>(d_o), n_rows, workspace);
  const bool split = dkv_split_by_query_head(n_kv_heads, G, T);
  unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
  float* dk_part = reinterpret_cast<float*>(ws + align256((size_t)n_rows * sizeof(float)));
  float* dv_part = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(dk_part) + align256((size_t)n_rows * kHeadDim * sizeof(float)));
  float* dm_part = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(dv_part) + align256((size_t)n_rows * kHeadDim * sizeof(float)));
  const int n_units = split ? n_q_heads : n_kv_heads;
  hipLaunchKernelGGL(masked_attn_bwd_dkv_kernel<1>, dim3((T + 127) / 128 * n_units), dim3(kDkvThreads), kDkvLds, stream,
                     static_cast<const uint4*>(q), static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v), m,
                     lse, workspace, static_cast<const uint4*>(d_o), T, n_kv_heads, G, split ? G : 1, scale,
                     split ? dk_part : dk, split ? dv_part : dv, split ? dm_part : dm);
  hipLaunchKernelGGL(masked_attn_bwd_dq_kernel<2>, dim3((T + 127) / 128 * n_q_heads), dim3(kMbThreads), kDqLds, stream,
                     static_cast<const uint16_t*>(q), static_cast<const uint4*>(k), static_cast<const uint4*>(v), m, lse,
                     workspace, static_cast<const uint16_t*>(d_o), T, n_q_heads, G, scale, dq);
  if (split) {
    const int64_t vec_per_head = (int64_t)T * kHeadDim / 4;
    const dim3 grid_v((unsigned)((vec_per_head + 255) / 256), n_kv_heads);
    hipLaunchKernelGGL(masked_attn_bwd_reduce_kernel<float4>, grid_v, dim3(256), 0, stream,
                       reinterpret_cast<const float4*>(dk_part), reinterpret_cast<float4*>(dk), vec_per_head, G);
    hipLaunchKernelGGL(masked_attn_bwd_reduce_kernel<float4>, grid_v, dim3(256), 0, stream,
                       reinterpret_cast<const float4*>(dv_part), reinterpret_cast<float4*>(dv), vec_per_head, G);
    hipLaunchKernelGGL(masked_attn_bwd_reduce_kernel<float>, dim3((unsigned)((T + 255) / 256), n_kv_heads), dim3(256), 0,
                       stream, dm_part, dm, (int64_t)T, G);
  }
}

}  // namespace lkv
