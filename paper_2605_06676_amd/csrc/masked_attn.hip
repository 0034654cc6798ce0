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
// Tiling (flash-attention style, for 64-wide waves and the 16x16x32 bf16 matrix instruction).  A block of four waves
// owns one query head and 64 * kQB consecutive queries, 16 * kQB per wave; it walks the key
// tiles of 32 up to its diagonal.  A tile's K and V rows (and its 32 mask weights) are staged
// once per block in LDS, double buffered with one barrier per tile, and read back as operands
// by all four waves.  Per wave and tile:
//   S^T[key, query] = K[key, :] . Q[query, :]^T      (A = K tile from LDS, B = Q^T held in registers)
//   O[query, ch]   += P[query, key] V[key, ch]       (A = P, B = V tile by the transposing LDS read)
// The accumulator layout of S^T (lane (rb, query) holds keys 4 rb .. 4 rb + 3 of a 16-key
// half) is the A-operand layout of P for one K-step over the 32 keys, so probabilities go from
// the first product to the second without leaving their lanes.  Each K and V operand read is
// shared by the kQB query blocks of the wave.
#include "lkv_common.h"
#include "lkv_kernels.h"

namespace lkv {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

constexpr int kMaThreads = 256;
constexpr int kMaWaves = kMaThreads / 64;
constexpr int kMaKeys = 32;                   // keys per tile: one K-step of the P.V product
constexpr int kMaKStride = 272;               // LDS bytes per staged K row (conflict-free 16-byte reads)
constexpr int kMaVStride = 288;               // LDS bytes per staged V row (conflict-free transposing reads)
constexpr int kMaTileLds = kMaKeys * (kMaKStride + kMaVStride) + kMaKeys * 4;   // K, V and the mask weights
constexpr float kMaLog2e = 1.4426950408889634f;
constexpr float kMaLn2 = 0.6931471805599453f;

__device__ __forceinline__ float ma_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ s16x4_t ma_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(p));
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
  bf16x2_t v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

}  // namespace

template <int kQB>
__global__ void __launch_bounds__(kMaThreads, kQB >= 4 ? 1 : 2)
masked_attn_fwd_kernel(const uint16_t* __restrict__ q, const uint4* __restrict__ k, const uint4* __restrict__ v,
                       const float* __restrict__ m, int T, int G, float scale, uint16_t* __restrict__ o,
                       float* __restrict__ lse) {
  __shared__ __align__(16) unsigned char smem[2 * kMaTileLds];
  constexpr int kWaveQ = 16 * kQB;
  constexpr int kBlockQ = kMaWaves * kWaveQ;
  const int n_qtiles = (T + kBlockQ - 1) / kBlockQ;
  const int qtile = n_qtiles - 1 - (int)blockIdx.x;    // the longest rows of the causal triangle start first
  const int hq = blockIdx.y;
  const int h = hq / G;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r = lane >> 4;
  const int c = lane & 15;
  const int q0 = qtile * kBlockQ;
  const int qw0 = q0 + wave * kWaveQ;                  // first query of this wave
  const int n_tiles = (min(q0 + kBlockQ, T) + kMaKeys - 1) / kMaKeys;
  const float qscale = scale * kMaLog2e;

  // B operand of the first product: Q^T, lane (query c of block qb, K-block r) holds q[query][32 ks + 8 r .. +7]
  bf16x8_t qfrag[kQB][4];
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    const int query = qw0 + 16 * qb + c;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      uint4 x = make_uint4(0, 0, 0, 0);
      if (query < T) x = reinterpret_cast<const uint4*>(q + ((size_t)hq * T + query) * kHeadDim)[ks * 4 + r];
      qfrag[qb][ks] = __builtin_bit_cast(bf16x8_t, x);
    }
  }
  float m_run[kQB], l_run[kQB];     // per query c of block qb: running maximum (log2 domain), this lane's share of the denominator
  f32x4_t acc_o[kQB][8];            // O[query 4 r + e of block qb][channel 16 ct + c]
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) acc_o[qb][ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }

  // staging: thread (row slot tid / 16, piece tid % 16) moves rows slot and slot + 16 of the tile
  const uint4* kh = k + (size_t)h * T * kChunksPerRow;
  const uint4* vh = v + (size_t)h * T * kChunksPerRow;
  const float* mh = m + (size_t)h * T;
  const int srow = tid >> 4, spiece = tid & 15;
  // named registers, loaded unconditionally: an array that is assigned under a condition ends up in scratch memory
  uint4 k_a, k_b, v_a, v_b;
  float mk;
  auto load_tile = [&](int t) {
    const int key_a = min(t * kMaKeys + srow, T - 1);        // rows past the end re-read the last row; never used
    const int key_b = min(t * kMaKeys + srow + 16, T - 1);
    k_a = kh[(size_t)key_a * kChunksPerRow + spiece];
    k_b = kh[(size_t)key_b * kChunksPerRow + spiece];
    v_a = vh[(size_t)key_a * kChunksPerRow + spiece];
    v_b = vh[(size_t)key_b * kChunksPerRow + spiece];
    mk = mh[min(t * kMaKeys + (tid & (kMaKeys - 1)), T - 1)];
  };
  load_tile(0);

#pragma unroll 1
  for (int t = 0; t < n_tiles; ++t) {
    unsigned char* k_lds = smem + (t & 1) * kMaTileLds;
    unsigned char* v_lds = k_lds + kMaKeys * kMaKStride;
    float* m_lds = reinterpret_cast<float*>(v_lds + kMaKeys * kMaVStride);
    *reinterpret_cast<uint4*>(k_lds + srow * kMaKStride + spiece * 16) = k_a;
    *reinterpret_cast<uint4*>(k_lds + (srow + 16) * kMaKStride + spiece * 16) = k_b;
    *reinterpret_cast<uint4*>(v_lds + srow * kMaVStride + spiece * 16) = v_a;
    *reinterpret_cast<uint4*>(v_lds + (srow + 16) * kMaVStride + spiece * 16) = v_b;
    if (tid < kMaKeys) m_lds[tid] = mk;
    load_tile(min(t + 1, n_tiles - 1));   // the last iteration re-reads its own tile: no branch around the loads
    // One barrier per tile is enough with two buffers: a wave that runs ahead writes the other
    // buffer, and it cannot come back to this one before every wave has passed the next barrier.
    __syncthreads();
    const int key0 = t * kMaKeys;
    if (key0 > qw0 + kWaveQ - 1 || qw0 >= T) continue;   // wave-uniform: the tile lies wholly above this wave's diagonal

    // S^T for the two 16-key halves: lane (rb = r, query c) gets keys 16 tt + 4 r + e
    f32x4_t sacc[kQB][2];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) sacc[qb][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const uint4 kx = *reinterpret_cast<const uint4*>(k_lds + (tt * 16 + c) * kMaKStride + ks * 64 + r * 16);
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb)
          sacc[qb][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kx), qfrag[qb][ks],
                                                                 sacc[qb][tt], 0, 0, 0);
      }
    // the mask weights of this lane's eight keys
    float mw[8];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const float4 x = *reinterpret_cast<const float4*>(m_lds + 16 * tt + 4 * r);
      mw[tt * 4 + 0] = x.x; mw[tt * 4 + 1] = x.y; mw[tt * 4 + 2] = x.z; mw[tt * 4 + 3] = x.w;
    }
    const bool diagonal = key0 + kMaKeys - 1 > qw0;   // wave-uniform: some (query, key) pair of the tile has key > query

    bf16x8_t pfrag[kQB];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
      const int query = qw0 + 16 * qb + c;
      float sv[8];
      float mx = -INFINITY;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float s = sacc[qb][tt][e];
          if (diagonal) s = key0 + 16 * tt + 4 * r + e <= query ? s : -INFINITY;
          sv[tt * 4 + e] = s;
          mx = fmaxf(mx, s);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      mx = fmaxf(m_run[qb], mx * qscale);              // qscale > 0: scaling commutes with the maximum
      const float ref = mx == -INFINITY ? 0.f : mx;
      const float alpha = ma_exp2(m_run[qb] - ref);    // exp2(-inf) = 0 on the first tile
      m_run[qb] = mx;
      float psum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        sv[i] = ma_exp2(fmaf(sv[i], qscale, -ref)) * mw[i];   // the mask multiplies the exponential (App. B.2)
        psum += sv[i];
      }
      l_run[qb] = l_run[qb] * alpha + psum;
#pragma unroll
      for (int i = 0; i < 8; ++i) pfrag[qb][i] = (__bf16)sv[i];
      // rescale the output rows (queries 4 r + e) when any running maximum of the block moved
      if (__ballot(alpha != 1.f) != 0ull) {
        float al[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) al[e] = __shfl(alpha, 4 * r + e, 64);
#pragma unroll
        for (int ct = 0; ct < 8; ++ct)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc_o[qb][ct][e] *= al[e];
      }
    }
    // O += P V: B operand lane (channel c of tile ct, K-block r) holds V[keys 4r..4r+3 and 16+4r..16+4r+3][channel]
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) {
      const unsigned char* base = v_lds + (4 * r + (c >> 2)) * kMaVStride + ct * 32 + (c & 3) * 8;
      const s16x4_t v0 = ma_read_tr16(base);
      const s16x4_t v1 = ma_read_tr16(base + 16 * kMaVStride);
      const s16x8_t vb = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb)
        acc_o[qb][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pfrag[qb], __builtin_bit_cast(bf16x8_t, vb),
                                                                acc_o[qb][ct], 0, 0, 0);
    }
  }

  // normalise and store: lane (r, c) holds O[query 4 r + e][channels 16 ct + c]
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    float l = l_run[qb];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    const int query = qw0 + 16 * qb + c;
    if (r == 0 && query < T)
      lse[(size_t)hq * T + query] = l > 0.f ? m_run[qb] * kMaLn2 + __logf(l) : -INFINITY;
    const float linv = l > 0.f ? 1.f / l : 0.f;     // no weight in the whole prefix: zero output
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float li = __shfl(linv, 4 * r + e, 64);
      const int qrow = qw0 + 16 * qb + 4 * r + e;
      // neighbouring channels sit in neighbouring lanes: pair them so that each even lane stores 4 bytes
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const float mine = acc_o[qb][ct][e] * li;
        const float next = __shfl_down(mine, 1, 64);
        if ((c & 1) == 0 && qrow < T)
          *reinterpret_cast<uint32_t*>(o + ((size_t)hq * T + qrow) * kHeadDim + 16 * ct + c) = pack_bf16x2(mine, next);
      }
    }
  }
}

int masked_attn_block_queries(int T) { return T >= 8192 ? 256 : 128; }

void launch_masked_attn_fwd(const void* q, const void* k, const void* v, const float* m, int n_q_heads, int n_kv_heads,
                            int T, float scale, void* o, float* lse, hipStream_t stream) {
  const int G = n_q_heads / n_kv_heads;
  if (masked_attn_block_queries(T) == 256) {
    hipLaunchKernelGGL(masked_attn_fwd_kernel<4>, dim3((T + 255) / 256, n_q_heads), dim3(kMaThreads), 0, stream,
                       static_cast<const uint16_t*>(q), static_cast<const uint4*>(k), static_cast<const uint4*>(v), m, T,
                       G, scale, static_cast<uint16_t*>(o), lse);
  } else {
    hipLaunchKernelGGL(masked_attn_fwd_kernel<2>, dim3((T + 127) / 128, n_q_heads), dim3(kMaThreads), 0, stream,
                       static_cast<const uint16_t*>(q), static_cast<const uint4*>(k), static_cast<const uint4*>(v), m, T,
                       G, scale, static_cast<uint16_t*>(o), lse);
  }
}

}  // namespace lkv
