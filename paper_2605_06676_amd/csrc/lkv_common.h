// Shared device-side definitions of the LKV eviction kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lkv {

constexpr int kHeadDim = 128;          // d; a K or V row is 128 bf16 = 256 bytes = 16 lanes x 16 bytes
constexpr int kChunksPerRow = 16;      // 16-byte pieces per row
constexpr int kMaxSeqPerLaunch = 32;   // sequences described by one by-value launch table

// Register types of the matrix instructions (v_mfma_f32_16x16x32_bf16: eight bf16 per lane for the A and B
// operands, four fp32 per lane for the accumulator) and of the transposing LDS read.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

// Per-launch description of up to kMaxSeqPerLaunch sequences, passed by value
// in the kernel arguments (about 1 KB) so that no device-side table has to be
// uploaded.  `first[i]` is the first work unit (block or segment) of sequence
// i in this launch; first[n] is the total.
struct SeqTable {
  const uint16_t* k[kMaxSeqPerLaunch];
  const uint16_t* v[kMaxSeqPerLaunch];
  float* scores[kMaxSeqPerLaunch];
  int32_t T[kMaxSeqPerLaunch];
  int32_t first[kMaxSeqPerLaunch + 1];
  int32_t n;
};

// The same for the observation-window scorer, which reads keys and window queries and needs a
// workspace array per sequence.
struct WinTable {
  const uint16_t* k[kMaxSeqPerLaunch];
  const uint16_t* q[kMaxSeqPerLaunch];           // window queries [L, Hq, W, 128]
  float* scores[kMaxSeqPerLaunch];               // [L, H, T]
  float* partial[kMaxSeqPerLaunch];              // workspace [L H, blocks per head, padded rows, 2]
  const float* lse[kMaxSeqPerLaunch];            // optional: log-normalisers of the window rows [L, Hq, W], or null
  int32_t T[kMaxSeqPerLaunch];
  int32_t first[kMaxSeqPerLaunch + 1];
  int32_t n;
};

// Order-preserving key of a score: unsigned comparison of keys is the comparison of the scores, with NaN ranked
// as -inf and -0.0 below +0.0 (the total order of the fp32 bit patterns).
__device__ __forceinline__ uint32_t order_key(float u) {
  uint32_t bits = __float_as_uint(u);
  if ((bits & 0x7fffffffu) > 0x7f800000u) bits = 0xff800000u;   // NaN ranks as -inf
  return (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
}

// First level of the top-k's radix descent: the top 11 bits of the key.  A scoring launch can count them per
// segment on the way out (`counts`: uint32 [segments][kLevel0Bins], zero before the launch), which saves the
// top-k one pass over the scores.
constexpr int kLevel0Bins = 2048;
constexpr int kLevel0Shift = 21;

// Adds a block's LDS histogram of first-level digits to the segment's global one.  Most bins are empty (scores of
// one head span a few dozen quarter-octaves), so only the occupied ones cost an atomic.
__device__ __forceinline__ void flush_level0_counts(const uint32_t* hist_lds, uint32_t* __restrict__ counts, size_t seg,
                                                    int n_threads) {
  uint32_t* dst = counts + seg * kLevel0Bins;
  for (int i = threadIdx.x; i < kLevel0Bins; i += n_threads) {
    const uint32_t v = hist_lds[i];
    if (v != 0) atomicAdd(dst + i, v);
  }
}

// Index of the sequence that owns work unit `unit`.  `unit` is wave-uniform,
// so this runs on the scalar unit.
__device__ __forceinline__ int seq_of_unit(const SeqTable& tab, int unit) {
  int s = 0;
  while (s + 1 < tab.n && unit >= tab.first[s + 1]) ++s;
  return s;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Unpack the eight bf16 values of a 16-byte piece to fp32 (exact).
__device__ __forceinline__ void unpack8(const uint4& p, float (&f)[8]) {
  f[0] = bf16_lo(p.x); f[1] = bf16_hi(p.x);
  f[2] = bf16_lo(p.y); f[3] = bf16_hi(p.y);
  f[4] = bf16_lo(p.z); f[5] = bf16_hi(p.z);
  f[6] = bf16_lo(p.w); f[7] = bf16_hi(p.w);
}

// DPP controls: lane permutations inside a row of 16 lanes, free on the VALU.
constexpr int kDppQuadXor1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

template <int kCtrl>
__device__ __forceinline__ float dpp_f32(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xf, 0xf, true));
}

// Sum over the 16 lanes of a DPP row; every lane of the row gets the total.
// A K or V row is spread over exactly such a row of lanes.
__device__ __forceinline__ float row16_allreduce_sum(float x) {
  x += dpp_f32<kDppQuadXor1>(x);
  x += dpp_f32<kDppQuadXor2>(x);
  x += dpp_f32<kDppRowHalfMirror>(x);
  x += dpp_f32<kDppRowMirror>(x);
  return x;
}

// Sum (or maximum) of x over the four lanes c, c + 16, c + 32, c + 48 -- the same position in the four rows of 16
// lanes, which is where the matrix instructions leave the four K blocks (or accumulator row blocks) of one column --
// in every one of them.  Row swaps on the vector ALU: v_permlane16_swap exchanges the odd rows of its first operand
// with the even rows of its second, v_permlane32_swap the upper half of the first with the lower half of the second;
// with both operands equal the two results are x[lane] and x[lane ^ 16], resp. x[lane ^ 32], in some order, and the
// operations that follow are symmetric.  A shuffle through the LDS crossbar (ds_bpermute) gives the same values bit
// for bit but costs an LDS round trip that an in-order wave has to sit out.
typedef unsigned u32x2_swap_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float sum_over_row_blocks(float x) {
  const u32x2_swap_t a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(a.x) + __uint_as_float(a.y);
  const u32x2_swap_t b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(b.x) + __uint_as_float(b.y);
}
__device__ __forceinline__ float max_over_row_blocks(float x) {
  const u32x2_swap_t a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(a.x), __uint_as_float(a.y));
  const u32x2_swap_t b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(b.x), __uint_as_float(b.y));
}

// Largest s in [0, n - 1] with table[s] <= p, for a non-decreasing table with table[0] <= p.
// The whole wave takes part (p must be wave-uniform): 64 probes per round, so two rounds
// of loads cover 4096 entries where a binary search needs twelve dependent ones.
__device__ __forceinline__ int wave_upper_segment(const int32_t* __restrict__ table, int n, int64_t p, int lane) {
  int lo = 0, len = n;
  while (len > 1) {
    const int step = (len + 63) >> 6;
    const int i = lo + lane * step;
    const bool le = i < lo + len && (int64_t)table[i] <= p;
    const int cnt = max(1, __popcll(__ballot(le)));   // table[lo] <= p in a well-formed table; never steps below lo
    const int new_lo = lo + (cnt - 1) * step;
    len = min(step, lo + len - new_lo);
    lo = new_lo;
  }
  return lo;
}

// 16-byte load of cache data that this kernel reads exactly once.  Marked non-temporal: the
// rows then stream past the caches instead of displacing lines that will be re-used; measured
// 5 % (scoring) to 12 % (decode) faster than plain loads.
typedef unsigned int u32x4_native __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const uint4* p) {
  const u32x4_native v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_native*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// 16-byte store of data that this kernel will not touch again (the packed cache).  Non-temporal:
// the rows are written through instead of lingering dirty in the memory-side cache, where their
// write-back would otherwise land on whatever kernel runs next (measured: the decode step that
// follows a compaction ran 25 % slower with plain stores).
__device__ __forceinline__ void store_stream16(uint4* p, const uint4& v) {
  u32x4_native n;
  n.x = v.x; n.y = v.y; n.z = v.z; n.w = v.w;
  __builtin_nontemporal_store(n, reinterpret_cast<u32x4_native*>(p));
}

}  // namespace lkv
