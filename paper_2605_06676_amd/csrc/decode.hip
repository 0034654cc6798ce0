// One decode step of grouped-query attention over the ragged packed cache:
// Eq. 1 of the paper restricted to the kept tokens of each KV head, with all
// query heads of a GQA group reading the same segment (Sec. 3.1).
//
// Split-K over a flat list of fixed-size chunks of packed rows: block c owns
// packed rows [c*C, (c+1)*C) whatever segments they belong to, so every block
// streams the same number of bytes however skewed the head budgets are.  A
// chunk that crosses segment boundaries is processed piece by piece.  Each
// piece produces, per query head of its segment, an online-softmax partial
// (running max m, denominator l, unnormalised output acc[128]).  A piece that
// is a whole segment is normalised and written straight to the output; other
// pieces go to the workspace slot (segment + chunk) -- distinct pieces have
// distinct slots because segment and chunk indices both grow along the packed
// rows -- and a second kernel merges the slots of each segment.
//
// K and V rows are read once each with 16-byte loads, 16 lanes per row.  Lane
// (r, c) keeps channels 8c..8c+7 of the output for the rows of its row slot.
#include "lkv_common.h"

namespace lkv {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / 64;
constexpr int kDecChunk = 256;          // packed rows per block
constexpr int kDecStates = kDecWaves * 4;   // independent online-softmax states per block (wave x row slot)
constexpr int kDecUnroll = 4;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int G>
struct DecShared {
  float m[kDecStates][G];
  float l[kDecStates][G];
  float acc[kDecStates][G][kHeadDim];
};

template <int G>
__global__ void __launch_bounds__(kDecThreads)
decode_partial_kernel(const uint16_t* __restrict__ q, const uint4* __restrict__ kp,
                      const uint4* __restrict__ vp, const int32_t* __restrict__ offsets, int n_segments,
                      int64_t total_kept, float scale, float* __restrict__ out, float* __restrict__ lse,
                      float* __restrict__ ws_acc, float* __restrict__ ws_m, float* __restrict__ ws_l) {
  extern __shared__ __align__(16) unsigned char smem[];
  DecShared<G>& sh = *reinterpret_cast<DecShared<G>*>(smem);

  const int chunk = blockIdx.x;
  const int64_t p0 = (int64_t)chunk * kDecChunk;
  const int64_t p1 = min(p0 + (int64_t)kDecChunk, total_kept);
  // last segment with offsets[s] <= p0: the segment that contains row p0
  int lo = 0, hi = n_segments;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)offsets[mid] <= p0) lo = mid; else hi = mid;
  }

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r = lane >> 4;
  const int c = lane & 15;
  const int state = wave * 4 + r;
  const float qscale = scale * kLog2e;   // scores are kept in the log2 domain

#pragma unroll 1
  for (int s = lo; s < n_segments; ++s) {
    const int64_t seg_lo = offsets[s], seg_hi = offsets[s + 1];
    if (seg_lo >= p1) break;
    const int64_t a = max(p0, seg_lo), b = min(p1, seg_hi);
    if (b <= a) continue;   // empty segment

    // this lane's slice (channels 8c..8c+7) of the G query vectors of segment s
    float qv[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const uint4 qq = reinterpret_cast<const uint4*>(q + ((size_t)s * G + h) * kHeadDim)[c];
      unpack8(qq, qv[h]);
#pragma unroll
      for (int e = 0; e < 8; ++e) qv[h][e] *= qscale;
    }
    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      m[h] = -INFINITY; l[h] = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
    }

    const int n_rows = (int)(b - a);
#pragma unroll 1
    for (int i0 = 0; i0 * 16 < n_rows; i0 += kDecUnroll) {
      uint4 kk[kDecUnroll], vv[kDecUnroll];
      bool valid[kDecUnroll];
#pragma unroll
      for (int u = 0; u < kDecUnroll; ++u) {
        int row = (i0 + u) * 16 + state;
        valid[u] = row < n_rows;
        row = valid[u] ? row : n_rows - 1;
        kk[u] = load_stream16(kp + (a + row) * kChunksPerRow + c);
        vv[u] = load_stream16(vp + (a + row) * kChunksPerRow + c);
      }
      float sc[kDecUnroll][G];
#pragma unroll
      for (int u = 0; u < kDecUnroll; ++u) {
        float fk[8];
        unpack8(kk[u], fk);
#pragma unroll
        for (int h = 0; h < G; ++h) {
          float d = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) d = fmaf(fk[e], qv[h][e], d);
          d = row16_allreduce_sum(d);
          sc[u][h] = valid[u] ? d : -INFINITY;
        }
      }
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float mx = m[h];
#pragma unroll
        for (int u = 0; u < kDecUnroll; ++u) mx = fmaxf(mx, sc[u][h]);
        const float ref = mx == -INFINITY ? 0.f : mx;
        const float alpha = fast_exp2(m[h] - ref);
        m[h] = mx;
        l[h] *= alpha;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] *= alpha;
#pragma unroll
        for (int u = 0; u < kDecUnroll; ++u) sc[u][h] = fast_exp2(sc[u][h] - ref);
      }
#pragma unroll
      for (int u = 0; u < kDecUnroll; ++u) {
        float fv[8];
        unpack8(vv[u], fv);
#pragma unroll
        for (int h = 0; h < G; ++h) {
          l[h] += sc[u][h];
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[h][e] = fmaf(sc[u][h], fv[e], acc[h][e]);
        }
      }
    }

    // combine the 16 states of the block through LDS
#pragma unroll
    for (int h = 0; h < G; ++h) {
      if (c == 0) { sh.m[state][h] = m[h]; sh.l[state][h] = l[h]; }
      float4* dst = reinterpret_cast<float4*>(&sh.acc[state][h][c * 8]);
      dst[0] = make_float4(acc[h][0], acc[h][1], acc[h][2], acc[h][3]);
      dst[1] = make_float4(acc[h][4], acc[h][5], acc[h][6], acc[h][7]);
    }
    __syncthreads();
    const bool whole = seg_lo >= p0 && seg_hi <= p1;
    const size_t slot = (size_t)s + (size_t)chunk;
    for (int o = tid; o < G * kHeadDim; o += kDecThreads) {
      const int h = o / kHeadDim, ch = o - h * kHeadDim;
      float mx = -INFINITY;
#pragma unroll
      for (int st = 0; st < kDecStates; ++st) mx = fmaxf(mx, sh.m[st][h]);
      float num = 0.f, den = 0.f;
#pragma unroll
      for (int st = 0; st < kDecStates; ++st) {
        const float wgt = fast_exp2(sh.m[st][h] - mx);   // exp2(-inf) = 0 for states that saw no row
        num = fmaf(sh.acc[st][h][ch], wgt, num);
        den = fmaf(sh.l[st][h], wgt, den);
      }
      if (whole) {
        out[((size_t)s * G + h) * kHeadDim + ch] = num / den;
        if (ch == 0 && lse != nullptr) lse[(size_t)s * G + h] = mx * kLn2 + __logf(den);
      } else {
        ws_acc[(slot * G + h) * kHeadDim + ch] = num;
        if (ch == 0) { ws_m[slot * G + h] = mx; ws_l[slot * G + h] = den; }
      }
    }
    __syncthreads();   // the LDS states are rewritten by the next piece
  }
}

// Merge of the per-piece partials of one (segment, query head); 128 threads, one per channel.
__global__ void __launch_bounds__(kHeadDim)
decode_merge_kernel(const int32_t* __restrict__ offsets, int G, const float* __restrict__ ws_acc,
                    const float* __restrict__ ws_m, const float* __restrict__ ws_l,
                    float* __restrict__ out, float* __restrict__ lse) {
  const int s = blockIdx.x / G;
  const int h = blockIdx.x - s * G;
  const int ch = threadIdx.x;
  const int64_t a = offsets[s], b = offsets[s + 1];
  const size_t row = (size_t)s * G + h;
  if (b <= a) {   // empty segment: zero output, lse = -inf
    out[row * kHeadDim + ch] = 0.f;
    if (ch == 0 && lse != nullptr) lse[row] = -INFINITY;
    return;
  }
  const int c_first = (int)(a / kDecChunk), c_last = (int)((b - 1) / kDecChunk);
  if (c_first == c_last) return;   // a whole segment inside one chunk was finished by the first kernel
  float mx = -INFINITY;
  for (int cc = c_first; cc <= c_last; ++cc) mx = fmaxf(mx, ws_m[((size_t)s + cc) * G + h]);
  float num = 0.f, den = 0.f;
  for (int cc = c_first; cc <= c_last; ++cc) {
    const size_t slot = (size_t)s + cc;
    const float wgt = fast_exp2(ws_m[slot * G + h] - mx);
    num = fmaf(ws_acc[(slot * G + h) * kHeadDim + ch], wgt, num);
    den = fmaf(ws_l[slot * G + h], wgt, den);
  }
  out[row * kHeadDim + ch] = num / den;
  if (ch == 0 && lse != nullptr) lse[row] = mx * kLn2 + __logf(den);
}

size_t decode_slots(int n_segments, int64_t total_kept) {
  return (size_t)n_segments + (size_t)((total_kept + kDecChunk - 1) / kDecChunk);
}

size_t decode_workspace_bytes(int n_segments, int64_t total_kept, int G) {
  const size_t per_head = (size_t)(kHeadDim + 2) * sizeof(float);
  const size_t bytes = decode_slots(n_segments, total_kept) * (size_t)G * per_head;
  return (bytes + 255) & ~(size_t)255;
}

template <int G>
static hipError_t launch_decode_g(const void* q, const void* kp, const void* vp, const int32_t* offsets,
                                  int n_segments, int64_t total_kept, float scale, float* out, float* lse,
                                  float* ws, hipStream_t stream) {
  const size_t slots = decode_slots(n_segments, total_kept);
  float* ws_acc = ws;
  float* ws_m = ws + slots * G * kHeadDim;
  float* ws_l = ws_m + slots * G;
  const size_t lds = sizeof(DecShared<G>);
  const int chunks = (int)((total_kept + kDecChunk - 1) / kDecChunk);
  if (chunks > 0) {
    hipLaunchKernelGGL(decode_partial_kernel<G>, dim3(chunks), dim3(kDecThreads), lds, stream,
                       reinterpret_cast<const uint16_t*>(q), reinterpret_cast<const uint4*>(kp),
                       reinterpret_cast<const uint4*>(vp), offsets, n_segments, total_kept, scale, out, lse,
                       ws_acc, ws_m, ws_l);
  }
  hipLaunchKernelGGL(decode_merge_kernel, dim3(n_segments * G), dim3(kHeadDim), 0, stream, offsets, G,
                     ws_acc, ws_m, ws_l, out, lse);
  return hipGetLastError();
}

// The LDS block of the larger groups exceeds the default 64 KB limit per workgroup.
hipError_t decode_prepare() {
#define LKV_DEC_PREP(g)                                                                              \
  {                                                                                                  \
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_partial_kernel<g>),      \
                                       hipFuncAttributeMaxDynamicSharedMemorySize,                   \
                                       (int)sizeof(DecShared<g>));                                   \
    if (e != hipSuccess) return e;                                                                   \
  }
  LKV_DEC_PREP(1) LKV_DEC_PREP(2) LKV_DEC_PREP(3) LKV_DEC_PREP(4)
  LKV_DEC_PREP(5) LKV_DEC_PREP(6) LKV_DEC_PREP(7) LKV_DEC_PREP(8)
#undef LKV_DEC_PREP
  return hipSuccess;
}

hipError_t launch_decode(int G, const void* q, const void* kp, const void* vp, const int32_t* offsets,
                         int n_segments, int64_t total_kept, float scale, float* out, float* lse, float* ws,
                         hipStream_t stream) {
#define LKV_DEC_CASE(g) \
  case g: return launch_decode_g<g>(q, kp, vp, offsets, n_segments, total_kept, scale, out, lse, ws, stream);
  switch (G) {
    LKV_DEC_CASE(1) LKV_DEC_CASE(2) LKV_DEC_CASE(3) LKV_DEC_CASE(4)
    LKV_DEC_CASE(5) LKV_DEC_CASE(6) LKV_DEC_CASE(7) LKV_DEC_CASE(8)
    default: return hipErrorInvalidValue;
  }
#undef LKV_DEC_CASE
}

}  // namespace lkv
