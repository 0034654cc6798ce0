// One decode step of grouped-query attention over the ragged packed cache:
// Eq. 1 of the paper restricted to the kept tokens of each KV head, with all
// query heads of a GQA group reading the same segment (Sec. 3.1).
//
// Work decomposition.  Split-K over a flat list of equal chunks of packed rows:
// block c owns packed rows [c*C, (c+1)*C) whatever segments they belong to, so
// every block streams the same number of bytes however skewed the head budgets
// are.  C is chosen on the host so that the grid is a few blocks per compute
// unit.  A chunk that crosses segment boundaries is processed piece by piece.
// Each piece yields, per query head of its segment, an online-softmax partial
// (running max m, denominator l, unnormalised output acc[128]).  A piece that
// is a whole segment is normalised and written straight to the output; other
// pieces go to workspace slot (segment + chunk) -- distinct pieces get distinct
// slots because segment and chunk indices both grow along the packed rows --
// and a second, small kernel merges the slots of each segment.  A piece of at most 64 rows is
// not worth four waves and three block barriers: such pieces are dealt round robin to single
// waves, which run them on their own from load to store, so that a run of short segments inside
// a chunk (skewed budgets leave dozens of heads at the floor) costs a quarter of the serial
// latency chains it would otherwise.  (Merging inside
// the first kernel, by the block that delivers a segment's last piece, needs
// device-scope fences; with one L2 per XCD those write back and invalidate L2
// and were measured to cost more than the second launch.)
//
// Arithmetic.  With up to 16 query heads per KV head the two products are
// skinny GEMMs, and doing them on the vector ALUs costs more issue slots per
// byte than the HBM stream leaves room for, so both run on the matrix cores
// (v_mfma_f32_16x16x32_bf16, fp32 accumulate):
//   S^T[token, head] = K[token, :] . Q[head, :]^T     (A = K tile, B = Q^T)
//   O[head, ch]     += P[head, token] V[token, ch]    (A = P,      B = V tile)
// The accumulator layout of S^T (lane (rb, head) holds tokens 4rb..4rb+3 of a
// 16-token tile) is exactly the A-operand layout of P for a K-step made of two
// such tiles, so probabilities go from the first product to the second without
// leaving their lanes.  Rows are read from HBM once with coalesced 16-byte
// loads, staged in a wave-private LDS tile, and read back as operands: K by
// 16-byte reads (row stride 272 B), V by the transposing 8-byte LDS read of
// gfx950 (row stride 288 B); both strides make the reads bank-conflict free.
// The next 32 rows are prefetched into registers while the current 32 are
// multiplied.  Softmax runs in fp32 in the log2 domain.
#include "lkv_common.h"

namespace lkv {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / 64;
constexpr int kDecTile = 32;                 // rows per wave iteration: one K-step of the P.V product
constexpr int kDecKStride = 272;             // LDS bytes per staged K row
constexpr int kDecVStride = 288;             // LDS bytes per staged V row
constexpr int kDecWaveLds = kDecTile * (kDecKStride + kDecVStride);   // 17920
constexpr int kDecMaxGroup = 16;
constexpr int kDecSmallPiece = 2 * kDecTile; // pieces of at most this many rows are taken by one wave each (see below)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

constexpr int kDecTargetBlocks = 512;        // chunks per launch: one round of resident blocks (2 per compute unit)
constexpr int kDecMinChunk = 128;            // rows; shorter chunks only add partials to merge

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Per-block LDS: the four wave tiles; after a piece, reused for the cross-wave merge.
struct DecMerge {
  float m[kDecWaves][kDecMaxGroup];
  float l[kDecWaves][kDecMaxGroup];
  float acc[kDecWaves][kDecMaxGroup][kHeadDim];
};
static_assert(sizeof(DecMerge) <= (size_t)kDecWaves * kDecWaveLds, "merge scratch must fit the staging tiles");

__device__ __forceinline__ s16x4_t lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4_t*)(p));
}

// kMasked: every row carries a retention weight m in [0, 1] and the probabilities are
// p_i = e^{s_i} m_i / sum_j e^{s_j} m_j (the multiplicative mask of App. B.2, which is softmax(s + log m));
// the rows are then those of the uncompacted cache.
template <bool kMasked>
__global__ void __launch_bounds__(kDecThreads, 2)
decode_partial_kernel(const uint16_t* __restrict__ q, const uint4* __restrict__ kp,
                      const uint4* __restrict__ vp, const int32_t* __restrict__ offsets,
                      const int32_t* __restrict__ lengths /* rows in use per segment, or null: all of them */,
                      int n_segments, int64_t total_kept, int chunk_rows, int G, float scale, float* __restrict__ out,
                      float* __restrict__ lse, float* __restrict__ ws_acc, float* __restrict__ ws_m,
                      float* __restrict__ ws_l, const float* __restrict__ mask) {
  extern __shared__ __align__(16) unsigned char smem[];

  const int chunk = blockIdx.x;
  const int64_t p0 = (int64_t)chunk * chunk_rows;
  const int64_t p1 = min(p0 + (int64_t)chunk_rows, total_kept);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r = lane >> 4;     // load view: row slot.   operand view: K-block kb / accumulator row block rb
  const int c = lane & 15;     // load view: 16-byte piece. operand view: token / head / channel index
  unsigned char* k_lds = smem + wave * kDecWaveLds;
  unsigned char* v_lds = k_lds + kDecTile * kDecKStride;
  DecMerge& mg = *reinterpret_cast<DecMerge*>(smem);
  const float qscale = scale * kLog2e;
  // first segment of this block: the one that contains row p0, i.e. the last with offsets[s] <= p0
  const int s_first = wave_upper_segment(offsets, n_segments, p0, lane);
  int small_seen = 0;   // short pieces met so far in this chunk (the same count in every wave)

#pragma unroll 1
  for (int s = s_first; s < n_segments; ++s) {
    const int64_t seg_lo = offsets[s];
    if (seg_lo >= p1) break;
    // rows behind the ones in use (spare rows for later tokens) are never read
    const int64_t seg_hi = lengths != nullptr ? seg_lo + lengths[s] : (int64_t)offsets[s + 1];
    const int64_t a = max(p0, seg_lo), b = min(p1, seg_hi);
    if (b <= a) continue;   // empty segment (the merge kernel zeroes its output)
    const int n_rows = (int)(b - a);
    const int n_tiles = (n_rows + kDecTile - 1) / kDecTile;

    // Short pieces go to one wave each, in turn; the other waves move on to the next segment.
    const bool small = n_rows <= kDecSmallPiece;
    int t_first = wave, t_step = kDecWaves;
    if (small) {
      const int owner = small_seen & (kDecWaves - 1);
      ++small_seen;
      if (wave != owner) continue;
      t_first = 0;
      t_step = 1;
    }

    // B operand of the first product: Q^T, lane (head c, K-block r) holds q[head c][32 ks + 8 r .. +7]
    bf16x8_t qfrag[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (c < G) v = reinterpret_cast<const uint4*>(q + ((size_t)s * G + c) * kHeadDim)[ks * 4 + r];
      qfrag[ks] = __builtin_bit_cast(bf16x8_t, v);
    }
    float m_run = -INFINITY;   // running max of head c (log2 domain), identical in the four lanes of a head
    float l_run = 0.f;         // this lane's share of the denominator
    f32x4_t acc_o[8];          // O[head 4r+e][channel 16 ct + c]
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) acc_o[ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    uint4 kk[8], vv[8];
    auto load_tile = [&](int t) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        int row = t * kDecTile + 4 * j + r;
        row = row < n_rows ? row : n_rows - 1;   // rows past the piece re-read its last row; zeroed when staged
        kk[j] = load_stream16(kp + (a + row) * kChunksPerRow + c);
        vv[j] = load_stream16(vp + (a + row) * kChunksPerRow + c);
      }
    };
    if (t_first < n_tiles) load_tile(t_first);

#pragma unroll 1
    for (int t = t_first; t < n_tiles; t += t_step) {
      // stage 32 rows: row 4j + r, piece c
      if ((t + 1) * kDecTile <= n_rows) {   // wave-uniform: a full tile
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          *reinterpret_cast<uint4*>(k_lds + (4 * j + r) * kDecKStride + c * 16) = kk[j];
          *reinterpret_cast<uint4*>(v_lds + (4 * j + r) * kDecVStride + c * 16) = vv[j];
        }
      } else {   // last tile of the piece: zero the rows past its end
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const uint32_t keep = t * kDecTile + 4 * j + r < n_rows ? 0xffffffffu : 0u;
          *reinterpret_cast<uint4*>(k_lds + (4 * j + r) * kDecKStride + c * 16) =
              make_uint4(kk[j].x & keep, kk[j].y & keep, kk[j].z & keep, kk[j].w & keep);
          *reinterpret_cast<uint4*>(v_lds + (4 * j + r) * kDecVStride + c * 16) =
              make_uint4(vv[j].x & keep, vv[j].y & keep, vv[j].z & keep, vv[j].w & keep);
        }
      }
      if (t + t_step < n_tiles) load_tile(t + t_step);   // prefetch
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

      // S^T for the two 16-token halves: lane (rb = r, head c) gets tokens 16 tt + 4 r + e
      f32x4_t sacc[2];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        sacc[tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const uint4 kx = *reinterpret_cast<const uint4*>(k_lds + (tt * 16 + c) * kDecKStride + ks * 64 + r * 16);
          sacc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kx), qfrag[ks], sacc[tt],
                                                             0, 0, 0);
        }
      }
      // online softmax for head c over the 8 tokens of this lane and the other three lanes of the head
      float sv[8];
      float mx = m_run;
      const int tok0 = t * kDecTile;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int tok = tok0 + tt * 16 + 4 * r + e;
          const bool ok = tok < n_rows;
          float sc = sacc[tt][e] * qscale;
          if (kMasked) sc += __log2f(mask[a + (ok ? tok : 0)]);   // log2(0) = -inf drops the row
          sv[tt * 4 + e] = ok ? sc : -INFINITY;
          mx = fmaxf(mx, sv[tt * 4 + e]);
        }
      mx = max_over_row_blocks(mx);
      const float ref = mx == -INFINITY ? 0.f : mx;
      const float alpha = fast_exp2(m_run - ref);     // exp2(-inf) = 0 on the first tile
      m_run = mx;
      float psum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) { sv[i] = fast_exp2(sv[i] - ref); psum += sv[i]; }
      l_run = l_run * alpha + psum;
      // A operand of the second product: P[head c][K-slots 8 r .. 8 r + 7] = this lane's own 8 values
      bf16x8_t pfrag;
#pragma unroll
      for (int i = 0; i < 8; ++i) pfrag[i] = (__bf16)sv[i];
      // rescale the output rows (heads 4r+e) when any running max moved
      if (__ballot(alpha != 1.f) != 0ull) {
        float al[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) al[e] = __shfl(alpha, 4 * r + e, 64);
#pragma unroll
        for (int ct = 0; ct < 8; ++ct)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc_o[ct][e] *= al[e];
      }
      // O += P V: B operand lane (channel c of tile ct, K-block r) holds V[tokens 4r..4r+3 and 16+4r..16+4r+3][ch]
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const unsigned char* base = v_lds + (4 * r + (c >> 2)) * kDecVStride + ct * 32 + (c & 3) * 8;
        const s16x4_t v0 = lds_read_tr16(base);
        const s16x4_t v1 = lds_read_tr16(base + 16 * kDecVStride);
        const s16x8_t vb = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
        acc_o[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pfrag, __builtin_bit_cast(bf16x8_t, vb), acc_o[ct], 0, 0, 0);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }

    l_run = sum_over_row_blocks(l_run);
    const bool whole = seg_lo >= p0 && seg_hi <= p1;
    const size_t slot = (size_t)s + (size_t)chunk;
    if (small) {
      // ---- one wave had the whole piece: it writes the result (or the partial) straight from its registers;
      // head h's maximum and denominator sit in lane h ----
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int h = 4 * r + e;
        const float mxh = __shfl(m_run, h, 64);
        const float den = __shfl(l_run, h, 64);
        if (h < G) {
#pragma unroll
          for (int ct = 0; ct < 8; ++ct) {
            const float num = acc_o[ct][e];
            if (whole) out[((size_t)s * G + h) * kHeadDim + ct * 16 + c] = den > 0.f ? num / den : 0.f;
            else ws_acc[(slot * G + h) * kHeadDim + ct * 16 + c] = num;
          }
          if (c == 0) {
            if (whole) {
              if (lse != nullptr) lse[(size_t)s * G + h] = den > 0.f ? mxh * kLn2 + __logf(den) : -INFINITY;
            } else {
              ws_m[slot * G + h] = mxh;
              ws_l[slot * G + h] = den;
            }
          }
        }
      }
      continue;
    }
    // ---- combine the four waves through LDS (the staging tiles are free now) ----
    __syncthreads();   // every wave is done with its staging tile
    if (r == 0 && c < G) { mg.m[wave][c] = m_run; mg.l[wave][c] = l_run; }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int h = 4 * r + e;
      if (h < G) {
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) mg.acc[wave][h][ct * 16 + c] = acc_o[ct][e];
      }
    }
    __syncthreads();
    for (int o = tid; o < G * kHeadDim; o += kDecThreads) {
      const int h = o / kHeadDim, ch = o - h * kHeadDim;
      float mxw = -INFINITY;
#pragma unroll
      for (int w = 0; w < kDecWaves; ++w) mxw = fmaxf(mxw, mg.m[w][h]);
      const float refw = mxw == -INFINITY ? 0.f : mxw;   // -inf: no row of this piece carries weight
      float num = 0.f, den = 0.f;
#pragma unroll
      for (int w = 0; w < kDecWaves; ++w) {
        const float wgt = fast_exp2(mg.m[w][h] - refw);   // 0 for a wave that saw no row (m = -inf)
        num = fmaf(mg.acc[w][h][ch], wgt, num);
        den = fmaf(mg.l[w][h], wgt, den);
      }
      if (whole) {
        // den = 0 only when every row of the segment carries weight 0: zero output, lse = -inf
        out[((size_t)s * G + h) * kHeadDim + ch] = den > 0.f ? num / den : 0.f;
        if (ch == 0 && lse != nullptr) lse[(size_t)s * G + h] = den > 0.f ? mxw * kLn2 + __logf(den) : -INFINITY;
      } else {
        ws_acc[(slot * G + h) * kHeadDim + ch] = num;
        if (ch == 0) { ws_m[slot * G + h] = mxw; ws_l[slot * G + h] = den; }
      }
    }
    __syncthreads();   // the merge scratch becomes staging tiles again
  }
}

// Merge of the per-piece partials of one segment; also zeroes the output of empty segments.
// Each thread owns one output element (query head h, channel ch); a segment takes
// ceil(G * 128 / 256) blocks.  The kernel is a short chain of dependent memory latencies, so
// the partials of up to eight pieces are loaded together and folded in with a running maximum:
// the chain is the offsets load plus one round per eight pieces.
__global__ void __launch_bounds__(kDecThreads)
decode_merge_kernel(const int32_t* __restrict__ offsets, const int32_t* __restrict__ lengths, int G,
                    int blocks_per_segment, int chunk_rows,
                    const float* __restrict__ ws_acc, const float* __restrict__ ws_m,
                    const float* __restrict__ ws_l, float* __restrict__ out, float* __restrict__ lse) {
  const int s = blockIdx.x / blocks_per_segment;
  const int o = (blockIdx.x - s * blocks_per_segment) * kDecThreads + threadIdx.x;
  if (o >= G * kHeadDim) return;
  const int h = o / kHeadDim, ch = o - h * kHeadDim;
  const int64_t a = offsets[s];
  const int64_t b = lengths != nullptr ? a + lengths[s] : (int64_t)offsets[s + 1];
  const size_t row = (size_t)s * G + h;
  if (b <= a) {   // empty segment: zero output, lse = -inf
    out[row * kHeadDim + ch] = 0.f;
    if (ch == 0 && lse != nullptr) lse[row] = -INFINITY;
    return;
  }
  const int c_first = (int)(a / chunk_rows), c_last = (int)((b - 1) / chunk_rows);
  if (c_first == c_last) return;   // a whole segment inside one chunk was finished by the first kernel
  constexpr int kU = 8;
  float mx = -INFINITY, num = 0.f, den = 0.f;
  for (int c0 = c_first; c0 <= c_last; c0 += kU) {
    float mv[kU], lv[kU], av[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int cc = min(c0 + u, c_last);
      const size_t sl = (size_t)s + cc;
      mv[u] = ws_m[sl * G + h];
      lv[u] = ws_l[sl * G + h];
      av[u] = ws_acc[(sl * G + h) * kHeadDim + ch];
    }
    float mnew = mx;
#pragma unroll
    for (int u = 0; u < kU; ++u) mnew = fmaxf(mnew, mv[u]);   // -inf only if every row so far carries weight 0
    const float ref = mnew == -INFINITY ? 0.f : mnew;
    const float keep = fast_exp2(mx - ref);                    // 0 in the first round
    num *= keep;
    den *= keep;
    mx = mnew;
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const float wgt = c0 + u <= c_last ? fast_exp2(mv[u] - ref) : 0.f;
      num = fmaf(av[u], wgt, num);
      den = fmaf(lv[u], wgt, den);
    }
  }
  out[row * kHeadDim + ch] = den > 0.f ? num / den : 0.f;
  if (ch == 0 && lse != nullptr) lse[row] = den > 0.f ? mx * kLn2 + __logf(den) : -INFINITY;
}

// Rows per block: a multiple of the wave tile, sized for kDecTargetBlocks blocks.
int decode_chunk_rows(int64_t total_kept) {
  int64_t c = (total_kept + kDecTargetBlocks - 1) / kDecTargetBlocks;
  c = (c + kDecTile - 1) / kDecTile * kDecTile;
  if (c < kDecMinChunk) c = kDecMinChunk;
  return (int)c;
}

static size_t decode_slots(int n_segments, int64_t total_kept) {
  const int chunk = decode_chunk_rows(total_kept);
  return (size_t)n_segments + (size_t)((total_kept + chunk - 1) / chunk);
}

size_t decode_workspace_bytes(int n_segments, int64_t total_kept, int G) {
  const size_t per_head = (size_t)(kHeadDim + 2) * sizeof(float);
  const size_t bytes = decode_slots(n_segments, total_kept) * (size_t)G * per_head;
  return (bytes + 255) & ~(size_t)255;
}

// Split-K partials of the decode call that allocates nothing and takes no workspace argument: a
// fixed array in the library's device image.  Every GPU the library runs on holds its own copy at
// its own address until the process ends.  The name below is only a host-side handle for the
// symbol; the device address is looked up once per device and everything on the host side uses
// that address.
constexpr size_t kDecStaticBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kDecStaticBytes];
constexpr int kDecMaxDevices = 64;
static void* g_scratch_ptr[kDecMaxDevices] = {};

size_t decode_static_scratch_bytes() { return kDecStaticBytes; }

// Device address of the static scratch array on `device`, or null if decode_prepare has not run there.
void* decode_static_scratch(int device) {
  return device >= 0 && device < kDecMaxDevices ? g_scratch_ptr[device] : nullptr;
}

// Once per device, with that device current (lkv_create calls it right after selecting the device).
// The four staging tiles exceed the default 64 KB of LDS per workgroup.
hipError_t decode_prepare(int device) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_partial_kernel<false>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kDecWaves * kDecWaveLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_partial_kernel<true>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kDecWaves * kDecWaveLds);
  if (e != hipSuccess) return e;
  if (device < 0 || device >= kDecMaxDevices) return hipErrorInvalidDevice;
  if (g_scratch_ptr[device] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = ptr;
  }
  return hipSuccess;
}

// offsets[s] = s * len for s = 0..n_segments: the uncompacted cache of one sequence seen as a packed cache
__global__ void uniform_offsets_kernel(int n_segments, int len, int32_t* __restrict__ offsets) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s <= n_segments) offsets[s] = s * len;
}

void launch_uniform_offsets(int n_segments, int len, int32_t* offsets, hipStream_t stream) {
  hipLaunchKernelGGL(uniform_offsets_kernel, dim3((n_segments + 256) / 256), dim3(256), 0, stream, n_segments, len,
                     offsets);
}

hipError_t launch_decode(int G, const void* q, const void* kp, const void* vp, const int32_t* offsets,
                         const int32_t* lengths, int n_segments, int64_t total_kept, float scale, float* out, float* lse, float* ws,
                         hipStream_t stream, const float* mask) {
  if (G < 1 || G > kDecMaxGroup) return hipErrorInvalidValue;
  const size_t slots = decode_slots(n_segments, total_kept);
  float* ws_acc = ws;
  float* ws_m = ws + slots * G * kHeadDim;
  float* ws_l = ws_m + slots * G;
  const int chunk_rows = decode_chunk_rows(total_kept);
  const int chunks = (int)((total_kept + chunk_rows - 1) / chunk_rows);
  if (chunks > 0 && mask == nullptr) {
    hipLaunchKernelGGL(decode_partial_kernel<false>, dim3(chunks), dim3(kDecThreads), kDecWaves * kDecWaveLds, stream,
                       reinterpret_cast<const uint16_t*>(q), reinterpret_cast<const uint4*>(kp),
                       reinterpret_cast<const uint4*>(vp), offsets, lengths, n_segments, total_kept, chunk_rows, G, scale,
                       out, lse, ws_acc, ws_m, ws_l, mask);
  } else if (chunks > 0) {
    hipLaunchKernelGGL(decode_partial_kernel<true>, dim3(chunks), dim3(kDecThreads), kDecWaves * kDecWaveLds, stream,
                       reinterpret_cast<const uint16_t*>(q), reinterpret_cast<const uint4*>(kp),
                       reinterpret_cast<const uint4*>(vp), offsets, lengths, n_segments, total_kept, chunk_rows, G, scale,
                       out, lse, ws_acc, ws_m, ws_l, mask);
  }
  const int blocks_per_segment = (G * kHeadDim + kDecThreads - 1) / kDecThreads;
  hipLaunchKernelGGL(decode_merge_kernel, dim3(n_segments * blocks_per_segment), dim3(kDecThreads), 0, stream,
                     offsets, lengths, G, blocks_per_segment, chunk_rows, ws_acc, ws_m, ws_l, out, lse);
  return hipGetLastError();
}

}  // namespace lkv
