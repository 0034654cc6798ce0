// LKV-H at inference time (Sec. 3.3) and the Soft-TopK operator ST_k (Sec. 3.2, Eq. 2, App. A.1;
// its backward pass, App. A.2, further down), in fp64.  Both are tiny next to the cache kernels (L * H <= a few hundred heads,
// computed once and frozen), so one workgroup does the whole operator and the arithmetic is
// double precision throughout: the ratios decide integer budgets floor(r t).
//
// ST_k(x)_i = f(x_i / tau - lambda), f the Laplace CDF, lambda such that the outputs sum to k.
// With the inputs in descending order and m = #{i : x_i / tau >= lambda}, App. A.1 gives lambda in
// closed form from S1 = sum_{i <= m} e^{-x_i}, S2 = sum_{i > m} e^{x_i}.  The split index is found
// without trying every m: g(v) = sum_i f(x_i - v) - k decreases in v, so x_j >= lambda exactly
// when g(x_j) <= 0, and g at the element of rank j needs only the prefix sum S1(j) and the suffix
// sum S2(j).  All sums are carried as logarithms so that x / tau with a tiny tau cannot overflow.
// Inputs too long for the LDS sort go through soft_topk_large_kernel further down (no sort: the
// threshold is bracketed by passes over the input).
#include <hip/hip_runtime.h>

#include <cmath>

#include "lkv_kernels.h"

namespace lkv {

namespace {

constexpr int kStThreads = 1024;
constexpr int kStKeyBytes = 128 * 1024;   // LDS given to the sort keys
constexpr int kStLocal = 32;              // elements per thread chunk at the largest n

__device__ inline double log_add_exp(double a, double b) {   // log(e^a + e^b); -inf means an empty sum
  const double hi = fmax(a, b);
  const double lo = fmin(a, b);
  if (lo == -INFINITY) return hi;
  return hi + log1p(exp(lo - hi));
}

// keys whose unsigned order is the numeric order of the values
__device__ inline uint32_t to_key(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u >> 31) ? ~u : (u | 0x80000000u);
}
__device__ inline uint64_t to_key(double x) {
  const uint64_t u = (uint64_t)__double_as_longlong(x);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ inline double from_key(uint32_t k) {
  const uint32_t u = (k >> 31) ? (k & 0x7fffffffu) : ~k;
  return (double)__uint_as_float(u);
}
__device__ inline double from_key(uint64_t k) {
  const uint64_t u = (k >> 63) ? (k & 0x7fffffffffffffffull) : ~k;
  return __longlong_as_double((long long)u);
}

// log( sqrt(d^2 + e^L) + d ) for d >= 0
__device__ inline double log_root_plus(double d, double L) {
  const double h = 0.5 * L;
  if (d == 0.0) return h;
  if (h > 300.0) return h + asinh(d * exp(-h));
  return log(hypot(d, exp(h)) + d);
}

// value of sum_i f(x_i - v) - k at the element v of rank j (1-based, descending), given
// log S1(j) = log sum_{i <= j} e^{-x_i} and log S2(j) = log sum_{i > j} e^{x_i}
__device__ inline double constraint_at(double v, int j, double log_s1, double log_s2, double k) {
  return ((double)j - k) - 0.5 * exp(v + log_s1) + 0.5 * exp(log_s2 - v);
}

// In a batched launch block b works on vector b: rows of x, y and info, and its own target sum, which the paper
// keeps strictly inside (0, n) (App. A.1, "Numerical Stability at Boundaries"); the same is enforced here by clamping.
template <typename X>
__device__ inline void select_vector(const X*& x, double*& y, double* __restrict__& info,
                                     double& k, const double* __restrict__ k_vec, int n) {
  if (k_vec == nullptr) return;
  const size_t b = blockIdx.x;
  x += b * n;
  if (y != nullptr) y += b * n;
  if (info != nullptr) info += 2 * b;
  k = fmin(fmax(k_vec[b], 1e-6), (double)n - 1e-6);
}

struct StShared {
  double lambda;
  int m;
  int pad;
};

template <typename X, typename Key>
__global__ void __launch_bounds__(kStThreads)
soft_topk_kernel(const X* x, int n, int P, double k, double tau, double* y /* may alias x */,
                 double* __restrict__ info, int32_t* __restrict__ budgets, double t, const double* __restrict__ k_vec) {
  extern __shared__ __align__(16) unsigned char smem[];
  select_vector(x, y, info, k, k_vec, n);   // batched call: this block's vector and target
  Key* keys = reinterpret_cast<Key*>(smem);                                  // [P]
  double* pre = reinterpret_cast<double*>(smem + (size_t)P * sizeof(Key));  // [1024] prefix of log S1
  double* suf = pre + kStThreads;                                            // [1024] suffix of log S2
  double* loc = suf + kStThreads;                                            // [kStLocal]
  StShared* sh = reinterpret_cast<StShared*>(loc + kStLocal);
  const int tid = threadIdx.x;

  for (int i = tid; i < P; i += kStThreads) keys[i] = i < n ? to_key(x[i]) : (Key)0;
  __syncthreads();

  // bitonic sort, descending
  for (int span = 2; span <= P; span <<= 1) {
    for (int j = span >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < (P >> 1); i += kStThreads) {
        const int a = ((i & ~(j - 1)) << 1) | (i & (j - 1));
        const int b = a | j;
        const Key ka = keys[a], kb = keys[b];
        const bool descending = (a & span) == 0;
        if (descending ? (ka < kb) : (ka > kb)) {
          keys[a] = kb;
          keys[b] = ka;
        }
      }
      __syncthreads();
    }
  }

  // per-thread chunk of the sorted values
  const int c = (n + kStThreads - 1) / kStThreads;
  const int start = min(n, tid * c);
  const int end = min(n, start + c);
  double a_loc = -INFINITY, b_loc = -INFINITY;
  for (int i = start; i < end; ++i) {
    const double v = from_key(keys[i]) / tau;
    a_loc = log_add_exp(a_loc, -v);
    b_loc = log_add_exp(b_loc, v);
  }
  pre[tid] = a_loc;
  suf[tid] = b_loc;
  __syncthreads();
  for (int off = 1; off < kStThreads; off <<= 1) {
    const double pa = tid >= off ? pre[tid - off] : -INFINITY;
    const double sb = tid + off < kStThreads ? suf[tid + off] : -INFINITY;
    __syncthreads();
    pre[tid] = log_add_exp(pre[tid], pa);
    suf[tid] = log_add_exp(suf[tid], sb);
    __syncthreads();
  }
  const double before = tid > 0 ? pre[tid - 1] : -INFINITY;               // log S1 of everything ahead of the chunk
  const double after = tid + 1 < kStThreads ? suf[tid + 1] : -INFINITY;   // log S2 of everything behind it

  // chunks whose last element is still at or above the threshold are wholly in the head
  bool whole = false;
  if (end > start) {
    const double v = from_key(keys[end - 1]) / tau;
    whole = constraint_at(v, end, pre[tid], after, k) <= 0.0;
  }
  const int full_chunks = __syncthreads_count(whole);
  const int used_chunks = (n + c - 1) / c;

  if (tid == min(full_chunks, kStThreads - 1)) {
    int m;
    double log_s1, log_s2;
    if (full_chunks >= used_chunks) {   // every element is at or above the threshold
      m = n;
      log_s1 = pre[kStThreads - 1];
      log_s2 = -INFINITY;
    } else {
      // the split lies in this thread's chunk: suffix sums inside the chunk, then a forward walk
      const int cnt = end - start;
      double run = -INFINITY;
      for (int i = cnt - 1; i >= 0; --i) {
        loc[i] = run;   // log sum of e^{x} over the chunk elements behind element i
        run = log_add_exp(run, from_key(keys[start + i]) / tau);
      }
      m = start;
      log_s1 = before;
      log_s2 = log_add_exp(run, after);
      double s1 = before;
      for (int i = 0; i < cnt; ++i) {
        const double v = from_key(keys[start + i]) / tau;
        s1 = log_add_exp(s1, -v);
        const double s2 = log_add_exp(loc[i], after);
        if (constraint_at(v, start + i + 1, s1, s2, k) > 0.0) break;
        m = start + i + 1;
        log_s1 = s1;
        log_s2 = s2;
      }
    }
    // closed form of App. A.1 for y = e^lambda: S1 y^2 + 2 (k - m) y - S2 = 0, positive root,
    // written so that neither a difference of close numbers nor an overflow occurs
    const double d = k - (double)m;
    double lambda;
    if (m == 0) lambda = log_s2 - log(2.0 * k);
    else if (m == n) lambda = log(2.0 * ((double)n - k)) - log_s1;
    else if (d >= 0.0) lambda = log_s2 - log_root_plus(d, log_s1 + log_s2);
    else lambda = log_root_plus(-d, log_s1 + log_s2) - log_s1;
    sh->lambda = lambda;
    sh->m = m;
  }
  __syncthreads();
  const double lambda = sh->lambda;
  if (tid == 0 && info != nullptr) {
    info[0] = lambda;
    info[1] = (double)sh->m;
  }
  for (int i = tid; i < n; i += kStThreads) {
    const double z = (double)x[i] / tau - lambda;
    const double r = z >= 0.0 ? 1.0 - 0.5 * exp(-z) : 0.5 * exp(z);
    if (y != nullptr) y[i] = r;
    if (budgets != nullptr) budgets[i] = (int32_t)floor(r * t);
  }
}

// ---- inputs too long to sort in LDS ---------------------------------------------------------------
// The threshold is the root of g(v) = sum_i f(x_i / tau - v) - k, which decreases in v.  One workgroup
// brackets it from the extremes of the input, then halves the bracket, one pass over the input per
// step, until no input value lies inside: from then on the split index m is known, the sums S1 and
// S2 take one more pass, and lambda comes out of the same closed form as above (App. A.1).  No sort,
// any n; about 50 passes over an input that stays in the L2 cache.
constexpr int kStLargeMaxN = 1 << 22;

struct StLargeShared {
  double d[4][16];
  long long c[2][16];
  double out_d[4];
  long long out_c[2];
};

// block-wide sums of up to four doubles and two counters (fixed order: reproducible), result to every thread
__device__ inline void st_block_sum(StLargeShared* sh, double (&v)[4], long long (&cnt)[2]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] += __shfl_xor(v[i], off, 64);
#pragma unroll
    for (int i = 0; i < 2; ++i) cnt[i] += __shfl_xor(cnt[i], off, 64);
  }
  __syncthreads();   // the previous round's results have been read
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) sh->d[i][wave] = v[i];
#pragma unroll
    for (int i = 0; i < 2; ++i) sh->c[i][wave] = cnt[i];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 0; i < 4; ++i) {
      double a = 0.0;
      for (int w = 0; w < kStThreads / 64; ++w) a += sh->d[i][w];
      sh->out_d[i] = a;
    }
    for (int i = 0; i < 2; ++i) {
      long long a = 0;
      for (int w = 0; w < kStThreads / 64; ++w) a += sh->c[i][w];
      sh->out_c[i] = a;
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = sh->out_d[i];
#pragma unroll
  for (int i = 0; i < 2; ++i) cnt[i] = sh->out_c[i];
}

template <typename X>
__global__ void __launch_bounds__(kStThreads)
soft_topk_large_kernel(const X* x, int n, double k, double tau, double* y /* may alias x */,
                       double* __restrict__ info, int32_t* __restrict__ budgets, double t,
                       const double* __restrict__ k_vec) {
  __shared__ StLargeShared sh;
  select_vector(x, y, info, k, k_vec, n);   // batched call: this block's vector and target
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;

  // extremes of z = x / tau
  double zmin = INFINITY, zmax = -INFINITY;
  for (int i = tid; i < n; i += kStThreads) {
    const double z = (double)x[i] / tau;
    zmin = fmin(zmin, z);
    zmax = fmax(zmax, z);
  }
  for (int off = 32; off > 0; off >>= 1) {
    zmin = fmin(zmin, __shfl_xor(zmin, off, 64));
    zmax = fmax(zmax, __shfl_xor(zmax, off, 64));
  }
  if (lane == 0) { sh.d[0][wave] = zmin; sh.d[1][wave] = zmax; }
  __syncthreads();
  for (int w = 0; w < kStThreads / 64; ++w) { zmin = fmin(zmin, sh.d[0][w]); zmax = fmax(zmax, sh.d[1][w]); }
  // g > 0 at lo: every f is at least 1 - e^{-L} / 2 with L >= 1 + log(n / (2 (n - k))), so the sum exceeds
  // n - (n - k) / e > k; g < 0 at hi: every f is at most e^{-U} / 2 with U >= 1 + log(n / (2 k)): sum <= k / e
  double lo = zmin - 1.0 - fmax(0.0, log((double)n / (2.0 * ((double)n - k))));
  double hi = zmax + 1.0 + fmax(0.0, log((double)n / (2.0 * k)));

  for (int step = 0; step < 200; ++step) {
    const double mid = 0.5 * (lo + hi);
    if (!(mid > lo && mid < hi)) break;   // the bracket is down to neighbouring numbers: what is inside ties with the root
    double v[4] = {0.0, 0.0, 0.0, 0.0};
    long long cnt[2] = {0, 0};
    for (int i = tid; i < n; i += kStThreads) {
      const double z = (double)x[i] / tau;
      const double d = z - mid;
      v[0] += d >= 0.0 ? 1.0 - 0.5 * exp(-d) : 0.5 * exp(d);
      cnt[0] += (z >= lo && z < mid) ? 1 : 0;
      cnt[1] += (z >= mid && z < hi) ? 1 : 0;
    }
    st_block_sum(&sh, v, cnt);
    long long inside;
    if (v[0] - k > 0.0) { lo = mid; inside = cnt[1]; }
    else { hi = mid; inside = cnt[0]; }
    if (inside == 0) break;
  }

  // split: the head is {z >= hi}; log S1 = log sum_head e^{-z}, log S2 = log sum_rest e^{z}, each against its own maximum
  double s1_ref = -INFINITY, s2_ref = -INFINITY;
  for (int i = tid; i < n; i += kStThreads) {
    const double z = (double)x[i] / tau;
    if (z >= hi) s1_ref = fmax(s1_ref, -z);
    else s2_ref = fmax(s2_ref, z);
  }
  for (int off = 32; off > 0; off >>= 1) {
    s1_ref = fmax(s1_ref, __shfl_xor(s1_ref, off, 64));
    s2_ref = fmax(s2_ref, __shfl_xor(s2_ref, off, 64));
  }
  __syncthreads();
  if (lane == 0) { sh.d[2][wave] = s1_ref; sh.d[3][wave] = s2_ref; }
  __syncthreads();
  for (int w = 0; w < kStThreads / 64; ++w) { s1_ref = fmax(s1_ref, sh.d[2][w]); s2_ref = fmax(s2_ref, sh.d[3][w]); }
  double v[4] = {0.0, 0.0, 0.0, 0.0};
  long long cnt[2] = {0, 0};
  for (int i = tid; i < n; i += kStThreads) {
    const double z = (double)x[i] / tau;
    if (z >= hi) { v[0] += exp(-z - s1_ref); cnt[0] += 1; }
    else v[1] += exp(z - s2_ref);
  }
  st_block_sum(&sh, v, cnt);
  const int m = (int)cnt[0];
  const double log_s1 = m > 0 ? s1_ref + log(v[0]) : -INFINITY;
  const double log_s2 = m < n ? s2_ref + log(v[1]) : -INFINITY;
  // closed form of App. A.1 for y = e^lambda: S1 y^2 + 2 (k - m) y - S2 = 0, positive root
  const double d = k - (double)m;
  double lambda;
  if (m == 0) lambda = log_s2 - log(2.0 * k);
  else if (m == n) lambda = log(2.0 * ((double)n - k)) - log_s1;
  else if (d >= 0.0) lambda = log_s2 - log_root_plus(d, log_s1 + log_s2);
  else lambda = log_root_plus(-d, log_s1 + log_s2) - log_s1;
  if (tid == 0 && info != nullptr) {
    info[0] = lambda;
    info[1] = (double)m;
  }
  for (int i = tid; i < n; i += kStThreads) {
    const double z = (double)x[i] / tau - lambda;
    const double r = z >= 0.0 ? 1.0 - 0.5 * exp(-z) : 0.5 * exp(z);
    if (y != nullptr) y[i] = r;
    if (budgets != nullptr) budgets[i] = (int32_t)floor(r * t);
  }
}

// Backward of ST_k (App. A.2).  With z_i = x_i / tau - lambda and f'(z) = e^{-|z|} / 2 the implicit
// function theorem gives d lambda / d x_j = f'(z_j) / sum_i f'(z_i) = w_j and d lambda / d k =
// -1 / sum_i f'(z_i), hence for an upstream gradient g = dL/dy
//   dL/dx_j = (f'(z_j) / tau) (g_j - gbar),   dL/dk = gbar = sum_i g_i w_i.
// One workgroup, three passes over the input: the smallest |z| (the weights are formed relative to
// it, so a cold temperature at which every f'(z) underflows still yields the ratios), the two sums,
// the output.  lambda is read from the forward call's `info`.  Sums in a fixed order.
template <typename X>
__global__ void __launch_bounds__(kStThreads)
soft_topk_backward_kernel(const X* __restrict__ x, int n, double tau, const double* __restrict__ info,
                          const double* g, double* dx /* may alias g */, double* __restrict__ dk) {
  __shared__ StLargeShared sh;
  {   // one vector per block
    const size_t b = blockIdx.x;
    x += b * n;
    g += b * n;
    dx += b * n;
    info += 2 * b;
    if (dk != nullptr) dk += b;
  }
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const double lambda = info[0];
  double amin = INFINITY;
  for (int i = tid; i < n; i += kStThreads) amin = fmin(amin, fabs((double)x[i] / tau - lambda));
  for (int off = 32; off > 0; off >>= 1) amin = fmin(amin, __shfl_xor(amin, off, 64));
  if (lane == 0) sh.d[0][wave] = amin;
  __syncthreads();
  for (int w = 0; w < kStThreads / 64; ++w) amin = fmin(amin, sh.d[0][w]);
  double v[4] = {0.0, 0.0, 0.0, 0.0};
  long long cnt[2] = {0, 0};
  for (int i = tid; i < n; i += kStThreads) {
    const double e = exp(amin - fabs((double)x[i] / tau - lambda));
    v[0] += e;
    v[1] += g[i] * e;
  }
  st_block_sum(&sh, v, cnt);
  const double gbar = v[1] / v[0];
  if (tid == 0 && dk != nullptr) dk[0] = gbar;
  const double inv_tau = 1.0 / tau;
  for (int i = tid; i < n; i += kStThreads) {
    const double a = fabs((double)x[i] / tau - lambda);
    dx[i] = 0.5 * exp(-a) * (g[i] - gbar) * inv_tau;
  }
}

// s = w2 . SiLU(W1 e + b1) (+ b2) for one head per block
__global__ void __launch_bounds__(256)
head_scores_kernel(const float* __restrict__ emb, const float* __restrict__ w1, const float* __restrict__ b1,
                   const float* __restrict__ w2, const float* __restrict__ b2, int d_e, int hidden,
                   double* __restrict__ s) {
  extern __shared__ __align__(16) unsigned char smem[];
  double* part = reinterpret_cast<double*>(smem);   // [hidden]
  const float* e = emb + (size_t)blockIdx.x * d_e;
  for (int j = threadIdx.x; j < hidden; j += blockDim.x) {
    const float* w = w1 + (size_t)j * d_e;
    double z = 0.0;
    for (int q = 0; q < d_e; ++q) z = fma((double)w[q], (double)e[q], z);
    z += (double)b1[j];
    part[j] = (double)w2[j] * (z / (1.0 + exp(-z)));
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double acc = 0.0;
    for (int j = 0; j < hidden; ++j) acc += part[j];
    if (b2 != nullptr) acc += (double)b2[0];
    s[blockIdx.x] = acc;
  }
}

int padded_size(int n) {
  int P = 2;
  while (P < n) P <<= 1;
  return P;
}

size_t soft_topk_lds(int P, size_t key_bytes) {
  return (size_t)P * key_bytes + (size_t)(2 * kStThreads + kStLocal) * sizeof(double) + sizeof(StShared);
}

}  // namespace

int soft_topk_sorted_max_n(bool is_f64) { return kStKeyBytes / (int)(is_f64 ? sizeof(uint64_t) : sizeof(uint32_t)); }
int soft_topk_max_n(bool) { return kStLargeMaxN; }
int head_scores_max_hidden() { return 4096; }

hipError_t lkv_h_prepare() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(soft_topk_kernel<float, uint32_t>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)soft_topk_lds(kStKeyBytes / 4, 4));
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(soft_topk_kernel<double, uint64_t>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)soft_topk_lds(kStKeyBytes / 8, 8));
}

// y, info and budgets may each be null; y may alias x when x is fp64.  k_vec != nullptr: n_vec vectors of n values,
// one block each, targets read from the device.
void launch_soft_topk(const void* x, bool is_f64, int n, double k, double tau, double* y, double* info,
                      int32_t* budgets, double t, hipStream_t stream, int n_vec, const double* k_vec) {
  if (n > soft_topk_sorted_max_n(is_f64)) {   // too long to sort in LDS: bracketing passes over the input
    if (is_f64)
      hipLaunchKernelGGL(soft_topk_large_kernel<double>, dim3(n_vec), dim3(kStThreads), 0, stream,
                         static_cast<const double*>(x), n, k, tau, y, info, budgets, t, k_vec);
    else
      hipLaunchKernelGGL(soft_topk_large_kernel<float>, dim3(n_vec), dim3(kStThreads), 0, stream,
                         static_cast<const float*>(x), n, k, tau, y, info, budgets, t, k_vec);
    return;
  }
  const int P = padded_size(n);
  if (is_f64)
    hipLaunchKernelGGL((soft_topk_kernel<double, uint64_t>), dim3(n_vec), dim3(kStThreads), soft_topk_lds(P, 8), stream,
                       static_cast<const double*>(x), n, P, k, tau, y, info, budgets, t, k_vec);
  else
    hipLaunchKernelGGL((soft_topk_kernel<float, uint32_t>), dim3(n_vec), dim3(kStThreads), soft_topk_lds(P, 4), stream,
                       static_cast<const float*>(x), n, P, k, tau, y, info, budgets, t, k_vec);
}

void launch_soft_topk_backward(const void* x, bool is_f64, int n, double tau, const double* info, const double* g,
                               double* dx, double* dk, hipStream_t stream, int n_vec) {
  if (is_f64)
    hipLaunchKernelGGL(soft_topk_backward_kernel<double>, dim3(n_vec), dim3(kStThreads), 0, stream,
                       static_cast<const double*>(x), n, tau, info, g, dx, dk);
  else
    hipLaunchKernelGGL(soft_topk_backward_kernel<float>, dim3(n_vec), dim3(kStThreads), 0, stream,
                       static_cast<const float*>(x), n, tau, info, g, dx, dk);
}

void launch_head_scores(const float* emb, const float* w1, const float* b1, const float* w2, const float* b2,
                        int n_heads, int d_e, int hidden, double* s, hipStream_t stream) {
  hipLaunchKernelGGL(head_scores_kernel, dim3(n_heads), dim3(256), (size_t)hidden * sizeof(double), stream, emb, w1,
                     b1, w2, b2, d_e, hidden, s);
}

}  // namespace lkv
