// Stages 2-3 of Alg. 1 on the GPU: the multiple-choice knapsack of Eq. 6 solved by
// Lagrangian bisection (Alg. 2), one workgroup per item.
//
// For a multiplier lam the per-unit minimiser of w eps(b) + lam b is the highest
// vertex k of the lower convex hull of (b, eps(b)) with (double) w > lam * r_k,
// r_k the slope ratio of the hull edge into k (computed on the host).  Thresholds
// are fp64, the summed bits are integers, and the search returns the feasible
// iterate with the smallest multiplier (first one inside the tolerance band
// below the budget), so the result never exceeds the budget.
#include "rdkv_internal.h"

namespace rdkv {

namespace {

constexpr int kThreads = 1024;
constexpr int kMaxHull = 5;

struct AllocArgs {
  const float* w;
  const int64_t* item_off;
  const int32_t* item_U;
  const double* item_budget;   // average bits per unit
  uint8_t* bits;
  double r[kMaxHull];          // r[k-1]: threshold ratio into hull tier k
  int32_t tiers[kMaxHull];
  int32_t n_hull;
  int32_t max_iters;
  double need_frac;            // 1 - rel_tol
};

__device__ __forceinline__ long long block_sum(long long v, long long* sm) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[wave] = v;
  __syncthreads();
  long long t = 0;
  for (int i = 0; i < kThreads / 64; ++i) t += sm[i];
  return t;
}

__device__ __forceinline__ float block_max(float v, float* sm) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[wave] = v;
  __syncthreads();
  float t = sm[0];
  for (int i = 1; i < kThreads / 64; ++i) t = fmaxf(t, sm[i]);
  return t;
}

__global__ __launch_bounds__(kThreads) void bisect_kernel(AllocArgs a) {
  __shared__ long long sm_sum[kThreads / 64];
  __shared__ float sm_max[kThreads / 64];
  const int item = blockIdx.x;
  const int U = a.item_U[item];
  if (U == 0) return;
  const float* __restrict__ w = a.w + a.item_off[item];
  uint8_t* __restrict__ bits = a.bits + a.item_off[item];
  const int nh = a.n_hull;
  const long long B_int = static_cast<long long>(floor(a.item_budget[item] * static_cast<double>(U)));
  const int top = a.tiers[nh - 1];
  int fill = -1;
  if (B_int >= static_cast<long long>(top) * U) fill = top;
  else if (nh == 1 || B_int < a.tiers[1]) fill = a.tiers[0];
  if (fill >= 0) {
    for (int u = threadIdx.x; u < U; u += kThreads) bits[u] = static_cast<uint8_t>(fill);
    return;
  }
  const long long need = static_cast<long long>(ceil(a.need_frac * static_cast<double>(B_int)));

  float mx = 0.f;
  for (int u = threadIdx.x; u < U; u += kThreads) mx = fmaxf(mx, w[u]);
  mx = block_max(mx, sm_max);

  double lo = 0.0, hi = static_cast<double>(mx);
  double best = 0.0;
  bool have = false;
  // per-step increments of the bit sum when a threshold is passed: tiers[k] - tiers[k-1]
  for (int it = 0; it < a.max_iters; ++it) {
    const double lam = (lo + hi) * 0.5;
    double thr[kMaxHull - 1];
#pragma unroll
    for (int k = 0; k < kMaxHull - 1; ++k) thr[k] = (k < nh - 1) ? lam * a.r[k] : INFINITY;
    long long s = 0;
    for (int u = threadIdx.x; u < U; u += kThreads) {
      const double wu = static_cast<double>(w[u]);
      int idx = 0;
#pragma unroll
      for (int k = 0; k < kMaxHull - 1; ++k) idx += (wu > thr[k]) ? 1 : 0;
      s += a.tiers[idx];
    }
    s = block_sum(s, sm_sum);
    if (s <= B_int) {
      best = lam;
      have = true;
      hi = lam;
      if (s >= need) break;
    } else {
      lo = lam;
    }
  }
  double thr[kMaxHull - 1];
#pragma unroll
  for (int k = 0; k < kMaxHull - 1; ++k) thr[k] = (k < nh - 1) ? best * a.r[k] : INFINITY;
  for (int u = threadIdx.x; u < U; u += kThreads) {
    int idx = 0;
    if (have) {
      const double wu = static_cast<double>(w[u]);
#pragma unroll
      for (int k = 0; k < kMaxHull - 1; ++k) idx += (wu > thr[k]) ? 1 : 0;
    }
    bits[u] = static_cast<uint8_t>(a.tiers[idx]);
  }
}

// retained units (bit-width above zero) of every item: Stage 3 spreads the K budget over them
__global__ __launch_bounds__(256) void count_kept_kernel(const uint8_t* __restrict__ bits,
                                                         const int64_t* __restrict__ item_off,
                                                         const int32_t* __restrict__ item_U,
                                                         int32_t* __restrict__ kept) {
  __shared__ int sm[4];
  const int item = blockIdx.x;
  const uint8_t* b = bits + item_off[item];
  int c = 0;
  for (int u = threadIdx.x; u < item_U[item]; u += 256) c += b[u] != 0;
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) kept[item] = sm[0] + sm[1] + sm[2] + sm[3];
}

}  // namespace

hipError_t launch_count_kept(const uint8_t* bits, const int64_t* d_item_off, const int32_t* d_item_U, int n_items,
                             int32_t* kept, hipStream_t st) {
  if (n_items == 0) return hipSuccess;
  hipLaunchKernelGGL(count_kept_kernel, dim3(n_items), dim3(256), 0, st, bits, d_item_off, d_item_U, kept);
  return hipGetLastError();
}

hipError_t launch_allocate(const float* w, const int64_t* d_item_off, const int32_t* d_item_U,
                           const double* d_item_budget, int n_items, int n_hull, const int* hull_tiers,
                           const double* hull_r, double need_frac, int max_iters, uint8_t* bits, hipStream_t st) {
  if (n_items == 0) return hipSuccess;
  if (n_hull < 1 || n_hull > kMaxHull) return hipErrorInvalidValue;
  AllocArgs a;
  a.w = w; a.item_off = d_item_off; a.item_U = d_item_U; a.item_budget = d_item_budget; a.bits = bits;
  for (int k = 0; k < kMaxHull; ++k) {
    a.tiers[k] = k < n_hull ? hull_tiers[k] : 0;
    a.r[k] = k < n_hull - 1 ? hull_r[k] : 0.0;
  }
  a.n_hull = n_hull; a.max_iters = max_iters; a.need_frac = need_frac;
  hipLaunchKernelGGL(bisect_kernel, dim3(n_items), dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace rdkv
