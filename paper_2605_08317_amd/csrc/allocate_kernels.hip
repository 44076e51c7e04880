// Stages 2-3 of Alg. 1 on the GPU: the multiple-choice knapsack of Eq. 6 solved by
// Lagrangian bisection (Alg. 2), one workgroup per item.
//
// For a multiplier lam the per-unit minimiser of w eps(b) + lam b is the highest
// vertex k of the lower convex hull of (b, eps(b)) with (double) w > lam * r_k,
// r_k the slope ratio of the hull edge into k (computed on the host).  Thresholds
// are fp64, the summed bits are integers, and the search returns the feasible
// iterate with the smallest multiplier (first one inside the tolerance band
// below the budget), so the result never exceeds the budget.
#include <algorithm>

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
  double* lam_out;             // [items] or null: the multiplier of the returned allocation (NaN: no search ran)
  int32_t* iters_out;          // [items] or null: bisection steps taken
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

// Sum of a small int over the workgroup with one barrier: DPP row rotations inside a row of 16 lanes, four lane
// reads for the rows, one LDS slot per wavefront.  `sm` holds two sets of slots used alternately (parity), so that a
// call never overwrites slots another wavefront may still be reading from the previous call.
template <int CTRL>
__device__ __forceinline__ int dpp_add(int v) {
  return v + __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ int block_sum_small(int v, int* sm, int parity) {
  v = dpp_add<0x128>(v);   // row_ror:8
  v = dpp_add<0x124>(v);   // row_ror:4
  v = dpp_add<0x122>(v);   // row_ror:2
  v = dpp_add<0x121>(v);   // row_ror:1
  const int ws = __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
                 __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
  int* slots = sm + parity * (kThreads / 64);
  if ((threadIdx.x & 63) == 0) slots[threadIdx.x >> 6] = ws;
  __syncthreads();
  int t = 0;
#pragma unroll
  for (int i = 0; i < kThreads / 64; ++i) t += slots[i];
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

// Bit sum of one unit at thresholds thr: tiers[#thresholds strictly below w].
__device__ __forceinline__ int classify_tier(double wu, const double (&thr)[kMaxHull - 1], const int32_t (&tiers)[kMaxHull]) {
  int idx = 0;
#pragma unroll
  for (int k = 0; k < kMaxHull - 1; ++k) idx += (wu > thr[k]) ? 1 : 0;
  return tiers[idx];
}

// A unit is decided on the multiplier bracket [lo, hi] when no threshold lam * r_k, lam in [lo, hi], can change its
// tier: for every k either w > hi * r_k (above for all lam) or not w > lo * r_k (below for all lam).  Rounded fp64
// products are monotone in lam, so the test is exact.
__device__ __forceinline__ bool undecided(double wu, const double (&thr_lo)[kMaxHull - 1],
                                          const double (&thr_hi)[kMaxHull - 1]) {
  bool u = false;
#pragma unroll
  for (int k = 0; k < kMaxHull - 1; ++k) u |= (wu > thr_lo[k]) && !(wu > thr_hi[k]);
  return u;
}

constexpr int kListCap = 6144;    // undecided units kept in LDS (24 KiB)
constexpr int kBuckets = 8192;    // histogram over the top 13 bits of the positive fp32 pattern (32 KiB)
constexpr int kBucketShift = 18;

__device__ __forceinline__ int bucket_of(float w) {
  const uint32_t u = __float_as_uint(w);
  return (w > 0.0f) ? static_cast<int>(min(u, 0x7F7FFFFFu) >> kBucketShift) : 0;   // w <= 0 is never above a threshold
}

// An item's weights read as aligned 16-byte quads (one workgroup streams half a megabyte three times: with 4-byte
// loads the passes are bound by the number of load instructions in flight).  Quad q covers units 4 q - a .. 4 q - a + 3,
// a = how many floats the item's first weight sits past a 16-byte boundary; units outside [0, U) read as 0 and are
// skipped by the caller.  The first and the last quad are read element by element (their neighbours may lie outside
// the array).
struct Quads {
  const float* w;
  int a, U, nq;
  __device__ Quads(const float* w_, int U_) : w(w_), U(U_) {
    a = static_cast<int>((reinterpret_cast<uintptr_t>(w_) >> 2) & 3);
    nq = (U_ + a + 3) >> 2;
  }
  __device__ __forceinline__ int first_unit(int q) const { return 4 * q - a; }
  __device__ __forceinline__ void load(int q, float (&v)[4]) const {
    const int u0 = 4 * q - a;
    if (q > 0 && q + 1 < nq) {
      const float4 t = *reinterpret_cast<const float4*>(w + u0);
      v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = (q < nq && u0 + j >= 0 && u0 + j < U) ? w[u0 + j] : 0.0f;
    }
  }
};
constexpr int kQlp = 8;           // independent quad loads per thread in a streaming pass

// Units with w > thr: at least those in buckets above thr's bucket, at most those plus thr's own bucket.
// suffix[b] = number of units in buckets >= b (suffix[kBuckets] = 0).
__device__ __forceinline__ void count_bounds(double thr, const int* __restrict__ suffix, int* lo_cnt, int* hi_cnt) {
  // largest finite float <= thr (thr > 0): every float in a higher bucket exceeds thr, none in a lower bucket does
  float tf = static_cast<float>(fmin(thr, 3.4028234663852886e38));
  if (static_cast<double>(tf) > thr) tf = __uint_as_float(__float_as_uint(tf) - 1u);
  const int bt = static_cast<int>(__float_as_uint(tf) >> kBucketShift);
  *lo_cnt = suffix[bt + 1];
  *hi_cnt = suffix[bt];
}

__global__ __launch_bounds__(kThreads) void bisect_kernel(AllocArgs a) {
  __shared__ long long sm_sum[kThreads / 64];
  __shared__ float sm_max[kThreads / 64];
  __shared__ int s_hist[kBuckets + 1];
  __shared__ float s_list[kListCap];
  __shared__ int s_count;
  __shared__ int sm_small[2 * (kThreads / 64)];
  const int item = blockIdx.x;
  const int U = a.item_U[item];
  if (threadIdx.x == 0) {      // overwritten below when the search runs
    if (a.lam_out) a.lam_out[item] = __longlong_as_double(0x7FF8000000000000ll);
    if (a.iters_out) a.iters_out[item] = 0;
  }
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
  int32_t tiers[kMaxHull];
  double r[kMaxHull - 1];
#pragma unroll
  for (int k = 0; k < kMaxHull; ++k) tiers[k] = a.tiers[k];
#pragma unroll
  for (int k = 0; k < kMaxHull - 1; ++k) r[k] = a.r[k];

  // ---- one pass: maximum and histogram ------------------------------------------------------------------
  for (int i = threadIdx.x; i <= kBuckets; i += kThreads) s_hist[i] = 0;
  __syncthreads();
  float mx = 0.f;
  const Quads quads(w, U);
  for (int q0 = threadIdx.x; q0 < quads.nq; q0 += kQlp * kThreads) {
    float wv[kQlp][4];
#pragma unroll
    for (int j = 0; j < kQlp; ++j) quads.load(q0 + j * kThreads, wv[j]);
#pragma unroll
    for (int j = 0; j < kQlp; ++j) {
      const int u0 = quads.first_unit(q0 + j * kThreads);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (u0 + e >= 0 && u0 + e < U) {
          mx = fmaxf(mx, wv[j][e]);
          atomicAdd(&s_hist[bucket_of(wv[j][e])], 1);
        }
    }
  }
  mx = block_max(mx, sm_max);
  // suffix sums in place: s_hist[b] = units in buckets >= b (each thread owns 8 consecutive buckets)
  {
    const int b0 = threadIdx.x * (kBuckets / kThreads);
    int local = 0;
#pragma unroll
    for (int i = 0; i < kBuckets / kThreads; ++i) local += s_hist[b0 + i];
    __shared__ int s_part[kThreads];
    s_part[threadIdx.x] = local;
    __syncthreads();
    for (int off = 1; off < kThreads; off <<= 1) {   // inclusive suffix scan (Hillis-Steele)
      const int v = (threadIdx.x + off < kThreads) ? s_part[threadIdx.x + off] : 0;
      __syncthreads();
      s_part[threadIdx.x] += v;
      __syncthreads();
    }
    int run = s_part[threadIdx.x] - local;           // units in buckets above this thread's range
#pragma unroll
    for (int i = kBuckets / kThreads - 1; i >= 0; --i) {
      run += s_hist[b0 + i];
      s_hist[b0 + i] = run;
    }
    __syncthreads();
  }

  double lo = 0.0, hi = static_cast<double>(mx);
  double best = 0.0;
  bool have = false;
  // Every step decides exactly as Alg. 2 does at lam = (lo + hi) / 2.  While the histogram bounds on the bit sum
  // settle the comparisons, no unit is read.  At the first step they cannot, the units whose tier can still change
  // inside the bracket are moved to LDS (the others add a constant) and the remaining steps evaluate those exactly;
  // the same pass gives this step's exact sum, so if the units do not fit the search goes on with the bounds.
  int mode = 0;   // 0: histogram bounds, 1: list in LDS
  int n_list = 0;
  long long s_fixed = 0;
  int steps = 0;
  for (int it = 0; it < a.max_iters; ++it) {
    steps = it + 1;
    const double lam = (lo + hi) * 0.5;
    double thr[kMaxHull - 1];
#pragma unroll
    for (int k = 0; k < kMaxHull - 1; ++k) thr[k] = (k < nh - 1) ? lam * r[k] : INFINITY;
    long long s = 0;
    int verdict = -1;   // 0: over budget, 1: feasible (continue), 2: feasible and inside the band (stop)
    if (mode == 0) {
      long long s_min = static_cast<long long>(tiers[0]) * U, s_max = s_min;
#pragma unroll
      for (int k = 0; k < kMaxHull - 1; ++k) {
        if (k < nh - 1) {
          int c_lo, c_hi;
          count_bounds(thr[k], s_hist, &c_lo, &c_hi);
          s_min += static_cast<long long>(tiers[k + 1] - tiers[k]) * c_lo;
          s_max += static_cast<long long>(tiers[k + 1] - tiers[k]) * c_hi;
        }
      }
      if (s_min > B_int) verdict = 0;
      else if (s_max <= B_int && s_min >= need) verdict = 2;
      else if (s_max < need) verdict = 1;
      if (verdict < 0) {
        // ambiguous: collect the units still undecided on [lo, hi]
        double t_lo[kMaxHull - 1], t_hi[kMaxHull - 1];
#pragma unroll
        for (int k = 0; k < kMaxHull - 1; ++k) {
          t_lo[k] = (k < nh - 1) ? lo * r[k] : INFINITY;
          t_hi[k] = (k < nh - 1) ? hi * r[k] : INFINITY;
        }
        if (threadIdx.x == 0) s_count = 0;
        __syncthreads();
        long long sf = 0;
        for (int q0 = threadIdx.x; q0 < quads.nq; q0 += kQlp * kThreads) {
          float wv[kQlp][4];
#pragma unroll
          for (int j = 0; j < kQlp; ++j) quads.load(q0 + j * kThreads, wv[j]);
#pragma unroll
          for (int j = 0; j < kQlp; ++j) {
            const int u0 = quads.first_unit(q0 + j * kThreads);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (u0 + e >= 0 && u0 + e < U) {
                const double wu = static_cast<double>(wv[j][e]);
                s += classify_tier(wu, thr, tiers);                 // this step's exact bit sum
                if (undecided(wu, t_lo, t_hi)) {
                  const int pos = atomicAdd(&s_count, 1);
                  if (pos < kListCap) s_list[pos] = wv[j][e];
                } else {
                  sf += classify_tier(wu, t_hi, tiers);
                }
              }
          }
        }
        s = block_sum(s, sm_sum);
        s_fixed = block_sum(sf, sm_sum);
        __syncthreads();
        n_list = s_count;
        __syncthreads();                      // everyone has read the count before a later step resets it
        if (n_list <= kListCap) mode = 1;     // else: too many for LDS; try again at the next unsettled step
        verdict = s > B_int ? 0 : (s >= need ? 2 : 1);
      }
    } else if (mode == 1) {
      int sl = 0;   // at most kListCap * 16: fits an int
      for (int i = threadIdx.x; i < n_list; i += kThreads) sl += classify_tier(static_cast<double>(s_list[i]), thr, tiers);
      s = block_sum_small(sl, sm_small, it & 1) + s_fixed;
    }
    if (verdict < 0) verdict = s > B_int ? 0 : (s >= need ? 2 : 1);
    if (verdict == 0) {
      lo = lam;
    } else {
      best = lam;
      have = true;
      hi = lam;
      if (verdict == 2) break;
    }
  }
  if (threadIdx.x == 0) {
    if (a.lam_out && have) a.lam_out[item] = best;
    if (a.iters_out) a.iters_out[item] = steps;
  }
  double thr[kMaxHull - 1];
#pragma unroll
  for (int k = 0; k < kMaxHull - 1; ++k) thr[k] = (k < nh - 1) ? best * r[k] : INFINITY;
  for (int q0 = threadIdx.x; q0 < quads.nq; q0 += kQlp * kThreads) {
    float wv[kQlp][4];
#pragma unroll
    for (int j = 0; j < kQlp; ++j) quads.load(q0 + j * kThreads, wv[j]);
#pragma unroll
    for (int j = 0; j < kQlp; ++j) {
      const int u0 = quads.first_unit(q0 + j * kThreads);
      uint32_t packed = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int t = tiers[0];
        if (have) t = classify_tier(static_cast<double>(wv[j][e]), thr, tiers);
        packed |= static_cast<uint32_t>(t) << (8 * e);
      }
      if (u0 >= 0 && u0 + 3 < U && (reinterpret_cast<uintptr_t>(bits + u0) & 3) == 0) {
        *reinterpret_cast<uint32_t*>(bits + u0) = packed;          // four units' bytes at once
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (u0 + e >= 0 && u0 + e < U) bits[u0 + e] = static_cast<uint8_t>(packed >> (8 * e));
      }
    }
  }
}

// ---- the same search with an item's three streaming passes spread over many workgroups ---------------------------
// A long item (128K tokens) keeps one workgroup busy for 160 us in bisect_kernel while the rest of the chip idles.
// Here the passes that touch every unit run on kSlices workgroups per item, and only the steps of the search itself
// run on one:
//   hist_kernel      every slice histograms its units (top 13 bits of the fp32 pattern) and adds to the item's
//                    histogram and maximum;
//   steps_kernel<0>  the steps of Alg. 2 that the histogram's two-sided bounds on the bit sum decide, up to the first
//                    step they cannot; leaves the bracket [lo, hi] and the step index;
//   gather_kernel    every slice appends its units whose tier can still change inside the bracket to the item's list
//                    and adds the bits of the others (fixed from here on) to a sum;
//   steps_kernel<1>  the remaining steps, each evaluated exactly on the list plus the fixed sum;
//   write_kernel     the bit map at the multiplier found.
// Every verdict is the same integer comparison as in bisect_kernel, so the multipliers visited and the bit maps are
// the same bit for bit.  A list that would overflow makes steps_kernel<1> read all units of the item instead.
constexpr int kGlobalListCap = 32768;       // undecided units kept per item (floats)
struct SearchState {
  double lo, hi, best;
  long long s_fixed, B_int, need;
  float mx;
  int32_t have, it, done, fill, n_list, steps;
};
struct MultiArgs {
  AllocArgs a;
  int32_t* hist;        // [items][kBuckets + 1], zero on entry
  SearchState* state;   // [items], zero on entry
  float* list;          // [items][2][kGlobalListCap]: the list, and the half it moves to when it shrinks
  int32_t slices;
};

__device__ __forceinline__ void slice_range(const Quads& quads, int slices, int* q0, int* q1) {
  const int per = (quads.nq + slices - 1) / slices;
  *q0 = min(quads.nq, static_cast<int>(blockIdx.x) * per);
  *q1 = min(quads.nq, *q0 + per);
}

__global__ __launch_bounds__(kThreads) void hist_kernel(MultiArgs m) {
  __shared__ int s_hist[kBuckets + 1];
  __shared__ float sm_max[kThreads / 64];
  const AllocArgs& a = m.a;
  const int item = blockIdx.y;
  const int U = a.item_U[item];
  if (U == 0) return;
  const float* __restrict__ w = a.w + a.item_off[item];
  for (int i = threadIdx.x; i <= kBuckets; i += kThreads) s_hist[i] = 0;
  __syncthreads();
  const Quads quads(w, U);
  int q0, q1;
  slice_range(quads, m.slices, &q0, &q1);
  float mx = 0.f;
  for (int q = q0 + threadIdx.x; q < q1; q += kThreads) {
    float wv[4];
    quads.load(q, wv);
    const int u0 = quads.first_unit(q);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (u0 + e >= 0 && u0 + e < U) {
        mx = fmaxf(mx, wv[e]);
        atomicAdd(&s_hist[bucket_of(wv[e])], 1);
      }
  }
  mx = block_max(mx, sm_max);
  __syncthreads();
  int32_t* gh = m.hist + static_cast<int64_t>(item) * (kBuckets + 1);
  for (int i = threadIdx.x; i < kBuckets; i += kThreads)
    if (s_hist[i] != 0) atomicAdd(gh + i, s_hist[i]);
  // weights are non-negative here (a negative one never exceeds a threshold and mx starts at 0): integer order = float order
  if (threadIdx.x == 0 && mx > 0.f) atomicMax(reinterpret_cast<int*>(&m.state[item].mx), __float_as_int(mx));
}

// PHASE 0: steps decided by the histogram; PHASE 1: steps evaluated on the list (or on every unit after an overflow)
template <int PHASE>
__global__ __launch_bounds__(kThreads) void steps_kernel(MultiArgs m) {
  __shared__ long long sm_sum[kThreads / 64];
  __shared__ int s_hist[kBuckets + 1];
  __shared__ float s_list[kListCap];
  __shared__ int sm_small[2 * (kThreads / 64)];
  const AllocArgs& a = m.a;
  const int item = blockIdx.x;
  const int U = a.item_U[item];
  SearchState& st = m.state[item];
  const int nh = a.n_hull;
  int32_t tiers[kMaxHull];
  double r[kMaxHull - 1];
#pragma unroll
  for (int k = 0; k < kMaxHull; ++k) tiers[k] = a.tiers[k];
#pragma unroll
  for (int k = 0; k < kMaxHull - 1; ++k) r[k] = a.r[k];
  double lo, hi, best;
  bool have;
  int it0;
  long long B_int, need;
  if constexpr (PHASE == 0) {
    if (threadIdx.x == 0) {
      if (a.lam_out) a.lam_out[item] = __longlong_as_double(0x7FF8000000000000ll);
      if (a.iters_out) a.iters_out[item] = 0;
    }
    if (U == 0) { if (threadIdx.x == 0) { st.done = 1; st.fill = a.tiers[0]; } return; }
    B_int = static_cast<long long>(floor(a.item_budget[item] * static_cast<double>(U)));
    const int top = a.tiers[nh - 1];
    int fill = -1;
    if (B_int >= static_cast<long long>(top) * U) fill = top;
    else if (nh == 1 || B_int < a.tiers[1]) fill = a.tiers[0];
    if (fill >= 0) { if (threadIdx.x == 0) { st.done = 1; st.fill = fill; } return; }
    need = static_cast<long long>(ceil(a.need_frac * static_cast<double>(B_int)));
    const int32_t* gh = m.hist + static_cast<int64_t>(item) * (kBuckets + 1);
    for (int i = threadIdx.x; i <= kBuckets; i += kThreads) s_hist[i] = i < kBuckets ? gh[i] : 0;
    __syncthreads();
    {   // suffix sums in place: s_hist[b] = units in buckets >= b (each thread owns 8 consecutive buckets)
      const int b0 = threadIdx.x * (kBuckets / kThreads);
      int local = 0;
#pragma unroll
      for (int i = 0; i < kBuckets / kThreads; ++i) local += s_hist[b0 + i];
      __shared__ int s_part[kThreads];
      s_part[threadIdx.x] = local;
      __syncthreads();
      for (int off = 1; off < kThreads; off <<= 1) {
        const int v = (threadIdx.x + off < kThreads) ? s_part[threadIdx.x + off] : 0;
        __syncthreads();
        s_part[threadIdx.x] += v;
        __syncthreads();
      }
      int run = s_part[threadIdx.x] - local;
#pragma unroll
      for (int i = kBuckets / kThreads - 1; i >= 0; --i) {
        run += s_hist[b0 + i];
        s_hist[b0 + i] = run;
      }
      __syncthreads();
    }
    lo = 0.0; hi = static_cast<double>(st.mx); best = 0.0; have = false; it0 = 0;
  } else {
    if (st.done) return;
    lo = st.lo; hi = st.hi; best = st.best; have = st.have != 0; it0 = st.it;
    B_int = st.B_int; need = st.need;
  }
  const float* __restrict__ w = a.w + a.item_off[item];
  int n_list = 0;
  bool overflow = false;
  long long s_fixed = 0;
  float* gsrc = m.list + static_cast<int64_t>(item) * (2 * kGlobalListCap);   // the list, and where it moves when it shrinks
  float* gdst = gsrc + kGlobalListCap;
  if constexpr (PHASE == 1) {
    n_list = st.n_list;
    s_fixed = st.s_fixed;
    overflow = n_list > kGlobalListCap;
    if (!overflow && n_list <= kListCap) {
      for (int i = threadIdx.x; i < n_list; i += kThreads) s_list[i] = gsrc[i];
      __syncthreads();
    }
  }
  int steps = it0;
  for (int it = it0; it < a.max_iters; ++it) {
    const double lam = (lo + hi) * 0.5;
    double thr[kMaxHull - 1];
#pragma unroll
    for (int k = 0; k < kMaxHull - 1; ++k) thr[k] = (k < nh - 1) ? lam * r[k] : INFINITY;
    int verdict = -1;   // 0: over budget, 1: feasible (continue), 2: feasible and inside the band (stop)
    if constexpr (PHASE == 0) {
      long long s_min = static_cast<long long>(tiers[0]) * U, s_max = s_min;
#pragma unroll
      for (int k = 0; k < kMaxHull - 1; ++k)
        if (k < nh - 1) {
          int c_lo, c_hi;
          count_bounds(thr[k], s_hist, &c_lo, &c_hi);
          s_min += static_cast<long long>(tiers[k + 1] - tiers[k]) * c_lo;
          s_max += static_cast<long long>(tiers[k + 1] - tiers[k]) * c_hi;
        }
      if (s_min > B_int) verdict = 0;
      else if (s_max <= B_int && s_min >= need) verdict = 2;
      else if (s_max < need) verdict = 1;
      if (verdict < 0) {     // the histogram cannot decide this step: hand over to the list
        if (threadIdx.x == 0) {
          st.lo = lo; st.hi = hi; st.best = best; st.have = have; st.it = it; st.B_int = B_int; st.need = need;
          st.done = 0; st.n_list = 0; st.s_fixed = 0;
        }
        return;
      }
    } else {
      long long s;
      if (overflow) {        // every unit of the item
        long long sl = 0;
        for (int u = threadIdx.x; u < U; u += kThreads) sl += classify_tier(static_cast<double>(w[u]), thr, tiers);
        s = block_sum(sl, sm_sum);
      } else if (n_list <= kListCap) {
        int sl = 0;
        for (int i = threadIdx.x; i < n_list; i += kThreads) sl += classify_tier(static_cast<double>(s_list[i]), thr, tiers);
        s = block_sum_small(sl, sm_small, it & 1) + s_fixed;
      } else {
        int sl = 0;
        for (int i = threadIdx.x; i < n_list; i += kThreads) sl += classify_tier(static_cast<double>(gsrc[i]), thr, tiers);
        s = block_sum_small(sl, sm_small, it & 1) + s_fixed;
      }
      verdict = s > B_int ? 0 : (s >= need ? 2 : 1);
      if (!overflow && n_list > kListCap && verdict != 2) {
        // The list does not fit LDS yet.  The bracket has just halved: the units it has decided leave the list (their
        // bits join the fixed sum) and the rest moves to the other half of the item's list area, or into LDS once
        // few enough are left.  The order of a list does not matter: every sum over it is an integer sum.
        const double nlo = verdict == 0 ? lam : lo, nhi = verdict == 0 ? hi : lam;
        double t_lo[kMaxHull - 1], t_hi[kMaxHull - 1];
#pragma unroll
        for (int k = 0; k < kMaxHull - 1; ++k) {
          t_lo[k] = (k < nh - 1) ? nlo * r[k] : INFINITY;
          t_hi[k] = (k < nh - 1) ? nhi * r[k] : INFINITY;
        }
        __shared__ int s_keep;
        if (threadIdx.x == 0) s_keep = 0;
        __syncthreads();
        long long sf = 0;
        for (int i = threadIdx.x; i < n_list; i += kThreads) {
          const float wf = gsrc[i];
          const double wu = static_cast<double>(wf);
          if (undecided(wu, t_lo, t_hi)) gdst[atomicAdd(&s_keep, 1)] = wf;
          else sf += classify_tier(wu, t_hi, tiers);
        }
        s_fixed += block_sum(sf, sm_sum);
        __syncthreads();
        n_list = s_keep;
        __syncthreads();
        float* t = gsrc; gsrc = gdst; gdst = t;
        if (n_list <= kListCap) {
          __threadfence_block();
          for (int i = threadIdx.x; i < n_list; i += kThreads) s_list[i] = gsrc[i];
          __syncthreads();
        }
      }
    }
    steps = it + 1;
    if (verdict == 0) {
      lo = lam;
    } else {
      best = lam;
      have = true;
      hi = lam;
      if (verdict == 2) break;
    }
  }
  if (threadIdx.x == 0) {   // the search is over
    st.best = best; st.have = have; st.done = 1; st.fill = -1; st.steps = steps;
    if (a.lam_out && have) a.lam_out[item] = best;
    if (a.iters_out) a.iters_out[item] = steps;
  }
}

__global__ __launch_bounds__(kThreads) void gather_kernel(MultiArgs m) {
  __shared__ long long sm_sum[kThreads / 64];
  const AllocArgs& a = m.a;
  const int item = blockIdx.y;
  SearchState& st = m.state[item];
  if (st.done) return;
  const int U = a.item_U[item];
  const float* __restrict__ w = a.w + a.item_off[item];
  const int nh = a.n_hull;
  int32_t tiers[kMaxHull];
#pragma unroll
  for (int k = 0; k < kMaxHull; ++k) tiers[k] = a.tiers[k];
  double t_lo[kMaxHull - 1], t_hi[kMaxHull - 1];
#pragma unroll
  for (int k = 0; k < kMaxHull - 1; ++k) {
    t_lo[k] = (k < nh - 1) ? st.lo * a.r[k] : INFINITY;
    t_hi[k] = (k < nh - 1) ? st.hi * a.r[k] : INFINITY;
  }
  float* gl = m.list + static_cast<int64_t>(item) * (2 * kGlobalListCap);
  const Quads quads(w, U);
  int q0, q1;
  slice_range(quads, m.slices, &q0, &q1);
  // undecided units are collected in LDS first, so that the item's list counter sees one atomic per workgroup and
  // round of 1024 quads instead of one per unit
  __shared__ float s_buf[4 * kThreads];
  __shared__ int s_cnt, s_base;
  long long sf = 0;
  for (int base = q0; base < q1; base += kThreads) {
    if (threadIdx.x == 0) s_cnt = 0;
    __syncthreads();
    const int q = base + threadIdx.x;
    if (q < q1) {
      float wv[4];
      quads.load(q, wv);
      const int u0 = quads.first_unit(q);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (u0 + e >= 0 && u0 + e < U) {
          const double wu = static_cast<double>(wv[e]);
          if (undecided(wu, t_lo, t_hi)) s_buf[atomicAdd(&s_cnt, 1)] = wv[e];
          else sf += classify_tier(wu, t_hi, tiers);
        }
    }
    __syncthreads();
    const int cnt = s_cnt;
    if (cnt > 0) {
      if (threadIdx.x == 0) s_base = atomicAdd(&st.n_list, cnt);
      __syncthreads();
      const int b0 = s_base;
      for (int i = threadIdx.x; i < cnt; i += kThreads)
        if (b0 + i < kGlobalListCap) gl[b0 + i] = s_buf[i];
    }
    __syncthreads();
  }
  sf = block_sum(sf, sm_sum);
  if (threadIdx.x == 0 && sf != 0) atomicAdd(reinterpret_cast<unsigned long long*>(&st.s_fixed), static_cast<unsigned long long>(sf));
}

__global__ __launch_bounds__(kThreads) void write_kernel(MultiArgs m) {
  const AllocArgs& a = m.a;
  const int item = blockIdx.y;
  const int U = a.item_U[item];
  if (U == 0) return;
  const SearchState& st = m.state[item];
  const float* __restrict__ w = a.w + a.item_off[item];
  uint8_t* __restrict__ bits = a.bits + a.item_off[item];
  const int nh = a.n_hull;
  int32_t tiers[kMaxHull];
#pragma unroll
  for (int k = 0; k < kMaxHull; ++k) tiers[k] = a.tiers[k];
  const int fill = st.fill >= 0 ? st.fill : (st.have ? -1 : tiers[0]);
  double thr[kMaxHull - 1];
#pragma unroll
  for (int k = 0; k < kMaxHull - 1; ++k) thr[k] = (k < nh - 1) ? st.best * a.r[k] : INFINITY;
  const Quads quads(w, U);
  int q0, q1;
  slice_range(quads, m.slices, &q0, &q1);
  for (int q = q0 + threadIdx.x; q < q1; q += kThreads) {
    float wv[4];
    if (fill < 0) quads.load(q, wv);
    const int u0 = quads.first_unit(q);
    uint32_t packed = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int t = fill >= 0 ? fill : classify_tier(static_cast<double>(wv[e]), thr, tiers);
      packed |= static_cast<uint32_t>(t) << (8 * e);
    }
    if (u0 >= 0 && u0 + 3 < U && (reinterpret_cast<uintptr_t>(bits + u0) & 3) == 0) {
      *reinterpret_cast<uint32_t*>(bits + u0) = packed;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (u0 + e >= 0 && u0 + e < U) bits[u0 + e] = static_cast<uint8_t>(packed >> (8 * e));
    }
  }
}

// Stage 3 of Alg. 1: the K budget r_K * B_head of an item is spread over its retained tokens (bit-width above zero)
// only: k_avg = min(16, 2 r_K avg_bits T / n_kept) average bits per channel unit, 0 if nothing is retained; rounded
// to fp32 like every budget.  fp64 in this operation order (the file is compiled without contraction).
__global__ __launch_bounds__(1024) void stage3_budget_kernel(const uint8_t* __restrict__ bits,
                                                             const int64_t* __restrict__ item_off,
                                                             const int32_t* __restrict__ item_U,
                                                             const double* __restrict__ item_avg, double rk,
                                                             int32_t* __restrict__ kept,
                                                             double* __restrict__ k_budget) {
  __shared__ int sm[16];
  const int item = blockIdx.x;
  const int U = item_U[item];
  const uint8_t* b = bits + item_off[item];
  int c = 0;
  // 16 bytes per load once the pointer is aligned
  const int head = min(U, static_cast<int>((16 - (reinterpret_cast<uintptr_t>(b) & 15)) & 15));
  for (int u = threadIdx.x; u < head; u += 1024) c += b[u] != 0;
  const int nq = (U - head) >> 4;
  const uint4* q = reinterpret_cast<const uint4*>(b + head);
  for (int i = threadIdx.x; i < nq; i += 1024) {
    const uint4 v = q[i];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int e = 0; e < 4; ++e) c += ((w[k] >> (8 * e)) & 0xFFu) != 0;
  }
  for (int u = head + 16 * nq + threadIdx.x; u < U; u += 1024) c += b[u] != 0;
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    int n = 0;
    for (int i = 0; i < 16; ++i) n += sm[i];
    kept[item] = n;
    double k_avg = 0.0;
    if (n > 0) k_avg = fmin(16.0, 2.0 * rk * item_avg[item] * static_cast<double>(U) / static_cast<double>(n));
    k_budget[item] = static_cast<double>(static_cast<float>(k_avg));
  }
}

}  // namespace

hipError_t launch_stage3_budget(const uint8_t* bits, const int64_t* d_item_off, const int32_t* d_item_U,
                                const double* d_item_avg, double rk, int n_items, int32_t* kept, double* k_budget,
                                hipStream_t st) {
  if (n_items == 0) return hipSuccess;
  hipLaunchKernelGGL(stage3_budget_kernel, dim3(n_items), dim3(1024), 0, st, bits, d_item_off, d_item_U, d_item_avg,
                     rk, kept, k_budget);
  return hipGetLastError();
}

hipError_t launch_allocate(const float* w, const int64_t* d_item_off, const int32_t* d_item_U,
                           const double* d_item_budget, int n_items, int n_hull, const int* hull_tiers,
                           const double* hull_r, double need_frac, int max_iters, uint8_t* bits, double* lam_out,
                           int32_t* iters_out, void* multi_scratch, hipStream_t st) {
  if (n_items == 0) return hipSuccess;
  if (n_hull < 1 || n_hull > kMaxHull) return hipErrorInvalidValue;
  AllocArgs a;
  a.w = w; a.item_off = d_item_off; a.item_U = d_item_U; a.item_budget = d_item_budget; a.bits = bits;
  for (int k = 0; k < kMaxHull; ++k) {
    a.tiers[k] = k < n_hull ? hull_tiers[k] : 0;
    a.r[k] = k < n_hull - 1 ? hull_r[k] : 0.0;
  }
  a.n_hull = n_hull; a.max_iters = max_iters; a.need_frac = need_frac;
  a.lam_out = lam_out; a.iters_out = iters_out;
  if (multi_scratch != nullptr) {   // long items: the streaming passes on many workgroups
    MultiArgs m;
    m.a = a;
    uint8_t* p = static_cast<uint8_t*>(multi_scratch);
    const size_t hist_b = (static_cast<size_t>(n_items) * (kBuckets + 1) * sizeof(int32_t) + 255) / 256 * 256;
    const size_t state_b = (static_cast<size_t>(n_items) * sizeof(SearchState) + 255) / 256 * 256;
    m.hist = reinterpret_cast<int32_t*>(p);
    m.state = reinterpret_cast<SearchState*>(p + hist_b);
    m.list = reinterpret_cast<float*>(p + hist_b + state_b);
    m.slices = std::max(1, std::min(64, 512 / n_items));
    hipError_t e = hipMemsetAsync(p, 0, hist_b + state_b, st);
    if (e != hipSuccess) return e;
    const dim3 wide(m.slices, n_items), one(n_items), block(kThreads);
    hipLaunchKernelGGL(hist_kernel, wide, block, 0, st, m);
    hipLaunchKernelGGL(steps_kernel<0>, one, block, 0, st, m);
    hipLaunchKernelGGL(gather_kernel, wide, block, 0, st, m);
    hipLaunchKernelGGL(steps_kernel<1>, one, block, 0, st, m);
    hipLaunchKernelGGL(write_kernel, wide, block, 0, st, m);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(bisect_kernel, dim3(n_items), dim3(kThreads), 0, st, a);
  return hipGetLastError();
}

// device scratch launch_allocate needs to spread long items over many workgroups
size_t allocate_multi_scratch_bytes(int n_items) {
  const size_t hist_b = (static_cast<size_t>(n_items) * (kBuckets + 1) * sizeof(int32_t) + 255) / 256 * 256;
  const size_t state_b = (static_cast<size_t>(n_items) * sizeof(SearchState) + 255) / 256 * 256;
  return hist_b + state_b + static_cast<size_t>(n_items) * 2 * kGlobalListCap * sizeof(float);
}

}  // namespace rdkv
