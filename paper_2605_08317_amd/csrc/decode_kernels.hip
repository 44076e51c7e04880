// The log-sum-exp merge of the uncompressed path's split partials, and the kernels that keep the appended-token
// zone (Sec. 3.3 Zone C): append a row, gather the rows back for re-budgeting.
#include "decode_merge.h"
#include "rdkv_internal.h"

namespace rdkv {

namespace {

constexpr float kNegBig = -1.0e30f;   // finite "minus infinity": keeps exp2(m_old - m_new) defined

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Log-sum-exp merge of the partial results of one (item, query head).  512 threads: 4 slot groups x 128
// channels.  Every thread issues all the loads of its (up to kMergeBatch) slots before anything waits on them: the
// running maxima, the sums and the accumulators of a batch arrive together, so a merge of a few dozen partials costs
// two dependent memory round trips (slot range, then data) instead of one per pass.  Fixed summation order.
constexpr int kMergeThreads = 512;
constexpr int kMergeBatch = 16;   // slots per thread and round: 64 slots per (item, head) and round

__device__ __forceinline__ void merge_slots(const float* __restrict__ part_acc, const float* __restrict__ part_ml,
                                            int64_t slot0, int n, int g, int h, float* __restrict__ out,
                                            float* __restrict__ lse) {
  __shared__ float sm_m[4], sm_l[4];
  __shared__ float sm_o[4][kHeadDim];
  const int tid = threadIdx.x, c = tid & (kHeadDim - 1), grp = tid >> 7;
  float m_run = kNegBig, l_run = 0.f, o_run = 0.f;      // of this thread's slots: grp, grp + 4, ...
  for (int base = grp; base < n; base += 4 * kMergeBatch) {
    float2 ml[kMergeBatch];
    float a[kMergeBatch];
#pragma unroll
    for (int u = 0; u < kMergeBatch; ++u) {
      const int i = base + 4 * u;
      ml[u] = make_float2(kNegBig, 0.f);
      a[u] = 0.f;
      if (i < n) {
        const int64_t s = slot0 + i;
        ml[u] = *reinterpret_cast<const float2*>(part_ml + (s * g + h) * 2);
        a[u] = part_acc[(s * g + h) * kHeadDim + c];
      }
    }
    float mb = m_run;
#pragma unroll
    for (int u = 0; u < kMergeBatch; ++u) mb = fmaxf(mb, ml[u].x);
    const float f0 = fast_exp2(m_run - mb);
    l_run *= f0;
    o_run *= f0;
#pragma unroll
    for (int u = 0; u < kMergeBatch; ++u) {
      const float f = fast_exp2(ml[u].x - mb);
      l_run = __builtin_fmaf(ml[u].y, f, l_run);
      o_run = __builtin_fmaf(a[u], f, o_run);
    }
    m_run = mb;
  }
  // the four slot groups: every thread of a group holds the same (m, l)
  if (c == 0) {
    sm_m[grp] = m_run;
    sm_l[grp] = l_run;
  }
  sm_o[grp][c] = o_run;
  __syncthreads();
  if (grp == 0) {
    const float mstar = fmaxf(fmaxf(sm_m[0], sm_m[1]), fmaxf(sm_m[2], sm_m[3]));
    float l = 0.f, t = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float f = fast_exp2(sm_m[k] - mstar);
      l = __builtin_fmaf(sm_l[k], f, l);
      t = __builtin_fmaf(sm_o[k][c], f, t);
    }
    const bool empty = !(l > 0.f);
    out[c] = empty ? 0.f : t / l;
    if (lse != nullptr && c == 0) *lse = empty ? -INFINITY : (mstar + __log2f(l)) * 0.6931471805599453f;
  }
}

__global__ __launch_bounds__(kMergeThreads) void merge_dense_kernel(DenseArgs a, int g) {
  const int h = blockIdx.x % g;
  const int item = blockIdx.x / g;            // local: sl * hkv + head
  const int sl = item / a.hkv, head = item % a.hkv;
  const int T = a.T[sl];
  const int n = (T + a.chunk_rows - 1) / a.chunk_rows;
  const int64_t qh = static_cast<int64_t>(a.seq_base + sl) * a.hq + head * g + h;
  merge_slots(a.part_acc, a.part_ml, static_cast<int64_t>(item) * a.max_splits, n, g, h,
              a.out + qh * kHeadDim, a.lse ? a.lse + qh : nullptr);
}

}  // namespace

hipError_t launch_decode_dense_merge(const DenseArgs& a, int g, int n_seqs, hipStream_t st) {
  hipLaunchKernelGGL(merge_dense_kernel, dim3(n_seqs * a.hkv * g), dim3(kMergeThreads), 0, st, a, g);
  return hipGetLastError();
}

// Zone C: one new bf16 K row and V row per item, scattered into the item's tail at the token index held in the
// cache's device word tail_state[0] (so that a captured launch appends at the right place on every replay).  The
// tail is kept in the 64-token tiles the decode kernels read (see process_tail_tiles): per item tail_tiles tiles of
// 16 KiB for K, then (after the K tiles of all items) the same for V.  tail_state[1] counts the workgroups that are
// done: the last one advances the length and clears the count.  A full tail is left as it is.
__global__ __launch_bounds__(256) void append_rows_kernel(const uint16_t* __restrict__ k_new,
                                                          const uint16_t* __restrict__ v_new, uint8_t* __restrict__ tail,
                                                          int64_t n_items, int32_t tail_tiles, int32_t tail_cap,
                                                          int32_t* tail_state) {
  const int64_t item = blockIdx.x;
  const int t = threadIdx.x;
  const int row = __hip_atomic_load(tail_state, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const int tile = row >> 6, r = row & 63;
  constexpr int kTileBytes = 64 * kHeadDim * 2;
  if (row < tail_cap) {
    if (t < 16) {          // K: words 4t .. 4t+3 of the token's row = 16 bytes at 1024 t + 16 r
      const uint4 v = *reinterpret_cast<const uint4*>(k_new + item * kHeadDim + t * 8);
      uint8_t* dst = tail + (item * tail_tiles + tile) * static_cast<int64_t>(kTileBytes) + 1024 * t + 16 * r;
      *reinterpret_cast<uint4*>(dst) = v;
    } else if (t >= 128) {  // V: channel c of the token: unit u = 4 (c / 32) + (r % 32) / 8, lane 32 (r / 32) + c % 32
      const int c = t - 128;
      const int lane = 32 * (r >> 5) + (c & 31), u = 4 * (c >> 5) + ((r & 31) >> 3);
      uint8_t* dst = tail + ((n_items + item) * tail_tiles + tile) * static_cast<int64_t>(kTileBytes) + 1024 * u +
                     16 * lane + 2 * (r & 7);
      *reinterpret_cast<uint16_t*>(dst) = v_new[item * kHeadDim + c];
    }
  }
  __syncthreads();         // every thread has read the length (and written its part of the row)
  if (t == 0) {
    const int done = __hip_atomic_fetch_add(tail_state + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (done == static_cast<int>(n_items) - 1) {   // every workgroup has read the length: advance it
      __hip_atomic_store(tail_state + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (row < tail_cap) __hip_atomic_store(tail_state, row + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

hipError_t launch_append_rows(const uint16_t* k_new, const uint16_t* v_new, uint8_t* tail, int64_t n_items,
                              int32_t tail_tiles, int32_t tail_cap, int32_t* tail_state, hipStream_t st) {
  if (n_items == 0) return hipSuccess;
  hipLaunchKernelGGL(append_rows_kernel, dim3(static_cast<unsigned>(n_items)), dim3(256), 0, st, k_new, v_new, tail,
                     n_items, tail_tiles, tail_cap, tail_state);
  return hipGetLastError();
}

// Inverse of append_rows_kernel: the first n tokens of every item's tail, as row-major bf16 [items][n][128] K and V
// (the input format of the compression pass).  One workgroup = one 64-token tile of one item.
__global__ __launch_bounds__(256) void gather_tail_rows_kernel(const uint8_t* __restrict__ tail, int64_t n_items,
                                                               int32_t tail_tiles, int32_t n,
                                                               uint16_t* __restrict__ k_rows, uint16_t* __restrict__ v_rows) {
  const int64_t item = blockIdx.y;
  const int tile = blockIdx.x, t = threadIdx.x;
  constexpr int kTileBytes = 64 * kHeadDim * 2;
  const uint8_t* kt = tail + (item * tail_tiles + tile) * static_cast<int64_t>(kTileBytes);
  const uint8_t* vt = tail + ((n_items + item) * tail_tiles + tile) * static_cast<int64_t>(kTileBytes);
  const int64_t row_base = item * n + static_cast<int64_t>(tile) * 64;
#pragma unroll
  for (int j = 0; j < 4; ++j) {   // K: 16-byte unit (w, r) at 1024 w + 16 r holds channels 8w .. 8w+7 of token r
    const int idx = j * 256 + t, w = idx >> 6, r = idx & 63;
    if (tile * 64 + r < n)
      *reinterpret_cast<uint4*>(k_rows + (row_base + r) * kHeadDim + 8 * w) =
          *reinterpret_cast<const uint4*>(kt + 1024 * w + 16 * r);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {   // V: unit (u, lane) holds channel 32 (u / 4) + lane % 32 of 8 consecutive tokens
    const int idx = j * 256 + t, u = idx >> 6, lane = idx & 63;
    const uint4 v = *reinterpret_cast<const uint4*>(vt + 1024 * u + 16 * lane);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    const int c = 32 * (u >> 2) + (lane & 31), r0 = 32 * (lane >> 5) + 8 * (u & 3);
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (tile * 64 + r0 + k < n)
        v_rows[(row_base + r0 + k) * kHeadDim + c] = static_cast<uint16_t>(w[k >> 1] >> (16 * (k & 1)));
  }
}

hipError_t launch_gather_tail_rows(const uint8_t* tail, int64_t n_items, int32_t tail_tiles, int32_t n,
                                   uint16_t* k_rows, uint16_t* v_rows, hipStream_t st) {
  if (n_items == 0 || n == 0) return hipSuccess;
  hipLaunchKernelGGL(gather_tail_rows_kernel, dim3((n + 63) / 64, static_cast<unsigned>(n_items)), dim3(256), 0, st,
                     tail, n_items, tail_tiles, n, k_rows, v_rows);
  return hipGetLastError();
}

}  // namespace rdkv
