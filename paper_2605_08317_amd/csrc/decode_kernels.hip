// Split-K flash-decode over row-major bf16 rows (Sec. 3.3, Eq. 7) for gfx950: the uncompressed path and the
// 16-bit tier of a token-wise cache, and the log-sum-exp merge of split partials.
//
// One workgroup (4 wavefronts) streams one chunk of rows of one (sequence, KV head).  Sixteen lanes share a token:
// each lane owns 8 of the 128 channels, so a wavefront covers 4 tokens per load and a K/V byte is read once for
// all g query heads of the group.  Online softmax runs per 16-lane row with DPP reductions; rows, wavefronts and
// chunks are merged by log-sum-exp weights (rows and wavefronts in LDS, chunks by the merge kernels).
#include "decode_merge.h"
#include "rdkv_internal.h"

namespace rdkv {

namespace {

constexpr int kWG = 256;
constexpr int kWaves = 4;
constexpr float kNegBig = -1.0e30f;   // finite "minus infinity": keeps exp2(m_old - m_new) defined

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over the 16 lanes of a DPP row; every lane receives the same bits.
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_mov<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_mov<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_mov<0x141>(v);   // row_half_mirror
  v += dpp_mov<0x140>(v);   // row_mirror
  return v;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// 8 bf16 channel values of one row held by a lane, as floats
__device__ __forceinline__ void unpack8(const uint4& r, float (&x)[8]) {
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __uint_as_float(w[i] << 16);
    x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
  }
}

__device__ __forceinline__ uint4 load_lane(const uint8_t* __restrict__ base, int row, int c16) {
  return *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(row) * (kHeadDim * 2) + c16 * 16);
}

// Streams `rows` rows and leaves the chunk's unnormalised result in part_acc / part_ml (AGENT: with agent-scope
// stores, for a merge inside the same launch).
template <int G, bool AGENT>
__device__ __forceinline__ void process_rows(const uint8_t* __restrict__ kd, const uint8_t* __restrict__ vd,
                                             int rows, const uint16_t* __restrict__ q,
                                             float* __restrict__ part_acc, float* __restrict__ part_ml,
                                             float* smem) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane >> 4, c16 = lane & 15;
  // logits are kept in the log2 domain: q is scaled by log2(e) / sqrt(d)
  const float qscale = 1.4426950408889634f * 0.08838834764831845f;

  float qv[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    unpack8(*reinterpret_cast<const uint4*>(q + h * kHeadDim + c16 * 8), qv[h]);
#pragma unroll
    for (int c = 0; c < 8; ++c) qv[h][c] *= qscale;
  }

  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m[h] = kNegBig;
    l[h] = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[h][c] = 0.f;
  }

  const int last = rows - 1;
  for (int base = wave * 16; base < rows; base += kWaves * 16) {
    uint4 kr[4], vr[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) kr[u] = load_lane(kd, min(base + u * 4 + r, last), c16);
#pragma unroll
    for (int u = 0; u < 4; ++u) vr[u] = load_lane(vd, min(base + u * 4 + r, last), c16);

    float s[4][G];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float kx[8];
      unpack8(kr[u], kx);
      const bool valid = (base + u * 4 + r) < rows;
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float dot = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) dot = __builtin_fmaf(qv[h][c], kx[c], dot);
        dot = row16_sum(dot);
        s[u][h] = valid ? dot : -INFINITY;
      }
    }

    // online softmax, one update per 4 rows
    float p[4][G];
    bool changed = false;
    float alpha[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float mt = fmaxf(fmaxf(s[0][h], s[1][h]), fmaxf(s[2][h], s[3][h]));
      const float mn = fmaxf(m[h], mt);
      alpha[h] = fast_exp2(m[h] - mn);
      changed |= (mn != m[h]);
      m[h] = mn;
      float ls = 0.f;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        p[u][h] = fast_exp2(s[u][h] - mn);
        ls += p[u][h];
      }
      l[h] = __builtin_fmaf(l[h], alpha[h], ls);
    }
    if (__any(changed)) {
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[h][c] *= alpha[h];
    }

#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float vx[8];
      unpack8(vr[u], vx);
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[h][c] = __builtin_fmaf(p[u][h], vx[c], acc[h][c]);
    }
  }

  // ---- merge the 16 (wavefront, row) streams of this workgroup -------------
  float* s_ml = smem;                    // [16][G][2]
  float* s_acc = smem + 16 * G * 2;      // [4][G][128]
  const int sid = wave * 4 + r;
  if (c16 == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      s_ml[(sid * G + h) * 2] = m[h];
      s_ml[(sid * G + h) * 2 + 1] = l[h];
    }
  }
  __syncthreads();
  float mstar[G], lstar[G];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float mm = kNegBig;
    for (int i = 0; i < 16; ++i) mm = fmaxf(mm, s_ml[(i * G + h) * 2]);
    float ll = 0.f;
    for (int i = 0; i < 16; ++i) ll += s_ml[(i * G + h) * 2 + 1] * fast_exp2(s_ml[(i * G + h) * 2] - mm);
    mstar[h] = mm;
    lstar[h] = ll;
    const float f = fast_exp2(m[h] - mm);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      float v = acc[h][c] * f;
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      acc[h][c] = v;
    }
  }
  if (r == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int c = 0; c < 8; ++c) s_acc[(wave * G + h) * kHeadDim + c16 * 8 + c] = acc[h][c];
  }
  __syncthreads();
  for (int i = tid; i < G * kHeadDim; i += kWG) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) v += s_acc[w * G * kHeadDim + i];
    if constexpr (AGENT) merge::store_agent(part_acc + i, v); else part_acc[i] = v;
  }
  if (tid < G) {
    if constexpr (AGENT) {
      merge::store_agent(part_ml + tid * 2, mstar[tid]);
      merge::store_agent(part_ml + tid * 2 + 1, lstar[tid]);
    } else {
      part_ml[tid * 2] = mstar[tid];
      part_ml[tid * 2 + 1] = lstar[tid];
    }
  }
}

template <int G>
__global__ __launch_bounds__(kWG) void decode_dense_kernel(DenseArgs a) {
  __shared__ float smem[16 * G * 2 + kWaves * G * kHeadDim];
  const int split = blockIdx.x, head = blockIdx.y, sl = blockIdx.z;
  const int T = a.T[sl];
  const int row0 = split * a.chunk_rows;
  if (row0 >= T) return;
  const int rows = min(a.chunk_rows, T - row0);
  const int64_t first = a.row_off[sl] + static_cast<int64_t>(head) * T + row0;
  const uint8_t* kd = reinterpret_cast<const uint8_t*>(a.K) + first * (kHeadDim * 2);
  const uint8_t* vd = reinterpret_cast<const uint8_t*>(a.V) + first * (kHeadDim * 2);
  const int seq = a.seq_base + sl;
  const uint16_t* q = a.q + (static_cast<int64_t>(seq) * a.hq + head * G) * kHeadDim;
  const int64_t slot = (static_cast<int64_t>(sl) * a.hkv + head) * a.max_splits + split;
  process_rows<G, false>(kd, vd, rows, q, a.part_acc + slot * G * kHeadDim, a.part_ml + slot * G * 2, smem);
}

template <int G>
__global__ __launch_bounds__(kWG) void decode_tiered_kernel(const Chunk* __restrict__ chunks,
                                                            const uint8_t* __restrict__ arena,
                                                            const uint16_t* __restrict__ q, MergeArgs ma) {
  constexpr int kSplit = 16 * G * 2 + kWaves * G * kHeadDim;
  constexpr int kMerge = merge::merge_lds_floats(kWG, G);
  __shared__ float smem[kSplit > kMerge ? kSplit : kMerge];
  const Chunk ch = chunks[blockIdx.x];
  const int seq = ch.item / ma.hkv, head = ch.item % ma.hkv;
  const uint16_t* qp = q + (static_cast<int64_t>(seq) * ma.hq + head * G) * kHeadDim;
  float* pa = ma.part_acc + static_cast<int64_t>(ch.slot) * G * kHeadDim;
  float* pm = ma.part_ml + static_cast<int64_t>(ch.slot) * G * 2;
  // row-major bf16 rows: the 16-bit tier of a token-wise cache
  process_rows<G, true>(arena + ch.k_data, arena + ch.v_data, ch.rows, qp, pa, pm, smem);
  merge::partial_stores_done();
  __syncthreads();
  merge::arrive_and_merge<kWG>(ma, ch.item, ch.slot0, ch.nslots, G, smem);
}

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

hipError_t launch_decode_dense_split(const DenseArgs& a, int g, int n_seqs, hipStream_t st) {
  dim3 grid(a.max_splits, a.hkv, n_seqs), block(kWG);
  switch (g) {
    case 1: hipLaunchKernelGGL(decode_dense_kernel<1>, grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL(decode_dense_kernel<2>, grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL(decode_dense_kernel<4>, grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL(decode_dense_kernel<8>, grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_decode_dense_merge(const DenseArgs& a, int g, int n_seqs, hipStream_t st) {
  hipLaunchKernelGGL(merge_dense_kernel, dim3(n_seqs * a.hkv * g), dim3(kMergeThreads), 0, st, a, g);
  return hipGetLastError();
}

hipError_t launch_decode_tiered_split(const Chunk* chunks, int n_chunks, const uint8_t* arena, const uint16_t* q,
                                      const MergeArgs& ma, hipStream_t st) {
  const int g = ma.hq / ma.hkv;
  if (n_chunks == 0) return hipSuccess;
  dim3 grid(n_chunks), block(kWG);
  switch (g) {
    case 1: hipLaunchKernelGGL(decode_tiered_kernel<1>, grid, block, 0, st, chunks, arena, q, ma); break;
    case 2: hipLaunchKernelGGL(decode_tiered_kernel<2>, grid, block, 0, st, chunks, arena, q, ma); break;
    case 4: hipLaunchKernelGGL(decode_tiered_kernel<4>, grid, block, 0, st, chunks, arena, q, ma); break;
    case 8: hipLaunchKernelGGL(decode_tiered_kernel<8>, grid, block, 0, st, chunks, arena, q, ma); break;
    default: return hipErrorInvalidValue;
  }
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
