// Log-sum-exp merge of the split partials of a decode step (the last step of Eq. 7's evaluation as a split-K
// flash-decode) inside the decode kernels themselves: every workgroup stores its chunk's partial result, announces
// it on the item's arrival counter, and the workgroup that arrives last merges all partials of the item and writes
// the output rows.  One launch per decode step instead of a split launch and a merge launch.
//
// Memory ordering across the chip's eight L2 caches: partials are written and read with agent-scope accesses (they
// go through to memory instead of staying in one XCD's L2), every thread waits for its stores to drain before the
// workgroup's barrier, and one thread then bumps the counter with an agent-scope atomic.  The merging workgroup resets the
// counter, so a cache's workspace is ready for the next step on the same stream.  The merge has a fixed summation
// order (slot order), so results do not depend on which workgroup happens to arrive last.
#pragma once
#include "rdkv_internal.h"

namespace rdkv {

struct MergeArgs {
  float* part_acc;     // [slots][g][128] unnormalised partial outputs
  float* part_ml;      // [slots][g][2]   running maximum (log2 domain) and sum of each partial
  int32_t* arrive;     // [items] arrival counters, zero between steps
  float* out;          // [batch][hq][128]
  float* lse;          // [batch][hq] or null
  int32_t hq, hkv;
};

inline hipError_t launch_decode_mixed(const Chunk* chunks, int n_chunks, const uint8_t* arena, const ItemK* items_k,
                                      int max_words, int max_steps, int max_qsteps, const uint16_t* q,
                                      const MergeArgs& ma, const int32_t* tail_len, int per_unit, int waves,
                                      hipStream_t st) {
  const bool hs2 = ma.hq / ma.hkv > 4, lng = max_words > 32;
  return (hs2 ? (lng ? launch_decode_mixed_hs2_long1 : launch_decode_mixed_hs2_long0)
              : (lng ? launch_decode_mixed_hs1_long1 : launch_decode_mixed_hs1_long0))(
      chunks, n_chunks, arena, items_k, max_words, max_steps, max_qsteps, q, ma, tail_len, per_unit, waves, st);
}

namespace merge {

constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ void store_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float load_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Every thread calls this after its last store_agent of the partial and before the workgroup barrier that precedes
// arrive_and_merge(): agent-scope stores are written through to memory, so once the wave's store counter has drained
// they are visible to every XCD.  (A release fence would add a write-back of the whole L2, which has nothing of
// ours to write back and costs the launch tens of microseconds when hundreds of workgroups issue it.)
__device__ __forceinline__ void partial_stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// The merge proper for G query heads per KV head: thread = (slot group, channel).  Every load of a thread's slots is
// issued before anything waits (one memory round trip for up to SG * kBatch slots); each slot group reduces its slots
// with running maxima, and the SG groups are combined through LDS.
template <int NT, int G>
__device__ __forceinline__ void merge_item(const MergeArgs& ma, int item, int slot0, int nslots, float* smem) {
  constexpr int SG = NT / 128;
  constexpr int kBatch = G >= 8 ? 4 : 8;
  const int tid = threadIdx.x;
  const int c = tid & 127, sg = tid >> 7;
  float* s_m = smem + 16;                   // [SG][G]
  float* s_l = s_m + SG * 8;                // [SG][G]
  float* s_red = smem + 16 + 2 * SG * 8;    // [SG][G][128]
  const float* ml0 = ma.part_ml + static_cast<int64_t>(slot0) * G * 2;
  const float* acc0 = ma.part_acc + static_cast<int64_t>(slot0) * G * kHeadDim;
  float m_run[G], l_run[G], o_run[G];
#pragma unroll
  for (int h = 0; h < G; ++h) { m_run[h] = kNegBig; l_run[h] = 0.f; o_run[h] = 0.f; }
  for (int s0 = sg; s0 < nslots; s0 += SG * kBatch) {
    float a[kBatch][G], mv[kBatch][G], lv[kBatch][G];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int s = s0 + u * SG;
#pragma unroll
      for (int h = 0; h < G; ++h) {
        a[u][h] = 0.f; mv[u][h] = kNegBig; lv[u][h] = 0.f;
        if (s < nslots) {
          const float* pa = acc0 + (static_cast<int64_t>(s) * G + h) * kHeadDim + c;
          const float* pm = ml0 + (static_cast<int64_t>(s) * G + h) * 2;
          a[u][h] = load_agent(pa);
          mv[u][h] = load_agent(pm);
          lv[u][h] = load_agent(pm + 1);
        }
      }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float mb = m_run[h];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) mb = fmaxf(mb, mv[u][h]);
      const float f0 = __builtin_amdgcn_exp2f(m_run[h] - mb);
      float l = l_run[h] * f0, o = o_run[h] * f0;
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const float f = __builtin_amdgcn_exp2f(mv[u][h] - mb);
        l = __builtin_fmaf(lv[u][h], f, l);
        o = __builtin_fmaf(a[u][h], f, o);
      }
      m_run[h] = mb; l_run[h] = l; o_run[h] = o;
    }
  }
#pragma unroll
  for (int h = 0; h < G; ++h) {
    s_red[(sg * G + h) * kHeadDim + c] = o_run[h];
    if (c == 0) { s_m[sg * 8 + h] = m_run[h]; s_l[sg * 8 + h] = l_run[h]; }
  }
  __syncthreads();
  const int seq = item / ma.hkv, head = item % ma.hkv;
  const int64_t qh0 = static_cast<int64_t>(seq) * ma.hq + head * G;
  for (int idx = tid; idx < G * kHeadDim; idx += NT) {
    const int h = idx >> 7;
    float mm = kNegBig;
#pragma unroll
    for (int k = 0; k < SG; ++k) mm = fmaxf(mm, s_m[k * 8 + h]);
    float l = 0.f, t = 0.f;
#pragma unroll
    for (int k = 0; k < SG; ++k) {
      const float f = __builtin_amdgcn_exp2f(s_m[k * 8 + h] - mm);
      l = __builtin_fmaf(s_l[k * 8 + h], f, l);
      t = __builtin_fmaf(s_red[k * G * kHeadDim + idx], f, t);
    }
    ma.out[qh0 * kHeadDim + idx] = l > 0.f ? t / l : 0.f;
    if ((idx & 127) == 0 && ma.lse != nullptr)
      ma.lse[qh0 + h] = l > 0.f ? (mm + __log2f(l)) * 0.6931471805599453f : -INFINITY;
  }
}

// Called by all NT threads of a workgroup after a barrier that follows partial_stores_done().  Returns after the
// item's output rows are written if this workgroup arrived last, at once otherwise.
// smem: merge_lds_floats(NT, g) floats of LDS that nothing else uses any more.
// GMAX: the most query heads per KV head the calling kernel is built for (larger merges are not compiled into it)
template <int NT, int GMAX = 8>
__device__ __forceinline__ void arrive_and_merge(const MergeArgs& ma, int item, int slot0, int nslots, int g,
                                                 float* smem) {
  static_assert(NT % 128 == 0 && NT >= 128, "the merge assigns 128 channel threads per slot group");
  const int tid = threadIdx.x;
  int* s_flag = reinterpret_cast<int*>(smem);
  if (tid == 0) {
    const int old = __hip_atomic_fetch_add(ma.arrive + item, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *s_flag = old == nslots - 1;
  }
  __syncthreads();
  if (*s_flag == 0) return;
  // the partials are read with agent-scope loads, which do not hit stale lines of this XCD's caches
  if constexpr (GMAX > 4) {
    if (g > 4) merge_item<NT, 8>(ma, item, slot0, nslots, smem);
  }
  switch (g) {
    case 1: merge_item<NT, 1>(ma, item, slot0, nslots, smem); break;
    case 2: merge_item<NT, 2>(ma, item, slot0, nslots, smem); break;
    case 4: merge_item<NT, 4>(ma, item, slot0, nslots, smem); break;
    default: break;
  }
  if (tid == 0) __hip_atomic_store(ma.arrive + item, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS floats arrive_and_merge needs for NT threads and g heads
__host__ __device__ constexpr int merge_lds_floats(int nt, int g) { return 16 + 2 * (nt / 128) * 8 + (nt / 128) * g * 128; }

}  // namespace merge
}  // namespace rdkv
