// Stage 4 of Alg. 1 on the GPU: stable per-tier partition of the token bit map and
// group-wise quantize-and-pack into row-major tier segments.
//
// The quantizer is fp32 in a fixed operation order (this file is compiled with
// floating-point contraction off) so that codes, scales and offsets are
// reproducible bit for bit:
//   mn = min x, mx = max x            over a group of 32 channels
//   s  = fp16_rn((mx - mn) / Q)        Q = 2^b - 1, IEEE divide
//   m  = fp16_rn(mn)
//   code = clamp(rint((x - m) / s), 0, Q), all zero when s == 0
// Codes are packed little-endian: element i of a row sits at bit i*b (App. B).
#include "rdkv_internal.h"

namespace rdkv {

namespace {

constexpr int kPartBlock = 1024;   // tokens per partition block

__device__ __forceinline__ int tier_slot(uint8_t b) {   // 16,8,4,2 -> 0..3 ; else -1
  return b == 16 ? 0 : b == 8 ? 1 : b == 4 ? 2 : b == 2 ? 3 : -1;
}

// counts of each stored tier inside every block of 1024 tokens of every item
__global__ __launch_bounds__(256) void tier_count_kernel(const uint8_t* __restrict__ bits,
                                                         const int64_t* __restrict__ item_tok_off,
                                                         const int32_t* __restrict__ item_T,
                                                         const int32_t* __restrict__ item_blk_off,
                                                         int32_t* __restrict__ blk_counts) {
  const int item = blockIdx.y;
  const int T = item_T[item];
  const int t0 = blockIdx.x * kPartBlock;
  if (t0 >= T) return;
  const uint8_t* b = bits + item_tok_off[item];
  int c[4] = {0, 0, 0, 0};
  for (int t = t0 + threadIdx.x; t < min(T, t0 + kPartBlock); t += 256) {
    const int s = tier_slot(b[t]);
#pragma unroll
    for (int k = 0; k < 4; ++k) c[k] += (s == k);
  }
  __shared__ int sm[4][4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    int v = c[k];
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6][k] = v;
  }
  __syncthreads();
  if (threadIdx.x < 4) {
    const int k = threadIdx.x;
    blk_counts[(item_blk_off[item] + blockIdx.x) * 4 + k] = sm[0][k] + sm[1][k] + sm[2][k] + sm[3][k];
  }
}

// exclusive scan of the block counts of one item (one thread per tier; blocks are few)
__global__ void tier_scan_kernel(const int32_t* __restrict__ item_T, const int32_t* __restrict__ item_blk_off,
                                 int32_t* __restrict__ blk_counts, int32_t* __restrict__ item_counts) {
  const int item = blockIdx.x, k = threadIdx.x;
  if (k >= 4) return;
  const int nblk = (item_T[item] + kPartBlock - 1) / kPartBlock;
  int run = 0;
  int32_t* p = blk_counts + static_cast<int64_t>(item_blk_off[item]) * 4 + k;
  for (int i = 0; i < nblk; ++i) {
    const int v = p[i * 4];
    p[i * 4] = run;
    run += v;
  }
  item_counts[item * 4 + k] = run;
}

// writes the ascending position lists: tier_idx[item_base + tier_base + rank]
__global__ __launch_bounds__(256) void tier_scatter_kernel(const uint8_t* __restrict__ bits,
                                                           const int64_t* __restrict__ item_tok_off,
                                                           const int32_t* __restrict__ item_T,
                                                           const int32_t* __restrict__ item_blk_off,
                                                           const int32_t* __restrict__ blk_offsets,
                                                           const int64_t* __restrict__ idx_base /* [items][4] */,
                                                           int32_t* __restrict__ tier_idx) {
  const int item = blockIdx.y;
  const int T = item_T[item];
  const int t0 = blockIdx.x * kPartBlock;
  if (t0 >= T) return;
  const uint8_t* b = bits + item_tok_off[item];
  __shared__ int wave_cnt[4][4];
  __shared__ int run_base[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x < 4) run_base[threadIdx.x] = blk_offsets[(item_blk_off[item] + blockIdx.x) * 4 + threadIdx.x];
  __syncthreads();
  for (int sub = 0; sub < kPartBlock; sub += 256) {
    const int t = t0 + sub + threadIdx.x;
    const int s = t < T ? tier_slot(b[t]) : -1;
    int rank_in_wave = 0;
    int cnt[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const unsigned long long mask = __ballot(s == k);
      cnt[k] = __popcll(mask);
      if (s == k) rank_in_wave = __popcll(mask & ((1ull << lane) - 1ull));
    }
    if (lane == 0) {
#pragma unroll
      for (int k = 0; k < 4; ++k) wave_cnt[wave][k] = cnt[k];
    }
    __syncthreads();
    if (s >= 0) {
      int before = run_base[s];
      for (int w = 0; w < wave; ++w) before += wave_cnt[w][s];
      tier_idx[idx_base[item * 4 + s] + before + rank_in_wave] = t;
    }
    __syncthreads();
    if (threadIdx.x < 4) {
      const int k = threadIdx.x;
      run_base[k] += wave_cnt[0][k] + wave_cnt[1][k] + wave_cnt[2][k] + wave_cnt[3][k];
    }
    __syncthreads();
  }
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Quantize one group of 32 values (already in registers) and store codes + metadata.
template <int BITS>
__device__ __forceinline__ void quant_store_group(const float (&x)[32], uint8_t* __restrict__ data,
                                                  uint8_t* __restrict__ meta) {
  float mn = x[0], mx = x[0];
#pragma unroll
  for (int i = 1; i < 32; ++i) {
    mn = fminf(mn, x[i]);
    mx = fmaxf(mx, x[i]);
  }
  mn = mn + 0.0f;   // canonical +0
  constexpr float Q = static_cast<float>((1 << BITS) - 1);
  const _Float16 sh = static_cast<_Float16>((mx - mn) / Q);   // round to nearest even
  const _Float16 mh = static_cast<_Float16>(mn);
  const float s = static_cast<float>(sh), m = static_cast<float>(mh);
  uint32_t words[BITS];   // 32 codes * BITS bits = BITS 32-bit words
#pragma unroll
  for (int w = 0; w < BITS; ++w) words[w] = 0u;
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    float t = rintf((x[i] - m) / s);
    t = fminf(fmaxf(t, 0.0f), Q);
    const uint32_t code = (s == 0.0f) ? 0u : static_cast<uint32_t>(t);
    const int bit = i * BITS;
    words[bit >> 5] |= code << (bit & 31);
  }
  uint32_t* dst = reinterpret_cast<uint32_t*>(data);
#pragma unroll
  for (int w = 0; w < BITS; ++w) dst[w] = words[w];
  *reinterpret_cast<uint32_t*>(meta) =
      static_cast<uint32_t>(__builtin_bit_cast(unsigned short, sh)) |
      (static_cast<uint32_t>(__builtin_bit_cast(unsigned short, mh)) << 16);
}

struct PackArgs {
  const uint16_t* K;
  const uint16_t* V;
  const int32_t* tier_idx;
  const int64_t* idx_base;     // [items][4]
  const int32_t* counts;       // [items][4]
  const int64_t* seg_off;      // [items][4][4]
  const int64_t* item_row_off; // [items]: first row of the item's [T][d] block in K / V
  uint8_t* arena;
  int32_t ti;                  // which stored tier this launch packs
};

// one thread = one group of 32 channels of one kept row, for K and for V
template <int BITS>
__global__ __launch_bounds__(256) void quant_pack_kernel(PackArgs a) {
  const int item = blockIdx.y;
  const int n = a.counts[item * 4 + a.ti];
  const int row = blockIdx.x * 64 + (threadIdx.x >> 2);
  if (row >= n) return;
  const int grp = threadIdx.x & 3;
  const int pos = a.tier_idx[a.idx_base[item * 4 + a.ti] + row];
  const int64_t src_row = a.item_row_off[item] + pos;
  const int64_t* so = a.seg_off + (static_cast<int64_t>(item) * 4 + a.ti) * 4;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const uint16_t* src = (which == 0 ? a.K : a.V) + src_row * kHeadDim + grp * kGroup;
    uint8_t* data = a.arena + so[which * 2] + static_cast<int64_t>(row) * (kHeadDim * BITS / 8);
    const uint4* s4 = reinterpret_cast<const uint4*>(src);
    if constexpr (BITS == 16) {
      uint4* d4 = reinterpret_cast<uint4*>(data + grp * 64);
#pragma unroll
      for (int i = 0; i < 4; ++i) d4[i] = s4[i];
    } else {
      float x[32];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint4 v = s4[i];
        x[8 * i + 0] = bf16_lo(v.x); x[8 * i + 1] = bf16_hi(v.x);
        x[8 * i + 2] = bf16_lo(v.y); x[8 * i + 3] = bf16_hi(v.y);
        x[8 * i + 4] = bf16_lo(v.z); x[8 * i + 5] = bf16_hi(v.z);
        x[8 * i + 6] = bf16_lo(v.w); x[8 * i + 7] = bf16_hi(v.w);
      }
      uint8_t* meta = a.arena + so[which * 2 + 1] + static_cast<int64_t>(row) * 16 + grp * 4;
      quant_store_group<BITS>(x, data + grp * (kGroup * BITS / 8), meta);
    }
  }
}

}  // namespace

hipError_t launch_tier_count(const uint8_t* bits, const int64_t* item_tok_off, const int32_t* item_T,
                             const int32_t* item_blk_off, int32_t* blk_counts, int32_t* item_counts,
                             int n_items, int max_T, hipStream_t st) {
  const int max_blk = (max_T + kPartBlock - 1) / kPartBlock;
  if (n_items == 0 || max_blk == 0) return hipSuccess;
  hipLaunchKernelGGL(tier_count_kernel, dim3(max_blk, n_items), dim3(256), 0, st, bits, item_tok_off, item_T,
                     item_blk_off, blk_counts);
  hipLaunchKernelGGL(tier_scan_kernel, dim3(n_items), dim3(64), 0, st, item_T, item_blk_off, blk_counts,
                     item_counts);
  return hipGetLastError();
}

hipError_t launch_tier_scatter(const uint8_t* bits, const int64_t* item_tok_off, const int32_t* item_T,
                               const int32_t* item_blk_off, const int32_t* blk_offsets, const int64_t* idx_base,
                               int32_t* tier_idx, int n_items, int max_T, hipStream_t st) {
  const int max_blk = (max_T + kPartBlock - 1) / kPartBlock;
  if (n_items == 0 || max_blk == 0) return hipSuccess;
  hipLaunchKernelGGL(tier_scatter_kernel, dim3(max_blk, n_items), dim3(256), 0, st, bits, item_tok_off, item_T,
                     item_blk_off, blk_offsets, idx_base, tier_idx);
  return hipGetLastError();
}

hipError_t launch_quant_pack(const uint16_t* K, const uint16_t* V, const int32_t* tier_idx,
                             const int64_t* idx_base, const int32_t* counts, const int64_t* seg_off,
                             const int64_t* item_row_off, uint8_t* arena, int n_items,
                             const int32_t max_count[4], hipStream_t st) {
  for (int ti = 0; ti < 4; ++ti) {
    if (max_count[ti] == 0) continue;
    PackArgs a{K, V, tier_idx, idx_base, counts, seg_off, item_row_off, arena, ti};
    dim3 grid((max_count[ti] + 63) / 64, n_items), block(256);
    switch (ti) {
      case 0: hipLaunchKernelGGL(quant_pack_kernel<16>, grid, block, 0, st, a); break;
      case 1: hipLaunchKernelGGL(quant_pack_kernel<8>, grid, block, 0, st, a); break;
      case 2: hipLaunchKernelGGL(quant_pack_kernel<4>, grid, block, 0, st, a); break;
      default: hipLaunchKernelGGL(quant_pack_kernel<2>, grid, block, 0, st, a); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

int partition_block() { return kPartBlock; }

}  // namespace rdkv
