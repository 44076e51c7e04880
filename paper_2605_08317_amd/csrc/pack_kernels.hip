// Stage 4 of Alg. 1 on the GPU: stable per-tier partition of the token bit map and
// group-wise quantize-and-pack into tier segments (16-bit rows row-major, quantized tiers in 64-row tiles in
// token-wise mode and 32-row tiles in mixed mode).
//
// The quantizer is fp32 in a fixed operation order (this file is compiled with
// floating-point contraction off) so that codes, scales and offsets are
// reproducible bit for bit:
//   mn = min x, mx = max x            over a group of 32 channels
//   s  = fp16_rn((mx - mn) / Q)        Q = 2^b - 1, IEEE divide
//   m  = fp16_rn(mn)
//   code = clamp(rint((x - m) / s), 0, Q), all zero when s == 0
// Codes occupy b-bit fields of little-endian words (App. B: fields at bit offsets 0,2,4,6 / 0,4 of a byte).
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
                                                         int32_t* __restrict__ blk_counts,
                                                         int32_t* __restrict__ invalid) {
  const int item = blockIdx.y;
  const int T = item_T[item];
  const int t0 = blockIdx.x * kPartBlock;
  if (t0 >= T) return;
  const uint8_t* b = bits + item_tok_off[item];
  int c[4] = {0, 0, 0, 0};
  bool bad = false;
  for (int t = t0 + threadIdx.x; t < min(T, t0 + kPartBlock); t += 256) {
    const int s = tier_slot(b[t]);
    bad |= s < 0 && b[t] != 0;           // neither a stored tier nor 0 (evicted)
#pragma unroll
    for (int k = 0; k < 4; ++k) c[k] += (s == k);
  }
  if (bad) atomicOr(invalid, 1);
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

// exclusive scan of the block counts of one item: one wavefront per tier, 64 blocks per step
__global__ __launch_bounds__(256) void tier_scan_kernel(const int32_t* __restrict__ item_T,
                                                        const int32_t* __restrict__ item_blk_off,
                                                        int32_t* __restrict__ blk_counts,
                                                        int32_t* __restrict__ item_counts) {
  const int item = blockIdx.x, k = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nblk = (item_T[item] + kPartBlock - 1) / kPartBlock;
  int32_t* p = blk_counts + static_cast<int64_t>(item_blk_off[item]) * 4 + k;
  int run = 0;
  for (int b0 = 0; b0 < nblk; b0 += 64) {
    const int i = b0 + lane;
    const int v = i < nblk ? p[i * 4] : 0;
    int incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(incl, o);
      if (lane >= o) incl += t;
    }
    if (i < nblk) p[i * 4] = run + incl - v;
    run += __shfl(incl, 63);
  }
  if (lane == 0) item_counts[item * 4 + k] = run;
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
  int32_t v_only;              // mixed mode: K is packed channel-wise by pack_k_mixed_kernel
  const ItemK* items_k;        // [items] (mixed mode)
  const uint8_t* bits_ch;      // [items][128] (mixed mode)
  uint32_t* k_range;           // [items][128][2]: ordered-integer images of a channel's minimum and maximum over all
                               // retained tokens (one scale per channel, App. B), or null (groups of 32 tokens)
  int32_t row_wide;            // token rows: one scale and offset per row (App. B's per-token format), repeated in
                               // the row's four metadata slots, instead of one per group of 32 channels
};

// monotone map float -> uint32 (and back), so that integer atomic min / max order floats
__device__ __forceinline__ uint32_t float_to_ordered(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// 16-bit tier: the kept bf16 rows are copied verbatim, row-major (one thread = 64 bytes of K and of V)
__global__ __launch_bounds__(256) void copy_rows_kernel(PackArgs a) {
  const int item = blockIdx.y;
  const int n = a.counts[item * 4 + a.ti];
  const int row = blockIdx.x * 64 + (threadIdx.x >> 2);
  if (row >= n) return;
  const int part = threadIdx.x & 3;
  const int pos = a.tier_idx[a.idx_base[item * 4 + a.ti] + row];
  const int64_t src_row = a.item_row_off[item] + pos;
  const int64_t* so = a.seg_off + (static_cast<int64_t>(item) * 4 + a.ti) * 4;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const uint4* s4 = reinterpret_cast<const uint4*>((which == 0 ? a.K : a.V) + src_row * kHeadDim + part * 32);
    uint4* d4 = reinterpret_cast<uint4*>(a.arena + so[which * 2] + static_cast<int64_t>(row) * (kHeadDim * 2) + part * 64);
#pragma unroll
    for (int i = 0; i < 4; ++i) d4[i] = s4[i];
  }
}

// Tiers 8/4/2: one workgroup = one tile of 64 kept rows, K and V (mixed mode: V only, v_only set).
//
// Tile layout (what the decode kernel's 4x4x4 MFMA steps want).  A wavefront lane owns a run of 4*BITS 32-bit words,
// word W of lane L stored at byte 1024*(W/4) + 16*L + 4*(W%4).  The run holds four groups of BITS words; a group is
// read in eight steps of four codes: with F = 16/BITS fields per 16-bit half, step s reads field s % F of both
// halves of the word pair s / F, i.e. code k of step s sits at word 2*(s/F) + k/2, bit 16*(k%2) + BITS*(s%F).
//   K: lane = token r; group = c / 32; c % 32 = 4*step + k        (a lane holds one token's row)
//   V: lane = 32*(r/32) + c % 32; group = c / 32; r % 32 = 4*step + k   (a lane holds one channel for 32 tokens)
// Metadata tile = 1024 bytes: K row-major per token [4 scales][4 offsets]; V per block of 4 tokens 4 groups x 16
// bytes: the group's scales of the 4 tokens, then its offsets.
template <int BITS>
__global__ __launch_bounds__(256) void quant_pack_tile64_kernel(PackArgs a) {
  constexpr int kRows = 64;
  constexpr int kRowStride = kHeadDim + 8;                 // bf16 elements; 272-byte rows
  __shared__ __align__(16) uint16_t s_rows[2][kRows][kRowStride];
  __shared__ __align__(16) uint8_t s_codes[2][kRows][kHeadDim];
  const int item = blockIdx.y;
  const int n = a.counts[item * 4 + a.ti];
  const int r0 = blockIdx.x * kRows;
  if (r0 >= n) return;
  const int valid = min(kRows, n - r0);
  const int tid = threadIdx.x;
  const int64_t* so = a.seg_off + (static_cast<int64_t>(item) * 4 + a.ti) * 4;

  {  // gather the tile's rows: 4 threads per row, 64 bytes of K and of V each
    const int row = tid >> 2, part = tid & 3;
    uint4 kv[2][4];
#pragma unroll
    for (int w = 0; w < 2; ++w)
#pragma unroll
      for (int i = 0; i < 4; ++i) kv[w][i] = make_uint4(0, 0, 0, 0);
    if (row < valid) {
      const int pos = a.tier_idx[a.idx_base[item * 4 + a.ti] + r0 + row];
      const int64_t src = (a.item_row_off[item] + pos) * kHeadDim + part * 32;
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        const uint4* p = reinterpret_cast<const uint4*>((w == 0 ? a.K : a.V) + src);
#pragma unroll
        for (int i = 0; i < 4; ++i) kv[w][i] = p[i];
      }
    }
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      uint4* d = reinterpret_cast<uint4*>(&s_rows[w][row][part * 32]);
#pragma unroll
      for (int i = 0; i < 4; ++i) d[i] = kv[w][i];
    }
  }
  __syncthreads();

  // quantize: one task = one group of 32 channels of one row of K or V (fixed-order fp32); 512 tasks
  for (int task = tid; task < 2 * kRows * 4; task += 256) {
    const int w = task >> 8, row = (task >> 2) & 63, grp = task & 3;
    float x[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) x[i] = __uint_as_float(static_cast<uint32_t>(s_rows[w][row][grp * 32 + i]) << 16);
    float mn = x[0], mx = x[0];
#pragma unroll
    for (int i = 1; i < 32; ++i) {
      mn = fminf(mn, x[i]);
      mx = fmaxf(mx, x[i]);
    }
    if (a.row_wide) {   // the four groups of a row are the four lanes of a quad (task % 4 = lane % 4)
      mn = fminf(mn, __shfl_xor(mn, 1));
      mx = fmaxf(mx, __shfl_xor(mx, 1));
      mn = fminf(mn, __shfl_xor(mn, 2));
      mx = fmaxf(mx, __shfl_xor(mx, 2));
    }
    mn = mn + 0.0f;   // canonical +0
    constexpr float Q = static_cast<float>((1 << BITS) - 1);
    const _Float16 sh = static_cast<_Float16>((mx - mn) / Q);   // round to nearest even
    const _Float16 mh = static_cast<_Float16>(mn);
    const float s = static_cast<float>(sh), m = static_cast<float>(mh);
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      float t = rintf((x[i] - m) / s);
      t = fminf(fmaxf(t, 0.0f), Q);
      s_codes[w][row][grp * 32 + i] = (s == 0.0f) ? uint8_t(0) : static_cast<uint8_t>(t);
    }
    if (row < valid && !(a.v_only && w == 0)) {
      int si, oi;
      if (w == 0) {
        si = 8 * row + grp;
        oi = si + 4;
      } else {
        si = 32 * (row >> 2) + 8 * grp + (row & 3);
        oi = si + 4;
      }
      uint16_t* meta = reinterpret_cast<uint16_t*>(a.arena + so[w * 2 + 1] + static_cast<int64_t>(blockIdx.x) * 1024);
      meta[si] = __builtin_bit_cast(unsigned short, sh);
      meta[oi] = __builtin_bit_cast(unsigned short, mh);
    }
  }
  __syncthreads();

  // emit the tile's data words in their physical order (coalesced 32-bit stores)
  constexpr int kWords = kRows * kHeadDim * BITS / 32;      // 2048 / 1024 / 512
  constexpr int F = 16 / BITS;
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    if (a.v_only && w == 0) continue;
    uint32_t* dst = reinterpret_cast<uint32_t*>(a.arena + so[w * 2] +
                                                static_cast<int64_t>(blockIdx.x) * (kRows * kHeadDim * BITS / 8));
    for (int word = tid; word < kWords; word += 256) {
      const int chunk = word >> 8, lane = (word >> 2) & 63, dd = word & 3;
      const int W = 4 * chunk + dd;
      const int grp = W / BITS, wl = W % BITS;
      const int pair = wl >> 1, kw = wl & 1;
      uint32_t out = 0;
#pragma unroll
      for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int f = 0; f < F; ++f) {
          const int idx = 4 * (pair * F + f) + 2 * kw + half;      // position inside the group: 4*step + k
          int r, c;
          if (w == 0) {
            r = lane;
            c = 32 * grp + idx;
          } else {
            r = 32 * (lane >> 5) + idx;
            c = 32 * grp + (lane & 31);
          }
          out |= static_cast<uint32_t>(s_codes[w][r][c]) << (16 * half + BITS * f);
        }
      dst[word] = out;
    }
  }
}

// ---- mixed mode -------------------------------------------------------------------------------------------------
// 16-bit V rows as 64-token tiles with the lane assignment of the quantized V tiers: lane 32 (r / 32) + c % 32 holds
// channel c for the 32 tokens of its tile half, eight tokens per 16-byte unit; unit u = 4 (c / 32) + (r % 32) / 8
// sits at byte 1024 u + 16 lane of the 16 KiB tile.
__global__ __launch_bounds__(256) void pack_v16_tile64_kernel(PackArgs a) {
  constexpr int kRows = 64;
  constexpr int kRowStride = kHeadDim + 8;
  __shared__ __align__(16) uint16_t s_rows[kRows][kRowStride];
  const int item = blockIdx.y;
  const int n = a.counts[item * 4 + a.ti];
  const int r0 = blockIdx.x * kRows;
  if (r0 >= n) return;
  const int valid = min(kRows, n - r0);
  const int tid = threadIdx.x;
  const int64_t* so = a.seg_off + (static_cast<int64_t>(item) * 4 + a.ti) * 4;
  {
    const int row = tid >> 2, part = tid & 3;
    uint4 v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = make_uint4(0, 0, 0, 0);
    if (row < valid) {
      const int pos = a.tier_idx[a.idx_base[item * 4 + a.ti] + r0 + row];
      const uint4* p = reinterpret_cast<const uint4*>(a.V + (a.item_row_off[item] + pos) * kHeadDim + part * 32);
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = p[i];
    }
    uint4* d = reinterpret_cast<uint4*>(&s_rows[row][part * 32]);
#pragma unroll
    for (int i = 0; i < 4; ++i) d[i] = v[i];
  }
  __syncthreads();
  uint32_t* dst = reinterpret_cast<uint32_t*>(a.arena + so[2] + static_cast<int64_t>(blockIdx.x) * (kRows * kHeadDim * 2));
  for (int word = tid; word < kRows * kHeadDim / 2; word += 256) {
    const int u = word >> 8, lane = (word >> 2) & 63, t8 = 2 * (word & 3);
    const int r = 32 * (lane >> 5) + 8 * (u & 3) + t8, c = 32 * (u >> 2) + (lane & 31);
    dst[word] = s_rows[r][c] | (static_cast<uint32_t>(s_rows[r + 1][c]) << 16);
  }
}

// One scale per channel over all retained tokens (App. B): the channel's minimum and maximum over the kept rows of
// all four tiers of the item.  k_range starts at (0xFFFFFFFF, 0).
__global__ __launch_bounds__(256) void k_channel_range_kernel(PackArgs a) {
  __shared__ uint32_t s_mn[2][kHeadDim], s_mx[2][kHeadDim];
  const int item = blockIdx.y;
  const int64_t first = a.idx_base[item * 4];
  const int kept = a.counts[item * 4] + a.counts[item * 4 + 1] + a.counts[item * 4 + 2] + a.counts[item * 4 + 3];
  const int c = threadIdx.x & (kHeadDim - 1), sub = threadIdx.x >> 7;
  uint32_t mn = 0xFFFFFFFFu, mx = 0u;
  for (int r = blockIdx.x * 2 + sub; r < kept; r += gridDim.x * 2) {
    const int pos = a.tier_idx[first + r];
    const float x = __uint_as_float(static_cast<uint32_t>(a.K[(a.item_row_off[item] + pos) * kHeadDim + c]) << 16);
    const uint32_t k = float_to_ordered(x);
    mn = min(mn, k);
    mx = max(mx, k);
  }
  s_mn[sub][c] = mn;
  s_mx[sub][c] = mx;
  __syncthreads();
  if (sub == 0 && kept > 0) {
    atomicMin(&a.k_range[(static_cast<int64_t>(item) * kHeadDim + c) * 2], min(s_mn[0][c], s_mn[1][c]));
    atomicMax(&a.k_range[(static_cast<int64_t>(item) * kHeadDim + c) * 2 + 1], max(s_mx[0][c], s_mx[1][c]));
  }
}

// Channel-wise K of one 64-token tile (Sec. 3.2 Stage 3 on the retained tokens): every channel is quantized at
// its own bit-width over each half of the tile (one group = 32 consecutive retained tokens of one channel) and the
// codes are written in sorted-channel order.  Token r of the tile owns n_words_padded 32-bit words: word W at byte
// 1024 (W / 4) + 16 r + 4 (W % 4), the last two words of a row whose word count is not a multiple of four at
// 1024 (n / 4) + 8 r + 4 (W % 2).  Inside a word, slot 4k + e of a b-bit tier sits at bit
// 16 (e % 2) + b (e / 2) + 2 b k; a 16-bit word holds its two slots in its halves.
// Metadata: per token group G and quantized step sq (4 slots) 4 fp16 scales then 4 fp16 offsets at fp16 index
// 8 (G n_qsteps + sq).
__global__ __launch_bounds__(256) void pack_k_mixed_kernel(PackArgs a) {
  constexpr int kRows = 64;
  constexpr int kRowStride = kHeadDim + 8;
  __shared__ __align__(16) uint16_t s_rows[kRows][kRowStride];
  __shared__ uint16_t s_codes[kRows][kHeadDim + 2];
  __shared__ uint16_t s_sc[2][kHeadDim], s_of[2][kHeadDim];
  __shared__ ItemK s_ik;
  const int item = blockIdx.y;
  const int n = a.counts[item * 4 + a.ti];
  const int r0 = blockIdx.x * kRows;
  if (r0 >= n) return;
  const int valid = min(kRows, n - r0);
  const int tid = threadIdx.x;
  const int64_t* so = a.seg_off + (static_cast<int64_t>(item) * 4 + a.ti) * 4;
  for (int i = tid; i < static_cast<int>(sizeof(ItemK) / 4); i += 256)
    reinterpret_cast<uint32_t*>(&s_ik)[i] = reinterpret_cast<const uint32_t*>(a.items_k + item)[i];
  {
    const int row = tid >> 2, part = tid & 3;
    uint4 v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = make_uint4(0, 0, 0, 0);
    if (row < valid) {
      const int pos = a.tier_idx[a.idx_base[item * 4 + a.ti] + r0 + row];
      const uint4* p = reinterpret_cast<const uint4*>(a.K + (a.item_row_off[item] + pos) * kHeadDim + part * 32);
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = p[i];
    }
    uint4* d = reinterpret_cast<uint4*>(&s_rows[row][part * 32]);
#pragma unroll
    for (int i = 0; i < 4; ++i) d[i] = v[i];
  }
  __syncthreads();
  {  // one thread = one (token group, channel)
    const int G = tid >> 7, c = tid & 127;
    const int rb = kKTokenGroup * G, vg = min(max(valid - rb, 0), kKTokenGroup);
    const int b = a.bits_ch[item * kHeadDim + c];
    uint16_t sc = 0, of = 0;
    if (b == 16) {
      for (int r = 0; r < kKTokenGroup; ++r) s_codes[rb + r][c] = s_rows[rb + r][c];   // rows beyond `valid` are zero
    } else if ((b == 8 || b == 4 || b == 2) && vg > 0) {
      float mn, mx;
      if (a.k_range) {   // the range of the whole unit
        mn = ordered_to_float(a.k_range[(static_cast<int64_t>(item) * kHeadDim + c) * 2]);
        mx = ordered_to_float(a.k_range[(static_cast<int64_t>(item) * kHeadDim + c) * 2 + 1]);
      } else {
        mn = __uint_as_float(static_cast<uint32_t>(s_rows[rb][c]) << 16);
        mx = mn;
        for (int r = 1; r < vg; ++r) {
          const float x = __uint_as_float(static_cast<uint32_t>(s_rows[rb + r][c]) << 16);
          mn = fminf(mn, x);
          mx = fmaxf(mx, x);
        }
      }
      mn = mn + 0.0f;
      const float Q = static_cast<float>((1 << b) - 1);
      const _Float16 sh = static_cast<_Float16>((mx - mn) / Q);
      const _Float16 mh = static_cast<_Float16>(mn);
      const float s = static_cast<float>(sh), m = static_cast<float>(mh);
      for (int r = 0; r < kKTokenGroup; ++r) {
        const float x = __uint_as_float(static_cast<uint32_t>(s_rows[rb + r][c]) << 16);
        float t = rintf((x - m) / s);
        t = fminf(fmaxf(t, 0.0f), Q);
        s_codes[rb + r][c] = (s == 0.0f || r >= vg) ? uint16_t(0) : static_cast<uint16_t>(t);
      }
      sc = __builtin_bit_cast(unsigned short, sh);
      of = __builtin_bit_cast(unsigned short, mh);
    } else {
      for (int r = 0; r < kKTokenGroup; ++r) s_codes[rb + r][c] = 0;
    }
    s_sc[G][c] = sc;
    s_of[G][c] = of;
  }
  __syncthreads();

  const int nwp = s_ik.n_words_padded, full = nwp & ~3;
  uint32_t* dst = reinterpret_cast<uint32_t*>(a.arena + so[0] + static_cast<int64_t>(blockIdx.x) * s_ik.kt_bytes);
  for (int idx = tid; idx < kRows * nwp; idx += 256) {
    int W, r;
    if (idx < kRows * full) {
      W = 4 * (idx >> 8) + (idx & 3);
      r = (idx >> 2) & 63;
    } else {
      W = full + (idx & 1);
      r = (idx - kRows * full) >> 1;
    }
    uint32_t out = 0;
    if (W < s_ik.n_words) {
      int t = 0;
      while (W >= s_ik.word_end[t]) ++t;
      const int b = 16 >> t, per_word = 32 / b;
      const int lw = W - (t > 0 ? s_ik.word_end[t - 1] : 0);
      const int16_t* sl = s_ik.slot_ch + s_ik.slot_base[t] + lw * per_word;
      for (int jj = 0; jj < per_word; ++jj) {
        const int c = sl[jj];
        if (c < 0) continue;
        const int k = jj >> 2, e = jj & 3;
        const int bit = b == 16 ? 16 * jj : 16 * (e & 1) + b * (e >> 1) + 2 * b * k;
        out |= static_cast<uint32_t>(s_codes[r][c]) << bit;
      }
    }
    dst[idx] = out;
  }
  const int nqs = s_ik.n_qsteps;
  if (a.k_range) {   // one record for the whole segment, written by its first tile
    if (blockIdx.x == 0) {
      uint16_t* meta1 = reinterpret_cast<uint16_t*>(a.arena + so[1]);
      for (int idx = tid; idx < 8 * nqs; idx += 256) {
        const int sq = idx >> 3, e = idx & 3, is_off = (idx >> 2) & 1;
        const int c = s_ik.slot_ch[s_ik.slot_base[1] + 4 * sq + e];
        meta1[idx] = c >= 0 ? (is_off ? s_of[0][c] : s_sc[0][c]) : uint16_t(0);
      }
    }
    return;
  }
  uint16_t* meta = reinterpret_cast<uint16_t*>(a.arena + so[1] + static_cast<int64_t>(blockIdx.x) * s_ik.km_bytes);
  for (int idx = tid; idx < 16 * nqs; idx += 256) {
    const int G = idx / (8 * nqs), rem = idx - G * 8 * nqs;
    const int sq = rem >> 3, e = rem & 3, is_off = (rem >> 2) & 1;
    const int c = s_ik.slot_ch[s_ik.slot_base[1] + 4 * sq + e];
    meta[idx] = c >= 0 ? (is_off ? s_of[G][c] : s_sc[G][c]) : uint16_t(0);
  }
}

}  // namespace

hipError_t launch_tier_count(const uint8_t* bits, const int64_t* item_tok_off, const int32_t* item_T,
                             const int32_t* item_blk_off, int32_t* blk_counts, int32_t* item_counts,
                             int32_t* invalid, int n_items, int max_T, hipStream_t st) {
  const int max_blk = (max_T + kPartBlock - 1) / kPartBlock;
  if (n_items == 0 || max_blk == 0) return hipSuccess;
  // `invalid` (zero on entry) is set when the map holds a value that is no bit-width of the method
  hipLaunchKernelGGL(tier_count_kernel, dim3(max_blk, n_items), dim3(256), 0, st, bits, item_tok_off, item_T,
                     item_blk_off, blk_counts, invalid);
  hipLaunchKernelGGL(tier_scan_kernel, dim3(n_items), dim3(256), 0, st, item_T, item_blk_off, blk_counts,
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
                             const int32_t max_count[4], const ItemK* items_k, const uint8_t* bits_ch,
                             uint32_t* k_range, int row_wide, hipStream_t st) {
  const bool mixed = items_k != nullptr;
  if (k_range) {   // k_range must hold (0xFFFFFFFF, 0) pairs on entry
    PackArgs a{K, V, tier_idx, idx_base, counts, seg_off, item_row_off, arena, 0, 1, items_k, bits_ch, k_range,
               row_wide};
    hipLaunchKernelGGL(k_channel_range_kernel, dim3(64, n_items), dim3(256), 0, st, a);
  }
  for (int ti = 0; ti < 4; ++ti) {
    if (max_count[ti] == 0) continue;
    PackArgs a{K, V, tier_idx, idx_base, counts, seg_off, item_row_off, arena, ti, mixed ? 1 : 0, items_k, bits_ch,
               k_range, row_wide};
    dim3 grid64((max_count[ti] + 63) / 64, n_items);   // 64 rows per workgroup in every kernel below
    dim3 block(256);
    if (mixed) hipLaunchKernelGGL(pack_k_mixed_kernel, grid64, block, 0, st, a);
    switch (ti) {
      case 0:
        if (mixed) hipLaunchKernelGGL(pack_v16_tile64_kernel, grid64, block, 0, st, a);
        else hipLaunchKernelGGL(copy_rows_kernel, grid64, block, 0, st, a);
        break;
      case 1: hipLaunchKernelGGL(quant_pack_tile64_kernel<8>, grid64, block, 0, st, a); break;
      case 2: hipLaunchKernelGGL(quant_pack_tile64_kernel<4>, grid64, block, 0, st, a); break;
      default: hipLaunchKernelGGL(quant_pack_tile64_kernel<2>, grid64, block, 0, st, a); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

int partition_block() { return kPartBlock; }

}  // namespace rdkv
