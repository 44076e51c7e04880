// Device helpers shared by the tile decode kernels (token-wise and mixed mode): operand types, the subnormal-fp16
// unpack of packed codes, tile loads, and the stages both kernels run after the logits of a 64-token tile are
// known: online softmax, P V over a token-wise V tile, and the end-of-chunk merge of a workgroup's wavefronts.
//
// Lane roles (v_mfma_f32_4x4x4_16B_f16, sixteen independent 4x4x4 blocks, lane = 4 * block + x):
//   logits    lane (block b, x = head j) holds tokens 4b..4b+3 of the tile in its four result registers
//   P V       A = p * scale of lane (b, head j) for its tokens, broadcast from block a to blocks 0..7 and from
//             block 8 + a to blocks 8..15 (cbsz = 3);  B = V codes: lane = (token half, channel of the group),
//             4 tokens per step;  D: lane holds 4 heads of one channel, summed over its token half.
#pragma once
#include "decode_merge.h"
#include "rdkv_internal.h"

namespace rdkv {
namespace tile {

typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kTile = 64;   // tokens per tile
constexpr float kNegBig = -1.0e30f;
constexpr float kLogitScale = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)

// Codes enter the matrix cores as fp16 subnormals: a 16-bit pattern with a zero exponent field and the code in
// mantissa bits [fb, fb + b) is the number code * 2^fb * 2^-24 exactly, so one AND per pair of codes is the whole
// conversion.  The query operand of the K product is pre-multiplied by 2^(kQExp - fb); on the V side the power of
// two goes into p (per lane) and the accumulators are rescaled once per chunk.
constexpr int kQExp = 4;                                   // keeps the scaled query clear of fp16 underflow
constexpr float kKUnit = 1.0f / static_cast<float>(1 << (24 - kQExp));   // K partial products come out times this
constexpr float kXScale = kLogitScale * static_cast<float>(1 << (24 - kQExp));

// The probabilities exp2(x - running maximum) are carried times 2^kPExp, so that after the multiplication by a
// V scale they stay in fp16's normal range for flat attention over tens of thousands of tokens (p ~ 1e-5); the
// factor is returned by reporting the running maximum kPExp lower to the merge.  2^kPExp * scale must stay below
// 65504, which holds for V scales below 1023.
constexpr float kPExp = 6.0f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef short short4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

// four bf16 of an operand from two 32-bit words (a bit cast: a union of the two types is left in scratch memory)
__device__ __forceinline__ short4v bf4(uint32_t lo, uint32_t hi) { return __builtin_bit_cast(short4v, uint2v{lo, hi}); }

// the probabilities of a lane's four tokens as two truncated bf16 terms (the remainder of the first is exact in fp32)
__device__ __forceinline__ void split_bf16(const float (&p)[4], short4v& hi, short4v& lo) {
  uint32_t hb[4], lb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    hb[i] = __float_as_uint(p[i]) & 0xFFFF0000u;
    lb[i] = __float_as_uint(p[i] - __uint_as_float(hb[i]));
  }
  hi = bf4((hb[0] >> 16) | hb[1], (hb[2] >> 16) | hb[3]);
  lo = bf4((lb[0] >> 16) | (lb[1] & 0xFFFF0000u), (lb[2] >> 16) | (lb[3] & 0xFFFF0000u));
}

union Pack4 {
  half4 h;
  half2v p[2];
  uint32_t u[2];
};

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, dpp_u32<CTRL>(__builtin_bit_cast(uint32_t, v)));
}
// reduction over the 16 lanes that hold the same head (lane % 4): lanes 4 apart inside a row of 16, then the rows
__device__ __forceinline__ float head_max(float v) {
  v = fmaxf(v, dpp_f32<0x124>(v));   // row_ror:4
  v = fmaxf(v, dpp_f32<0x128>(v));   // row_ror:8
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}
__device__ __forceinline__ float head_sum(float v) {
  v += dpp_f32<0x124>(v);
  v += dpp_f32<0x128>(v);
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}
// value held by lane i of this lane's quad
template <int I>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t v) { return dpp_u32<I * 0x55>(v); }

// Field position of step s inside a 16-bit half, which right-shifted copy of the word it is read from, and the bit
// offset that remains after that shift (the code then reads as code * 2^fb * 2^-24).
template <int TIER>
struct Step {
  static constexpr int F = 16 / TIER;                                     // fields per half
  __host__ __device__ static constexpr int pair(int s) { return s / F; }
  __host__ __device__ static constexpr int field(int s) { return s % F; }
  __host__ __device__ static constexpr int copy(int s) {
    return TIER == 8 ? 0 : TIER == 4 ? field(s) / 2 : field(s) / 3;
  }
  __host__ __device__ static constexpr int fb(int s) {
    return TIER == 8 ? 0 : TIER == 4 ? 4 * (field(s) % 2) : 2 * (field(s) % 3);
  }
  static constexpr int kCopies = TIER == 8 ? 1 : TIER == 4 ? 2 : 3;
  static constexpr int kShift = TIER == 4 ? 8 : 6;                        // right shift between copies
};

// The 4 codes of step s of a group whose words are gw[0..TIER): two words, fp16 subnormals in both halves.
template <int TIER>
__device__ __forceinline__ half4 step_operand(const uint32_t (&gw)[Step<TIER>::kCopies][TIER], int s) {
  using S = Step<TIER>;
  Pack4 r;
  const int p = S::pair(s);
  if constexpr (TIER == 8) {
    // byte f of each half, zero-extended: both selections go through the byte permute (mixing it with a plain
    // AND of the same register was seen to be scheduled with the AND done in place before the permute read it)
    const uint32_t sel = S::field(s) ? 0x0C030C01u : 0x0C020C00u;
    r.u[0] = __builtin_amdgcn_perm(0u, gw[0][2 * p], sel);
    r.u[1] = __builtin_amdgcn_perm(0u, gw[0][2 * p + 1], sel);
  } else {
    const uint32_t mask = (TIER == 4 ? 0x000F000Fu : 0x00030003u) << S::fb(s);
    r.u[0] = gw[S::copy(s)][2 * p] & mask;
    r.u[1] = gw[S::copy(s)][2 * p + 1] & mask;
  }
  return r.h;
}

template <int TIER>
__device__ __forceinline__ void group_words(const uint4 (&raw)[TIER], int grp, uint32_t (&gw)[Step<TIER>::kCopies][TIER]) {
  using S = Step<TIER>;
#pragma unroll
  for (int w = 0; w < TIER; ++w) {
    const int W = grp * TIER + w;
    const uint4 c = raw[W >> 2];
    const uint32_t v = (W & 3) == 0 ? c.x : (W & 3) == 1 ? c.y : (W & 3) == 2 ? c.z : c.w;
    gw[0][w] = v;
#pragma unroll
    for (int k = 1; k < S::kCopies; ++k) gw[k][w] = v >> (k * S::kShift);
  }
}

template <int TIER>
__device__ __forceinline__ void load_tile_side(uint4 (&raw)[TIER], const uint8_t* __restrict__ data, int tile, int lane) {
  const uint8_t* p = data + static_cast<int64_t>(tile) * (kTile * 16 * TIER) + lane * 16;
#pragma unroll
  for (int i = 0; i < TIER; ++i) raw[i] = *reinterpret_cast<const uint4*>(p + i * 1024);
}

__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Running state of one wavefront over its tiles of a chunk: per head set the running maximum and sum of the
// online softmax (lanes of head j; the sum carries this lane's factor kappa), the output accumulators
// acc[hs][grp][i] (head 4 hs + i, channel 32 grp + lane % 32, summed over this lane's token half), and the offset
// sums offv[hs][i] = kappa * sum_t p m of head 4 hs + i and channel group lane % 4 over the tokens of this lane's block.
template <int HS>
struct Run {
  float m[HS], l[HS];
  floatx4 acc[HS][4];
  floatx4 offv[HS];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int hs = 0; hs < HS; ++hs) {
      m[hs] = kNegBig;
      l[hs] = 0.f;
      offv[hs] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int grp = 0; grp < 4; ++grp) acc[hs][grp] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
  }
};

// Padded rows of a chunk's last tile take no part in the softmax.
template <int HS>
__device__ __forceinline__ void mask_rows(float (&x)[HS][4], int tile, int rows, int blk) {
  if ((tile + 1) * kTile > rows) {
#pragma unroll
    for (int hs = 0; hs < HS; ++hs)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (tile * kTile + 4 * blk + i >= rows) x[hs][i] = -INFINITY;
  }
}

// Online softmax per head over the logits x (in units of 1 / kXScale) of a tile; probabilities carried times
// 2^(kPExp + lk): lk = log2 of the lane's factor kappa on the V side (0 where there is none), which the exponential
// applies for free; the running sum carries the same factor and finish_chunk takes it out again.
template <int HS>
__device__ __forceinline__ void softmax_tile(const float (&x)[HS][4], Run<HS>& run, float (&p)[HS][4], float lk = 0.f) {
#pragma unroll
  for (int hs = 0; hs < HS; ++hs) {
    const float mt = head_max(fmaxf(fmaxf(x[hs][0], x[hs][1]), fmaxf(x[hs][2], x[hs][3])));
    const float m_new = fmaxf(run.m[hs], mt);
    if (__any(m_new != run.m[hs])) {
      const float alpha = fast_exp2((run.m[hs] - m_new) * kXScale);
      run.l[hs] *= alpha;
      const uint32_t au = __builtin_bit_cast(uint32_t, alpha);
      const float ah[4] = {__builtin_bit_cast(float, quad_bcast<0>(au)), __builtin_bit_cast(float, quad_bcast<1>(au)),
                           __builtin_bit_cast(float, quad_bcast<2>(au)), __builtin_bit_cast(float, quad_bcast<3>(au))};
#pragma unroll
      for (int i = 0; i < 4; ++i) {   // row i of the accumulators is head i
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) run.acc[hs][grp][i] *= ah[i];
        run.offv[hs][i] *= ah[i];
      }
      run.m[hs] = m_new;
    }
    const float neg_mc = (kPExp + lk) - run.m[hs] * kXScale;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      p[hs][i] = fast_exp2(__builtin_fmaf(x[hs][i], kXScale, neg_mc));
      run.l[hs] += p[hs][i];
    }
  }
}

// log2 of kappa = 2^-fb of the field this lane's block is read from on the V side (block a = blk % 8 feeds step a)
template <int TIER>
__device__ __forceinline__ float v_log2_kappa(int blk) {
  float lk = 0.0f;
#pragma unroll
  for (int a = 0; a < 8; ++a)
    if ((blk & 7) == a) lk = -static_cast<float>(Step<TIER>::fb(a));
  return lk;
}

template <int G>
struct GroupIndex {
  static constexpr int value = G;
};

// P V over a token-wise V tile of tier TIER (8, 4, 2).  fill_gw(GroupIndex<G>, gw) delivers the code words of
// channel group G (and their shifted copies); vmeta = group (lane % 4)'s scales (x, y) and offsets (z, w) of
// tokens 4 blk + 0..3; p = the probabilities times the lane's kappa (softmax_tile with lk).
// The offsets go through one more product: A = p (4 heads x the block's 4 tokens), B = this lane's offsets (4 tokens
// of channel group lane % 4), so that lane (block, j) gathers sum_t p m of the four heads for group j -- with the
// same rounded p that multiplies the codes, which keeps the two halves of sum_t p (s code + m) consistent.
template <int TIER, int HS, class FillGw>
__device__ __forceinline__ void pv_tile_groups(FillGw&& fill_gw, const uint4& vmeta, const float (&p)[HS][4],
                                               Run<HS>& run) {
  using S = Step<TIER>;
  Pack4 ph[HS], ob;
  ob.u[0] = vmeta.z;
  ob.u[1] = vmeta.w;
#pragma unroll
  for (int hs = 0; hs < HS; ++hs) {
    ph[hs].p[0] = half2v{static_cast<_Float16>(p[hs][0]), static_cast<_Float16>(p[hs][1])};
    ph[hs].p[1] = half2v{static_cast<_Float16>(p[hs][2]), static_cast<_Float16>(p[hs][3])};
    run.offv[hs] = __builtin_amdgcn_mfma_f32_4x4x4f16(ph[hs].h, ob.h, run.offv[hs], 0, 0, 0);
  }
#define RDKV_PV_GROUP(G_)                                                                                      \
  {                                                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                                         \
    /* V scales of tokens 4 blk + 0..3: lane G_ of the quad holds group G_'s (x, y) */                         \
    Pack4 sv, pa[HS];                                                                                          \
    sv.u[0] = quad_bcast<G_>(vmeta.x); sv.u[1] = quad_bcast<G_>(vmeta.y);                                      \
    _Pragma("unroll") for (int hs = 0; hs < HS; ++hs) {                                                        \
      pa[hs].p[0] = ph[hs].p[0] * sv.p[0];                                                                     \
      pa[hs].p[1] = ph[hs].p[1] * sv.p[1];                                                                     \
    }                                                                                                          \
    uint32_t gw[S::kCopies][TIER];                                                                             \
    fill_gw(GroupIndex<G_>{}, gw);                                                                             \
    RDKV_PV_STEP(G_, 0) RDKV_PV_STEP(G_, 1) RDKV_PV_STEP(G_, 2) RDKV_PV_STEP(G_, 3)                            \
    RDKV_PV_STEP(G_, 4) RDKV_PV_STEP(G_, 5) RDKV_PV_STEP(G_, 6) RDKV_PV_STEP(G_, 7)                            \
  }
#define RDKV_PV_STEP(G_, A_)                                                                                   \
  {                                                                                                            \
    const half4 b = step_operand<TIER>(gw, A_);                                                                \
    _Pragma("unroll") for (int hs = 0; hs < HS; ++hs)                                                          \
        run.acc[hs][G_] = __builtin_amdgcn_mfma_f32_4x4x4f16(pa[hs].h, b, run.acc[hs][G_], 3, A_, 0);          \
  }
  RDKV_PV_GROUP(0) RDKV_PV_GROUP(1) RDKV_PV_GROUP(2) RDKV_PV_GROUP(3)
#undef RDKV_PV_STEP
#undef RDKV_PV_GROUP
}

// the same with the whole tile's code words in registers
template <int TIER, int HS>
__device__ __forceinline__ void pv_tile(const uint4 (&vraw)[TIER], const uint4& vmeta, const float (&p)[HS][4],
                                        Run<HS>& run) {
  pv_tile_groups<TIER, HS>(
      [&](auto gi, uint32_t (&gw)[Step<TIER>::kCopies][TIER]) __attribute__((always_inline)) {
        group_words<TIER>(vraw, decltype(gi)::value, gw);
      },
      vmeta, p, run);
}

// Where a chunk's partial result goes and what the merge of its item needs.
struct ChunkOut {
  int item, slot, slot0, nslots;   // the chunk's item and partial slot; the item's first slot and slot count
};

// End of a chunk: scale the accumulators back (acc_scale = 2^24 where the V codes entered as fp16 subnormals),
// take the lane's factor kappa = 2^lk out of the running sums, add the offset sums, merge the workgroup's NWV
// wavefronts through LDS, store the chunk's partial result and announce it; the workgroup that completes its item
// merges the item's partials (arrive_and_merge).
// s_ml: [NWV][4 HS heads][m, l] floats; s_acc: [2 NWV streams][g][128] floats (also the merge's LDS).  ALIAS: the
// two areas overlap LDS that the tile loop used, so a barrier separates the two uses.
template <int HS, bool ALIAS, int NWV>
__device__ __forceinline__ void finish_chunk(Run<HS>& run, float acc_scale, float lk, int g, float* s_ml,
                                             float* s_acc, const MergeArgs& ma, const ChunkOut& co) {
  constexpr int NT = NWV * 64;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int th = lane >> 5, cl = lane & 31;
  float* __restrict__ part_acc = ma.part_acc + static_cast<int64_t>(co.slot) * g * kHeadDim;
  float* __restrict__ part_ml = ma.part_ml + static_cast<int64_t>(co.slot) * g * 2;
  const float inv_kappa = __builtin_ldexpf(1.0f, static_cast<int>(-lk));   // lk is a small integer
#pragma unroll
  for (int hs = 0; hs < HS; ++hs) {
    run.l[hs] = head_sum(run.l[hs] * inv_kappa);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // lanes (block, j) hold head i's sum_t p m of channel group j over the block's tokens: all blocks, then to the
      // lanes of every group
      const uint32_t ou = __builtin_bit_cast(uint32_t, head_sum(run.offv[hs][i] * inv_kappa));
      const float og[4] = {__builtin_bit_cast(float, quad_bcast<0>(ou)), __builtin_bit_cast(float, quad_bcast<1>(ou)),
                           __builtin_bit_cast(float, quad_bcast<2>(ou)), __builtin_bit_cast(float, quad_bcast<3>(ou))};
#pragma unroll
      for (int grp = 0; grp < 4; ++grp)
        run.acc[hs][grp][i] = __builtin_fmaf(run.acc[hs][grp][i], acc_scale, th == 0 ? og[grp] : 0.f);
    }
  }
  if constexpr (ALIAS) __syncthreads();
#pragma unroll
  for (int hs = 0; hs < HS; ++hs)
    if (lane < 4) {
      s_ml[((wave * HS + hs) * 4 + lane) * 2] = run.m[hs] * kXScale - kPExp;   // log2 domain from here on
      s_ml[((wave * HS + hs) * 4 + lane) * 2 + 1] = run.l[hs];
    }
  __syncthreads();
#pragma unroll
  for (int hs = 0; hs < HS; ++hs)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int head = 4 * hs + i;
      float mm = kNegBig;
#pragma unroll
      for (int w = 0; w < NWV; ++w) mm = fmaxf(mm, s_ml[((w * HS + hs) * 4 + i) * 2]);
      const float f = fast_exp2(s_ml[((wave * HS + hs) * 4 + i) * 2] - mm);
      if (head < g) {
#pragma unroll
        for (int grp = 0; grp < 4; ++grp)
          s_acc[((wave * 2 + th) * g + head) * kHeadDim + 32 * grp + cl] = run.acc[hs][grp][i] * f;
      }
    }
  __syncthreads();
  for (int idx = tid; idx < g * kHeadDim; idx += NT) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < 2 * NWV; ++w) v += s_acc[w * g * kHeadDim + idx];
    merge::store_agent(part_acc + idx, v);
  }
  if (tid < g) {
    const int hs = tid >> 2, i = tid & 3;
    float mm = kNegBig;
#pragma unroll
    for (int w = 0; w < NWV; ++w) mm = fmaxf(mm, s_ml[((w * HS + hs) * 4 + i) * 2]);
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < NWV; ++w)
      ll += s_ml[((w * HS + hs) * 4 + i) * 2 + 1] * fast_exp2(s_ml[((w * HS + hs) * 4 + i) * 2] - mm);
    merge::store_agent(part_ml + tid * 2, mm);
    merge::store_agent(part_ml + tid * 2 + 1, ll);
  }
  merge::partial_stores_done();
  __syncthreads();     // every partial store has landed, and nobody reads s_ml / s_acc any more
  merge::arrive_and_merge<NT, 4 * HS>(ma, co.item, co.slot0, co.nslots, g, s_acc);
}

// A chunk of appended tokens (Sec. 3.3 Zone C: bf16 rows kept after the compression pass) on the same instruction
// and lane roles.  The tail is stored in 64-token tiles written by the append kernel: K tile = 16 KiB, word W (two
// bf16 channels 2W, 2W+1) of token r at byte 1024 (W / 4) + 16 r + 4 (W % 4), so a lane (= token) reads its row
// with sixteen coalesced 16-byte loads; V tile = 16 KiB in the layout of the 16-bit V tiles of mixed mode (lane
// 32 (r / 32) + c % 32 holds channel c, eight tokens per 16-byte unit u = 4 (c / 32) + (r % 32) / 8 at 1024 u).
// s_q: LDS for the query operands, [32 steps][HS][4 heads] x 8 bytes (raw bf16; the products are exact).
template <int HS, bool ALIAS, int NWV>
__device__ __forceinline__ void process_tail_tiles(const uint8_t* __restrict__ kd, const uint8_t* __restrict__ vd,
                                                   int rows, int g, const uint16_t* __restrict__ q, uint8_t* s_q,
                                                   float* s_ml, float* s_acc, const MergeArgs& ma,
                                                   const ChunkOut& co) {
  constexpr int kWG = NWV * 64, kWaves = NWV;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int blk = lane >> 2, j = lane & 3;
  const int ntiles = (rows + kTile - 1) / kTile;
  constexpr int kTileBytes = kTile * kHeadDim * 2;
  for (int e = tid; e < 32 * HS * 4; e += kWG) {
    const int s = e / (HS * 4), hs = (e >> 2) % HS, hj = e & 3;
    const int head = 4 * hs + hj;
    uint2 v = make_uint2(0, 0);
    if (head < g) v = *reinterpret_cast<const uint2*>(q + head * kHeadDim + 4 * s);
    *reinterpret_cast<uint2*>(s_q + ((s * HS + hs) * 4 + hj) * 8) = v;
  }
  __syncthreads();
  Run<HS> run;
  run.init();
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};
  for (int tile = wave; tile < ntiles; tile += kWaves) {
    const uint8_t* kp = kd + static_cast<int64_t>(tile) * kTileBytes + 16 * lane;
    const uint8_t* vp = vd + static_cast<int64_t>(tile) * kTileBytes + 16 * lane;
    uint4 kq[16], vq[3][4];   // the K row and the first channel group of V in one round trip
#pragma unroll
    for (int i = 0; i < 16; ++i) kq[i] = *reinterpret_cast<const uint4*>(kp + 1024 * i);
#pragma unroll
    for (int i = 0; i < 4; ++i) vq[0][i] = *reinterpret_cast<const uint4*>(vp + 1024 * i);
    floatx4 a16[HS];
#pragma unroll
    for (int hs = 0; hs < HS; ++hs) a16[hs] = zero4;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int s = 2 * i + half;   // step s = channels 4s .. 4s+3 = words 2s, 2s+1
        const short4v a = half ? bf4(kq[i].z, kq[i].w) : bf4(kq[i].x, kq[i].y);
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) {
          const uint2 braw = *reinterpret_cast<const uint2*>(s_q + ((s * HS + hs) * 4 + j) * 8);
          a16[hs] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, bf4(braw.x, braw.y), a16[hs], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);   // the K registers are free: the other three channel groups of V
#pragma unroll
    for (int i = 0; i < 4; ++i) vq[1][i] = *reinterpret_cast<const uint4*>(vp + 1024 * (4 + i));
#pragma unroll
    for (int i = 0; i < 4; ++i) vq[2][i] = *reinterpret_cast<const uint4*>(vp + 1024 * (8 + i));
    float x[HS][4];
#pragma unroll
    for (int hs = 0; hs < HS; ++hs)
#pragma unroll
      for (int i = 0; i < 4; ++i) x[hs][i] = a16[hs][i] * kKUnit;
    mask_rows<HS>(x, tile, rows, blk);
    float p[HS][4];
    softmax_tile<HS>(x, run, p);
    short4v phi[HS], plo[HS];
#pragma unroll
    for (int hs = 0; hs < HS; ++hs) split_bf16(p[hs], phi[hs], plo[hs]);
    // P V: step a of a channel group = tokens 4a..4a+3 of this lane's token half (rows past the end are zero in the
    // tile and carry p = 0)
#define RDKV_TAIL_STEP(G_, A_, X_, Y_)                                                                          \
  {                                                                                                            \
    const short4v b = bf4(X_, Y_);                                                                             \
    _Pragma("unroll") for (int hs = 0; hs < HS; ++hs) {                                                        \
      run.acc[hs][G_] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(phi[hs], b, run.acc[hs][G_], 3, A_, 0);         \
      run.acc[hs][G_] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(plo[hs], b, run.acc[hs][G_], 3, A_, 0);         \
    }                                                                                                          \
  }
#define RDKV_TAIL_GROUP(G_, V_)                                                                                \
  RDKV_TAIL_STEP(G_, 0, V_[0].x, V_[0].y) RDKV_TAIL_STEP(G_, 1, V_[0].z, V_[0].w)                              \
  RDKV_TAIL_STEP(G_, 2, V_[1].x, V_[1].y) RDKV_TAIL_STEP(G_, 3, V_[1].z, V_[1].w)                              \
  RDKV_TAIL_STEP(G_, 4, V_[2].x, V_[2].y) RDKV_TAIL_STEP(G_, 5, V_[2].z, V_[2].w)                              \
  RDKV_TAIL_STEP(G_, 6, V_[3].x, V_[3].y) RDKV_TAIL_STEP(G_, 7, V_[3].z, V_[3].w)
    RDKV_TAIL_GROUP(0, vq[0])
#pragma unroll
    for (int i = 0; i < 4; ++i) vq[0][i] = *reinterpret_cast<const uint4*>(vp + 1024 * (12 + i));   // group 3
    RDKV_TAIL_GROUP(1, vq[1])
    RDKV_TAIL_GROUP(2, vq[2])
    RDKV_TAIL_GROUP(3, vq[0])
#undef RDKV_TAIL_GROUP
#undef RDKV_TAIL_STEP
  }
  finish_chunk<HS, ALIAS, NWV>(run, 1.0f, 0.f, g, s_ml, s_acc, ma, co);
}

}  // namespace tile
}  // namespace rdkv
