// Split-K flash-decode over the quantized tiers (8/4/2 bit) of a token-wise cache (Sec. 3.3, Eq. 7) on the
// gfx950 matrix cores.
//
// With grouped-query attention the query heads of a KV head share every K/V byte.  The products run on
// v_mfma_f32_4x4x4_16B_f16: sixteen independent 4x4x4 blocks per instruction, four query heads on one side, so
// that no lane of the result is padding (a 16-wide head dimension would be three quarters empty at g = 4 and
// the plain ALUs, which apply the scales and the softmax to every result lane, are the scarce unit).
//
//   q K^T   A = K codes: lane = token (64 per tile), 4 channels per step;  B = the query, 4 heads x 4 channels,
//           the same in every block;  D: lane (block b, head j) holds tokens 4b..4b+3.  Eight steps cover a
//           quantization group of 32 channels; the group's scale multiplies the partial product (fusion identity
//           of App. B) and the offsets go through one more product with the group sums of q.
//   P V     A = p * scale of lane (b, head j) for its tokens 4b..4b+3, broadcast from block a to blocks 0..7 and
//           from block 8 + a to blocks 8..15 (cbsz = 3);  B = V codes: lane = (token half, channel of the group),
//           4 tokens per step;  D: lane holds 4 heads of one channel, summed over its token half.  One instruction
//           per (group, a): the V scale of a (token, group) is applied on the A side.
//
// Codes enter as fp16 subnormals: a 16-bit pattern with a zero exponent field and the code in mantissa bits
// [fb, fb + b) is the number code * 2^fb * 2^-24 exactly, so one AND per pair of codes is the whole conversion.
// The tile layout puts the four codes of a step in the two halves of two words at one field position; the
// power of two of the field is folded into the query operand (K side) or into p (V side, per lane).
// Everything a tile needs is loaded straight into registers in its final form; LDS holds only the query operands
// and the merge of the four wavefronts of a workgroup.
#include "decode_tile_common.h"

namespace rdkv {

namespace {

using namespace tile;

typedef _Float16 half4 __attribute__((ext_vector_type(4)));

constexpr int kTile = 64;   // tokens per tile

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

// LDS: query operands [HS][4 groups][8 steps][4 heads] x 8 bytes, group sums [HS][hi, lo][4 heads] x 8 bytes,
// then the merge area
template <int HS>
struct Lds {
  static constexpr int kQop = HS * 4 * 8 * 4 * 8;
  static constexpr int kQsum = HS * 2 * 4 * 8;
  static constexpr int kMl = kWaves * 8 * HS * 2 * 4;     // [4 waves][4 HS heads][m, l]
};

template <int TIER, int HS>
__device__ __forceinline__ void process_tiles(const uint8_t* __restrict__ kd, const uint8_t* __restrict__ km,
                                              const uint8_t* __restrict__ vd, const uint8_t* __restrict__ vm,
                                              int rows, int g, const uint16_t* __restrict__ q,
                                              float* __restrict__ part_acc, float* __restrict__ part_ml,
                                              uint8_t* smem) {
  using S = Step<TIER>;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int blk = lane >> 2, j = lane & 3;
  const uint8_t* s_qop = smem;
  const uint8_t* s_qsum = smem + Lds<HS>::kQop;
  float* s_ml = reinterpret_cast<float*>(smem + Lds<HS>::kQop + Lds<HS>::kQsum);   // [4][4 HS][2]
  float* s_acc = s_ml + kWaves * 4 * HS * 2;                                       // [8 streams][g][128]

  const int ntiles = (rows + kTile - 1) / kTile;

  // ---- first tile's loads, issued before anything waits ------------------------------------------------
  // The 4- and 2-bit tiers keep K and V of a tile in separate registers and refill each right after its last use,
  // so a wavefront always has its next tile in flight.  An 8-bit tile is 18 KiB: there the K and V codes take turns
  // in one register set (the other wavefronts of the SIMD cover the wait) and the kernel stays within 128 registers.
  constexpr bool kShare = TIER == 8;
  constexpr int kDepth = TIER == 2 ? 2 : 1;   // a 2-bit tile is only 6 KiB: two per wavefront in flight
  struct Regs {
    uint4 k[TIER], v[kShare ? 1 : TIER], kmeta, vmeta;
  };
  Regs regs[kDepth];
  auto load_k = [&](Regs& r, int t) __attribute__((always_inline)) {
    load_tile_side<TIER>(r.k, kd, t, lane);
    r.kmeta = *reinterpret_cast<const uint4*>(km + static_cast<int64_t>(t) * 1024 + lane * 16);
  };
  auto load_v = [&](Regs& r, int t) __attribute__((always_inline)) {
    if constexpr (kShare) load_tile_side<TIER>(r.k, vd, t, lane); else load_tile_side<TIER>(r.v, vd, t, lane);
    // lane (block, j) fetches group j's scales and offsets of tokens 4 blk + 0..3; the quad shares them below
    r.vmeta = *reinterpret_cast<const uint4*>(vm + static_cast<int64_t>(t) * 1024 + lane * 16);
  };
#pragma unroll
  for (int dd = 0; dd < kDepth; ++dd) {
    regs[dd].kmeta = regs[dd].vmeta = make_uint4(0, 0, 0, 0);
    if (wave + dd * kWaves < ntiles) {
      load_k(regs[dd], wave + dd * kWaves);
      if constexpr (!kShare) load_v(regs[dd], wave + dd * kWaves);
    }
  }

  // ---- query operands (once per workgroup) ------------------------------------------------------------------
  // B operand of (head set, group, step): lane head j holds q[head][32 grp + 4 step + 0..3] * 2^(kQExp - fb(step)).
  // The group sums of q (B operand of the K-offset product, k = group, as two fp16 terms) fall out of the same
  // loads: the eight steps of a (head, group) sit in lanes 4, 8 and 16 apart.
  for (int e = tid; e < HS * 128; e += kWG) {
    const int hs = e >> 7, grp = (e >> 5) & 3, st = (e >> 2) & 7, hj = e & 3;
    const int head = 4 * hs + hj;
    Pack4 o;
    o.u[0] = o.u[1] = 0;
    float psum = 0.f;
    if (head < g) {
      const uint2 raw = *reinterpret_cast<const uint2*>(q + head * kHeadDim + grp * 32 + st * 4);
      const float f = ldexpf(1.0f, kQExp - S::fb(st));
      const float v0 = __uint_as_float(raw.x << 16), v1 = __uint_as_float(raw.x & 0xFFFF0000u);
      const float v2 = __uint_as_float(raw.y << 16), v3 = __uint_as_float(raw.y & 0xFFFF0000u);
      o.h[0] = static_cast<_Float16>(v0 * f);
      o.h[1] = static_cast<_Float16>(v1 * f);
      o.h[2] = static_cast<_Float16>(v2 * f);
      o.h[3] = static_cast<_Float16>(v3 * f);
      psum = (v0 + v1) + (v2 + v3);
    }
    *reinterpret_cast<uint2*>(smem + e * 8) = make_uint2(o.u[0], o.u[1]);
    psum += __shfl_xor(psum, 4);
    psum += __shfl_xor(psum, 8);
    psum += __shfl_xor(psum, 16);
    if (st == 0) {
      const _Float16 hi = static_cast<_Float16>(psum);
      const _Float16 lo = static_cast<_Float16>(psum - static_cast<float>(hi));
      _Float16* dst = reinterpret_cast<_Float16*>(smem + Lds<HS>::kQop + (hs * 2 * 4 + hj) * 8);
      dst[grp] = hi;
      dst[16 + grp] = lo;      // the low terms follow the four heads' high terms (32 bytes on)
    }
  }
  __syncthreads();

  // 2^-fb of the field this lane's block is read from on the V side (block a = blk % 8 feeds step a)
  float kappa = 1.0f;
#pragma unroll
  for (int a = 0; a < 8; ++a)
    if ((blk & 7) == a) kappa = 1.0f / static_cast<float>(1 << S::fb(a));

  float m_run[HS], l_run[HS];
  floatx4 acc[HS][4];
  float off[HS][4];
#pragma unroll
  for (int hs = 0; hs < HS; ++hs) {
    m_run[hs] = kNegBig;
    l_run[hs] = 0.f;
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
      acc[hs][grp] = floatx4{0.f, 0.f, 0.f, 0.f};
      off[hs][grp] = 0.f;
    }
  }
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};

  auto do_tile = [&](Regs& r, const int tile) __attribute__((always_inline)) {
    const int next = tile + kDepth * kWaves;
    const bool more = next < ntiles;
    auto& kraw = r.k;
    auto& vraw = [&]() -> auto& { if constexpr (kShare) return r.k; else return r.v; }();
    const uint4& kmeta = r.kmeta;
    const uint4& vmeta = r.vmeta;

    // ---- logits x[hs][i] of token 4 blk + i and head 4 hs + j, in units of kKUnit --------------------------
    float x[HS][4];
    {
      // offsets x group sums of q (A: this lane's own token, k = group)
      Pack4 aoff;
      aoff.u[0] = kmeta.z;
      aoff.u[1] = kmeta.w;
#pragma unroll
      for (int hs = 0; hs < HS; ++hs) {
        Pack4 bh, bl;
        const uint2 h2 = *reinterpret_cast<const uint2*>(s_qsum + (hs * 2 * 4 + j) * 8);
        const uint2 l2 = *reinterpret_cast<const uint2*>(s_qsum + (hs * 2 * 4 + j) * 8 + 32);
        bh.u[0] = h2.x; bh.u[1] = h2.y;
        bl.u[0] = l2.x; bl.u[1] = l2.y;
        floatx4 d = __builtin_amdgcn_mfma_f32_4x4x4f16(aoff.h, bh.h, zero4, 0, 0, 0);
        d = __builtin_amdgcn_mfma_f32_4x4x4f16(aoff.h, bl.h, d, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) x[hs][i] = d[i] * kKUnit;
      }
#pragma unroll
      for (int grp = 0; grp < 4; ++grp) {
        __builtin_amdgcn_sched_barrier(0);   // keep a group's operand reads next to their use (register pressure)
        uint32_t gw[S::kCopies][TIER];
        group_words<TIER>(kraw, grp, gw);
        floatx4 dg[HS];
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) dg[hs] = zero4;
#pragma unroll
        for (int st = 0; st < 8; ++st) {
          const half4 a = step_operand<TIER>(gw, st);
#pragma unroll
          for (int hs = 0; hs < HS; ++hs) {
            Pack4 b;
            const uint2 braw = *reinterpret_cast<const uint2*>(s_qop + (((hs * 4 + grp) * 8 + st) * 4 + j) * 8);
            b.u[0] = braw.x;
            b.u[1] = braw.y;
            dg[hs] = __builtin_amdgcn_mfma_f32_4x4x4f16(a, b.h, dg[hs], 0, 0, 0);
          }
        }
        // scale of (token 4 blk + i, group): held by lane i of this quad in half grp of its (x, y)
        const uint32_t sw = grp < 2 ? kmeta.x : kmeta.y;
        const uint32_t s4[4] = {quad_bcast<0>(sw), quad_bcast<1>(sw), quad_bcast<2>(sw), quad_bcast<3>(sw)};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const half2v sp = __builtin_bit_cast(half2v, s4[i]);
          const float sf = static_cast<float>(sp[grp & 1]);
#pragma unroll
          for (int hs = 0; hs < HS; ++hs) x[hs][i] = __builtin_fmaf(sf, dg[hs][i], x[hs][i]);
        }
      }
    }
    if constexpr (kShare) load_v(r, tile);   // the K codes are used up: their registers take this tile's V codes
    else if (more) load_k(r, next);          // K registers are free again

    if ((tile + 1) * kTile > rows) {   // padded rows of the last tile
#pragma unroll
      for (int hs = 0; hs < HS; ++hs)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (tile * kTile + 4 * blk + i >= rows) x[hs][i] = -INFINITY;
    }

    // ---- online softmax per head; probabilities carried times 2^kPExp ----------------------------------
    float p[HS][4];
#pragma unroll
    for (int hs = 0; hs < HS; ++hs) {
      const float mt = head_max(fmaxf(fmaxf(x[hs][0], x[hs][1]), fmaxf(x[hs][2], x[hs][3])));
      const float m_new = fmaxf(m_run[hs], mt);
      if (__any(m_new != m_run[hs])) {
        const float alpha = fast_exp2((m_run[hs] - m_new) * kXScale);
        l_run[hs] *= alpha;
        const uint32_t au = __builtin_bit_cast(uint32_t, alpha);
        const float ah[4] = {__builtin_bit_cast(float, quad_bcast<0>(au)), __builtin_bit_cast(float, quad_bcast<1>(au)),
                             __builtin_bit_cast(float, quad_bcast<2>(au)), __builtin_bit_cast(float, quad_bcast<3>(au))};
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[hs][grp][i] *= ah[i];   // acc row i is head i
          off[hs][grp] *= alpha;
        }
        m_run[hs] = m_new;
      }
      const float neg_mc = kPExp - m_run[hs] * kXScale;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        p[hs][i] = fast_exp2(__builtin_fmaf(x[hs][i], kXScale, neg_mc));
        l_run[hs] += p[hs][i];
      }
    }

    // ---- P V ------------------------------------------------------------------------------------------------
    {
      Pack4 ph[HS];
#pragma unroll
      for (int hs = 0; hs < HS; ++hs) {
        ph[hs].p[0] = half2v{static_cast<_Float16>(p[hs][0] * kappa), static_cast<_Float16>(p[hs][1] * kappa)};
        ph[hs].p[1] = half2v{static_cast<_Float16>(p[hs][2] * kappa), static_cast<_Float16>(p[hs][3] * kappa)};
      }
#define RDKV_PV_GROUP(G_)                                                                                      \
  {                                                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                                         \
    /* V metadata of tokens 4 blk + 0..3: lane G_ of the quad holds group G_'s scales (x, y), offsets (z, w) */ \
    Pack4 sv, ov, pa[HS];                                                                                      \
    sv.u[0] = quad_bcast<G_>(vmeta.x); sv.u[1] = quad_bcast<G_>(vmeta.y);                                      \
    ov.u[0] = quad_bcast<G_>(vmeta.z); ov.u[1] = quad_bcast<G_>(vmeta.w);                                      \
    _Pragma("unroll") for (int hs = 0; hs < HS; ++hs) {                                                        \
      pa[hs].p[0] = ph[hs].p[0] * sv.p[0];                                                                     \
      pa[hs].p[1] = ph[hs].p[1] * sv.p[1];                                                                     \
      float o = off[hs][G_];                                                                                   \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) o = __builtin_fmaf(p[hs][i], static_cast<float>(ov.h[i]), o); \
      off[hs][G_] = o;                                                                                         \
    }                                                                                                          \
    uint32_t gw[S::kCopies][TIER];                                                                             \
    group_words<TIER>(vraw, G_, gw);                                                                           \
    RDKV_PV_STEP(G_, 0) RDKV_PV_STEP(G_, 1) RDKV_PV_STEP(G_, 2) RDKV_PV_STEP(G_, 3)                            \
    RDKV_PV_STEP(G_, 4) RDKV_PV_STEP(G_, 5) RDKV_PV_STEP(G_, 6) RDKV_PV_STEP(G_, 7)                            \
  }
#define RDKV_PV_STEP(G_, A_)                                                                                   \
  {                                                                                                            \
    const half4 b = step_operand<TIER>(gw, A_);                                                                \
    _Pragma("unroll") for (int hs = 0; hs < HS; ++hs)                                                          \
        acc[hs][G_] = __builtin_amdgcn_mfma_f32_4x4x4f16(pa[hs].h, b, acc[hs][G_], 3, A_, 0);                  \
  }
      RDKV_PV_GROUP(0) RDKV_PV_GROUP(1) RDKV_PV_GROUP(2) RDKV_PV_GROUP(3)
#undef RDKV_PV_STEP
#undef RDKV_PV_GROUP
    }
    if (more) {               // V registers are free again
      if constexpr (kShare) load_k(r, next); else load_v(r, next);
    }
  };
  for (int tile = wave; tile < ntiles; tile += kDepth * kWaves) {
#pragma unroll
    for (int dd = 0; dd < kDepth; ++dd)
      if (tile + dd * kWaves < ntiles) do_tile(regs[dd], tile + dd * kWaves);
  }

  // ---- end of the chunk: undo the subnormal unit, add the offsets, merge the 4 wavefronts --------------------
  // acc[hs][grp][i]: head 4 hs + i, channel 32 grp + lane % 32, summed over this lane's token half
  const int th = lane >> 5, cl = lane & 31;
#pragma unroll
  for (int hs = 0; hs < HS; ++hs) {
    l_run[hs] = head_sum(l_run[hs]);
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
      const uint32_t ou = __builtin_bit_cast(uint32_t, head_sum(off[hs][grp]));   // lanes of head j hold sum_t p m
      const float oh[4] = {__builtin_bit_cast(float, quad_bcast<0>(ou)), __builtin_bit_cast(float, quad_bcast<1>(ou)),
                           __builtin_bit_cast(float, quad_bcast<2>(ou)), __builtin_bit_cast(float, quad_bcast<3>(ou))};
#pragma unroll
      for (int i = 0; i < 4; ++i)
        acc[hs][grp][i] = __builtin_fmaf(acc[hs][grp][i], 16777216.0f, th == 0 ? oh[i] : 0.f);
    }
    if (lane < 4) {
      s_ml[((wave * HS + hs) * 4 + lane) * 2] = m_run[hs] * kXScale - kPExp;   // log2 domain from here on
      s_ml[((wave * HS + hs) * 4 + lane) * 2 + 1] = l_run[hs];
    }
  }
  __syncthreads();
#pragma unroll
  for (int hs = 0; hs < HS; ++hs)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int head = 4 * hs + i;
      float mm = kNegBig;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, s_ml[((w * HS + hs) * 4 + i) * 2]);
      const float f = fast_exp2(s_ml[((wave * HS + hs) * 4 + i) * 2] - mm);
      if (head < g) {
#pragma unroll
        for (int grp = 0; grp < 4; ++grp)
          s_acc[((wave * 2 + th) * g + head) * kHeadDim + 32 * grp + cl] = acc[hs][grp][i] * f;
      }
    }
  __syncthreads();
  for (int idx = tid; idx < g * kHeadDim; idx += kWG) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < 2 * kWaves; ++w) v += s_acc[w * g * kHeadDim + idx];
    part_acc[idx] = v;
  }
  if (tid < g) {
    const int hs = tid >> 2, i = tid & 3;
    float mm = kNegBig;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, s_ml[((w * HS + hs) * 4 + i) * 2]);
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w)
      ll += s_ml[((w * HS + hs) * 4 + i) * 2 + 1] * fast_exp2(s_ml[((w * HS + hs) * 4 + i) * 2] - mm);
    part_ml[tid * 2] = mm;
    part_ml[tid * 2 + 1] = ll;
  }
}

template <int HS>
__global__ __launch_bounds__(kWG, HS == 1 ? 4 : 3) void decode_tiles_kernel(const Chunk* __restrict__ chunks,
                                                                           const uint8_t* __restrict__ arena,
                                                                           const uint16_t* __restrict__ q,
                                                                           float* part_acc, float* part_ml, int hq,
                                                                           int hkv) {
  extern __shared__ __align__(16) uint8_t smem[];
  const Chunk ch = chunks[blockIdx.x];
  const int g = hq / hkv;
  const int seq = ch.item / hkv, head = ch.item % hkv;
  const uint16_t* qp = q + (static_cast<int64_t>(seq) * hq + head * g) * kHeadDim;
  float* pa = part_acc + static_cast<int64_t>(ch.slot) * g * kHeadDim;
  float* pm = part_ml + static_cast<int64_t>(ch.slot) * g * 2;
  const uint8_t* kd = arena + ch.k_data;
  const uint8_t* km = arena + ch.k_meta;
  const uint8_t* vd = arena + ch.v_data;
  const uint8_t* vm = arena + ch.v_meta;
  switch (ch.tier) {
    case 8: process_tiles<8, HS>(kd, km, vd, vm, ch.rows, g, qp, pa, pm, smem); break;
    case 4: process_tiles<4, HS>(kd, km, vd, vm, ch.rows, g, qp, pa, pm, smem); break;
    default: process_tiles<2, HS>(kd, km, vd, vm, ch.rows, g, qp, pa, pm, smem); break;
  }
}

}  // namespace

hipError_t launch_decode_tiles(const Chunk* chunks, int n_chunks, const uint8_t* arena, const uint16_t* q,
                               float* part_acc, float* part_ml, int hq, int hkv, hipStream_t st) {
  if (n_chunks == 0) return hipSuccess;
  const int g = hq / hkv;
  const int hs = g > 4 ? 2 : 1;
  const size_t lds = (hs == 1 ? Lds<1>::kQop + Lds<1>::kQsum : Lds<2>::kQop + Lds<2>::kQsum) +
                     kWaves * 4 * hs * 2 * sizeof(float) + static_cast<size_t>(2 * kWaves) * g * kHeadDim * sizeof(float);
  if (hs == 1)
    hipLaunchKernelGGL(decode_tiles_kernel<1>, dim3(n_chunks), dim3(kWG), lds, st, chunks, arena, q, part_acc, part_ml,
                       hq, hkv);
  else
    hipLaunchKernelGGL(decode_tiles_kernel<2>, dim3(n_chunks), dim3(kWG), lds, st, chunks, arena, q, part_acc, part_ml,
                       hq, hkv);
  return hipGetLastError();
}

}  // namespace rdkv
