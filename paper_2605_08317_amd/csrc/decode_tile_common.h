// Device helpers shared by the tile decode kernels: operand types, the subnormal-fp16 unpack of packed codes,
// tile loads and the wavefront-level LDS fence.
#pragma once
#include "rdkv_internal.h"

namespace rdkv {
namespace tile {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kWG = 256;
constexpr int kWaves = 4;
constexpr int kQBytes = 9 * 64 * 16;   // LDS copy of the query operands: 8 x (m-block, group) and the group sums
constexpr float kNegBig = -1.0e30f;
constexpr float kLogitScale = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)

// Codes enter the matrix cores as fp16 subnormals: a 16-bit pattern with a zero exponent field and the code in
// mantissa bits [fb, fb + b) is the number code * 2^fb * 2^-24 exactly, so one AND per pair of codes is the whole
// conversion.  The layout gives all eight slots of an operand the same fb; the query operand of the K product is
// pre-multiplied by 2^(kQExp - fb) and the V accumulators are rescaled once per chunk.
constexpr int kQExp = 4;                                   // keeps the scaled query clear of fp16 underflow
constexpr float kKUnit = 1.0f / static_cast<float>(1 << (24 - kQExp));   // K partial products come out times this
constexpr float kXScale = kLogitScale * static_cast<float>(1 << (24 - kQExp));

// The probabilities exp2(x - running maximum) are carried times 2^kPExp, so that after the multiplication by a
// V scale they stay in fp16's normal range for flat attention over tens of thousands of tokens (p ~ 1e-5); the
// factor is returned by reporting the running maximum kPExp lower to the merge.  2^kPExp * scale must stay below
// 65504, which holds for V scales below 1023.
constexpr float kPExp = 6.0f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

union Pack8 {
  half8 h;
  half2v p[4];
  uint32_t u[4];
  uint4 q;
};

// bit offset (inside a 16-bit half, after the pre-shift) of the field that operand o reads
template <int TIER>
__host__ __device__ constexpr int field_bit(int o) {
  return TIER == 8 ? 0 : TIER == 4 ? 4 * (o & 1) : (o < 5 ? 2 * o : 2 * (o - 5));
}

// Raw bytes of one tile side held by a lane, plus the right-shifted copy that brings the fields lying in the exponent
// bits of a half down into its mantissa bits (2-bit: fields 5..7, shift 10; 4-bit: nibbles 2 and 3, shift 8).
template <int TIER>
struct Side {
  uint4 raw[TIER / 2];
};
template <int TIER>
struct Shifted {
  uint4 s[TIER == 8 ? 1 : TIER / 2];
};

template <int TIER>
__device__ __forceinline__ Shifted<TIER> pre_shift(const Side<TIER>& a) {
  Shifted<TIER> r;
  if constexpr (TIER != 8) {
    constexpr int kSh = TIER == 2 ? 10 : 8;
#pragma unroll
    for (int i = 0; i < TIER / 2; ++i)
      r.s[i] = make_uint4(a.raw[i].x >> kSh, a.raw[i].y >> kSh, a.raw[i].z >> kSh, a.raw[i].w >> kSh);
  }
  return r;
}

// operand o (0..7) of this lane: eight codes as fp16 subnormals
template <int TIER>
__device__ __forceinline__ half8 unpack_operand(const Side<TIER>& a, const Shifted<TIER>& sh, int o) {
  Pack8 r;
  if constexpr (TIER == 8) {
    const uint4 c = a.raw[o >> 1];
    // bytes (0, 2) of every word for an even operand, (1, 3) for an odd one, zero-extended to 16 bits each.
    // Both go through the byte permute: mixing it with a plain AND of the same register was seen to be
    // scheduled with the AND done in place before the permute read its source.
    const uint32_t sel = (o & 1) ? 0x0C030C01u : 0x0C020C00u;
    r.u[0] = __builtin_amdgcn_perm(0u, c.x, sel);
    r.u[1] = __builtin_amdgcn_perm(0u, c.y, sel);
    r.u[2] = __builtin_amdgcn_perm(0u, c.z, sel);
    r.u[3] = __builtin_amdgcn_perm(0u, c.w, sel);
  } else if constexpr (TIER == 4) {
    const int n = o & 3;
    const uint4 c = n < 2 ? a.raw[o >> 2] : sh.s[o >> 2];
    const uint32_t mask = 0x000F000Fu << (4 * (n & 1));
    r.q = make_uint4(c.x & mask, c.y & mask, c.z & mask, c.w & mask);
  } else {
    const uint4 c = o < 5 ? a.raw[0] : sh.s[0];
    const uint32_t mask = 0x00030003u << field_bit<2>(o);
    r.q = make_uint4(c.x & mask, c.y & mask, c.z & mask, c.w & mask);
  }
  return r.h;
}

template <int TIER>
__device__ __forceinline__ void load_side(Side<TIER>& r, const uint8_t* __restrict__ data, int tile, int lane) {
  constexpr int kTileBytes = kRowPad * kHeadDim * TIER / 8;
  const uint8_t* p = data + static_cast<int64_t>(tile) * kTileBytes + lane * 16;
#pragma unroll
  for (int i = 0; i < TIER / 2; ++i) r.raw[i] = *reinterpret_cast<const uint4*>(p + i * 1024);
}

__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace tile
}  // namespace rdkv
