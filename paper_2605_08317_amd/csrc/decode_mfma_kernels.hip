// Split-K flash-decode over the quantized tiers (8/4/2 bit) of the packed cache
// (Sec. 3.3, Eq. 7) on the gfx950 matrix cores.
//
// With grouped-query attention the g query heads of a KV head share every K/V
// byte, so per quantization group q K^T is a [16 (g padded) x 32 channels] x
// [32 x 16 tokens] contraction and P V a [16 x 32 tokens] x [32 x 16 channels]
// one: both run on v_mfma_f32_16x16x32_f16 with the integer codes as exact fp16
// operands (the same device the paper uses on tensor cores, App. B).  The plain
// ALUs are left with unpacking, the per-(token, group) scales and the softmax:
// at 8 TB/s they could not also carry g multiply-adds per code.
//
// Tile = 32 tokens.  K codes are MFMA A operands (tokens on M, one quantization
// group on K), the query is the B operand (heads on N), so the logits come out as
// x[token 16mb + 4quad + i][head l16]; exactly the lane layout the P operand of the
// second product needs (heads on M, tokens on K), because V is stored transposed
// inside the tile with its 8 slots per lane in the order (mb, i).  Scales are
// applied to the per-group partial products (fusion identity of App. B); offsets
// go through one extra MFMA per product (K: offsets x group sums of q, V: P x offsets).
// One wavefront owns a tile; 4 wavefronts of a workgroup interleave over a chunk.
#include "rdkv_internal.h"

namespace rdkv {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kWG = 256;
constexpr int kWaves = 4;
constexpr int kQBytes = 5 * 64 * 16;   // LDS copy of the query operands
constexpr float kNegBig = -1.0e30f;
constexpr float kLogitScale = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

union Pack8 {
  half8 h;
  half2v p[4];
  uint32_t u[4];
  uint4 q;
};

// fields of a word -> pair of exact fp16 integers: (w & mask) | 0x6400 is 1024 + code * 2^shift in each half
template <int SHIFT>
__device__ __forceinline__ uint32_t field_pair(uint32_t w, uint32_t mask) {
  // one v_and_or_b32: the mask rides in a scalar register, the fp16 pattern in a vector register
  // (a gfx9 VALU instruction may read only one scalar or literal operand)
  uint32_t x;
  const uint32_t magic = 0x64006400u;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(x) : "v"(w), "s"(mask), "v"(magic));
  const half2v v = __builtin_bit_cast(half2v, x);
  constexpr float inv = 1.0f / static_cast<float>(1 << SHIFT);
  const half2v scale = {static_cast<_Float16>(inv), static_cast<_Float16>(inv)};
  const half2v bias = {static_cast<_Float16>(-1024.0f * inv), static_cast<_Float16>(-1024.0f * inv)};
  const half2v r = __builtin_elementwise_fma(v, scale, bias);
  return __builtin_bit_cast(uint32_t, r);
}

// operand o (0..7) of this lane out of the raw tile bytes it loaded
template <int TIER>
__device__ __forceinline__ half8 unpack_operand(const uint4 (&raw)[TIER / 2], int o) {
  Pack8 r;
  if constexpr (TIER == 8) {
    const uint4 c = raw[o >> 1];
    const uint32_t w0 = (o & 1) ? c.z : c.x, w1 = (o & 1) ? c.w : c.y;
    const half2v k1024 = {static_cast<_Float16>(1024.0f), static_cast<_Float16>(1024.0f)};
    const uint32_t ws[2] = {w0, w1};
#pragma unroll
    for (int d = 0; d < 2; ++d) {
      const uint32_t lo = __builtin_amdgcn_perm(0x64646464u, ws[d], 0x04010400u);   // bytes 0,1 -> 0x64bb 0x64bb
      const uint32_t hi = __builtin_amdgcn_perm(0x64646464u, ws[d], 0x04030402u);   // bytes 2,3
      r.p[2 * d] = __builtin_bit_cast(half2v, lo) - k1024;
      r.p[2 * d + 1] = __builtin_bit_cast(half2v, hi) - k1024;
    }
  } else if constexpr (TIER == 4) {
    const uint4 c = raw[o >> 2];
    const uint32_t w = (o & 3) == 0 ? c.x : (o & 3) == 1 ? c.y : (o & 3) == 2 ? c.z : c.w;
    const uint32_t t = w >> 8;
    r.u[0] = field_pair<0>(w, 0x000F000Fu);
    r.u[1] = field_pair<4>(w, 0x00F000F0u);
    r.u[2] = field_pair<0>(t, 0x000F000Fu);
    r.u[3] = field_pair<4>(t, 0x00F000F0u);
  } else {
    const uint4 c = raw[0];
    const int d = o >> 1;
    uint32_t w = d == 0 ? c.x : d == 1 ? c.y : d == 2 ? c.z : c.w;
    if (o & 1) w >>= 8;
    r.u[0] = field_pair<0>(w, 0x00030003u);
    r.u[1] = field_pair<2>(w, 0x000C000Cu);
    r.u[2] = field_pair<4>(w, 0x00300030u);
    r.u[3] = field_pair<6>(w, 0x00C000C0u);
  }
  return r.h;
}

// Raw bytes of NT consecutive tiles held by one lane.  K and V registers are refilled right after their last
// use (K after the logits, V after the second product), so loads of the next tiles overlap the rest of the
// iteration without a second register buffer.
template <int TIER, int NT>
struct SuperRaw {
  uint4 k[NT][TIER / 2];
  uint4 v[NT][TIER / 2];
  uint4 kmeta;   // NT == 2: K metadata of tile (lane / 32); NT == 1: K metadata (lanes 0..31) and V metadata (32..63)
  uint4 vmeta;   // NT == 2 only
};

template <int TIER, int NT>
__device__ __forceinline__ void load_k(SuperRaw<TIER, NT>& r, const uint8_t* __restrict__ kd,
                                       const uint8_t* __restrict__ km, const uint8_t* __restrict__ vm, int st,
                                       int ntiles, int lane) {
  constexpr int kTileBytes = kRowPad * kHeadDim * TIER / 8;
#pragma unroll
  for (int u = 0; u < NT; ++u) {
    const int tile = min(st * NT + u, ntiles - 1);
    const uint8_t* kp = kd + static_cast<int64_t>(tile) * kTileBytes + lane * 16;
#pragma unroll
    for (int i = 0; i < TIER / 2; ++i) r.k[u][i] = *reinterpret_cast<const uint4*>(kp + i * 1024);
  }
  if constexpr (NT == 2) {
    const int tile = min(st * 2 + (lane >> 5), ntiles - 1);
    r.kmeta = *reinterpret_cast<const uint4*>(km + static_cast<int64_t>(tile) * 512 + (lane & 31) * 16);
  } else {
    const int tile = min(st, ntiles - 1);
    r.kmeta = *reinterpret_cast<const uint4*>((lane < 32 ? km : vm) + static_cast<int64_t>(tile) * 512 + (lane & 31) * 16);
  }
}

template <int TIER, int NT>
__device__ __forceinline__ void load_v(SuperRaw<TIER, NT>& r, const uint8_t* __restrict__ vd,
                                       const uint8_t* __restrict__ vm, int st, int ntiles, int lane) {
  constexpr int kTileBytes = kRowPad * kHeadDim * TIER / 8;
#pragma unroll
  for (int u = 0; u < NT; ++u) {
    const int tile = min(st * NT + u, ntiles - 1);
    const uint8_t* vp = vd + static_cast<int64_t>(tile) * kTileBytes + lane * 16;
#pragma unroll
    for (int i = 0; i < TIER / 2; ++i) r.v[u][i] = *reinterpret_cast<const uint4*>(vp + i * 1024);
  }
  if constexpr (NT == 2) {
    const int tile = min(st * 2 + (lane >> 5), ntiles - 1);
    r.vmeta = *reinterpret_cast<const uint4*>(vm + static_cast<int64_t>(tile) * 512 + (lane & 31) * 16);
  }
}

struct QOperands {
  half8 q[4];      // B operand per channel group: q[head l16][32 grp + 8 quad + 0..7]
  half8 qsum;      // B operand of the K-offset product: slots 0..3 group sums (hi), 4..7 (lo); quad 0 only
};

__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int TIER, int NT>
__device__ __forceinline__ void process_tiles(const uint8_t* __restrict__ kd, const uint8_t* __restrict__ km,
                                              const uint8_t* __restrict__ vd, const uint8_t* __restrict__ vm,
                                              int rows, int g, float* __restrict__ part_acc,
                                              float* __restrict__ part_ml, uint8_t* smem) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // scalar: tile indices and branches stay uniform
  const int quad = lane >> 4, l16 = lane & 15;
  const uint8_t* s_q = smem + lane * 16;                           // query operands: [5][64 lanes][16 B]
  uint8_t* s_meta_k = smem + kQBytes + wave * 2048;                // this wavefront's metadata staging
  uint8_t* s_meta_v = s_meta_k + NT * 512;
  float* s_ml = reinterpret_cast<float*>(smem + kQBytes + kWaves * 2048);    // [4][16][2]
  float* s_acc = s_ml + kWaves * 16 * 2;                           // [4][g][128]

  const int ntiles = (rows + kRowPad - 1) / kRowPad;
  const int nsuper = (ntiles + NT - 1) / NT;
  float m_run = kNegBig, l_run = 0.f;
  floatx4 acc[8], acc_off;
#pragma unroll
  for (int nt = 0; nt < 8; ++nt) acc[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  acc_off = floatx4{0.f, 0.f, 0.f, 0.f};
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};

  SuperRaw<TIER, NT> raw;
  if (wave < nsuper) {
    load_k<TIER, NT>(raw, kd, km, vm, wave, ntiles, lane);
    load_v<TIER, NT>(raw, vd, vm, wave, ntiles, lane);
  }
  for (int st = wave; st < nsuper; st += kWaves) {
    const bool more = st + kWaves < nsuper;

    // stage the metadata for broadcast reads (K tiles at s_meta_k + 512u, V tiles at s_meta_v + 512u)
    *reinterpret_cast<uint4*>(s_meta_k + lane * 16) = raw.kmeta;
    wave_lds_sync();

    // ---- logits: x[u][mb][i] for token 32(st NT + u) + 16mb + 4quad + i, head l16 -----------
    float x[NT][2][4];
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      Pack8 ks[4];   // scales of (mb, grp, i): 32 fp16
#pragma unroll
      for (int j = 0; j < 4; ++j) ks[j].q = *reinterpret_cast<const uint4*>(s_meta_k + u * 512 + quad * 64 + j * 16);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        // offsets x group sums of q
        const uint2 mo = *reinterpret_cast<const uint2*>(s_meta_k + u * 512 + 256 + (mb * 16 + l16) * 8);
        Pack8 a_off;
        a_off.u[0] = a_off.u[2] = quad == 0 ? mo.x : 0u;
        a_off.u[1] = a_off.u[3] = quad == 0 ? mo.y : 0u;
        const floatx4 d_off = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_off.h, *reinterpret_cast<const half8*>(s_q + 4 * 1024), zero4, 0, 0, 0);
        float sum[4] = {d_off[0], d_off[1], d_off[2], d_off[3]};
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
          const half8 a = unpack_operand<TIER>(raw.k[u], mb * 4 + grp);
          const floatx4 dd = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, *reinterpret_cast<const half8*>(s_q + grp * 1024), zero4, 0, 0, 0);
          const int e = (mb * 4 + grp) * 4;           // scale index of i = 0
#pragma unroll
          for (int i = 0; i < 4; ++i)
            sum[i] = __builtin_fmaf(static_cast<float>(ks[e >> 3].h[(e & 7) + i]), dd[i], sum[i]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) x[u][mb][i] = sum[i];   // raw q.k; the 1/sqrt(d) and log2(e) factors enter at the exp
      }
    }
    if (more) load_k<TIER, NT>(raw, kd, km, vm, st + kWaves, ntiles, lane);   // K registers are free again

    if ((st + 1) * NT * kRowPad > rows) {   // padded rows (and a missing second tile) of the last super-tile
#pragma unroll
      for (int u = 0; u < NT; ++u)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if ((st * NT + u) * kRowPad + 16 * mb + 4 * quad + i >= rows) x[u][mb][i] = -INFINITY;
    }

    // ---- online softmax (head l16; the four quads hold different tokens) ----------------------
    float mt = kNegBig;
#pragma unroll
    for (int u = 0; u < NT; ++u)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int i = 0; i < 4; ++i) mt = fmaxf(mt, x[u][mb][i]);
    mt = fmaxf(mt, __shfl_xor(mt, 16));
    mt = fmaxf(mt, __shfl_xor(mt, 32));
    const float m_new = fmaxf(m_run, mt);
    if (__any(m_new != m_run)) {
      const float alpha = fast_exp2((m_run - m_new) * kLogitScale);
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float ah = __shfl(alpha, 4 * quad + i);   // factor of head 4quad+i, the row of acc[.][i]
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) acc[nt][i] *= ah;
        acc_off[i] *= ah;
      }
      m_run = m_new;
    }

    if constexpr (NT == 2) {
      *reinterpret_cast<uint4*>(s_meta_v + lane * 16) = raw.vmeta;
      wave_lds_sync();
    }
    // ---- P V: slot j = 4mb + i of this lane is token 16mb + 4quad + i of tile u ----------------
    const float neg_mc = -m_run * kLogitScale;
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      float p[8];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          p[mb * 4 + i] = fast_exp2(__builtin_fmaf(x[u][mb][i], kLogitScale, neg_mc));
          l_run += p[mb * 4 + i];
        }
      Pack8 ph;
#pragma unroll
      for (int j = 0; j < 4; ++j) ph.p[j] = half2v{static_cast<_Float16>(p[2 * j]), static_cast<_Float16>(p[2 * j + 1])};
      Pack8 voff;
      voff.q = *reinterpret_cast<const uint4*>(s_meta_v + u * 512 + 256 + (quad * 4 + (l16 & 3)) * 16);
      if (l16 >= 4) voff.q = make_uint4(0, 0, 0, 0);
      acc_off = __builtin_amdgcn_mfma_f32_16x16x32_f16(ph.h, voff.h, acc_off, 0, 0, 0);
#pragma unroll
      for (int grp = 0; grp < 4; ++grp) {
        Pack8 vs, pa;
        vs.q = *reinterpret_cast<const uint4*>(s_meta_v + u * 512 + (quad * 4 + grp) * 16);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          pa.p[j] = half2v{static_cast<_Float16>(__builtin_fmaf(static_cast<float>(vs.h[2 * j]), p[2 * j], 0.0f)),
                           static_cast<_Float16>(__builtin_fmaf(static_cast<float>(vs.h[2 * j + 1]), p[2 * j + 1], 0.0f))};
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const int nt = grp * 2 + h2;
          const half8 b = unpack_operand<TIER>(raw.v[u], nt);
          acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa.h, b, acc[nt], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();   // all reads of the staging area are issued before it is overwritten
    if (more) load_v<TIER, NT>(raw, vd, vm, st + kWaves, ntiles, lane);       // V registers are free again
  }

  // ---- merge the 4 wavefronts; acc[nt][i] is head 4quad+i, channel 16nt + l16 -----------------
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (quad == 0) {
    s_ml[(wave * 16 + l16) * 2] = m_run * kLogitScale;   // running maximum in the log2 domain from here on
    s_ml[(wave * 16 + l16) * 2 + 1] = l_run;
  }
  __syncthreads();
  float f_own[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int h = 4 * quad + i;
    float mm = kNegBig;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, s_ml[(w * 16 + h) * 2]);
    f_own[i] = fast_exp2(s_ml[(wave * 16 + h) * 2] - mm);
  }
  // the V-offset product left sum_t p m_v[t][grp] in lane (quad, l16 = grp); bring it to every channel lane
#pragma unroll
  for (int grp = 0; grp < 4; ++grp)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float o = __shfl(acc_off[i], quad * 16 + grp);
      acc[2 * grp][i] += o;
      acc[2 * grp + 1][i] += o;
    }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int h = 4 * quad + i;
    if (h < g) {
#pragma unroll
      for (int nt = 0; nt < 8; ++nt) s_acc[(wave * g + h) * kHeadDim + nt * 16 + l16] = acc[nt][i] * f_own[i];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < g * kHeadDim; idx += kWG) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) v += s_acc[w * g * kHeadDim + idx];
    part_acc[idx] = v;
  }
  if (tid < g) {
    float mm = kNegBig;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, s_ml[(w * 16 + tid) * 2]);
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) ll += s_ml[(w * 16 + tid) * 2 + 1] * fast_exp2(s_ml[(w * 16 + tid) * 2] - mm);
    part_ml[tid * 2] = mm;
    part_ml[tid * 2 + 1] = ll;
  }
}

template <int TIER_SEL>
__global__ __launch_bounds__(kWG) void decode_tiles_kernel(const Chunk* __restrict__ chunks,
                                                           const uint8_t* __restrict__ arena,
                                                           const uint16_t* __restrict__ q, float* part_acc,
                                                           float* part_ml, int hq, int hkv) {
  extern __shared__ __align__(16) uint8_t smem[];
  const Chunk ch = chunks[blockIdx.x];
  const int g = hq / hkv;
  const int seq = ch.item / hkv, head = ch.item % hkv;
  const int lane = threadIdx.x & 63, quad = lane >> 4, l16 = lane & 15;

  // query operands: lane (head l16, quad) holds q[head][32 grp + 8 quad + 0..7] as fp16
  QOperands qo;
  float gsum[4];
#pragma unroll
  for (int grp = 0; grp < 4; ++grp) {
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (l16 < g)
      raw = *reinterpret_cast<const uint4*>(q + (static_cast<int64_t>(seq) * hq + head * g + l16) * kHeadDim +
                                             grp * 32 + quad * 8);
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float lo = __uint_as_float(w[j] << 16), hi = __uint_as_float(w[j] & 0xFFFF0000u);
      qo.q[grp][2 * j] = static_cast<_Float16>(lo);
      qo.q[grp][2 * j + 1] = static_cast<_Float16>(hi);
      s += lo + hi;
    }
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    gsum[grp] = s;
  }
#pragma unroll
  for (int grp = 0; grp < 4; ++grp) {
    const _Float16 hi = static_cast<_Float16>(gsum[grp]);
    const _Float16 lo = static_cast<_Float16>(gsum[grp] - static_cast<float>(hi));
    qo.qsum[grp] = quad == 0 ? hi : static_cast<_Float16>(0.0f);
    qo.qsum[4 + grp] = quad == 0 ? lo : static_cast<_Float16>(0.0f);
  }

  if (threadIdx.x < 64) {
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) *reinterpret_cast<half8*>(smem + grp * 1024 + lane * 16) = qo.q[grp];
    *reinterpret_cast<half8*>(smem + 4 * 1024 + lane * 16) = qo.qsum;
  }
  __syncthreads();

  float* pa = part_acc + static_cast<int64_t>(ch.slot) * g * kHeadDim;
  float* pm = part_ml + static_cast<int64_t>(ch.slot) * g * 2;
  const uint8_t* kd = arena + ch.k_data;
  const uint8_t* km = arena + ch.k_meta;
  const uint8_t* vd = arena + ch.v_data;
  const uint8_t* vm = arena + ch.v_meta;
  // TIER_SEL == 0: any quantized tier in one launch; otherwise the launch holds chunks of one tier only
  const int tier = TIER_SEL == 0 ? ch.tier : TIER_SEL;
  switch (tier) {
    case 8: process_tiles<8, 1>(kd, km, vd, vm, ch.rows, g, pa, pm, smem); break;
    case 4: process_tiles<4, 1>(kd, km, vd, vm, ch.rows, g, pa, pm, smem); break;
    default: process_tiles<2, 1>(kd, km, vd, vm, ch.rows, g, pa, pm, smem); break;
  }
}

}  // namespace

hipError_t launch_decode_tiles(const Chunk* chunks, int n_chunks, const uint8_t* arena, const uint16_t* q,
                               float* part_acc, float* part_ml, int hq, int hkv, hipStream_t st) {
  if (n_chunks == 0) return hipSuccess;
  const int g = hq / hkv;
  const size_t lds = kQBytes + kWaves * 2048 + kWaves * 16 * 2 * sizeof(float) + static_cast<size_t>(kWaves) * g * kHeadDim * sizeof(float);
  hipLaunchKernelGGL(decode_tiles_kernel<0>, dim3(n_chunks), dim3(kWG), lds, st, chunks, arena, q, part_acc, part_ml,
                     hq, hkv);
  if (false) {
    hipLaunchKernelGGL(decode_tiles_kernel<8>, dim3(n_chunks), dim3(kWG), lds, st, chunks, arena, q, part_acc, part_ml, hq, hkv);
    hipLaunchKernelGGL(decode_tiles_kernel<4>, dim3(n_chunks), dim3(kWG), lds, st, chunks, arena, q, part_acc, part_ml, hq, hkv);
    hipLaunchKernelGGL(decode_tiles_kernel<2>, dim3(n_chunks), dim3(kWG), lds, st, chunks, arena, q, part_acc, part_ml, hq, hkv);
  }
  return hipGetLastError();
}

}  // namespace rdkv
