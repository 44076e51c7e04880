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
#include "decode_tile_common.h"

namespace rdkv {

namespace {

using namespace tile;

// K metadata (lanes 0..31) and V metadata (lanes 32..63) of a tile: 16 bytes per lane
__device__ __forceinline__ uint4 load_meta(const uint8_t* __restrict__ km, const uint8_t* __restrict__ vm, int tile,
                                           int lane) {
  return *reinterpret_cast<const uint4*>((lane < 32 ? km : vm) + static_cast<int64_t>(tile) * 512 + (lane & 31) * 16);
}

// One workgroup streams the tiles of one chunk; a wavefront owns a tile and the four wavefronts interleave.
// A wavefront keeps DEPTH tiles in registers; the K (and metadata) registers of a tile are refilled right after the
// logits, the V registers right after the second product, with the tile DEPTH rounds ahead, so DEPTH - 1 to DEPTH
// tiles per wavefront are in flight at any time (the low-bit tiers need two to cover the HBM latency).
template <int TIER, int DEPTH>
__device__ __forceinline__ void process_tiles(const uint8_t* __restrict__ kd, const uint8_t* __restrict__ km,
                                              const uint8_t* __restrict__ vd, const uint8_t* __restrict__ vm,
                                              int rows, int g, const uint16_t* __restrict__ q,
                                              float* __restrict__ part_acc, float* __restrict__ part_ml,
                                              uint8_t* smem) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // scalar: tile indices and branches stay uniform
  const int quad = lane >> 4, l16 = lane & 15;
  const uint8_t* s_q = smem + lane * 16;                           // query operands: [9][64 lanes][16 B]
  uint8_t* s_meta_k = smem + kQBytes + wave * 1024;                // this wavefront's metadata staging
  uint8_t* s_meta_v = s_meta_k + 512;
  float* s_ml = reinterpret_cast<float*>(smem + kQBytes + kWaves * 1024);    // [4][16][2]
  float* s_acc = s_ml + kWaves * 16 * 2;                           // [4][g][128]

  const int ntiles = (rows + kRowPad - 1) / kRowPad;

  // ---- issue the query loads, then the first tile's loads, before anything waits ---------------------------
  uint4 qraw[4];
#pragma unroll
  for (int grp = 0; grp < 4; ++grp) {
    qraw[grp] = make_uint4(0, 0, 0, 0);
    if (wave == 0 && l16 < g) qraw[grp] = *reinterpret_cast<const uint4*>(q + l16 * kHeadDim + grp * 32 + quad * 8);
  }
  Side<TIER> rk[DEPTH], rv[DEPTH];
  uint4 rmeta[DEPTH];
#pragma unroll
  for (int dd = 0; dd < DEPTH; ++dd) {
    const int t = wave + dd * kWaves;
    rmeta[dd] = make_uint4(0, 0, 0, 0);
    if (t < ntiles) {
      load_side<TIER>(rk[dd], kd, t, lane);
      rmeta[dd] = load_meta(km, vm, t, lane);
      load_side<TIER>(rv[dd], vd, t, lane);
    }
  }

  // ---- query operands: lane (head l16, quad) holds q[head][32 grp + 8 quad + 0..7]; B operand of (mb, grp) is
  //      q * 2^(kQExp - fb(4 mb + grp)); the group sums go through one more product with the offsets -------------
  if (wave == 0) {
    float gsum[4];
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
      const uint32_t w[4] = {qraw[grp].x, qraw[grp].y, qraw[grp].z, qraw[grp].w};
      float v[8];
      float s = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[2 * j] = __uint_as_float(w[j] << 16);
        v[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
        s += v[2 * j] + v[2 * j + 1];
      }
      s += __shfl_xor(s, 16);
      s += __shfl_xor(s, 32);
      gsum[grp] = s;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const float f = static_cast<float>(1 << kQExp) / static_cast<float>(1 << field_bit<TIER>(4 * mb + grp));
        half8 qo;
#pragma unroll
        for (int j = 0; j < 8; ++j) qo[j] = static_cast<_Float16>(v[j] * f);
        *reinterpret_cast<half8*>(smem + (mb * 4 + grp) * 1024 + lane * 16) = qo;
      }
    }
    half8 qsum;   // slots 0..3: high parts of the group sums, 4..7: low parts; quad 0 only
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
      const _Float16 hi = static_cast<_Float16>(gsum[grp]);
      const _Float16 lo = static_cast<_Float16>(gsum[grp] - static_cast<float>(hi));
      qsum[grp] = quad == 0 ? hi : static_cast<_Float16>(0.0f);
      qsum[4 + grp] = quad == 0 ? lo : static_cast<_Float16>(0.0f);
    }
    *reinterpret_cast<half8*>(smem + 8 * 1024 + lane * 16) = qsum;
  }
  __syncthreads();

  float m_run = kNegBig, l_run = 0.f;     // running maximum in units of kKUnit * (raw q.k)
  floatx4 acc[8], acc_off;
#pragma unroll
  for (int nt = 0; nt < 8; ++nt) acc[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  acc_off = floatx4{0.f, 0.f, 0.f, 0.f};
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};

  auto step = [&](Side<TIER>& rk, Side<TIER>& rv, uint4& rmeta, const int tile) __attribute__((always_inline)) {
    const int next = tile + DEPTH * kWaves;
    const bool more = next < ntiles;

    // stage the metadata for broadcast reads (K at s_meta_k, V at s_meta_v = s_meta_k + 512)
    *reinterpret_cast<uint4*>(s_meta_k + lane * 16) = rmeta;
    uint4 rmeta_next = rmeta;
    wave_lds_sync();

    // ---- logits x[mb][i] of token 16 mb + 4 quad + i and head l16, times kKUnit ---------------------------
    float x[2][4];
    {
      const Shifted<TIER> ks = pre_shift<TIER>(rk);
      Pack8 sc[4];   // scales of (mb, grp, i): 32 fp16
#pragma unroll
      for (int j = 0; j < 4; ++j) sc[j].q = *reinterpret_cast<const uint4*>(s_meta_k + quad * 64 + j * 16);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        // offsets x group sums of q
        const uint2 mo = *reinterpret_cast<const uint2*>(s_meta_k + 256 + (mb * 16 + l16) * 8);
        Pack8 a_off;
        a_off.u[0] = a_off.u[2] = quad == 0 ? mo.x : 0u;
        a_off.u[1] = a_off.u[3] = quad == 0 ? mo.y : 0u;
        const floatx4 d_off = __builtin_amdgcn_mfma_f32_16x16x32_f16(
            a_off.h, *reinterpret_cast<const half8*>(s_q + 8 * 1024), zero4, 0, 0, 0);
        float sum[4] = {d_off[0] * kKUnit, d_off[1] * kKUnit, d_off[2] * kKUnit, d_off[3] * kKUnit};
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
          const half8 a = unpack_operand<TIER>(rk, ks, mb * 4 + grp);
          const floatx4 dd = __builtin_amdgcn_mfma_f32_16x16x32_f16(
              a, *reinterpret_cast<const half8*>(s_q + (mb * 4 + grp) * 1024), zero4, 0, 0, 0);
          const int e = (mb * 4 + grp) * 4;           // scale index of i = 0
#pragma unroll
          for (int i = 0; i < 4; ++i)
            sum[i] = __builtin_fmaf(static_cast<float>(sc[e >> 3].h[(e & 7) + i]), dd[i], sum[i]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) x[mb][i] = sum[i];
      }
    }
    if (more) {                        // K registers are free again
      load_side<TIER>(rk, kd, next, lane);
      rmeta_next = load_meta(km, vm, next, lane);
    }

    if ((tile + 1) * kRowPad > rows) {   // padded rows of the last tile
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (tile * kRowPad + 16 * mb + 4 * quad + i >= rows) x[mb][i] = -INFINITY;
    }

    // ---- online softmax (head l16; the four quads hold different tokens) ----------------------
    float mt = fmaxf(fmaxf(fmaxf(x[0][0], x[0][1]), fmaxf(x[0][2], x[0][3])),
                     fmaxf(fmaxf(x[1][0], x[1][1]), fmaxf(x[1][2], x[1][3])));
    mt = fmaxf(mt, __shfl_xor(mt, 16));
    mt = fmaxf(mt, __shfl_xor(mt, 32));
    const float m_new = fmaxf(m_run, mt);
    if (__any(m_new != m_run)) {
      const float alpha = fast_exp2((m_run - m_new) * kXScale);
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

    // ---- P V: slot j = 4mb + i of this lane is token 16mb + 4quad + i ----------------
    {
      const float neg_mc = kPExp - m_run * kXScale;   // probabilities times 2^kPExp
      Pack8 ph;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const float p0 = fast_exp2(__builtin_fmaf(x[mb][2 * h2], kXScale, neg_mc));
          const float p1 = fast_exp2(__builtin_fmaf(x[mb][2 * h2 + 1], kXScale, neg_mc));
          l_run += p0 + p1;
          ph.p[mb * 2 + h2] = half2v{static_cast<_Float16>(p0), static_cast<_Float16>(p1)};
        }
      const Shifted<TIER> vs = pre_shift<TIER>(rv);
      Pack8 voff;
      voff.q = *reinterpret_cast<const uint4*>(s_meta_v + 256 + (quad * 4 + (l16 & 3)) * 16);
      if (l16 >= 4) voff.q = make_uint4(0, 0, 0, 0);
      acc_off = __builtin_amdgcn_mfma_f32_16x16x32_f16(ph.h, voff.h, acc_off, 0, 0, 0);
#pragma unroll
      for (int grp = 0; grp < 4; ++grp) {
        Pack8 sv, pa;
        sv.q = *reinterpret_cast<const uint4*>(s_meta_v + (quad * 4 + grp) * 16);
#pragma unroll
        for (int j = 0; j < 4; ++j) pa.p[j] = ph.p[j] * sv.p[j];      // p * scale in fp16
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const int nt = grp * 2 + h2;
          const half8 b = unpack_operand<TIER>(rv, vs, nt);
          acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa.h, b, acc[nt], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();   // all reads of the staging area are issued before it is overwritten
    if (more) load_side<TIER>(rv, vd, next, lane);       // V registers are free again
    rmeta = rmeta_next;
  };
  for (int tile = wave; tile < ntiles; tile += DEPTH * kWaves) {
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd)
      if (tile + dd * kWaves < ntiles) step(rk[dd], rv[dd], rmeta[dd], tile + dd * kWaves);
  }

  // ---- merge the 4 wavefronts; acc[nt][i] is head 4quad+i, channel 16nt + l16 -----------------
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (quad == 0) {
    s_ml[(wave * 16 + l16) * 2] = m_run * kXScale - kPExp;   // running maximum in the log2 domain from here on
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
  // undo the subnormal unit of the V codes; the V-offset product left sum_t p m_v[t][grp] in lane
  // (quad, l16 = grp): bring it to every channel lane
#pragma unroll
  for (int grp = 0; grp < 4; ++grp)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float o = __shfl(acc_off[i], quad * 16 + grp);
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        const int nt = 2 * grp + h2;
        constexpr float kBase = 16777216.0f;   // 2^24
        const float unit = kBase / static_cast<float>(1 << field_bit<TIER>(nt));
        acc[nt][i] = __builtin_fmaf(acc[nt][i], unit, o);
      }
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

__global__ __launch_bounds__(kWG, 3) void decode_tiles_kernel(const Chunk* __restrict__ chunks,
                                                           const uint8_t* __restrict__ arena,
                                                           const uint16_t* __restrict__ q, float* part_acc,
                                                           float* part_ml, int hq, int hkv) {
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
    case 8: process_tiles<8, 1>(kd, km, vd, vm, ch.rows, g, qp, pa, pm, smem); break;
    case 4: process_tiles<4, 2>(kd, km, vd, vm, ch.rows, g, qp, pa, pm, smem); break;
    default: process_tiles<2, 2>(kd, km, vd, vm, ch.rows, g, qp, pa, pm, smem); break;
  }
}

}  // namespace

hipError_t launch_decode_tiles(const Chunk* chunks, int n_chunks, const uint8_t* arena, const uint16_t* q,
                               float* part_acc, float* part_ml, int hq, int hkv, hipStream_t st) {
  if (n_chunks == 0) return hipSuccess;
  const int g = hq / hkv;
  const size_t lds = kQBytes + kWaves * 1024 + kWaves * 16 * 2 * sizeof(float) +
                     static_cast<size_t>(kWaves) * g * kHeadDim * sizeof(float);
  hipLaunchKernelGGL(decode_tiles_kernel, dim3(n_chunks), dim3(kWG), lds, st, chunks, arena, q, part_acc, part_ml,
                     hq, hkv);
  return hipGetLastError();
}

}  // namespace rdkv
