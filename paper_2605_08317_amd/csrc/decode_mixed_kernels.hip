// Split-K flash-decode over a mixed-mode cache (Sec. 3.2 Stages 2-3, Sec. 3.3, Eq. 7): V token-wise in tiers,
// K of the retained tokens channel-wise, on the gfx950 matrix cores.
//
// Per-channel quantization k_hat[t][c] = s_c code[t][c] + m_c (one scale and offset per channel and 32-token
// tile) turns the logits into  sum_c (s_c q_c) code[t][c] + sum_c m_c q_c  (the dequantization fusion of App. B):
// the query operand is scaled by the tile's channel scales (two fp16 terms whose sum is the exact product), the raw
// codes are the other MFMA operand, and the offsets go through one more MFMA whose rows are all equal.  Channels are stored
// sorted by bit-width (App. B: "the query is permuted to the same sorted order"): the permuted query operands are
// built once per workgroup.  Channels kept at 16 bits go through the bf16 MFMA with the bf16 query (exact products).
//
// A K tile has a run-time shape (it depends on the item's channel bit map), so a wavefront prefetches the next
// tile's bytes into registers as a flat run of 1 KiB pieces, parks them in its own LDS buffer, and picks operands
// out of LDS by address.  The V side is the tile layout of the token-wise tiers; 16-bit V rows (Zone B) are 32-token
// tiles of bf16 multiplied by the probabilities split into two bf16 terms.
#include "decode_tile_common.h"

namespace rdkv {

namespace {

using namespace tile;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kMaxOps = 8;                  // K operands of a tile: at most 7 (4 full + 3 partial tiers)
constexpr int kItemKBytes = (sizeof(ItemK) + 15) / 16 * 16;
constexpr int kKMetaBytes = 1024;           // per wavefront: K metadata of a tile (at most 4 * 152 bytes)
constexpr int kVMetaBytes = 512;

union PackB8 {
  bf16x8 h;
  uint32_t u[4];
  uint4 q;
};

// V side registers of one tile
template <int VT>
struct VRegs {
  Side<VT> s;
};
template <>
struct VRegs<16> {
  uint4 o[8];   // operand nt: 8 bf16 (tokens) of channel 16 nt + l16
};

template <int VT>
__device__ __forceinline__ void load_v(VRegs<VT>& r, const uint8_t* __restrict__ vd, int tile, int lane) {
  if constexpr (VT == 16) {
    const uint8_t* p = vd + static_cast<int64_t>(tile) * (kRowPad * kHeadDim * 2) + lane * 16;
#pragma unroll
    for (int i = 0; i < 8; ++i) r.o[i] = *reinterpret_cast<const uint4*>(p + i * 1024);
  } else {
    load_side<VT>(r.s, vd, tile, lane);
  }
}

template <int VT, int NK>
__device__ __forceinline__ void process_mixed(const ItemK& ik, const uint8_t* __restrict__ kd,
                                              const uint8_t* __restrict__ km, const uint8_t* __restrict__ vd,
                                              const uint8_t* __restrict__ vm, int rows, int g,
                                              float* __restrict__ part_acc, float* __restrict__ part_ml,
                                              const uint8_t* s_qop, uint8_t* s_wave, float* s_ml, float* s_acc) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int quad = lane >> 4, l16 = lane & 15;
  uint8_t* s_kbuf = s_wave;                        // [NK KiB] this wavefront's K tile
  uint8_t* s_kmeta = s_wave + NK * 1024;           // scales then offsets of the quantized slots
  uint8_t* s_vmeta = s_kmeta + kKMetaBytes;

  const int kt_bytes = ik.kt_bytes, km_bytes = ik.km_bytes;
  const int ntiles = (rows + kRowPad - 1) / kRowPad;

  uint4 kraw[NK], kmeta_r = make_uint4(0, 0, 0, 0), vmeta_r = make_uint4(0, 0, 0, 0);
  VRegs<VT> rv;
  auto load_k = [&](int t) __attribute__((always_inline)) {
    const uint8_t* p = kd + static_cast<int64_t>(t) * kt_bytes + lane * 16;
#pragma unroll
    for (int i = 0; i < NK; ++i) {
      kraw[i] = make_uint4(0, 0, 0, 0);
      if (i * 1024 + lane * 16 < kt_bytes) kraw[i] = *reinterpret_cast<const uint4*>(p + i * 1024);
    }
    if (lane * 16 < km_bytes) kmeta_r = *reinterpret_cast<const uint4*>(km + static_cast<int64_t>(t) * km_bytes + lane * 16);
    if constexpr (VT != 16) {
      if (lane < 32) vmeta_r = *reinterpret_cast<const uint4*>(vm + static_cast<int64_t>(t) * 512 + lane * 16);
    }
  };
  if (wave < ntiles) {
    load_k(wave);
    load_v<VT>(rv, vd, wave, lane);
  }

  float m_run = kNegBig, l_run = 0.f;     // running maximum in units of kKUnit * (raw q.k)
  floatx4 acc[8], acc_off;
#pragma unroll
  for (int nt = 0; nt < 8; ++nt) acc[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  acc_off = floatx4{0.f, 0.f, 0.f, 0.f};
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};

  for (int tile = wave; tile < ntiles; tile += kWaves) {
    const int next = tile + kWaves;
    const bool more = next < ntiles;

    // ---- park the K tile and the metadata in LDS, then start the loads of the next tile ------------
#pragma unroll
    for (int i = 0; i < NK; ++i)
      if (i * 1024 < kt_bytes) *reinterpret_cast<uint4*>(s_kbuf + i * 1024 + lane * 16) = kraw[i];
    *reinterpret_cast<uint4*>(s_kmeta + lane * 16) = kmeta_r;
    if constexpr (VT != 16) {
      if (lane < 32) *reinterpret_cast<uint4*>(s_vmeta + lane * 16) = vmeta_r;
    }
    wave_lds_sync();
    if (more) load_k(next);

    // ---- logits: x[mb][i] of token 16 mb + 4 quad + i and head l16, times kKUnit ---------------------
    floatx4 xq0 = zero4, xq1 = zero4;       // quantized channels, in units of kKUnit
    floatx4 xt0 = zero4, xt1 = zero4;       // 16-bit channels, true scale
    floatx4 xb = zero4;                     // sum_c m_c q_c: the same in every row
    int e = 0;
#pragma unroll 1
    for (int t = 0; t < 4; ++t) {
      const int nq = ik.nq[t];
      const int b = 16 >> t;
      const int qslot0 = ik.slot_base[t] - ik.slot_base[1];
#pragma unroll 1
      for (int o = 0; 4 * o < nq; ++o, ++e) {
        const int Q = 4 * o + quad;
        const bool have = Q < nq;
        const uint8_t* src = s_kbuf + ik.tier_base[t] + (have ? Q : 0) * 32 * b + l16 * 2 * b;
        const uint8_t* qop = s_qop + e * 2048 + lane * 16;
        if (t == 0) {
          PackB8 a0, a1, bq;
          a0.q = *reinterpret_cast<const uint4*>(src);
          a1.q = *reinterpret_cast<const uint4*>(src + 16);
          if (!have) a0.q = a1.q = make_uint4(0, 0, 0, 0);
          bq.q = *reinterpret_cast<const uint4*>(qop);
          xt0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0.h, bq.h, xt0, 0, 0, 0);
          xt1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1.h, bq.h, xt1, 0, 0, 0);
        } else {
          Pack8 sc, of, qpre, qpl, bq, bql, a0, a1;
          const int moff = (qslot0 + 8 * (have ? Q : 0)) * 2;
          sc.q = *reinterpret_cast<const uint4*>(s_kmeta + moff);
          of.q = *reinterpret_cast<const uint4*>(s_kmeta + (km_bytes >> 1) + moff);
          if (!have) sc.q = of.q = make_uint4(0, 0, 0, 0);
          qpre.q = *reinterpret_cast<const uint4*>(qop);
          qpl.q = *reinterpret_cast<const uint4*>(qop + 1024);
          // s_c q_c as an exact sum of two fp16 terms: the product of an 8-bit and an 11-bit significand
          // is the rounded product plus a remainder that the fused multiply-add returns exactly
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            bq.p[j] = qpre.p[j] * sc.p[j];
            bql.p[j] = __builtin_elementwise_fma(qpre.p[j], sc.p[j], -bq.p[j]);
          }
          if (t == 1) {
            uint4 w = *reinterpret_cast<const uint4*>(src);
            if (!have) w = make_uint4(0, 0, 0, 0);
            const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int p = 0; p < 4; ++p) {
              a0.u[p] = __builtin_amdgcn_perm(0u, ws[p], 0x0C020C00u);
              a1.u[p] = __builtin_amdgcn_perm(0u, ws[p], 0x0C030C01u);
            }
          } else if (t == 2) {
            uint2 w = *reinterpret_cast<const uint2*>(src);
            if (!have) w = make_uint2(0, 0);
            const uint32_t ws[2] = {w.x, w.y}, wh[2] = {w.x >> 8, w.y >> 8};
#pragma unroll
            for (int p = 0; p < 4; ++p) {
              const uint32_t mask = 0x000F000Fu << (4 * (p & 1));
              a0.u[p] = ws[p >> 1] & mask;
              a1.u[p] = wh[p >> 1] & mask;
            }
          } else {
            uint32_t w = *reinterpret_cast<const uint32_t*>(src);
            if (!have) w = 0;
            const uint32_t wh = w >> 8;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
              const uint32_t mask = 0x00030003u << (2 * p);
              a0.u[p] = w & mask;
              a1.u[p] = wh & mask;
            }
          }
          xq0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0.h, bq.h, xq0, 0, 0, 0);
          xq1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1.h, bq.h, xq1, 0, 0, 0);
          xq0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0.h, bql.h, xq0, 0, 0, 0);
          xq1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1.h, bql.h, xq1, 0, 0, 0);
          xb = __builtin_amdgcn_mfma_f32_16x16x32_f16(of.h, qpl.h, xb, 0, 0, 0);
        }
      }
    }
    float x[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[0][i] = __builtin_fmaf(xt0[i] + xb[i], kKUnit, xq0[i]);
      x[1][i] = __builtin_fmaf(xt1[i] + xb[i], kKUnit, xq1[i]);
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
        const float ah = __shfl(alpha, 4 * quad + i);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) acc[nt][i] *= ah;
        acc_off[i] *= ah;
      }
      m_run = m_new;
    }

    // ---- P V: slot j = 4mb + i of this lane is token 16mb + 4quad + i ----------------
    const float neg_mc = kPExp - m_run * kXScale;   // probabilities times 2^kPExp
    float p[8];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        p[4 * mb + i] = fast_exp2(__builtin_fmaf(x[mb][i], kXScale, neg_mc));
        l_run += p[4 * mb + i];
      }
    if constexpr (VT == 16) {
      PackB8 phi, plo;
      union { bf16x8 h; __bf16 e[8]; } hi, lo;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        hi.e[j] = static_cast<__bf16>(p[j]);
        lo.e[j] = static_cast<__bf16>(p[j] - static_cast<float>(hi.e[j]));
      }
      phi.h = hi.h;
      plo.h = lo.h;
#pragma unroll
      for (int nt = 0; nt < 8; ++nt) {
        PackB8 bv;
        bv.q = rv.o[nt];
        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi.h, bv.h, acc[nt], 0, 0, 0);
        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo.h, bv.h, acc[nt], 0, 0, 0);
      }
    } else {
      Pack8 ph;
#pragma unroll
      for (int j = 0; j < 4; ++j) ph.p[j] = half2v{static_cast<_Float16>(p[2 * j]), static_cast<_Float16>(p[2 * j + 1])};
      const Shifted<VT> vs = pre_shift<VT>(rv.s);
      Pack8 voff;
      voff.q = *reinterpret_cast<const uint4*>(s_vmeta + 256 + (quad * 4 + (l16 & 3)) * 16);
      if (l16 >= 4) voff.q = make_uint4(0, 0, 0, 0);
      acc_off = __builtin_amdgcn_mfma_f32_16x16x32_f16(ph.h, voff.h, acc_off, 0, 0, 0);
#pragma unroll
      for (int grp = 0; grp < 4; ++grp) {
        Pack8 sv, pa;
        sv.q = *reinterpret_cast<const uint4*>(s_vmeta + (quad * 4 + grp) * 16);
#pragma unroll
        for (int j = 0; j < 4; ++j) pa.p[j] = ph.p[j] * sv.p[j];
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const int nt = grp * 2 + h2;
          const half8 bv = unpack_operand<VT>(rv.s, vs, nt);
          acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa.h, bv, acc[nt], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();   // all reads of the LDS buffers are issued before they are overwritten
    if (more) load_v<VT>(rv, vd, next, lane);
  }

  // ---- merge the 4 wavefronts; acc[nt][i] is head 4quad+i, channel 16nt + l16 -----------------
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (quad == 0) {
    s_ml[(wave * 16 + l16) * 2] = m_run * kXScale - kPExp;   // log2 domain from here on
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
  if constexpr (VT != 16) {
#pragma unroll
    for (int grp = 0; grp < 4; ++grp)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float o = __shfl(acc_off[i], quad * 16 + grp);
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const int nt = 2 * grp + h2;
          const float unit = 16777216.0f / static_cast<float>(1 << field_bit<VT == 16 ? 8 : VT>(nt));
          acc[nt][i] = __builtin_fmaf(acc[nt][i], unit, o);
        }
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

template <int NK>
__global__ __launch_bounds__(kWG, 2) void decode_mixed_kernel(const Chunk* __restrict__ chunks,
                                                             const uint8_t* __restrict__ arena,
                                                             const ItemK* __restrict__ items_k,
                                                             const uint16_t* __restrict__ q, float* part_acc,
                                                             float* part_ml, int hq, int hkv) {
  extern __shared__ __align__(16) uint8_t smem[];
  // LDS: item layout | query rows (g x 128 bf16) | query operands (kMaxOps x 2 KiB) | per wavefront K tile, K and
  // V metadata | running maxima and sums | accumulators of the 4 wavefronts
  const Chunk ch = chunks[blockIdx.x];
  const int g = hq / hkv;
  const int seq = ch.item / hkv, head = ch.item % hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int quad = lane >> 4, l16 = lane & 15;
  ItemK& ik = *reinterpret_cast<ItemK*>(smem);
  uint16_t* s_qrow = reinterpret_cast<uint16_t*>(smem + kItemKBytes);
  uint8_t* s_qop = smem + kItemKBytes + 8 * kHeadDim * 2;
  uint8_t* s_waves = s_qop + kMaxOps * 2048;
  constexpr int kWaveBytes = NK * 1024 + kKMetaBytes + kVMetaBytes;
  float* s_ml = reinterpret_cast<float*>(s_waves + kWaves * kWaveBytes);
  float* s_acc = s_ml + kWaves * 16 * 2;

  for (int i = tid; i < static_cast<int>(sizeof(ItemK) / 4); i += kWG)
    reinterpret_cast<uint32_t*>(smem)[i] = reinterpret_cast<const uint32_t*>(items_k + ch.item)[i];
  const uint16_t* qp = q + (static_cast<int64_t>(seq) * hq + head * g) * kHeadDim;
  for (int i = tid; i < g * kHeadDim; i += kWG) s_qrow[i] = qp[i];
  __syncthreads();

  // query operands in sorted-channel order: lane (head l16, quad) of operand e holds the 8 slots of its quad.
  // Quantized tiers: slot pair p carries 2^(b (p % (8/b))) from its field position, undone here (times 2^kQExp).
  {
    int e = 0;
    for (int t = 0; t < 4; ++t) {
      const int nq = ik.nq[t], b = 16 >> t;
      for (int o = 0; 4 * o < nq; ++o, ++e) {
        if ((e & 3) != wave) continue;
        const int Q = 4 * o + quad;
        uint16_t raw[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int c = Q < nq ? ik.slot_ch[ik.slot_base[t] + 8 * Q + j] : -1;
          raw[j] = (c >= 0 && l16 < g) ? s_qrow[l16 * kHeadDim + c] : uint16_t(0);
        }
        uint8_t* dst = s_qop + e * 2048 + lane * 16;
        if (t == 0) {
          uint4 v;
          v.x = raw[0] | (static_cast<uint32_t>(raw[1]) << 16);
          v.y = raw[2] | (static_cast<uint32_t>(raw[3]) << 16);
          v.z = raw[4] | (static_cast<uint32_t>(raw[5]) << 16);
          v.w = raw[6] | (static_cast<uint32_t>(raw[7]) << 16);
          *reinterpret_cast<uint4*>(dst) = v;
        } else {
          half8 pre, plain;
          const int P = 8 / b;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float v = __uint_as_float(static_cast<uint32_t>(raw[j]) << 16);
            const int ex = kQExp - b * ((j >> 1) % P);
            plain[j] = static_cast<_Float16>(v);
            pre[j] = static_cast<_Float16>(ldexpf(v, ex));
          }
          *reinterpret_cast<half8*>(dst) = pre;
          *reinterpret_cast<half8*>(dst + 1024) = plain;
        }
      }
    }
  }
  __syncthreads();

  float* pa = part_acc + static_cast<int64_t>(ch.slot) * g * kHeadDim;
  float* pm = part_ml + static_cast<int64_t>(ch.slot) * g * 2;
  const uint8_t* kd = arena + ch.k_data;
  const uint8_t* km = arena + ch.k_meta;
  const uint8_t* vd = arena + ch.v_data;
  const uint8_t* vm = arena + ch.v_meta;
  uint8_t* s_wave = s_waves + wave * kWaveBytes;
  switch (ch.tier) {
    case 16: process_mixed<16, NK>(ik, kd, km, vd, vm, ch.rows, g, pa, pm, s_qop, s_wave, s_ml, s_acc); break;
    case 8: process_mixed<8, NK>(ik, kd, km, vd, vm, ch.rows, g, pa, pm, s_qop, s_wave, s_ml, s_acc); break;
    case 4: process_mixed<4, NK>(ik, kd, km, vd, vm, ch.rows, g, pa, pm, s_qop, s_wave, s_ml, s_acc); break;
    default: process_mixed<2, NK>(ik, kd, km, vd, vm, ch.rows, g, pa, pm, s_qop, s_wave, s_ml, s_acc); break;
  }
}

}  // namespace

hipError_t launch_decode_mixed(const Chunk* chunks, int n_chunks, const uint8_t* arena, const ItemK* items_k,
                               int max_kt_bytes, const uint16_t* q, float* part_acc, float* part_ml, int hq, int hkv,
                               hipStream_t st) {
  if (n_chunks == 0) return hipSuccess;
  const int g = hq / hkv;
  const int nk = max_kt_bytes <= 2048 ? 2 : max_kt_bytes <= 4096 ? 4 : 8;
  if (max_kt_bytes > 8192) return hipErrorInvalidValue;
  const size_t lds = kItemKBytes + 8 * kHeadDim * 2 + kMaxOps * 2048 +
                     static_cast<size_t>(kWaves) * (nk * 1024 + kKMetaBytes + kVMetaBytes) +
                     kWaves * 16 * 2 * sizeof(float) + static_cast<size_t>(kWaves) * g * kHeadDim * sizeof(float);
  dim3 grid(n_chunks), block(kWG);
  switch (nk) {
    case 2: hipLaunchKernelGGL(decode_mixed_kernel<2>, grid, block, lds, st, chunks, arena, items_k, q, part_acc, part_ml, hq, hkv); break;
    case 4: hipLaunchKernelGGL(decode_mixed_kernel<4>, grid, block, lds, st, chunks, arena, items_k, q, part_acc, part_ml, hq, hkv); break;
    default: hipLaunchKernelGGL(decode_mixed_kernel<8>, grid, block, lds, st, chunks, arena, items_k, q, part_acc, part_ml, hq, hkv); break;
  }
  return hipGetLastError();
}

}  // namespace rdkv
