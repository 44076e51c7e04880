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

// LDS: query operands [HS][4 groups][8 steps][4 heads] x 8 bytes, group sums [HS][hi, lo][4 heads] x 8 bytes,
// then the merge area
template <int HS>
struct Lds {
  static constexpr int kQop = HS * 4 * 8 * 4 * 8;
  static constexpr int kQsum = HS * 2 * 4 * 8;
};

// One piece of a workgroup's work: `rows` rows of one tier of one item, NWV wavefronts interleaving over its tiles.
// The running softmax state `run` carries over from piece to piece (a workgroup may go through several tiers of its
// item); the sums that carry the lane's factor kappa of this tier take it on entry and give it back on exit.
template <int TIER, int HS, int NWV>
__device__ __forceinline__ void process_tiles(const uint8_t* __restrict__ kd, const uint8_t* __restrict__ km,
                                              const uint8_t* __restrict__ vd, const uint8_t* __restrict__ vm,
                                              int rows, int g, const uint16_t* __restrict__ q, Run<HS>& run,
                                              uint8_t* smem) {
  constexpr int kWG = NWV * 64, kWaves = NWV;
  using S = Step<TIER>;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int blk = lane >> 2, j = lane & 3;
  const uint8_t* s_qop = smem;
  const uint8_t* s_qsum = smem + Lds<HS>::kQop;

  const int ntiles = (rows + kTile - 1) / kTile;

  // ---- first tile's loads, issued before anything waits ------------------------------------------------
  // The 4- and 2-bit tiers keep K and V of a tile in separate registers and refill each right after its last use,
  // so a wavefront always has its next tile in flight.  An 8-bit tile is 18 KiB: there the K and V codes take turns
  // in one register set (the other wavefronts of the SIMD cover the wait) and the kernel stays within 128 registers.
  constexpr bool kShare = TIER == 8;
  constexpr int kDepth = (TIER == 2 && HS == 1) ? 2 : 1;   // a 2-bit tile is only 6 KiB: two per wavefront in flight
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

  // ---- query operands (once per piece: the field positions folded into them depend on the tier; the caller puts
  // a barrier between two pieces) ------------------------------------------------------------------------------
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

  const float lk = v_log2_kappa<TIER>(blk);
  {
    const float kappa = __builtin_ldexpf(1.0f, static_cast<int>(lk));
#pragma unroll
    for (int hs = 0; hs < HS; ++hs) {
      run.l[hs] *= kappa;
#pragma unroll
      for (int i = 0; i < 4; ++i) run.offv[hs][i] *= kappa;
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
      // The query operands come from LDS two steps at a time.  With one head set the read of the next pair of steps
      // is issued before the products of the current pair, so that they cover the LDS latency; with two head sets
      // the extra operand registers would spill, and the pair is read where it is used.
      constexpr bool kAhead = HS == 1;
      auto qread = [&](int hs, int grp, int st) __attribute__((always_inline)) {
        return *reinterpret_cast<const uint2*>(s_qop + (((hs * 4 + grp) * 8 + st) * 4 + j) * 8);
      };
      uint2 bq[kAhead ? 2 : 1][HS][2];
      if constexpr (kAhead) {
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) {
          bq[0][hs][0] = qread(hs, 0, 0);
          bq[0][hs][1] = qread(hs, 0, 1);
        }
      }
#pragma unroll
      for (int grp = 0; grp < 4; ++grp) {
        __builtin_amdgcn_sched_barrier(0);   // keep a group's unpacked words next to their use (register pressure)
        uint32_t gw[S::kCopies][TIER];
        group_words<TIER>(kraw, grp, gw);
        floatx4 dg[HS];
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) dg[hs] = zero4;
#pragma unroll
        for (int sp = 0; sp < 4; ++sp) {
          const int cur = kAhead ? (grp * 4 + sp) & 1 : 0;
          if constexpr (kAhead) {
            if (!(grp == 3 && sp == 3)) {
              const int ngrp = sp == 3 ? grp + 1 : grp, nst = sp == 3 ? 0 : 2 * (sp + 1);
#pragma unroll
              for (int hs = 0; hs < HS; ++hs) {
                bq[cur ^ 1][hs][0] = qread(hs, ngrp, nst);
                bq[cur ^ 1][hs][1] = qread(hs, ngrp, nst + 1);
              }
            }
            __builtin_amdgcn_sched_barrier(0);
          } else {
#pragma unroll
            for (int hs = 0; hs < HS; ++hs) {
              bq[0][hs][0] = qread(hs, grp, 2 * sp);
              bq[0][hs][1] = qread(hs, grp, 2 * sp + 1);
            }
          }
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const half4 a = step_operand<TIER>(gw, 2 * sp + e);
#pragma unroll
            for (int hs = 0; hs < HS; ++hs) {
              Pack4 b;
              b.u[0] = bq[cur][hs][e].x;
              b.u[1] = bq[cur][hs][e].y;
              dg[hs] = __builtin_amdgcn_mfma_f32_4x4x4f16(a, b.h, dg[hs], 0, 0, 0);
            }
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

    mask_rows<HS>(x, tile, rows, blk);
    float p[HS][4];
    softmax_tile<HS>(x, run, p, lk);
    pv_tile<TIER, HS>(vraw, vmeta, p, run);
    if (more) {               // V registers are free again
      if constexpr (kShare) load_k(r, next); else load_v(r, next);
    }
  };
  for (int tile = wave; tile < ntiles; tile += kDepth * kWaves) {
#pragma unroll
    for (int dd = 0; dd < kDepth; ++dd)
      if (tile + dd * kWaves < ntiles) do_tile(regs[dd], tile + dd * kWaves);
  }

  {   // the piece is done: the lane's factor leaves the sums again
    const float inv_kappa = __builtin_ldexpf(1.0f, static_cast<int>(-lk));
#pragma unroll
    for (int hs = 0; hs < HS; ++hs) {
      run.l[hs] *= inv_kappa;
#pragma unroll
      for (int i = 0; i < 4; ++i) run.offv[hs][i] *= inv_kappa;
    }
  }
}

// MULTI: workgroups may go through several tiers of their item (Chunk::next); without it every chunk is one tier and
// the tier's body ends in its own copy of the chunk's end, which saves a latency-bound launch 0.3 us.
template <int HS, int NWV, bool MULTI>
__global__ __launch_bounds__(NWV * 64, HS == 1 ? 4 : 3) void decode_tiles_kernel(
    const Chunk* __restrict__ chunks, int first, const uint8_t* __restrict__ arena, const uint16_t* __restrict__ q,
    MergeArgs ma, const int32_t* __restrict__ tail_len) {
  extern __shared__ __align__(16) uint8_t smem[];
  Chunk ch = chunks[first + blockIdx.x];
  const int g = ma.hq / ma.hkv;
  const int seq = ch.item / ma.hkv, head = ch.item % ma.hkv;
  const uint16_t* qp = q + (static_cast<int64_t>(seq) * ma.hq + head * g) * kHeadDim;
  const ChunkOut co{ch.item, ch.slot, ch.slot0, ch.nslots};
  float* s_ml = reinterpret_cast<float*>(smem + Lds<HS>::kQop + Lds<HS>::kQsum);   // [NWV][4 HS][2]
  float* s_acc = s_ml + NWV * 4 * HS * 2;                                          // [2 NWV streams][g][128]
  if (ch.tier == kTierTail) {   // appended tokens: 64-token tiles of bf16 rows, as many rows as exist so far
    const int rows = max(0, min(ch.rows, *tail_len - ch.row0));
    process_tail_tiles<HS, false, NWV>(arena + ch.k_data, arena + ch.v_data, rows, g, qp, smem, s_ml, s_acc, ma, co);
    return;
  }
  if constexpr (!MULTI) {
#define RDKV_ONE(TIER_)                                                                                           \
  {                                                                                                               \
    Run<HS> run;                                                                                                  \
    run.init();                                                                                                   \
    process_tiles<TIER_, HS, NWV>(arena + ch.k_data, arena + ch.k_meta, arena + ch.v_data, arena + ch.v_meta,     \
                                  ch.rows, g, qp, run, smem);                                                     \
    finish_chunk<HS, false, NWV>(run, 16777216.0f, 0.f, g, s_ml, s_acc, ma, co);                                  \
  }
    switch (ch.tier) {
      case 8: RDKV_ONE(8) break;
      case 4: RDKV_ONE(4) break;
      default: RDKV_ONE(2) break;
    }
#undef RDKV_ONE
    return;
  }
  // The workgroup's pieces: runs of rows of the item's quantized tiers on one softmax state.  A share of an item's
  // work goes through the tiers in the order 2, 4, 8 bits, so the chain is at most three pieces long and the three
  // tier bodies follow each other in a straight line (a loop around a switch made the compiler spill the state).
  Run<HS> run;
  run.init();
#define RDKV_PIECE(TIER_)                                                                                         \
  if (ch.tier == (TIER_)) {                                                                                       \
    const int next = ch.next;                                                                                     \
    process_tiles<TIER_, HS, NWV>(arena + ch.k_data, arena + ch.k_meta, arena + ch.v_data, arena + ch.v_meta,     \
                                  ch.rows, g, qp, run, smem);                                                     \
    if (next >= 0) {                                                                                              \
      __syncthreads(); /* this piece's readers of the query operands are done */                                  \
      ch = chunks[next];                                                                                          \
    } else {                                                                                                      \
      ch.tier = 0;                                                                                                \
    }                                                                                                             \
  }
  RDKV_PIECE(2)
  RDKV_PIECE(4)
  RDKV_PIECE(8)
#undef RDKV_PIECE
  // ---- undo the subnormal unit, add the offsets, merge the wavefronts, hand the partial over -------------------
  finish_chunk<HS, false, NWV>(run, 16777216.0f, 0.f, g, s_ml, s_acc, ma, co);
}

template <int HS, int NWV, bool MULTI>
hipError_t launch_tiles(const Chunk* chunks, int first, int n_chunks, const uint8_t* arena, const uint16_t* q,
                        const MergeArgs& ma, const int32_t* tail_len, hipStream_t st) {
  const int g = ma.hq / ma.hkv;
  const size_t merge_area = static_cast<size_t>(2 * NWV) * g * kHeadDim * sizeof(float);
  static_assert(2 * NWV * 128 >= merge::merge_lds_floats(NWV * 64, 1), "the merge reuses the wavefront merge area");
  const size_t lds = Lds<HS>::kQop + Lds<HS>::kQsum + NWV * 4 * HS * 2 * sizeof(float) + merge_area;
  hipLaunchKernelGGL((decode_tiles_kernel<HS, NWV, MULTI>), dim3(n_chunks), dim3(NWV * 64), lds, st, chunks, first,
                     arena, q, ma, tail_len);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_tiles(const Chunk* chunks, int first, int n_chunks, bool multi, const uint8_t* arena,
                               const uint16_t* q, const MergeArgs& ma, const int32_t* tail_len, hipStream_t st) {
  if (n_chunks == 0) return hipSuccess;
  const int g = ma.hq / ma.hkv;
  // up to 4 query heads per KV head: one head set, workgroups of eight wavefronts; 8 heads: two head sets (166
  // registers, three wavefronts per SIMD), workgroups of four
  if (g > 4) {
    if (multi) return launch_tiles<2, 4, true>(chunks, first, n_chunks, arena, q, ma, tail_len, st);
    return launch_tiles<2, 4, false>(chunks, first, n_chunks, arena, q, ma, tail_len, st);
  }
  if (multi) return launch_tiles<1, 8, true>(chunks, first, n_chunks, arena, q, ma, tail_len, st);
  return launch_tiles<1, 8, false>(chunks, first, n_chunks, arena, q, ma, tail_len, st);
}

}  // namespace rdkv
