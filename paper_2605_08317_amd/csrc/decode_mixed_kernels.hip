// Split-K flash-decode over a mixed-mode cache (Sec. 3.2 Stages 2-3, Sec. 3.3): V token-wise, K channel-wise on
// the retained tokens, on the gfx950 matrix cores (v_mfma_f32_4x4x4_16B, sixteen independent 4x4x4 blocks).
//
// K side.  A retained token's K row is a run of 32-bit words in sorted-channel order (16-bit words first, then
// 8-, 4- and 2-bit words); a lane of the wavefront is a token of the 64-token tile and holds its row in registers.
// With per-channel quantization the logit is sum_c (s_c q_c) code_c + sum_c m_c q_c (fusion identity of App. B).
// Here a channel's scale belongs to a group of 32 retained tokens (half a tile), so the scaled query is rebuilt
// per tile: lane i of a token group multiplies the four query heads of step i (4 channel slots) by the step's four
// scales, keeps the product as an exact sum of two fp16 terms (a single rounded term costs ~2.5e-3 of output error
// with x10 outlier channels), parks both in the wavefront's LDS table, and adds its share of sum_c m_c q_c, which
// a lane-transposing reduction turns into one bias per (token group, head).  The main loop then walks the row's
// words -- word index static, tier boundaries run-time but uniform -- turning each word into one, two or four
// steps of fp16-subnormal codes (one AND per pair of codes) times the step's scaled query from LDS.  16-bit
// channels go through the bf16 instruction with the raw bf16 query (exact products).
//
// V side, softmax and the end-of-chunk merge are the stages shared with the token-wise kernel; 16-bit V rows are
// 64-token tiles of bf16 with the same lane assignment, multiplied by the probabilities as two bf16 terms.
//
// This file is compiled once per head-set count (-DRDKV_MIXED_HS=1: up to 4 query heads per KV head, =2: 8) and row
// length class (-DRDKV_MIXED_LONG=0: K rows of up to 32 words, =1: up to 68), each into an object of its own, so
// that the many instantiations build in parallel.
#include "decode_tile_common.h"

#if !defined(RDKV_MIXED_HS) || !defined(RDKV_MIXED_LONG)
#error "compile with -DRDKV_MIXED_HS=1 or 2 and -DRDKV_MIXED_LONG=0 (K rows of up to 32 words) or 1 (up to 68)"
#endif

namespace rdkv {

namespace {

using namespace tile;

// Wavefronts per workgroup: four, or eight for launches that fit the chip in one round (half as many partials per
// item for the same number of wavefronts in flight; every chunk costs its item an arrival and a partial to merge).

// LDS: query operands per step [steps][HS][4 heads] x 8 bytes (raw bf16 for 16-bit steps, fp16 q * 2^(kQExp - fb)
// for quantized ones), fp16 q * 2^kQExp per quantized step (for the offsets), then per wavefront the scaled-query
// table [2 token groups][quantized steps][HS][4 heads] x 16 bytes (high terms, low terms).  The merge area of the
// chunk's end reuses the same memory.
struct LdsPlan {
  int qpre, qraw, wtab, wtab_wave, total;
  __host__ __device__ LdsPlan(int n_steps, int n_qsteps, int hs, int g, int kWaves) {
    qpre = 0;
    qraw = qpre + n_steps * hs * 32;
    wtab = qraw + n_qsteps * hs * 32;
    wtab_wave = (2 * n_qsteps + 1) * hs * 64;   // one entry of padding: the step loop reads one entry ahead
    const int tables = wtab + kWaves * wtab_wave;
    const int merge = kWaves * 4 * hs * 2 * 4 + 2 * kWaves * g * kHeadDim * 4;
    total = tables > merge ? tables : merge;
  }
};

// bit offset left after the copy shift of field f of a 16-bit half (tier b): the code reads as code * 2^fb * 2^-24
__device__ __forceinline__ int field_fb(int b, int f) { return b == 2 ? 2 * (f % 3) : b == 4 ? 4 * (f % 2) : 0; }

template <int VT, int NW, int HS, int NWV>
__device__ __forceinline__ void process_mixed(const Chunk& ch, const uint8_t* __restrict__ arena,
                                              const ItemK* __restrict__ ikp, int g, const uint16_t* __restrict__ q,
                                              const MergeArgs& ma, const ChunkOut& co,
                                              uint8_t* smem, int lds_steps, int lds_qsteps, bool per_unit) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int blk = lane >> 2, j = lane & 3, G = lane >> 5;
  const int rows = ch.rows;
  const int ntiles = (rows + kTile - 1) / kTile;

  // shape of the item's K rows (uniform over the workgroup; it travels with the chunk so that the first loads
  // need not wait for a second dependent fetch)
  const int e16 = ch.k_word_end[0], e8 = ch.k_word_end[1], e4 = ch.k_word_end[2], e2 = ch.k_word_end[3];
  const int nwp = (e2 + 1) & ~1;
  const int ns16 = e16 >> 1;
  const int nqs = (e8 - e16) + 2 * (e4 - e8) + 4 * (e2 - e4);
  const int n_steps = ns16 + nqs;
  const int kt_bytes = 256 * nwp, km_bytes = 32 * nqs;
  constexpr int kWaves = NWV, kWG = NWV * 64;
  const LdsPlan plan(lds_steps, lds_qsteps, HS, g, kWaves);   // the launch sized LDS for the largest item of the cache
  const uint8_t* s_qpre = smem + plan.qpre;
  const uint8_t* s_qraw = smem + plan.qraw;
  uint8_t* s_wtab = smem + plan.wtab + wave * plan.wtab_wave;

  const uint8_t* kd = arena + ch.k_data;
  const uint8_t* km = arena + ch.k_meta;
  const uint8_t* vd = arena + ch.v_data;
  const uint8_t* vm = arena + ch.v_meta;

  // ---- registers of a tile and their loads ------------------------------------------------------------------
  uint32_t kw[NW];      // the lane's token: its K row
  uint4 kmeta[2];       // scales (x, y), offsets (z, w) of quantized step lane % 32 (+ 32) of this lane's token group
  // V codes: 4- and 2-bit tiles sit whole in registers; 8- and 16-bit tiles stream through two 32-byte buffers
  // (an 8-bit channel group, half a 16-bit one), the next piece in flight while the current one is multiplied
  constexpr bool kStream = VT >= 8;
  constexpr int kVRegs = kStream ? 2 : VT;
  constexpr int kPieces = VT == 16 ? 8 : 4;          // pieces of a streamed tile
  uint4 vraw[kStream ? 2 : 1][kVRegs], vmeta;
  auto load_k = [&](int t) __attribute__((always_inline)) {
    const uint8_t* p = kd + static_cast<int64_t>(t) * kt_bytes;
#pragma unroll
    for (int u = 0; u < NW / 4; ++u) {
      // every word is assigned on every path (stores under the branches get merged into stores through a selected
      // pointer, which keeps the array out of registers)
      uint4 v = make_uint4(0, 0, 0, 0);
      if (4 * u + 3 < nwp) {
        v = *reinterpret_cast<const uint4*>(p + 1024 * u + 16 * lane);
      } else if (4 * u + 1 < nwp) {   // the row's last two words
        const uint2 t2 = *reinterpret_cast<const uint2*>(p + 1024 * u + 8 * lane);
        v.x = t2.x;
        v.y = t2.y;
      }
      kw[4 * u] = v.x; kw[4 * u + 1] = v.y; kw[4 * u + 2] = v.z; kw[4 * u + 3] = v.w;
    }
    if (!per_unit) {   // scales per group of 32 tokens: a record per tile and token group
      const uint8_t* pm = km + static_cast<int64_t>(t) * km_bytes;
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const int sq = (lane & 31) + 32 * it;
        kmeta[it] = make_uint4(0, 0, 0, 0);
        if (sq < nqs) kmeta[it] = *reinterpret_cast<const uint4*>(pm + (G * nqs + sq) * 16);
      }
    }
  };
  auto load_v_piece = [&](int t, int piece, uint4 (&dst)[kVRegs]) __attribute__((always_inline)) {
    const uint8_t* p = vd + static_cast<int64_t>(t) * (kTile * 16 * VT) + 2048 * piece + 16 * lane;
    dst[0] = *reinterpret_cast<const uint4*>(p);
    dst[1] = *reinterpret_cast<const uint4*>(p + 1024);
  };
  auto load_v = [&](int t) __attribute__((always_inline)) {
    if constexpr (kStream) load_v_piece(t, 0, vraw[0]);
    else load_tile_side<VT>(vraw[0], vd, t, lane);
    if constexpr (VT != 16) vmeta = *reinterpret_cast<const uint4*>(vm + static_cast<int64_t>(t) * 1024 + lane * 16);
  };
#pragma unroll
  for (int w = 0; w < NW; ++w) kw[w] = 0;
  kmeta[0] = kmeta[1] = vmeta = make_uint4(0, 0, 0, 0);
  if (per_unit) {      // one scale per channel over all retained tokens (App. B): a single record per segment
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int sq = (lane & 31) + 32 * it;
      if (sq < nqs) kmeta[it] = *reinterpret_cast<const uint4*>(km + sq * 16);
    }
  }
  if (wave < ntiles) {
    load_k(wave);
    load_v(wave);
  }

  // ---- query operands per step (once per workgroup) ---------------------------------------------------------
  for (int e = tid; e < n_steps * HS * 4; e += kWG) {
    const int s = e / (HS * 4), hs = (e >> 2) % HS, hj = e & 3;
    const int head = 4 * hs + hj;
    float v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int c = ikp->slot_ch[4 * s + k];
      v[k] = (c >= 0 && head < g) ? __uint_as_float(static_cast<uint32_t>(q[head * kHeadDim + c]) << 16) : 0.f;
    }
    uint2 out;
    if (s < ns16) {   // raw bf16
      out.x = (__float_as_uint(v[0]) >> 16) | (__float_as_uint(v[1]) & 0xFFFF0000u);
      out.y = (__float_as_uint(v[2]) >> 16) | (__float_as_uint(v[3]) & 0xFFFF0000u);
    } else {
      const int sq = s - ns16;
      int b, k;   // tier of the step and its position inside its word
      if (sq < e8 - e16) { b = 8; k = 0; }
      else if (sq < (e8 - e16) + 2 * (e4 - e8)) { b = 4; k = (sq - (e8 - e16)) & 1; }
      else { b = 2; k = (sq - (e8 - e16) - 2 * (e4 - e8)) & 3; }
      const float f0 = ldexpf(1.0f, kQExp - field_fb(b, 2 * k)), f1 = ldexpf(1.0f, kQExp - field_fb(b, 2 * k + 1));
      Pack4 o, r;
      o.h[0] = static_cast<_Float16>(v[0] * f0); o.h[1] = static_cast<_Float16>(v[1] * f0);
      o.h[2] = static_cast<_Float16>(v[2] * f1); o.h[3] = static_cast<_Float16>(v[3] * f1);
      const float fr = static_cast<float>(1 << kQExp);
#pragma unroll
      for (int k2 = 0; k2 < 4; ++k2) r.h[k2] = static_cast<_Float16>(v[k2] * fr);
      out = make_uint2(o.u[0], o.u[1]);
      *reinterpret_cast<uint2*>(smem + plan.qraw + ((sq * HS + hs) * 4 + hj) * 8) = make_uint2(r.u[0], r.u[1]);
    }
    *reinterpret_cast<uint2*>(smem + plan.qpre + ((s * HS + hs) * 4 + hj) * 8) = out;
  }
  __syncthreads();

  const float lk = VT == 16 ? 0.0f : v_log2_kappa<(VT == 16 ? 8 : VT)>(blk);
  Run<HS> run;
  run.init();
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};

  // ---- scaled query of a tile's two token groups, and the bias sum_c m_c q_c ------------------------------------
  // (per tile with 32-token groups; once per wavefront when a channel has one scale for all its tokens -- the
  // paper's "scaled query computed once per decode step")
  float bias[HS];
  auto prep = [&]() __attribute__((always_inline)) {
    {
      float bp[HS][4];
#pragma unroll
      for (int hs = 0; hs < HS; ++hs)
#pragma unroll
        for (int h = 0; h < 4; ++h) bp[hs][h] = 0.f;
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        if (32 * it < nqs) {   // uniform
          const int sq = (lane & 31) + 32 * it;
          Pack4 sc, mo;
          sc.u[0] = kmeta[it].x; sc.u[1] = kmeta[it].y;
          mo.u[0] = kmeta[it].z; mo.u[1] = kmeta[it].w;
          if (sq < nqs) {
#pragma unroll
            for (int hs = 0; hs < HS; ++hs) {
              const uint4* qp = reinterpret_cast<const uint4*>(s_qpre + ((ns16 + sq) * HS + hs) * 32);
              const uint4* qr = reinterpret_cast<const uint4*>(s_qraw + (sq * HS + hs) * 32);
              const uint4 qa = qp[0], qb = qp[1], ra = qr[0], rb = qr[1];
              const uint32_t qw[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
              const uint32_t rw[8] = {ra.x, ra.y, ra.z, ra.w, rb.x, rb.y, rb.z, rb.w};
              uint4* dst = reinterpret_cast<uint4*>(s_wtab + ((G * nqs + sq) * HS + hs) * 64);
#pragma unroll
              for (int h = 0; h < 4; ++h) {
                Pack4 qv, rv, hi, lo;
                qv.u[0] = qw[2 * h]; qv.u[1] = qw[2 * h + 1];
                rv.u[0] = rw[2 * h]; rv.u[1] = rw[2 * h + 1];
#pragma unroll
                for (int pr = 0; pr < 2; ++pr) {
                  hi.p[pr] = qv.p[pr] * sc.p[pr];
                  lo.p[pr] = __builtin_elementwise_fma(qv.p[pr], sc.p[pr], -hi.p[pr]);
                }
                dst[h] = make_uint4(hi.u[0], hi.u[1], lo.u[0], lo.u[1]);
                bp[hs][h] = __builtin_amdgcn_fdot2(rv.p[0], mo.p[0], bp[hs][h], false);
                bp[hs][h] = __builtin_amdgcn_fdot2(rv.p[1], mo.p[1], bp[hs][h], false);
              }
            }
          }
        }
      }
      // lane (block, head j) ends with the sum over its token group's 32 lanes of bp[.][j]
#pragma unroll
      for (int hs = 0; hs < HS; ++hs) {
        const bool o1 = (j & 1) != 0, o2 = (j & 2) != 0;
        float k0 = o1 ? bp[hs][1] : bp[hs][0], s0 = o1 ? bp[hs][0] : bp[hs][1];
        float k1 = o1 ? bp[hs][3] : bp[hs][2], s1 = o1 ? bp[hs][2] : bp[hs][3];
        k0 += dpp_f32<0xB1>(s0);   // quad_perm [1, 0, 3, 2]
        k1 += dpp_f32<0xB1>(s1);
        float kk = o2 ? k1 : k0, ss = o2 ? k0 : k1;
        kk += dpp_f32<0x4E>(ss);   // quad_perm [2, 3, 0, 1]
        kk += dpp_f32<0x124>(kk);  // row_ror:4
        kk += dpp_f32<0x128>(kk);  // row_ror:8
        kk += __shfl_xor(kk, 16);
        bias[hs] = kk;
      }
    }
    wave_lds_sync();
  };
  if (per_unit) prep();

  for (int tile = wave; tile < ntiles; tile += kWaves) {
    const int next = tile + kWaves;
    const bool more = next < ntiles;
    if (!per_unit) prep();

    // ---- logits x[hs][i] of token 4 blk + i and head 4 hs + j, in units of kKUnit ----------------------------
    float x[HS][4];
    {
      floatx4 a16[HS], aqh[HS], aql[HS];
#pragma unroll
      for (int hs = 0; hs < HS; ++hs) a16[hs] = aqh[hs] = aql[hs] = zero4;
      // The tier boundaries are laundered once per tile: as loop invariants the comparisons below would be
      // evaluated ahead of the tile loop and kept in scalar registers (thousands of spills).
      int t16 = e16, t8 = e8, t4 = e4, t2 = e2;
      asm volatile("" : "+s"(t16), "+s"(t8), "+s"(t4), "+s"(t2));
      // table address of word w's first step = tier base + w * (steps per word) * HS * 64
      const uint8_t* wt = s_wtab + G * nqs * HS * 64 + j * 16;
      const uint8_t* wt8 = wt - t16 * (HS * 64);
      const uint8_t* wt4 = wt + ((t8 - t16) - 2 * t8) * (HS * 64);
      const uint8_t* wt2 = wt + ((t8 - t16) + 2 * (t4 - t8) - 4 * t4) * (HS * 64);
      // The quantized steps of a row (8-, 4-, then 2-bit words) are consecutive entries of the table.  With one
      // head set every step asks for the next entry before its own products, so that they cover the LDS latency
      // (the entry after the last step is padding); with two head sets those registers would spill.
      constexpr bool kAhead = HS == 1;
      uint4 bq[HS];
      if constexpr (kAhead) {
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) bq[hs] = *reinterpret_cast<const uint4*>(wt + hs * 64);
      }
      auto qstep = [&](const Pack4& a, const uint8_t* o) __attribute__((always_inline)) {
        uint4 nx[HS];
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) {
          if constexpr (kAhead) nx[hs] = *reinterpret_cast<const uint4*>(o + (HS + hs) * 64);
          else bq[hs] = *reinterpret_cast<const uint4*>(o + hs * 64);
        }
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) {
          Pack4 bh, bl;
          bh.u[0] = bq[hs].x; bh.u[1] = bq[hs].y;
          bl.u[0] = bq[hs].z; bl.u[1] = bq[hs].w;
          aqh[hs] = __builtin_amdgcn_mfma_f32_4x4x4f16(a.h, bh.h, aqh[hs], 0, 0, 0);
          aql[hs] = __builtin_amdgcn_mfma_f32_4x4x4f16(a.h, bl.h, aql[hs], 0, 0, 0);
        }
        if constexpr (kAhead) {
#pragma unroll
          for (int hs = 0; hs < HS; ++hs) bq[hs] = nx[hs];
        }
      };
      // one word of each tier; the word index is a compile-time constant (registers cannot be indexed at run time)
      auto body16 = [&](auto wc) __attribute__((always_inline)) {   // a 16-bit step = two words = four bf16
        constexpr int w = decltype(wc)::value;
        if constexpr ((w & 1) == 0 && w + 1 < NW) {
          // the two words pass through an empty asm: read as one 8-byte vector straight from kw[], the pair would
          // keep the whole array out of registers (scalar replacement gives up on mixed-width accesses)
          uint32_t lo = kw[w], hi = kw[w + 1];
          asm("" : "+v"(lo), "+v"(hi));
          const short4v a = bf4(lo, hi);
#pragma unroll
          for (int hs = 0; hs < HS; ++hs) {
            const uint2 braw = *reinterpret_cast<const uint2*>(s_qpre + (((w >> 1) * HS + hs) * 4 + j) * 8);
            a16[hs] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, bf4(braw.x, braw.y), a16[hs], 0, 0, 0);
          }
        }
      };
      auto body8 = [&](auto wc) __attribute__((always_inline)) {
        constexpr int w = decltype(wc)::value;
        Pack4 a;
        a.u[0] = __builtin_amdgcn_perm(0u, kw[w], 0x0C020C00u);
        a.u[1] = __builtin_amdgcn_perm(0u, kw[w], 0x0C030C01u);
        qstep(a, wt8 + w * (HS * 64));
      };
      auto body4 = [&](auto wc) __attribute__((always_inline)) {
        constexpr int w = decltype(wc)::value;
        const uint32_t c0 = kw[w], c1 = c0 >> 8;
        const uint8_t* o = wt4 + 2 * w * (HS * 64);
        Pack4 a;
        a.u[0] = c0 & 0x000F000Fu; a.u[1] = c0 & 0x00F000F0u;
        qstep(a, o);
        a.u[0] = c1 & 0x000F000Fu; a.u[1] = c1 & 0x00F000F0u;
        qstep(a, o + HS * 64);
      };
      auto body2 = [&](auto wc) __attribute__((always_inline)) {
        constexpr int w = decltype(wc)::value;
        const uint32_t c0 = kw[w], c1 = c0 >> 6, c2 = c0 >> 12;
        const uint8_t* o = wt2 + 4 * w * (HS * 64);
        Pack4 a;
        a.u[0] = c0 & 0x00030003u; a.u[1] = c0 & 0x000C000Cu;     // fields 0, 1
        qstep(a, o);
        a.u[0] = c0 & 0x00300030u; a.u[1] = c1 & 0x00030003u;     // fields 2, 3
        qstep(a, o + HS * 64);
        a.u[0] = c1 & 0x000C000Cu; a.u[1] = c1 & 0x00300030u;     // fields 4, 5
        qstep(a, o + 2 * HS * 64);
        a.u[0] = c2 & 0x00030003u; a.u[1] = c2 & 0x000C000Cu;     // fields 6, 7
        qstep(a, o + 3 * HS * 64);
      };
      // A tier is a run of consecutive words [first, end): jump to its first word and fall through word by word
      // until the end (one uniform comparison per word; a test of every word against every tier costs several
      // times the branches and leaves accumulator copies at every merge).
#define RDKV_K_CASE(BODY_, END_, W_)                \
  case (W_):                                        \
    if constexpr ((W_) < NW) {                      \
      if ((W_) >= (END_)) break;                    \
      BODY_(GroupIndex<(W_)>{});                    \
    }                                               \
    [[fallthrough]];
#define RDKV_K_CASE4(BODY_, END_, W_) \
  RDKV_K_CASE(BODY_, END_, W_) RDKV_K_CASE(BODY_, END_, W_ + 1) RDKV_K_CASE(BODY_, END_, W_ + 2) RDKV_K_CASE(BODY_, END_, W_ + 3)
#define RDKV_K_CASE16(BODY_, END_, W_) \
  RDKV_K_CASE4(BODY_, END_, W_) RDKV_K_CASE4(BODY_, END_, W_ + 4) RDKV_K_CASE4(BODY_, END_, W_ + 8) RDKV_K_CASE4(BODY_, END_, W_ + 12)
#define RDKV_K_TIER(BODY_, FIRST_, END_)                                                                      \
  switch (FIRST_) {                                                                                           \
    RDKV_K_CASE16(BODY_, END_, 0) RDKV_K_CASE16(BODY_, END_, 16) RDKV_K_CASE16(BODY_, END_, 32)               \
    RDKV_K_CASE16(BODY_, END_, 48) RDKV_K_CASE4(BODY_, END_, 64)                                              \
    default: break;                                                                                           \
  }
      RDKV_K_TIER(body16, 0, t16)
      RDKV_K_TIER(body8, t16, t8)
      RDKV_K_TIER(body4, t8, t4)
      RDKV_K_TIER(body2, t4, t2)
#undef RDKV_K_TIER
#undef RDKV_K_CASE16
#undef RDKV_K_CASE4
#undef RDKV_K_CASE
#pragma unroll
      for (int hs = 0; hs < HS; ++hs)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          x[hs][i] = __builtin_fmaf(a16[hs][i], kKUnit, aqh[hs][i] + aql[hs][i]) + bias[hs] * (1.0f / 16777216.0f);
    }
    if (more) load_k(next);   // K registers are free again

    mask_rows<HS>(x, tile, rows, blk);
    float p[HS][4];
    softmax_tile<HS>(x, run, p, lk);

    // ---- P V ------------------------------------------------------------------------------------------------
    if constexpr (VT == 16) {
      // bf16 rows: p as two truncated bf16 terms (the remainder of the first is exact in fp32)
      short4v phi[HS], plo[HS];
#pragma unroll
      for (int hs = 0; hs < HS; ++hs) split_bf16(p[hs], phi[hs], plo[hs]);
#define RDKV_PV16_STEP(G_, A_, X_, Y_)                                                                          \
  {                                                                                                            \
    const short4v b = bf4(X_, Y_);                                                                             \
    _Pragma("unroll") for (int hs = 0; hs < HS; ++hs) {                                                        \
      run.acc[hs][G_] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(phi[hs], b, run.acc[hs][G_], 3, A_, 0);         \
      run.acc[hs][G_] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(plo[hs], b, run.acc[hs][G_], 3, A_, 0);         \
    }                                                                                                          \
  }
      // piece P_ = half H_ of channel group G_: tokens 16 H_ .. 16 H_ + 15 of this lane's token half
#define RDKV_PV16_PIECE(G_, H_)                                                                                \
  {                                                                                                            \
    constexpr int P_ = 2 * G_ + H_;                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                                         \
    if (P_ + 1 < kPieces) load_v_piece(tile, P_ + 1, vraw[(P_ + 1) & 1]);                                      \
    else if (more) load_v_piece(next, 0, vraw[0]);                                                             \
    const uint4(&v)[kVRegs] = vraw[P_ & 1];                                                                    \
    RDKV_PV16_STEP(G_, 4 * H_ + 0, v[0].x, v[0].y) RDKV_PV16_STEP(G_, 4 * H_ + 1, v[0].z, v[0].w)              \
    RDKV_PV16_STEP(G_, 4 * H_ + 2, v[1].x, v[1].y) RDKV_PV16_STEP(G_, 4 * H_ + 3, v[1].z, v[1].w)              \
  }
      RDKV_PV16_PIECE(0, 0) RDKV_PV16_PIECE(0, 1) RDKV_PV16_PIECE(1, 0) RDKV_PV16_PIECE(1, 1)
      RDKV_PV16_PIECE(2, 0) RDKV_PV16_PIECE(2, 1) RDKV_PV16_PIECE(3, 0) RDKV_PV16_PIECE(3, 1)
#undef RDKV_PV16_PIECE
#undef RDKV_PV16_STEP
    } else if constexpr (VT == 8) {
      pv_tile_groups<8, HS>(
          [&](auto gi, uint32_t (&gw)[1][8]) __attribute__((always_inline)) {
            constexpr int P = decltype(gi)::value;
            if (P + 1 < kPieces) load_v_piece(tile, P + 1, vraw[(P + 1) & 1]);
            else if (more) load_v_piece(next, 0, vraw[0]);
            const uint4(&v)[kVRegs] = vraw[P & 1];
            gw[0][0] = v[0].x; gw[0][1] = v[0].y; gw[0][2] = v[0].z; gw[0][3] = v[0].w;
            gw[0][4] = v[1].x; gw[0][5] = v[1].y; gw[0][6] = v[1].z; gw[0][7] = v[1].w;
          },
          vmeta, p, run);
      if (more) vmeta = *reinterpret_cast<const uint4*>(vm + static_cast<int64_t>(next) * 1024 + lane * 16);
    } else {
      pv_tile<VT, HS>(vraw[0], vmeta, p, run);
      if (more) load_v(next);   // V registers are free again
    }
  }

  finish_chunk<HS, true, NWV>(run, VT == 16 ? 1.0f : 16777216.0f, lk, g, reinterpret_cast<float*>(smem),
                                 reinterpret_cast<float*>(smem) + kWaves * 4 * HS * 2, ma, co);
}

template <int NW, int HS, int NWV>
__global__ __launch_bounds__(NWV * 64, (NW <= 32 && HS == 1) ? 3 : 2) void decode_mixed_kernel(
    const Chunk* __restrict__ chunks, const uint8_t* __restrict__ arena, const ItemK* __restrict__ items_k,
    const uint16_t* __restrict__ q, MergeArgs ma, int lds_steps, int lds_qsteps, const int32_t* __restrict__ tail_len,
    int per_unit) {
  extern __shared__ __align__(16) uint8_t smem[];
  const Chunk ch = chunks[blockIdx.x];
  const int g = ma.hq / ma.hkv;
  const int seq = ch.item / ma.hkv, head = ch.item % ma.hkv;
  const uint16_t* qp = q + (static_cast<int64_t>(seq) * ma.hq + head * g) * kHeadDim;
  const ChunkOut co{ch.item, ch.slot, ch.slot0, ch.nslots};
  const ItemK* ikp = items_k + ch.reserved;   // the K row layout of this chunk's (generation, item)
  switch (ch.tier) {
    case kTierTail: {   // appended tokens: 64-token tiles of bf16 rows, as many rows as exist so far
      const int rows = max(0, min(ch.rows, *tail_len - ch.row0));
      process_tail_tiles<HS, true, NWV>(arena + ch.k_data, arena + ch.v_data, rows, g, qp, smem,
                                        reinterpret_cast<float*>(smem),
                                        reinterpret_cast<float*>(smem) + NWV * 4 * HS * 2, ma, co);
      break;
    }
    case 16: process_mixed<16, NW, HS, NWV>(ch, arena, ikp, g, qp, ma, co, smem, lds_steps, lds_qsteps, per_unit != 0); break;
    case 8: process_mixed<8, NW, HS, NWV>(ch, arena, ikp, g, qp, ma, co, smem, lds_steps, lds_qsteps, per_unit != 0); break;
    case 4: process_mixed<4, NW, HS, NWV>(ch, arena, ikp, g, qp, ma, co, smem, lds_steps, lds_qsteps, per_unit != 0); break;
    default: process_mixed<2, NW, HS, NWV>(ch, arena, ikp, g, qp, ma, co, smem, lds_steps, lds_qsteps, per_unit != 0); break;
  }
}

template <int NW, int HS, int NWV>
hipError_t launch_one(const Chunk* chunks, int n_chunks, const uint8_t* arena, const ItemK* items_k, int lds_steps,
                      int lds_qsteps, const uint16_t* q, const MergeArgs& ma, const int32_t* tail_len, int per_unit,
                      hipStream_t st) {
  const size_t lds = static_cast<size_t>(LdsPlan(lds_steps, lds_qsteps, HS, ma.hq / ma.hkv, NWV).total);
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_mixed_kernel<NW, HS, NWV>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((decode_mixed_kernel<NW, HS, NWV>), dim3(n_chunks), dim3(NWV * 64), lds, st, chunks, arena,
                     items_k, q, ma, lds_steps, lds_qsteps, tail_len, per_unit);
  return hipGetLastError();
}

}  // namespace

#define RDKV_MIXED_NAME3(a_, b_, c_, d_) a_##b_##c_##d_
#define RDKV_MIXED_NAME(a_, b_, c_, d_) RDKV_MIXED_NAME3(a_, b_, c_, d_)
hipError_t RDKV_MIXED_NAME(launch_decode_mixed_hs, RDKV_MIXED_HS, _long, RDKV_MIXED_LONG)(
    const Chunk* chunks, int n_chunks, const uint8_t* arena, const ItemK* items_k, int max_words, int max_steps,
    int max_qsteps, const uint16_t* q, const MergeArgs& ma, const int32_t* tail_len, int per_unit, int waves,
    hipStream_t st) {
  if (n_chunks == 0) return hipSuccess;
#define RDKV_MIXED_LAUNCH(NW_, NWV_)                                                                            \
  return launch_one<NW_, RDKV_MIXED_HS, NWV_>(chunks, n_chunks, arena, items_k, max_steps, max_qsteps, q, ma,   \
                                              tail_len, per_unit, st)
  // kMaxKRowWords = 68 is the longest row a channel bit map can give (125 channels at 16 bits and one each at 8, 4
  // and 2 bits: 64 + 1 + 1 + 1 words, padded to an even count); the host refuses anything longer
  static_assert(kMaxKRowWords == 68, "the widest instantiation must hold the longest K row");
  if (max_words > kMaxKRowWords) return hipErrorInvalidValue;
  (void)waves;
#if RDKV_MIXED_LONG == 0
#if RDKV_MIXED_HS == 1
  // eight-wavefront workgroups exist for up to four query heads per KV head and rows of up to 32 words
  if (waves == 8 && max_words <= 16) RDKV_MIXED_LAUNCH(16, 8);
  if (waves == 8 && max_words <= 32) RDKV_MIXED_LAUNCH(32, 8);
#endif
  if (max_words <= 16) RDKV_MIXED_LAUNCH(16, 4);
  if (max_words <= 32) RDKV_MIXED_LAUNCH(32, 4);
  return hipErrorInvalidValue;
#else
  if (max_words <= 64) RDKV_MIXED_LAUNCH(64, 4);
  RDKV_MIXED_LAUNCH(68, 4);
#endif
#undef RDKV_MIXED_LAUNCH
}

}  // namespace rdkv
