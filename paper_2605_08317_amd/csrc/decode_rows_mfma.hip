// Split-K flash-decode over row-major bf16 rows (Sec. 3.3, Eq. 7) on the gfx950 matrix cores: the uncompressed path
// (the full-cache baseline of Sec. 4.2) and the 16-bit tier of a token-wise cache.
//
// Caller-owned rows are row-major [token][128 channels], so a coalesced load hands a lane 8 channels of one token,
// while the 4x4x4 products want a lane to be a token on the K side (4 consecutive channels per step) and a channel
// on the V side (4 consecutive tokens per step).  Each wavefront therefore passes its 64-token tiles through a
// region of LDS of its own: 16 coalesced 16-byte loads per lane and side, stored row by row with a row stride of 272
// bytes (so that the 16 lanes that read their own rows at the same column hit different banks), then
//   q K^T   lane = token reads its row back 64 bytes at a time: A = 4 channels of the token, B = the raw bf16 query
//           (exact products), D: lane (block b, head j) holds tokens 4b..4b+3;
//   P V     lane = channel pair (2 lane, 2 lane + 1) reads one 32-bit word per token: two byte permutes make the
//           B operands of 4 consecutive tokens for the even and the odd channel; A = the probabilities of those 4
//           tokens as two truncated bf16 terms, broadcast from the block that holds them (cbsz = 4).
// The V loads of a tile are in flight while its logits are computed, the next tile's K loads during P V.  With 8
// query heads per KV head the plain-ALU kernel this replaces spent 2 x 8 multiply-adds per loaded element; here the
// per-element work is one LDS write, one LDS read and a fraction of a byte permute, whatever the number of heads.
#include <utility>

#include "decode_tile_common.h"

namespace rdkv {

namespace {

using namespace tile;

constexpr int kRowsWaves = 4;
constexpr int kRowsWG = kRowsWaves * 64;
constexpr int kRowStride = 272;                       // bytes per token row in LDS (256 + 16 of padding)
constexpr int kStageBytes = kTile * kRowStride;       // one wavefront's staging region
template <int HS>
constexpr int rows_lds_bytes() {
  // query operands [32 steps][HS][4 heads] x 8 bytes, the wavefronts' staging regions, [waves][4 HS][m, l] floats;
  // the end-of-chunk areas (per-wavefront accumulators [waves][g][128] floats, then the merge) reuse the staging
  return 32 * HS * 32 + kRowsWaves * kStageBytes + kRowsWaves * 4 * HS * 2 * 4;
}

__device__ __forceinline__ uint4 load_row_chunk(const uint8_t* __restrict__ base, int row, int c16) {
  return *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(row) * (kHeadDim * 2) + c16 * 16);
}

// One step of P V: tokens 4 A .. 4 A + 3 (A is an instruction field, hence a template argument).
template <int A, int HS>
__device__ __forceinline__ void pv_step(const uint8_t* s_stage, int lane, const short4v (&phi)[HS],
                                        const short4v (&plo)[HS], Run<HS>& run) {
  uint32_t w[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) w[k] = *reinterpret_cast<const uint32_t*>(s_stage + (4 * A + k) * kRowStride + 4 * lane);
  // low halves of two tokens' words = the even channel, high halves = the odd channel
  const short4v be = bf4(__builtin_amdgcn_perm(w[1], w[0], 0x05040100u), __builtin_amdgcn_perm(w[3], w[2], 0x05040100u));
  const short4v bo = bf4(__builtin_amdgcn_perm(w[1], w[0], 0x07060302u), __builtin_amdgcn_perm(w[3], w[2], 0x07060302u));
#pragma unroll
  for (int hs = 0; hs < HS; ++hs) {
    run.acc[hs][0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(phi[hs], be, run.acc[hs][0], 4, A, 0);
    run.acc[hs][0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(plo[hs], be, run.acc[hs][0], 4, A, 0);
    run.acc[hs][1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(phi[hs], bo, run.acc[hs][1], 4, A, 0);
    run.acc[hs][1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(plo[hs], bo, run.acc[hs][1], 4, A, 0);
  }
}
template <int HS, int... A>
__device__ __forceinline__ void pv_steps(const uint8_t* s_stage, int lane, const short4v (&phi)[HS],
                                         const short4v (&plo)[HS], Run<HS>& run, std::integer_sequence<int, A...>) {
  (pv_step<A, HS>(s_stage, lane, phi, plo, run), ...);
}

// TIERED: the chunk's partial goes to the split workspace with agent-scope stores and the workgroup announces it
// (the item's last workgroup merges); otherwise plain stores for a merge kernel that follows.
template <int HS, bool TIERED>
__device__ __forceinline__ void process_rows_mfma(const uint8_t* __restrict__ kd, const uint8_t* __restrict__ vd,
                                                  int rows, int g, const uint16_t* __restrict__ q, uint8_t* smem,
                                                  float* __restrict__ part_acc, float* __restrict__ part_ml,
                                                  const MergeArgs* ma, const ChunkOut* co) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int blk = lane >> 2, j = lane & 3;
  uint8_t* s_q = smem;
  uint8_t* s_stage = smem + 32 * HS * 32 + wave * kStageBytes;
  float* s_ml = reinterpret_cast<float*>(smem + 32 * HS * 32 + kRowsWaves * kStageBytes);
  float* s_acc = reinterpret_cast<float*>(smem + 32 * HS * 32);   // after the tile loop: [waves][g][128], then the merge
  const int ntiles = (rows + kTile - 1) / kTile;
  const int last = rows - 1;
  const int lr = lane >> 4, lc = lane & 15;            // a load covers 4 rows x 16 chunks of 16 bytes

  uint4 st[16];
  auto load_tile = [&](const uint8_t* __restrict__ base, int t) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 16; ++i) st[i] = load_row_chunk(base, min(t * kTile + 4 * i + lr, last), lc);
  };
  auto store_tile = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 16; ++i) *reinterpret_cast<uint4*>(s_stage + (4 * i + lr) * kRowStride + 16 * lc) = st[i];
  };
  if (wave < ntiles) load_tile(kd, wave);

  // query operands of the K product: raw bf16, [step][HS][head] x 8 bytes
  for (int e = tid; e < 32 * HS * 4; e += kRowsWG) {
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
  for (int tile = wave; tile < ntiles; tile += kRowsWaves) {
    const int next = tile + kRowsWaves;
    store_tile();                       // K rows of this tile (the loads were issued a tile ago)
    load_tile(vd, tile);                // V rows: in flight during the logits
    wave_lds_sync();
    floatx4 a16[HS];
#pragma unroll
    for (int hs = 0; hs < HS; ++hs) a16[hs] = zero4;
#pragma unroll
    for (int part = 0; part < 4; ++part) {   // 64 bytes = 32 channels = 8 steps of the lane's own token row
      uint4 kr[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        kr[u] = *reinterpret_cast<const uint4*>(s_stage + lane * kRowStride + 64 * part + 16 * u);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int s = 8 * part + 2 * u + half;
          const short4v a = half ? bf4(kr[u].z, kr[u].w) : bf4(kr[u].x, kr[u].y);
#pragma unroll
          for (int hs = 0; hs < HS; ++hs) {
            const uint2 braw = *reinterpret_cast<const uint2*>(s_q + ((s * HS + hs) * 4 + j) * 8);
            a16[hs] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, bf4(braw.x, braw.y), a16[hs], 0, 0, 0);
          }
        }
    }
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

    wave_lds_sync();                    // every lane is done with the K rows
    store_tile();                       // V rows
    if (next < ntiles) load_tile(kd, next);   // the next tile's K rows: in flight during P V
    wave_lds_sync();
    // P V: step a = tokens 4a..4a+3; this lane's word of a token row = channels 2 lane, 2 lane + 1
    pv_steps<HS>(s_stage, lane, phi, plo, run, std::make_integer_sequence<int, 16>{});
    wave_lds_sync();                    // before the next tile's K rows overwrite the region
  }

  // ---- end of the chunk: merge the workgroup's wavefronts, store the partial ---------------------------------------
#pragma unroll
  for (int hs = 0; hs < HS; ++hs) run.l[hs] = head_sum(run.l[hs]);
  __syncthreads();                      // the staging regions become the accumulator area
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
      for (int w = 0; w < kRowsWaves; ++w) mm = fmaxf(mm, s_ml[((w * HS + hs) * 4 + i) * 2]);
      const float f = fast_exp2(s_ml[((wave * HS + hs) * 4 + i) * 2] - mm);
      if (head < g) {
        *reinterpret_cast<float2*>(s_acc + (wave * g + head) * kHeadDim + 2 * lane) =
            make_float2(run.acc[hs][0][i] * f, run.acc[hs][1][i] * f);
      }
    }
  __syncthreads();
  for (int idx = tid; idx < g * kHeadDim; idx += kRowsWG) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kRowsWaves; ++w) v += s_acc[w * g * kHeadDim + idx];
    if constexpr (TIERED) merge::store_agent(part_acc + idx, v); else part_acc[idx] = v;
  }
  if (tid < g) {
    const int hs = tid >> 2, i = tid & 3;
    float mm = kNegBig;
#pragma unroll
    for (int w = 0; w < kRowsWaves; ++w) mm = fmaxf(mm, s_ml[((w * HS + hs) * 4 + i) * 2]);
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < kRowsWaves; ++w)
      ll += s_ml[((w * HS + hs) * 4 + i) * 2 + 1] * fast_exp2(s_ml[((w * HS + hs) * 4 + i) * 2] - mm);
    if constexpr (TIERED) {
      merge::store_agent(part_ml + tid * 2, mm);
      merge::store_agent(part_ml + tid * 2 + 1, ll);
    } else {
      part_ml[tid * 2] = mm;
      part_ml[tid * 2 + 1] = ll;
    }
  }
  if constexpr (TIERED) {
    merge::partial_stores_done();
    __syncthreads();
    merge::arrive_and_merge<kRowsWG, 4 * HS>(*ma, co->item, co->slot0, co->nslots, g, s_acc);
  }
}

template <int HS>
__global__ __launch_bounds__(kRowsWG, 2) void decode_dense_mfma_kernel(DenseArgs a) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int split = blockIdx.x, head = blockIdx.y, sl = blockIdx.z;
  const int T = a.T[sl];
  const int row0 = split * a.chunk_rows;
  if (row0 >= T) return;
  const int g = a.hq / a.hkv;
  const int rows = min(a.chunk_rows, T - row0);
  const int64_t first = a.row_off[sl] + static_cast<int64_t>(head) * T + row0;
  const uint8_t* kd = reinterpret_cast<const uint8_t*>(a.K) + first * (kHeadDim * 2);
  const uint8_t* vd = reinterpret_cast<const uint8_t*>(a.V) + first * (kHeadDim * 2);
  const int seq = a.seq_base + sl;
  const uint16_t* q = a.q + (static_cast<int64_t>(seq) * a.hq + head * g) * kHeadDim;
  const int64_t slot = (static_cast<int64_t>(sl) * a.hkv + head) * a.max_splits + split;
  process_rows_mfma<HS, false>(kd, vd, rows, g, q, smem, a.part_acc + slot * g * kHeadDim, a.part_ml + slot * g * 2,
                               nullptr, nullptr);
}

template <int HS>
__global__ __launch_bounds__(kRowsWG, 2) void decode_tiered_mfma_kernel(const Chunk* __restrict__ chunks,
                                                                       const uint8_t* __restrict__ arena,
                                                                       const uint16_t* __restrict__ q, MergeArgs ma) {
  extern __shared__ __align__(16) uint8_t smem[];
  const Chunk ch = chunks[blockIdx.x];
  const int g = ma.hq / ma.hkv;
  const int seq = ch.item / ma.hkv, head = ch.item % ma.hkv;
  const uint16_t* qp = q + (static_cast<int64_t>(seq) * ma.hq + head * g) * kHeadDim;
  const ChunkOut co{ch.item, ch.slot, ch.slot0, ch.nslots};
  process_rows_mfma<HS, true>(arena + ch.k_data, arena + ch.v_data, ch.rows, g, qp, smem,
                              ma.part_acc + static_cast<int64_t>(ch.slot) * g * kHeadDim,
                              ma.part_ml + static_cast<int64_t>(ch.slot) * g * 2, &ma, &co);
}

template <class K>
hipError_t allow_lds(K kernel, size_t lds) {
  if (lds <= 48 * 1024) return hipSuccess;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             static_cast<int>(lds));
}

}  // namespace

hipError_t launch_decode_dense_split(const DenseArgs& a, int g, int n_seqs, hipStream_t st) {
  dim3 grid(a.max_splits, a.hkv, n_seqs), block(kRowsWG);
  if (g > 4) {
    const size_t lds = rows_lds_bytes<2>();
    hipError_t e = allow_lds(decode_dense_mfma_kernel<2>, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(decode_dense_mfma_kernel<2>, grid, block, lds, st, a);
  } else {
    const size_t lds = rows_lds_bytes<1>();
    hipError_t e = allow_lds(decode_dense_mfma_kernel<1>, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(decode_dense_mfma_kernel<1>, grid, block, lds, st, a);
  }
  return hipGetLastError();
}

hipError_t launch_decode_tiered_split(const Chunk* chunks, int n_chunks, const uint8_t* arena, const uint16_t* q,
                                      const MergeArgs& ma, hipStream_t st) {
  if (n_chunks == 0) return hipSuccess;
  const int g = ma.hq / ma.hkv;
  dim3 grid(n_chunks), block(kRowsWG);
  if (g > 4) {
    const size_t lds = rows_lds_bytes<2>();
    hipError_t e = allow_lds(decode_tiered_mfma_kernel<2>, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(decode_tiered_mfma_kernel<2>, grid, block, lds, st, chunks, arena, q, ma);
  } else {
    const size_t lds = rows_lds_bytes<1>();
    hipError_t e = allow_lds(decode_tiered_mfma_kernel<1>, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(decode_tiered_mfma_kernel<1>, grid, block, lds, st, chunks, arena, q, ma);
  }
  return hipGetLastError();
}

}  // namespace rdkv
