// Stage 1 of Alg. 1 on the GPU: token weights (Eq. 2) and channel weights (Eq. 4).
//
// The token weights need S = Q_obs K^T / sqrt(d) for the R = g * S_w window rows of
// a KV head against all T keys -- a dense [R x 128] x [128 x T] contraction, done
// with bf16 MFMA (v_mfma_f32_16x16x32_bf16) and never stored.  Two streaming
// passes over K: pass 1 produces the log-sum-exp of every row (softmax
// normaliser), pass 2 recomputes the logits and accumulates the column sums
// w_t = sum_rows exp(s - lse_row).  Pass 1 also accumulates the per-channel sum of
// squares of K for the channel weights.  One workgroup = 256 keys (64 per
// wavefront, held in registers as MFMA A operands) against all rows (Q_obs staged
// in LDS, read as B operands).
#include "rdkv_internal.h"

namespace rdkv {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

constexpr int kTokPerWG = 256;
constexpr int kRowsPerStage = 64;           // window rows staged in LDS at a time (19.5 KB per workgroup)
constexpr int kQStride = kHeadDim + 8;      // bf16 elements per LDS row (272 B: conflict-free 16-byte reads)
constexpr float kNegBig = -1.0e30f;
constexpr float kLogitScale = 1.4426950408889634f * 0.08838834764831845f;   // log2(e) / sqrt(128)

struct WeightArgs {
  const uint16_t* K;
  const uint16_t* Q;             // [batch][hq][s_obs][d]
  const int64_t* item_row_off;   // [items]
  const int32_t* item_T;         // [items]
  const int32_t* item_blk_off;   // [items] first 256-key block of the item
  float* row_part;               // [blocks][R_pad][2]  (m, l) in the log2 domain
  float* lse;                    // [items][R_pad]
  float* w_raw;                  // [total tokens] unpooled weights
  float* ksq_part;               // [blocks][128] or null
  int32_t hq, hkv, g, s_obs, R, R_pad, causal;
};

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  v += dpp_mov<0x141>(v);
  v += dpp_mov<0x140>(v);
  return v;
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int PASS>
__global__ __launch_bounds__(256, 3) void weights_kernel(WeightArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  uint16_t* sQ = reinterpret_cast<uint16_t*>(smem_raw);                              // [kRowsPerStage][kQStride]
  float* sStat = reinterpret_cast<float*>(smem_raw + kRowsPerStage * kQStride * 2);   // [4 waves][kRowsPerStage][2]

  const int item = blockIdx.y;
  const int T = a.item_T[item];
  const int tok0 = blockIdx.x * kTokPerWG;
  if (tok0 >= T) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, quad = lane >> 4;
  const int seq = item / a.hkv, head = item % a.hkv;
  const int64_t blk = a.item_blk_off[item] + blockIdx.x;

  const uint16_t* Qg = a.Q + (static_cast<int64_t>(seq) * a.hq + head * a.g) * a.s_obs * kHeadDim;

  // this wavefront's 64 keys as A operands: a_op[tt][kb] = key (tt*16 + l16), channels kb*32 + quad*8 .. +7
  const uint16_t* Kh = a.K + a.item_row_off[item] * kHeadDim;
  const int wtok0 = tok0 + wave * 64;
  bf16x8 a_op[4][4];
#pragma unroll
  for (int tt = 0; tt < 4; ++tt) {
    const int tok = min(wtok0 + tt * 16 + l16, T - 1);
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
      a_op[tt][kb] = *reinterpret_cast<const bf16x8*>(Kh + static_cast<int64_t>(tok) * kHeadDim + kb * 32 + quad * 8);
  }

  if (PASS == 1 && a.ksq_part != nullptr) {
    // per-channel sum of squares of K over the valid keys of this workgroup
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float s = 0.f;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const bool ok = (wtok0 + tt * 16 + l16) < T;
          const float x = ok ? static_cast<float>(a_op[tt][kb][j]) : 0.f;
          s = __builtin_fmaf(x, x, s);
        }
        s = row16_sum(s);
        if (l16 == 0) sStat[wave * kHeadDim + kb * 32 + quad * 8 + j] = s;
      }
    }
    __syncthreads();
    if (tid < kHeadDim)
      a.ksq_part[blk * kHeadDim + tid] = (sStat[tid] + sStat[kHeadDim + tid]) + (sStat[2 * kHeadDim + tid] + sStat[3 * kHeadDim + tid]);
  }
  __syncthreads();

  // does any row of this block need the causal mask?  keys <= T - s_obs are visible to every row
  const bool need_mask = a.causal && (tok0 + kTokPerWG > T - a.s_obs + 1);
  // nearly every block of a long context has 256 valid keys, all visible to every row: no masks, and the logit
  // scale goes into the fused multiply-add that feeds exp2 (4 plain-ALU instructions per logit instead of 9)
  const bool fast = !need_mask && (tok0 + kTokPerWG <= T) && (a.R == a.R_pad);
  float colsum[4][4];
#pragma unroll
  for (int tt = 0; tt < 4; ++tt)
#pragma unroll
    for (int i = 0; i < 4; ++i) colsum[tt][i] = 0.f;

  // The window rows pass through LDS kRowsPerStage at a time (the keys stay in registers).  A stage's rows are
  // fetched into registers while the previous stage is computed (4 x 16 bytes per thread) and stored to LDS between
  // two barriers, so that only the first stage's latency is waited for.
  uint4 qbuf[4];
  auto fetch = [&](int r0) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = tid + 256 * k, r = i >> 4, c8 = i & 15;
      qbuf[k] = make_uint4(0, 0, 0, 0);        // pad rows are zero
      if (r0 + r < a.R) qbuf[k] = *reinterpret_cast<const uint4*>(Qg + (r0 + r) * kHeadDim + c8 * 8);
    }
  };
  fetch(0);
  for (int r0 = 0; r0 < a.R_pad; r0 += kRowsPerStage) {
  const int nrows = min(kRowsPerStage, a.R_pad - r0);
  __syncthreads();   // the previous stage's readers are done
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int i = tid + 256 * k, r = i >> 4, c8 = i & 15;
    *reinterpret_cast<uint4*>(sQ + r * kQStride + c8 * 8) = qbuf[k];
  }
  if (PASS == 2)   // the rows' log-sum-exp, read once per row tile below
    for (int r = tid; r < nrows; r += 256) sStat[r] = a.lse[static_cast<int64_t>(item) * a.R_pad + r0 + r];
  if (r0 + kRowsPerStage < a.R_pad) fetch(r0 + kRowsPerStage);   // in flight during this stage's arithmetic
  __syncthreads();
  for (int rt = 0; rt < nrows / 16; ++rt) {
    floatx4 acc[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) acc[tt] = floatx4{0.f, 0.f, 0.f, 0.f};
    const int lrow = rt * 16 + l16, row = r0 + lrow;   // row inside the stage / of the window
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      const bf16x8 b_op = *reinterpret_cast<const bf16x8*>(sQ + lrow * kQStride + kb * 32 + quad * 8);
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
        acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_op[tt][kb], b_op, acc[tt], 0, 0, 0);
    }
    // acc[tt][i] = q_row . k_tok with tok = wtok0 + tt*16 + quad*4 + i, row = rt*16 + l16
    if (fast) {
      if (PASS == 1) {
        float mx = acc[0][0];
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
#pragma unroll
          for (int i = 0; i < 4; ++i) mx = fmaxf(mx, acc[tt][i]);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        mx *= kLogitScale;                       // the scale is positive: the maximum of the scaled logits
        float ls = 0.f;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
#pragma unroll
          for (int i = 0; i < 4; ++i) ls += fast_exp2(__builtin_fmaf(acc[tt][i], kLogitScale, -mx));
        ls += __shfl_xor(ls, 16);
        ls += __shfl_xor(ls, 32);
        if (quad == 0) {
          sStat[(wave * kRowsPerStage + lrow) * 2] = mx;
          sStat[(wave * kRowsPerStage + lrow) * 2 + 1] = ls;
        }
      } else {
        const float nlse = -sStat[lrow];
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
#pragma unroll
          for (int i = 0; i < 4; ++i) colsum[tt][i] += fast_exp2(__builtin_fmaf(acc[tt][i], kLogitScale, nlse));
      }
      continue;
    }
    const int limit = a.causal ? (T - a.s_obs + (row % a.s_obs)) : (T - 1);   // last visible key of this row
    const bool row_ok = row < a.R;
    float x[4][4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int tok = wtok0 + tt * 16 + quad * 4 + i;
        const bool ok = row_ok && (need_mask ? (tok <= limit) : true) && (tok < T);
        x[tt][i] = ok ? acc[tt][i] * kLogitScale : -INFINITY;
      }
    if (PASS == 1) {
      float mx = kNegBig;
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int i = 0; i < 4; ++i) mx = fmaxf(mx, x[tt][i]);
      // rows are shared by the 4 quads of the wavefront
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      float ls = 0.f;
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int i = 0; i < 4; ++i) ls += fast_exp2(x[tt][i] - mx);
      ls += __shfl_xor(ls, 16);
      ls += __shfl_xor(ls, 32);
      if (quad == 0) {
        sStat[(wave * kRowsPerStage + lrow) * 2] = mx;
        sStat[(wave * kRowsPerStage + lrow) * 2 + 1] = ls;
      }
    } else {
      const float lse = sStat[lrow];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int i = 0; i < 4; ++i) colsum[tt][i] += fast_exp2(x[tt][i] - lse);
    }
  }

  if (PASS == 1) {   // this block's (maximum, sum) of the stage's rows: merge the four wavefronts
    __syncthreads();
    for (int r = tid; r < nrows; r += 256) {
      float m = kNegBig;
#pragma unroll
      for (int w = 0; w < 4; ++w) m = fmaxf(m, sStat[(w * kRowsPerStage + r) * 2]);
      float l = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w)
        l += sStat[(w * kRowsPerStage + r) * 2 + 1] * fast_exp2(sStat[(w * kRowsPerStage + r) * 2] - m);
      a.row_part[(blk * a.R_pad + r0 + r) * 2] = m;
      a.row_part[(blk * a.R_pad + r0 + r) * 2 + 1] = l;
    }
  }
  }   // stages

  if (PASS == 2) {
    float* w_out = a.w_raw + a.item_row_off[item];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float s = row16_sum(colsum[tt][i]);
        const int tok = wtok0 + tt * 16 + quad * 4 + i;
        if (l16 == 0 && tok < T) w_out[tok] = s;
      }
  }
}

// log-sum-exp of every window row over the key blocks of its item (log2 domain);
// one wavefront per row, lanes stride over the blocks
__global__ __launch_bounds__(256) void row_lse_kernel(WeightArgs a) {
  const int item = blockIdx.y;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= a.R_pad) return;
  const int lane = threadIdx.x & 63;
  const int T = a.item_T[item];
  const int nblk = (T + kTokPerWG - 1) / kTokPerWG;
  const int64_t b0 = a.item_blk_off[item];
  float m = kNegBig;
  for (int b = lane; b < nblk; b += 64) m = fmaxf(m, a.row_part[((b0 + b) * a.R_pad + r) * 2]);
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  float l = 0.f;
  for (int b = lane; b < nblk; b += 64)
    l += a.row_part[((b0 + b) * a.R_pad + r) * 2 + 1] * fast_exp2(a.row_part[((b0 + b) * a.R_pad + r) * 2] - m);
  for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o);
  // a padded row has no visible key: give it +inf so that exp2(x - lse) = 0
  if (lane == 0) a.lse[static_cast<int64_t>(item) * a.R_pad + r] = (l > 0.f) ? m + __log2f(l) : INFINITY;
}

// AvgPool1d(kernel, stride 1, zero padding kernel/2, divisor kernel) along the keys of each item
__global__ __launch_bounds__(256) void pool_kernel(const float* __restrict__ w_raw, float* __restrict__ w_out,
                                                   const int64_t* __restrict__ item_row_off,
                                                   const int32_t* __restrict__ item_T, int kernel) {
  const int item = blockIdx.y;
  const int T = item_T[item];
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const float* w = w_raw + item_row_off[item];
  const int r = kernel / 2;
  float s = 0.f;
  for (int k = -r; k <= r; ++k) {
    const int u = t + k;
    if (u >= 0 && u < T) s += w[u];
  }
  w_out[item_row_off[item] + t] = s / static_cast<float>(kernel);
}

// w_c = ||Q[:,c]|| ||K[:,c]|| / sqrt(d): finishes the K sums of squares and adds the probe's column norms
__global__ __launch_bounds__(kHeadDim) void channel_weight_kernel(WeightArgs a, float* __restrict__ w_ch) {
  const int item = blockIdx.x, c = threadIdx.x;
  const int T = a.item_T[item];
  const int nblk = (T + kTokPerWG - 1) / kTokPerWG;
  const int64_t b0 = a.item_blk_off[item];
  float ksq = 0.f;
  for (int b = 0; b < nblk; ++b) ksq += a.ksq_part[(b0 + b) * kHeadDim + c];
  const int seq = item / a.hkv, head = item % a.hkv;
  const uint16_t* Qg = a.Q + (static_cast<int64_t>(seq) * a.hq + head * a.g) * a.s_obs * kHeadDim;
  float qsq = 0.f;
  for (int r = 0; r < a.R; ++r) {
    const float q = __uint_as_float(static_cast<uint32_t>(Qg[r * kHeadDim + c]) << 16);
    qsq = __builtin_fmaf(q, q, qsq);
  }
  w_ch[static_cast<int64_t>(item) * kHeadDim + c] = sqrtf(qsq) * sqrtf(ksq) * 0.08838834764831845f;
}

}  // namespace

int weights_block() { return kTokPerWG; }

// scratch layout (floats): row_part | lse | w_raw | ksq_part
size_t weights_scratch_floats(int64_t n_blocks, int64_t n_items, int64_t total_tokens, int R_pad, bool want_ch) {
  return static_cast<size_t>(n_blocks) * R_pad * 2 + static_cast<size_t>(n_items) * R_pad +
         static_cast<size_t>(total_tokens) + (want_ch ? static_cast<size_t>(n_blocks) * kHeadDim : 0) + 64;
}

hipError_t launch_weights(const rdkv_config& cfg, const int64_t* d_item_row_off, const int32_t* d_item_T,
                          const int32_t* d_item_blk_off, int64_t n_blocks, int64_t n_items, int64_t total_tokens,
                          int max_T, const uint16_t* K, const uint16_t* Q_obs, float* w_tok, float* w_ch,
                          float* scratch, hipStream_t st) {
  if (n_items == 0 || max_T == 0) return hipSuccess;
  WeightArgs a;
  a.K = K; a.Q = Q_obs; a.item_row_off = d_item_row_off; a.item_T = d_item_T; a.item_blk_off = d_item_blk_off;
  a.hq = cfg.hq; a.hkv = cfg.hkv; a.g = cfg.hq / cfg.hkv; a.s_obs = cfg.s_obs;
  a.R = a.g * cfg.s_obs; a.R_pad = (a.R + 15) / 16 * 16; a.causal = cfg.causal ? 1 : 0;
  a.row_part = scratch;
  a.lse = a.row_part + n_blocks * a.R_pad * 2;
  a.w_raw = a.lse + n_items * a.R_pad;
  a.ksq_part = w_ch ? a.w_raw + total_tokens : nullptr;
  const int max_blk = (max_T + kTokPerWG - 1) / kTokPerWG;
  const size_t lds = static_cast<size_t>(kRowsPerStage) * kQStride * 2 + 4 * kRowsPerStage * 2 * sizeof(float);
  hipError_t e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(weights_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          static_cast<int>(lds));
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(weights_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          static_cast<int>(lds));
  if (e != hipSuccess) return e;
  dim3 grid(max_blk, static_cast<unsigned>(n_items));
  hipLaunchKernelGGL(weights_kernel<1>, grid, dim3(256), lds, st, a);
  hipLaunchKernelGGL(row_lse_kernel, dim3((a.R_pad + 3) / 4, static_cast<unsigned>(n_items)), dim3(256), 0, st, a);
  hipLaunchKernelGGL(weights_kernel<2>, grid, dim3(256), lds, st, a);
  const bool pooled = cfg.pool_kernel > 1;
  if (pooled) {
    hipLaunchKernelGGL(pool_kernel, dim3((max_T + 255) / 256, static_cast<unsigned>(n_items)), dim3(256), 0, st,
                       a.w_raw, w_tok, d_item_row_off, d_item_T, cfg.pool_kernel);
  } else {
    e = hipMemcpyAsync(w_tok, a.w_raw, total_tokens * sizeof(float), hipMemcpyDeviceToDevice, st);
    if (e != hipSuccess) return e;
  }
  if (w_ch) hipLaunchKernelGGL(channel_weight_kernel, dim3(static_cast<unsigned>(n_items)), dim3(kHeadDim), 0, st, a, w_ch);
  return hipGetLastError();
}

}  // namespace rdkv
