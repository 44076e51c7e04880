// Distortion-table calibration (App. B "Calibration"; App. "Calibrated Distortion Tables", Table 9): the normalized
// squared error of the library's own quantizer at 2, 4 and 8 bits on supplied K and V, per (sequence, KV head)
// slice.  Every token is retained.
//   rows     : groups of 32 channels of a token row (V always; K when it shares the token map)
//   channels : groups of 32 consecutive tokens of a channel starting at token 0, or the whole channel (App. B)
// The codes are those of the pack kernels (same fp32 operations in the same order); the error of an element,
// x - (s code + m), and all sums are taken in fp64, so the result differs from an fp64 reference only by the order
// of the additions.  Every byte is read once (the whole-channel format reads K twice); three IEEE divisions and three
// fp64 error terms per element make the kernels bound by the plain ALUs, not by HBM.
#include "rdkv_internal.h"

namespace rdkv {
namespace {

constexpr int kCalibRowsPerBlock = 256;    // rows kernel: 16 iterations of 16 rows
constexpr int kCalibTokensPerBlock = 128;  // channels kernel: one 32-token group per wavefront

struct CalibArgs {
  const uint16_t* X;            // K or V, ragged [items][T][128] bf16
  const int64_t* item_row_off;  // [items]: first row of the item
  const int32_t* item_T;        // [items]
  double* acc;                  // [items][4]: squared error at 2, 4, 8 bits, then sum of squares
  uint32_t* range;              // [items][128][2] ordered-integer images of a channel's minimum / maximum, or null
  int32_t row_wide;             // rows kernel: one scale per token row instead of one per group of 32 channels
};

__device__ __forceinline__ uint32_t to_ordered(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float from_ordered(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

__device__ __forceinline__ void unpack8(const uint4& w, float x[8]) {
  const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __uint_as_float(u[i] << 16);
    x[2 * i + 1] = __uint_as_float(u[i] & 0xFFFF0000u);
  }
}

// squared error of N values of one group quantized at BITS bits with the group's range [mn, mx]
template <int BITS, int N>
__device__ __forceinline__ double group_error(const float (&x)[N], const bool (&ok)[N], float mn, float mx) {
  constexpr float Q = static_cast<float>((1 << BITS) - 1);
  mn = mn + 0.0f;   // canonical +0
  const _Float16 sh = static_cast<_Float16>((mx - mn) / Q);
  const _Float16 mh = static_cast<_Float16>(mn);
  const float s = static_cast<float>(sh), m = static_cast<float>(mh);
  double err = 0.0;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    float t = rintf((x[i] - m) / s);
    t = fminf(fmaxf(t, 0.0f), Q);
    if (s == 0.0f) t = 0.0f;
    const double xh = static_cast<double>(s) * static_cast<double>(t) + static_cast<double>(m);
    const double e = static_cast<double>(x[i]) - xh;
    if (ok[i]) err += e * e;
  }
  return err;
}

// adds the workgroup's four partial sums to the item's accumulators
__device__ __forceinline__ void block_accumulate(double v[4], double* acc) {
  __shared__ double s_part[4][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    double x = v[k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off);
    if (lane == 0) s_part[wave][k] = x;
  }
  __syncthreads();
  if (threadIdx.x < 4) {
    const int k = threadIdx.x;
    const double x = (s_part[0][k] + s_part[1][k]) + (s_part[2][k] + s_part[3][k]);
    if (x != 0.0) atomicAdd(acc + k, x);
  }
}

// One lane = 8 channels of one row (a 16-byte load); 4 consecutive lanes = one group of 32 channels.
__global__ __launch_bounds__(256) void calib_rows_kernel(CalibArgs a) {
  const int item = blockIdx.y;
  const int T = a.item_T[item];
  const int r0 = blockIdx.x * kCalibRowsPerBlock;
  if (r0 >= T) return;
  const uint4* src = reinterpret_cast<const uint4*>(a.X + a.item_row_off[item] * kHeadDim);
  double sum[4] = {0.0, 0.0, 0.0, 0.0};
  const int64_t n16 = static_cast<int64_t>(T) * (kHeadDim / 8);   // 16-byte units of the item
#pragma unroll 2
  for (int it = 0; it < kCalibRowsPerBlock / 16; ++it) {
    const int64_t u = static_cast<int64_t>(r0) * 16 + it * 256 + threadIdx.x;
    const bool live = u < n16;   // whole rows: the four lanes of a group are live together
    float x[8];
    unpack8(live ? src[u] : make_uint4(0, 0, 0, 0), x);
    float mn = x[0], mx = x[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) {
      mn = fminf(mn, x[i]);
      mx = fmaxf(mx, x[i]);
    }
    mn = fminf(mn, __shfl_xor(mn, 1));
    mx = fmaxf(mx, __shfl_xor(mx, 1));
    mn = fminf(mn, __shfl_xor(mn, 2));
    mx = fmaxf(mx, __shfl_xor(mx, 2));
    if (a.row_wide) {   // the 16 lanes of a row
      mn = fminf(mn, __shfl_xor(mn, 4));
      mx = fmaxf(mx, __shfl_xor(mx, 4));
      mn = fminf(mn, __shfl_xor(mn, 8));
      mx = fmaxf(mx, __shfl_xor(mx, 8));
    }
    const bool ok[8] = {live, live, live, live, live, live, live, live};
    sum[0] += group_error<2, 8>(x, ok, mn, mx);
    sum[1] += group_error<4, 8>(x, ok, mn, mx);
    sum[2] += group_error<8, 8>(x, ok, mn, mx);
#pragma unroll
    for (int i = 0; i < 8; ++i) sum[3] += static_cast<double>(x[i]) * static_cast<double>(x[i]);
  }
  block_accumulate(sum, a.acc + static_cast<int64_t>(item) * 4);
}

// Minimum and maximum of every channel over all tokens of the item.  range starts at (0xFFFFFFFF, 0).
__global__ __launch_bounds__(256) void calib_channel_range_kernel(CalibArgs a) {
  __shared__ uint32_t s_mn[16][kHeadDim], s_mx[16][kHeadDim];
  const int item = blockIdx.y;
  const int T = a.item_T[item];
  const int r0 = blockIdx.x * kCalibRowsPerBlock;
  if (r0 >= T) return;
  const uint4* src = reinterpret_cast<const uint4*>(a.X + a.item_row_off[item] * kHeadDim);
  const int cpart = threadIdx.x & 15, rsub = threadIdx.x >> 4;
  uint32_t mn[8], mx[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    mn[i] = 0xFFFFFFFFu;
    mx[i] = 0u;
  }
  for (int it = 0; it < kCalibRowsPerBlock / 16; ++it) {
    const int r = r0 + it * 16 + rsub;
    if (r < T) {
      float x[8];
      unpack8(src[static_cast<int64_t>(r) * 16 + cpart], x);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t k = to_ordered(x[i]);
        mn[i] = min(mn[i], k);
        mx[i] = max(mx[i], k);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    s_mn[rsub][8 * cpart + i] = mn[i];
    s_mx[rsub][8 * cpart + i] = mx[i];
  }
  __syncthreads();
  if (threadIdx.x < kHeadDim) {
    const int c = threadIdx.x;
    uint32_t lo = s_mn[0][c], hi = s_mx[0][c];
#pragma unroll
    for (int k = 1; k < 16; ++k) {
      lo = min(lo, s_mn[k][c]);
      hi = max(hi, s_mx[k][c]);
    }
    atomicMin(&a.range[(static_cast<int64_t>(item) * kHeadDim + c) * 2], lo);
    atomicMax(&a.range[(static_cast<int64_t>(item) * kHeadDim + c) * 2 + 1], hi);
  }
}

// One wavefront = one group of 32 tokens x 128 channels: lane (rsub = lane / 16, cpart = lane % 16) loads the 8
// channels 8 cpart.. of the rows 4 j + rsub, j = 0..7 (a wave-wide load covers 4 whole rows); the group's range of a
// channel is the minimum / maximum over j and over the four lanes that share cpart.
template <bool WHOLE_CHANNEL>
__global__ __launch_bounds__(256) void calib_channels_kernel(CalibArgs a) {
  const int item = blockIdx.y;
  const int T = a.item_T[item];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t0 = blockIdx.x * kCalibTokensPerBlock + wave * kKTokenGroup;
  if (blockIdx.x * kCalibTokensPerBlock >= T) return;
  const uint4* src = reinterpret_cast<const uint4*>(a.X + a.item_row_off[item] * kHeadDim);
  const int cpart = lane & 15, rsub = lane >> 4;
  double sum[4] = {0.0, 0.0, 0.0, 0.0};
  if (t0 < T) {
    float x[8][8];   // [j][channel]
    bool ok[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int r = t0 + 4 * j + rsub;
      ok[j] = r < T;
      unpack8(ok[j] ? src[static_cast<int64_t>(r) * 16 + cpart] : make_uint4(0, 0, 0, 0), x[j]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float col[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) col[j] = x[j][i];
      float mn, mx;
      if (WHOLE_CHANNEL) {
        const int64_t c = static_cast<int64_t>(item) * kHeadDim + 8 * cpart + i;
        mn = from_ordered(a.range[c * 2]);
        mx = from_ordered(a.range[c * 2 + 1]);
      } else {
        mn = __builtin_inff();
        mx = -__builtin_inff();
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (ok[j]) {
            mn = fminf(mn, col[j]);
            mx = fmaxf(mx, col[j]);
          }
        mn = fminf(mn, __shfl_xor(mn, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mn = fminf(mn, __shfl_xor(mn, 32));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
      }
      sum[0] += group_error<2, 8>(col, ok, mn, mx);
      sum[1] += group_error<4, 8>(col, ok, mn, mx);
      sum[2] += group_error<8, 8>(col, ok, mn, mx);
#pragma unroll
      for (int j = 0; j < 8; ++j) sum[3] += static_cast<double>(col[j]) * static_cast<double>(col[j]);
    }
  }
  block_accumulate(sum, a.acc + static_cast<int64_t>(item) * 4);
}

}  // namespace

// acc_k, acc_v: [items][4] doubles, zero on entry.  range: [items][128][2] holding (0xFFFFFFFF, 0) pairs on entry
// when k_whole_channel is set, else unused.
hipError_t launch_calibrate(const uint16_t* K, const uint16_t* V, const int64_t* item_row_off, const int32_t* item_T,
                            int n_items, int max_T, bool k_channelwise, bool k_whole_channel, bool row_wide,
                            double* acc_k, double* acc_v, uint32_t* range, hipStream_t st) {
  if (n_items == 0 || max_T == 0) return hipSuccess;
  const dim3 block(256);
  const dim3 grid_rows((max_T + kCalibRowsPerBlock - 1) / kCalibRowsPerBlock, n_items);
  const dim3 grid_ch((max_T + kCalibTokensPerBlock - 1) / kCalibTokensPerBlock, n_items);
  CalibArgs av{V, item_row_off, item_T, acc_v, nullptr, row_wide ? 1 : 0};
  hipLaunchKernelGGL(calib_rows_kernel, grid_rows, block, 0, st, av);
  CalibArgs ak{K, item_row_off, item_T, acc_k, range, row_wide ? 1 : 0};
  if (!k_channelwise) {
    hipLaunchKernelGGL(calib_rows_kernel, grid_rows, block, 0, st, ak);
  } else if (k_whole_channel) {
    hipLaunchKernelGGL(calib_channel_range_kernel, grid_rows, block, 0, st, ak);
    hipLaunchKernelGGL(calib_channels_kernel<true>, grid_ch, block, 0, st, ak);
  } else {
    hipLaunchKernelGGL(calib_channels_kernel<false>, grid_ch, block, 0, st, ak);
  }
  return hipGetLastError();
}

}  // namespace rdkv
