// Band SpMV over diagonal-major packed storage:
//
//   y(i) := sum_{d=-w..w, 0<=i+d<n} D(d,i) * x(i+d)
//
// The rule is the strided-band structure of Section 6.4 with unit stride and 2w+1 summands
// (w=0 is Table 2's SpMV_D).  Each diagonal is one summand with its own densely packed n-slot
// buffer (Section 4, per-summand buffers), addressed by band_offset(d,i) = (d+w)*n + i, so lane l of
// a wavefront reads slot i0+l of every diagonal: 2w+1 perfectly contiguous streams.  x is the only
// operand that is reused (each element by 2w+1 rows): a workgroup stages the window of x that its
// 1024 rows touch in LDS once and every lane keeps its own 4+2w values in registers.
//
// Padding slots (column outside the matrix) are never used for their value: interior workgroups
// cannot reach one, and the two edge workgroups select by the column predicate.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBlock = 256;
constexpr int kRowsPerThread = 4;
constexpr int kRowsPerBlock = kBlock * kRowsPerThread;

template <int W>
__global__ __launch_bounds__(kBlock) void band_tiled_kernel(int64_t n, const float *__restrict__ D,
                                                            const float *__restrict__ x, float *__restrict__ y) {
  static_assert(W % 2 == 0, "window must be a whole number of 16-byte LDS reads");
  constexpr int kWin = kRowsPerThread + 2 * W;  // x values one thread needs
  __shared__ __attribute__((aligned(16))) float xs[kRowsPerBlock + 2 * W];

  const int64_t b0 = (int64_t)blockIdx.x * kRowsPerBlock;
  for (int t = threadIdx.x; t < kRowsPerBlock + 2 * W; t += kBlock) {
    int64_t c = b0 - W + t;
    xs[t] = (c >= 0 && c < n) ? x[c] : 0.0f;
  }
  __syncthreads();

  float xw[kWin];
#pragma unroll
  for (int q = 0; q < kWin / 4; ++q) {
    f4a v = *reinterpret_cast<const f4a *>(&xs[threadIdx.x * kRowsPerThread + 4 * q]);
    xw[4 * q + 0] = v.x; xw[4 * q + 1] = v.y; xw[4 * q + 2] = v.z; xw[4 * q + 3] = v.w;
  }

  const int64_t i0 = b0 + (int64_t)threadIdx.x * kRowsPerThread;
  float acc[kRowsPerThread] = {0.0f, 0.0f, 0.0f, 0.0f};
  const bool interior = (b0 >= W) && (b0 + kRowsPerBlock + W <= n);
  if (interior) {
#pragma unroll
    for (int dd = 0; dd <= 2 * W; ++dd) {
      f4u dv = *reinterpret_cast<const f4u *>(D + (int64_t)dd * n + i0);
      acc[0] += dv.x * xw[dd + 0];
      acc[1] += dv.y * xw[dd + 1];
      acc[2] += dv.z * xw[dd + 2];
      acc[3] += dv.w * xw[dd + 3];
    }
    *reinterpret_cast<f4u *>(y + i0) = f4u{acc[0], acc[1], acc[2], acc[3]};
  } else {
#pragma unroll
    for (int dd = 0; dd <= 2 * W; ++dd) {
#pragma unroll
      for (int e = 0; e < kRowsPerThread; ++e) {
        int64_t i = i0 + e, c = i + dd - W;
        if (i < n && c >= 0 && c < n) acc[e] += D[(int64_t)dd * n + i] * xw[dd + e];
      }
    }
#pragma unroll
    for (int e = 0; e < kRowsPerThread; ++e)
      if (i0 + e < n) y[i0 + e] = acc[e];
  }
}

// Any half-width: one row per lane, x read through the vector cache.
__global__ __launch_bounds__(kBlock) void band_generic_kernel(int64_t n, int w, const float *__restrict__ D,
                                                              const float *__restrict__ x, float *__restrict__ y) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  float acc = 0.0f;
  for (int d = -w; d <= w; ++d) {
    int64_t c = i + d;
    if (c >= 0 && c < n) acc += D[(int64_t)(d + w) * n + i] * x[c];
  }
  y[i] = acc;
}

}  // namespace

extern "C" int dastac_band_spmv_f32(int64_t n, int64_t w, const float *D, const float *x, float *y, void *stream) {
  if (n < 0 || w < 0 || w > 64) return DASTAC_EINVAL;
  if (n > ((int64_t)1 << 40) / (2 * w + 1)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!D || !x || !y) return DASTAC_ENULL;
  if (overlaps(y, n * 4, D, (2 * w + 1) * n * 4) || overlaps(y, n * 4, x, n * 4)) return DASTAC_EALIAS;
  hipStream_t st = (hipStream_t)stream;
  unsigned tiled_blocks = (unsigned)ceil_div(n, kRowsPerBlock);
  switch (w) {
    case 16: band_tiled_kernel<16><<<tiled_blocks, kBlock, 0, st>>>(n, D, x, y); break;
    case 8: band_tiled_kernel<8><<<tiled_blocks, kBlock, 0, st>>>(n, D, x, y); break;
    case 4: band_tiled_kernel<4><<<tiled_blocks, kBlock, 0, st>>>(n, D, x, y); break;
    case 2: band_tiled_kernel<2><<<tiled_blocks, kBlock, 0, st>>>(n, D, x, y); break;
    case 0: band_tiled_kernel<0><<<tiled_blocks, kBlock, 0, st>>>(n, D, x, y); break;
    default:
      band_generic_kernel<<<(unsigned)ceil_div(n, kBlock), kBlock, 0, st>>>(n, (int)w, D, x, y);
  }
  return launch_status();
}
