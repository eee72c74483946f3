// Band SpMV over diagonal-major packed storage:
//
//   y(i) := sum_{d=-w..w, 0<=i+d<n} D(d,i) * x(i+d)
//
// The rule is the strided-band structure of Section 6.4 with unit stride and 2w+1 summands
// (w=0 is Table 2's SpMV_D).  Each diagonal is one summand with its own densely packed n-slot
// buffer (Section 4, per-summand buffers), addressed by band_offset(d,i) = (d+w)*n + i, so lane l of
// a wavefront reads slot i0+l of every diagonal: 2w+1 perfectly contiguous streams, each element
// used exactly once.  They are read with non-temporal loads (measured: about 15 % faster than
// cached loads, which evict x from L2 for nothing), one row per lane (measured faster than two or
// four rows per lane at this shape).  x is the only reused operand; its 2w+1-wide window per lane
// overlaps the neighbours' windows almost completely and is served by the vector L1 cache
// (staging it in LDS behind a workgroup barrier measured slower, because the barrier delays the
// issue of the diagonal loads).
//
// Padding slots (column outside the matrix) are never used for their value: interior lanes cannot
// reach one, and the w lanes at either end select by the column predicate.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBlock = 256;

// W >= 0: half-width known at compile time (fully unrolled); W < 0: run-time half-width `w`.
// With 33 streams per lane, four wavefronts per SIMD keep as much in flight as the memory system takes; the
// eight that the register count allows put more rows of more diagonals in flight at once and measured 2 % slower
// (n = 2^22: 97.6 -> 95.5 us; three: 95.0, five: 96.7, two: 102.9), so the widest instantiation is held to four.
template <int W, typename T>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(W == 16 ? 4 : 1, W == 16 ? 4 : 8)))
void band_kernel(int64_t n, int w, const T *__restrict__ D,
                                                      const T *__restrict__ x, T *__restrict__ y) {
  const int hw = W >= 0 ? W : w;
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  const T *d = D + i;
  T acc = T(0);
  if (i >= hw && i + hw < n) {  // interior row: every column exists
    const T *xw = x + (i - hw);
    if (W >= 0) {
#pragma unroll
      for (int dd = 0; dd <= 2 * (W >= 0 ? W : 0); ++dd)
        acc += __builtin_nontemporal_load(d + (int64_t)dd * n) * xw[dd];
    } else {
      for (int dd = 0; dd <= 2 * hw; ++dd) acc += __builtin_nontemporal_load(d + (int64_t)dd * n) * xw[dd];
    }
  } else {  // one of the first or last w rows: skip the padding slots
    for (int dd = 0; dd <= 2 * hw; ++dd) {
      const int64_t c = i + dd - hw;
      if (c >= 0 && c < n) acc += d[(int64_t)dd * n] * x[c];
    }
  }
  __builtin_nontemporal_store(acc, y + i);
}

// Element type T: float, or double (the paper's element type; same kernel, eight bytes per slot).
template <typename T>
int run(int64_t n, int64_t w, const T *D, const T *x, T *y, void *stream) {
  if (n < 0 || w < 0) return DASTAC_EINVAL;
  if (w > (1 << 20)) return DASTAC_EOVERFLOW;
  if (n > ((int64_t)1 << 40) / (2 * w + 1)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!D || !x || !y) return DASTAC_ENULL;
  const int64_t sz = (int64_t)sizeof(T);
  if (overlaps(y, n * sz, D, (2 * w + 1) * n * sz) || overlaps(y, n * sz, x, n * sz)) return DASTAC_EALIAS;
  hipStream_t st = (hipStream_t)stream;
  const unsigned blocks = (unsigned)ceil_div(n, kBlock);
  switch (w) {
    case 16: band_kernel<16, T><<<blocks, kBlock, 0, st>>>(n, 16, D, x, y); break;
    case 8: band_kernel<8, T><<<blocks, kBlock, 0, st>>>(n, 8, D, x, y); break;
    case 4: band_kernel<4, T><<<blocks, kBlock, 0, st>>>(n, 4, D, x, y); break;
    case 2: band_kernel<2, T><<<blocks, kBlock, 0, st>>>(n, 2, D, x, y); break;
    case 1: band_kernel<1, T><<<blocks, kBlock, 0, st>>>(n, 1, D, x, y); break;
    case 0: band_kernel<0, T><<<blocks, kBlock, 0, st>>>(n, 0, D, x, y); break;
    default: band_kernel<-1, T><<<blocks, kBlock, 0, st>>>(n, (int)w, D, x, y);
  }
  return launch_status();
}

}  // namespace

extern "C" int dastac_band_spmv_f32(int64_t n, int64_t w, const float *D, const float *x, float *y, void *stream) {
  return run<float>(n, w, D, x, y, stream);
}

extern "C" int dastac_band_spmv_f64(int64_t n, int64_t w, const double *D, const double *x, double *y,
                                    void *stream) {
  return run<double>(n, w, D, x, y, stream);
}
