// TRMM over a packed upper triangle:  C(i,c) := U(i,k) * B(k,c), i<=k.
// First version: one output element per lane, plain FMA loop (no matrix cores yet).
#include "common.h"

using namespace dastac;

namespace {
constexpr int kBlock = 256;

__global__ __launch_bounds__(kBlock) void trmm_simple_kernel(int64_t n, int64_t m, const float *__restrict__ U,
                                                             const float *__restrict__ B, int64_t ldb,
                                                             float *__restrict__ C, int64_t ldc) {
  const int64_t i = blockIdx.y;
  const int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (c >= m) return;
  const float *u = U + tri_row_start(n, i);
  float acc = 0.0f;
  for (int64_t k = i; k < n; ++k) acc += u[k - i] * B[k * ldb + c];
  C[i * ldc + c] = acc;
}
}  // namespace

extern "C" int dastac_trmm_f32(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C,
                               int64_t ldc, void *stream) {
  if (n < 0 || m < 1 || ldb < m || ldc < m) return DASTAC_EINVAL;
  if (n > 65535) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Up || !B || !C) return DASTAC_ENULL;
  if (overlaps(C, n * ldc * 4, Up, tri(n) * 4) || overlaps(C, n * ldc * 4, B, n * ldb * 4)) return DASTAC_EALIAS;
  dim3 grid((unsigned)ceil_div(m, kBlock), (unsigned)n);
  trmm_simple_kernel<<<grid, kBlock, 0, (hipStream_t)stream>>>(n, m, Up, B, ldb, C, ldc);
  return launch_status();
}
