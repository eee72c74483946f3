// MTTKRP over a packed upper tetrahedron:  M(i,r) := A(i,j,k) * B(j,r) * C(k,r), i<=j<=k.
// First version: one workgroup per slice i, one wavefront per row (i,j), plain FMA (no matrix cores yet).
#include "common.h"

using namespace dastac;

namespace {
constexpr int kBlock = 256;

__global__ __launch_bounds__(kBlock) void mttkrp_simple_kernel(int64_t n, int R, const float *__restrict__ A,
                                                               const float *__restrict__ B, int64_t ldb,
                                                               const float *__restrict__ C, int64_t ldc,
                                                               float *__restrict__ M, int64_t ldm) {
  __shared__ float part[kBlock / 64][32];
  const int64_t i = blockIdx.x;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int r = lane & 31, half = lane >> 5;
  float macc = 0.0f;
  for (int64_t j = i + wv; j < n; j += kBlock / 64) {
    const float *a = A + tet_row_start(n, i, j);
    float t = 0.0f;
    if (r < R)
      for (int64_t k = j + half; k < n; k += 2) t += a[k - j] * C[k * ldc + r];
    t += __shfl_xor(t, 32, 64);
    if (r < R) macc += t * B[j * ldb + r];
  }
  if (half == 0) part[wv][r] = macc;
  __syncthreads();
  if (threadIdx.x < R) {
    float s = 0.0f;
    for (int q = 0; q < kBlock / 64; ++q) s += part[q][threadIdx.x];
    M[i * ldm + threadIdx.x] = s;
  }
}
}  // namespace

extern "C" int dastac_tet_mttkrp_f32(int64_t n, int64_t R, const float *Ap, const float *B, int64_t ldb,
                                     const float *C, int64_t ldc, float *M, int64_t ldm, void *stream) {
  if (n < 0 || R < 1 || R > 32 || ldb < R || ldc < R || ldm < R) return DASTAC_EINVAL;
  if (n > DASTAC_TET_MAX_N || tet(n) > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Ap || !B || !C || !M) return DASTAC_ENULL;
  if (overlaps(M, n * ldm * 4, Ap, tet(n) * 4) || overlaps(M, n * ldm * 4, B, n * ldb * 4) ||
      overlaps(M, n * ldm * 4, C, n * ldc * 4))
    return DASTAC_EALIAS;
  mttkrp_simple_kernel<<<(unsigned)n, kBlock, 0, (hipStream_t)stream>>>(n, (int)R, Ap, B, ldb, C, ldc, M, ldm);
  return launch_status();
}
