// Three more structures, each a single-piece index polynomial over the same streaming pattern:
//
//   strided band   (Section 6.4, "Distance of Elements and Compression"): summands j-i = d*s,
//                  d=-w..w; the paper's experiment is w=1.  Same diagonal-major buffers as the
//                  unit-stride band, slot (d,i) holds A[i][i+d*s]; only the column a slot
//                  multiplies with changes, so the packed streams stay perfectly contiguous
//                  whatever the stride.
//   sub-triangular (Section 6.4, "Density and Compression"): j-i >= N-k.  Its unique set is the
//                  upper triangle of the k x k block in the top right corner, so
//                  subtri(N,k,i,j) = tri(k,i,j-(N-k)) and the product is the packed TRMV of order
//                  k on the last k entries of x; rows k..N-1 hold no element and give 0.
//   Leslie         (Table 2, SpMV_L): (i=0)(0<=j<n) + (1<=i<n)(j=i-1); two summands, two buffers:
//                  R[n], the first row in order of j, and S[n-1], the sub-diagonal in order of i.
//                  Output 0 is a dot product over the whole first row, every other output is one
//                  product; both read x(j) once.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBlock = 256;
constexpr int64_t kDenseMaxN = 1 << 20;
constexpr int kLeslieMaxBlocks = 1024;  // one atomic per workgroup lands on y(0)

inline unsigned grid_for(int64_t nblocks) { return (unsigned)(nblocks < (1 << 22) ? nblocks : (1 << 22)); }

// ---- strided band ---------------------------------------------------------------------------

// W >= 0: half-width known at compile time; W < 0: run-time half-width `w`.  One row per lane.
template <int W, typename T>
__global__ __launch_bounds__(kBlock) void sband_kernel(int64_t n, int w, int64_t s, const T *__restrict__ D,
                                                       const T *__restrict__ x, T *__restrict__ y) {
  const int hw = W >= 0 ? W : w;
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  const T *d = D + i;
  const int64_t reach = (int64_t)hw * s;
  T acc = T(0);
  if (i >= reach && i + reach < n) {  // interior row: every column exists
    const T *xw = x + (i - reach);
    if (W >= 0) {
#pragma unroll
      for (int dd = 0; dd <= 2 * (W >= 0 ? W : 0); ++dd)
        acc += __builtin_nontemporal_load(d + (int64_t)dd * n) * xw[(int64_t)dd * s];
    } else {
      for (int dd = 0; dd <= 2 * hw; ++dd)
        acc += __builtin_nontemporal_load(d + (int64_t)dd * n) * xw[(int64_t)dd * s];
    }
  } else {  // a row whose window leaves the matrix: skip the padding slots
    for (int dd = 0; dd <= 2 * hw; ++dd) {
      const int64_t c = i + (int64_t)(dd - hw) * s;
      if (c >= 0 && c < n) acc += d[(int64_t)dd * n] * x[c];
    }
  }
  __builtin_nontemporal_store(acc, y + i);
}

// The printed rule (w = 1): three streams of D and three windows of x carry too few bytes per lane when a lane
// takes one row, so a lane takes the 16 bytes of consecutive rows (four in single, two in double precision) of
// every stream at once.  Groups of rows whose windows leave the matrix take the tested path row by row.
template <typename T>
__global__ __launch_bounds__(kBlock) void sband_w1_kernel(int64_t n, int64_t s, const T *__restrict__ D,
                                                          const T *__restrict__ x, T *__restrict__ y) {
  constexpr int V = 16 / (int)sizeof(T);
  typedef T vecu __attribute__((ext_vector_type(V), aligned(sizeof(T))));  // rows start at any element
  const int64_t i = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * V;
  if (i >= n) return;
  if (i >= s && i + V - 1 + s < n) {  // interior rows: every column exists
    const vecu d0 = __builtin_nontemporal_load(reinterpret_cast<const vecu *>(D + i));
    const vecu d1 = __builtin_nontemporal_load(reinterpret_cast<const vecu *>(D + n + i));
    const vecu d2 = __builtin_nontemporal_load(reinterpret_cast<const vecu *>(D + 2 * n + i));
    const vecu x0 = *reinterpret_cast<const vecu *>(x + i - s);
    const vecu x1 = *reinterpret_cast<const vecu *>(x + i);
    const vecu x2 = *reinterpret_cast<const vecu *>(x + i + s);
    vecu acc;
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = ((T(0) + d0[v] * x0[v]) + d1[v] * x1[v]) + d2[v] * x2[v];  // from +0, like a running sum
    __builtin_nontemporal_store(acc, reinterpret_cast<vecu *>(y + i));
  } else {
    for (int64_t r = i; r < i + V && r < n; ++r) {
      T acc = T(0);
      for (int dd = 0; dd < 3; ++dd) {
        const int64_t c = r + (int64_t)(dd - 1) * s;
        if (c >= 0 && c < n) acc += D[(int64_t)dd * n + r] * x[c];
      }
      y[r] = acc;
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void pack_sband_kernel(int64_t n, int64_t w, int64_t s,
                                                            const T *__restrict__ dense, int64_t ld,
                                                            T *__restrict__ diag, int64_t pieces,
                                                            int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    const int64_t dw = b / pieces;  // d + w
    const int64_t i = (b - dw * pieces) * kBlock + threadIdx.x;
    if (i >= n) continue;
    const int64_t j = i + (dw - w) * s;
    diag[dw * n + i] = (j >= 0 && j < n) ? dense[i * ld + j] : T(0);
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void unpack_sband_kernel(int64_t n, int64_t w, int64_t s,
                                                              const T *__restrict__ diag,
                                                              T *__restrict__ dense, int64_t ld,
                                                              int64_t pieces, int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    const int64_t i = b / pieces;
    const int64_t j = (b - i * pieces) * kBlock + threadIdx.x;
    if (j >= n) continue;
    const int64_t dj = j - i, d = dj / s;  // exact only on a stored diagonal
    const bool stored = d * s == dj && d >= -w && d <= w;
    dense[i * ld + j] = stored ? diag[(d + w) * n + i] : T(0);
  }
}

// ---- sub-triangular -------------------------------------------------------------------------

template <typename T>
__global__ __launch_bounds__(kBlock) void unpack_subtri_kernel(int64_t N, int64_t k, const T *__restrict__ packed,
                                                               T *__restrict__ dense, int64_t ld,
                                                               int64_t pieces, int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    const int64_t i = b / pieces;
    const int64_t j = (b - i * pieces) * kBlock + threadIdx.x;
    if (j >= N) continue;
    const int64_t c = j - (N - k);  // column inside the k x k corner block
    dense[i * ld + j] = (i < k && c >= i) ? packed[tri_offset(k, i, c)] : T(0);
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void zero_tail_kernel(T *__restrict__ y, int64_t count) {
  const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (t < count) y[t] = T(0);
}

// ---- Leslie ---------------------------------------------------------------------------------

template <typename T>
__global__ __launch_bounds__(kBlock) void leslie_kernel(int64_t n, const T *__restrict__ R,
                                                        const T *__restrict__ S, const T *__restrict__ x,
                                                        T *__restrict__ y) {
  __shared__ T part[kBlock / 64];
  constexpr int V = 16 / (int)sizeof(T);  // a lane takes the 16 bytes of consecutive rows of every stream at once
  typedef T vecu __attribute__((ext_vector_type(V), aligned(sizeof(T))));
  const int64_t stride = (int64_t)gridDim.x * kBlock * V;
  T acc = T(0);
  int64_t j = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * V;
  for (; j + 3 * stride + V < n; j += 4 * stride) {  // four independent groups of rows in flight per lane, all with successors
    vecu xv[4], rv[4], sv[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      xv[q] = *reinterpret_cast<const vecu *>(x + j + q * stride);
      rv[q] = __builtin_nontemporal_load(reinterpret_cast<const vecu *>(R + j + q * stride));
      sv[q] = __builtin_nontemporal_load(reinterpret_cast<const vecu *>(S + j + q * stride));
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      vecu p;
#pragma unroll
      for (int v = 0; v < V; ++v) {
        acc += rv[q][v] * xv[q][v];
        p[v] = sv[q][v] * xv[q][v];
      }
      __builtin_nontemporal_store(p, reinterpret_cast<vecu *>(y + j + q * stride + 1));
    }
  }
  for (; j < n; j += stride)
    for (int64_t r = j; r < j + V && r < n; ++r) {
      const T xr = x[r];
      acc += R[r] * xr;
      if (r + 1 < n) y[r + 1] = S[r] * xr;
    }
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    T t = T(0);
    for (int v = 0; v < kBlock / 64; ++v) t += part[v];
    atomicAdd(y, t);  // y(0) was cleared by the launch before this one
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void pack_leslie_kernel(int64_t n, const T *__restrict__ dense, int64_t ld,
                                                             T *__restrict__ R, T *__restrict__ S) {
  const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (j >= n) return;
  R[j] = dense[j];
  if (j + 1 < n) S[j] = dense[(j + 1) * ld + j];
}

template <typename T>
__global__ __launch_bounds__(kBlock) void unpack_leslie_kernel(int64_t n, const T *__restrict__ R,
                                                               const T *__restrict__ S,
                                                               T *__restrict__ dense, int64_t ld, int64_t pieces,
                                                               int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    const int64_t i = b / pieces;
    const int64_t j = (b - i * pieces) * kBlock + threadIdx.x;
    if (j >= n) continue;
    dense[i * ld + j] = i == 0 ? R[j] : (j == i - 1 ? S[j] : T(0));
  }
}

int check_sband(int64_t n, int64_t w, int64_t s) {
  if (n < 0 || w < 0 || s < 1) return DASTAC_EINVAL;
  if (s > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  return DASTAC_OK;
}
// the packed upper-triangular entry points of either precision
inline int pack_triu(int64_t n, const float *d, int64_t ld, float *p, void *st) {
  return dastac_pack_triu_f32(n, d, ld, p, st);
}
inline int pack_triu(int64_t n, const double *d, int64_t ld, double *p, void *st) {
  return dastac_pack_triu_f64(n, d, ld, p, st);
}

template <typename T>
int pack_sband(int64_t n, int64_t w, int64_t s, const T *dense, int64_t ld, T *diag_major, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (int rc = check_sband(n, w, s)) return rc;
  if (ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN || w > kDenseMaxN || ld_too_large(ld)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !diag_major) return DASTAC_ENULL;
  if (overlaps(dense, view_bytes(n, ld, n, kB), diag_major, (2 * w + 1) * n * kB)) return DASTAC_EALIAS;
  const int64_t pieces = ceil_div(n, kBlock), nblocks = (2 * w + 1) * pieces;
  pack_sband_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, w, s, dense, ld, diag_major, pieces,
                                                                           nblocks);
  return launch_status();
}

template <typename T>
int unpack_sband(int64_t n, int64_t w, int64_t s, const T *diag_major, T *dense, int64_t ld, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (int rc = check_sband(n, w, s)) return rc;
  if (ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN || w > kDenseMaxN || ld_too_large(ld)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !diag_major) return DASTAC_ENULL;
  if (overlaps(dense, view_bytes(n, ld, n, kB), diag_major, (2 * w + 1) * n * kB)) return DASTAC_EALIAS;
  const int64_t pieces = ceil_div(n, kBlock), nblocks = n * pieces;
  unpack_sband_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, w, s, diag_major, dense, ld, pieces,
                                                                             nblocks);
  return launch_status();
}

template <typename T>
int sband_spmv(int64_t n, int64_t w, int64_t s, const T *D, const T *x, T *y, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (int rc = check_sband(n, w, s)) return rc;
  if (w > (1 << 20)) return DASTAC_EOVERFLOW;
  if (n > ((int64_t)1 << 40) / (2 * w + 1)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!D || !x || !y) return DASTAC_ENULL;
  if (overlaps(y, n * kB, D, (2 * w + 1) * n * kB) || overlaps(y, n * kB, x, n * kB)) return DASTAC_EALIAS;
  hipStream_t st = (hipStream_t)stream;
  const unsigned blocks = (unsigned)ceil_div(n, kBlock);
  if (w == 1)
    sband_w1_kernel<T><<<(unsigned)ceil_div(n, kBlock * (16 / kB)), kBlock, 0, st>>>(n, s, D, x, y);
  else
    sband_kernel<-1, T><<<blocks, kBlock, 0, st>>>(n, (int)w, s, D, x, y);
  return launch_status();
}

template <typename T>
int pack_subtri(int64_t N, int64_t k, const T *dense, int64_t ld, T *packed, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (N < 0 || k < 0 || k > N || ld < N) return DASTAC_EINVAL;
  if (N > kDenseMaxN || ld_too_large(ld)) return DASTAC_EOVERFLOW;
  if (k == 0) return DASTAC_OK;
  if (!dense || !packed) return DASTAC_ENULL;
  if (overlaps(dense, view_bytes(N, ld, N, kB), packed, tri(k) * kB)) return DASTAC_EALIAS;
  // the unique set is the upper triangle of the k x k block whose first column is N-k
  return pack_triu(k, dense + (N - k), ld, packed, stream);
}

template <typename T>
int unpack_subtri(int64_t N, int64_t k, const T *packed, T *dense, int64_t ld, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (N < 0 || k < 0 || k > N || ld < N) return DASTAC_EINVAL;
  if (N > kDenseMaxN || ld_too_large(ld)) return DASTAC_EOVERFLOW;
  if (N == 0) return DASTAC_OK;
  if (!dense || (k > 0 && !packed)) return DASTAC_ENULL;
  if (overlaps(dense, view_bytes(N, ld, N, kB), packed, tri(k) * kB)) return DASTAC_EALIAS;
  const int64_t pieces = ceil_div(N, kBlock), nblocks = N * pieces;
  unpack_subtri_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(N, k, packed, dense, ld, pieces,
                                                                              nblocks);
  return launch_status();
}

template <typename T>
int subtri_spmv(int64_t N, int64_t k, const T *Ap, const T *x, T *y, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (N < 0 || k < 0 || k > N) return DASTAC_EINVAL;
  if (N > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  if (N == 0) return DASTAC_OK;
  if (!x || !y || (k > 0 && !Ap)) return DASTAC_ENULL;
  if (overlaps(y, N * kB, x, N * kB) || overlaps(y, N * kB, Ap, tri(k) * kB)) return DASTAC_EALIAS;
  if (k > 0) return trmv_then_zeros(k, Ap, x + (N - k), y, N - k, stream);  // also bounds k
  zero_tail_kernel<T><<<(unsigned)ceil_div(N, kBlock), kBlock, 0, (hipStream_t)stream>>>(y, N);
  return launch_status();
}

template <typename T>
int pack_leslie(int64_t n, const T *dense, int64_t ld, T *R, T *S, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (n < 0 || ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN || ld_too_large(ld)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !R || (n > 1 && !S)) return DASTAC_ENULL;
  if (overlaps(dense, view_bytes(n, ld, n, kB), R, n * kB) || overlaps(dense, view_bytes(n, ld, n, kB), S, (n - 1) * kB) ||
      overlaps(R, n * kB, S, (n - 1) * kB))
    return DASTAC_EALIAS;
  pack_leslie_kernel<T><<<(unsigned)ceil_div(n, kBlock), kBlock, 0, (hipStream_t)stream>>>(n, dense, ld, R, S);
  return launch_status();
}

template <typename T>
int unpack_leslie(int64_t n, const T *R, const T *S, T *dense, int64_t ld, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (n < 0 || ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN || ld_too_large(ld)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !R || (n > 1 && !S)) return DASTAC_ENULL;
  if (overlaps(dense, view_bytes(n, ld, n, kB), R, n * kB) || overlaps(dense, view_bytes(n, ld, n, kB), S, (n - 1) * kB)) return DASTAC_EALIAS;
  const int64_t pieces = ceil_div(n, kBlock), nblocks = n * pieces;
  unpack_leslie_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, R, S, dense, ld, pieces, nblocks);
  return launch_status();
}

template <typename T>
int leslie_spmv(int64_t n, const T *R, const T *S, const T *x, T *y, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (n < 0) return DASTAC_EINVAL;
  if (n > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!R || !x || !y || (n > 1 && !S)) return DASTAC_ENULL;
  if (overlaps(y, n * kB, x, n * kB) || overlaps(y, n * kB, R, n * kB) || overlaps(y, n * kB, S, (n - 1) * kB))
    return DASTAC_EALIAS;
  hipStream_t st = (hipStream_t)stream;
  zero_tail_kernel<T><<<1, kBlock, 0, st>>>(y, 1);
  if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  const int64_t want = ceil_div(n, 4 * kBlock * (16 / kB));  // about four 16-byte groups of rows per lane before the cap
  const unsigned blocks = (unsigned)(want < 1 ? 1 : want > kLeslieMaxBlocks ? kLeslieMaxBlocks : want);
  leslie_kernel<T><<<blocks, kBlock, 0, st>>>(n, R, S, x, y);
  return launch_status();
}


}  // namespace

extern "C" {

int64_t dastac_subtri_offset(int64_t N, int64_t k, int64_t i, int64_t j) {
  if (N < 0 || N > DASTAC_TRI_MAX_N || k < 0 || k > N || i < 0 || j >= N || j - i < N - k) return -1;
  return tri_offset(k, i, j - (N - k));
}

int dastac_pack_sband_f32(int64_t n, int64_t w, int64_t s, const float *dense, int64_t ld, float *diag_major,
                          void *stream) {
  return pack_sband<float>(n, w, s, dense, ld, diag_major, stream);
}
int dastac_unpack_sband_f32(int64_t n, int64_t w, int64_t s, const float *diag_major, float *dense, int64_t ld,
                            void *stream) {
  return unpack_sband<float>(n, w, s, diag_major, dense, ld, stream);
}
int dastac_sband_spmv_f32(int64_t n, int64_t w, int64_t s, const float *D, const float *x, float *y, void *stream) {
  return sband_spmv<float>(n, w, s, D, x, y, stream);
}
int dastac_pack_subtri_f32(int64_t N, int64_t k, const float *dense, int64_t ld, float *packed, void *stream) {
  return pack_subtri<float>(N, k, dense, ld, packed, stream);
}
int dastac_unpack_subtri_f32(int64_t N, int64_t k, const float *packed, float *dense, int64_t ld, void *stream) {
  return unpack_subtri<float>(N, k, packed, dense, ld, stream);
}
int dastac_subtri_spmv_f32(int64_t N, int64_t k, const float *Ap, const float *x, float *y, void *stream) {
  return subtri_spmv<float>(N, k, Ap, x, y, stream);
}
int dastac_pack_leslie_f32(int64_t n, const float *dense, int64_t ld, float *R, float *S, void *stream) {
  return pack_leslie<float>(n, dense, ld, R, S, stream);
}
int dastac_unpack_leslie_f32(int64_t n, const float *R, const float *S, float *dense, int64_t ld, void *stream) {
  return unpack_leslie<float>(n, R, S, dense, ld, stream);
}
int dastac_leslie_spmv_f32(int64_t n, const float *R, const float *S, const float *x, float *y, void *stream) {
  return leslie_spmv<float>(n, R, S, x, y, stream);
}

int dastac_pack_sband_f64(int64_t n, int64_t w, int64_t s, const double *dense, int64_t ld, double *diag_major,
                          void *stream) {
  return pack_sband<double>(n, w, s, dense, ld, diag_major, stream);
}
int dastac_unpack_sband_f64(int64_t n, int64_t w, int64_t s, const double *diag_major, double *dense, int64_t ld,
                            void *stream) {
  return unpack_sband<double>(n, w, s, diag_major, dense, ld, stream);
}
int dastac_sband_spmv_f64(int64_t n, int64_t w, int64_t s, const double *D, const double *x, double *y, void *stream) {
  return sband_spmv<double>(n, w, s, D, x, y, stream);
}
int dastac_pack_subtri_f64(int64_t N, int64_t k, const double *dense, int64_t ld, double *packed, void *stream) {
  return pack_subtri<double>(N, k, dense, ld, packed, stream);
}
int dastac_unpack_subtri_f64(int64_t N, int64_t k, const double *packed, double *dense, int64_t ld, void *stream) {
  return unpack_subtri<double>(N, k, packed, dense, ld, stream);
}
int dastac_subtri_spmv_f64(int64_t N, int64_t k, const double *Ap, const double *x, double *y, void *stream) {
  return subtri_spmv<double>(N, k, Ap, x, y, stream);
}
int dastac_pack_leslie_f64(int64_t n, const double *dense, int64_t ld, double *R, double *S, void *stream) {
  return pack_leslie<double>(n, dense, ld, R, S, stream);
}
int dastac_unpack_leslie_f64(int64_t n, const double *R, const double *S, double *dense, int64_t ld, void *stream) {
  return unpack_leslie<double>(n, R, S, dense, ld, stream);
}
int dastac_leslie_spmv_f64(int64_t n, const double *R, const double *S, const double *x, double *y, void *stream) {
  return leslie_spmv<double>(n, R, S, x, y, stream);
}

}  // extern "C"
