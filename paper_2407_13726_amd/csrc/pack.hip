// Compression / decompression kernels (Section 3, "Data layout compression": iterate over the
// accessed indices and copy the data in and out of the packed buffer).
//
// One workgroup handles one 256-element piece of one dense row, so both sides of the copy are
// contiguous across the lanes of a wavefront; the packed row start is the index polynomial of the
// row, computed once per workgroup from wave-uniform values and added to the lane's column.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBlock = 256;

// flattened (row, piece) -> row index and first column of the piece; `pieces` per row
__device__ inline void split(int64_t b, int64_t pieces, int64_t &row, int64_t &col0) {
  row = b / pieces;
  col0 = (b - row * pieces) * kBlock;
}

template <typename T>
__global__ __launch_bounds__(kBlock) void pack_triu_kernel(int64_t n, const T *__restrict__ dense, int64_t ld,
                                                           T *__restrict__ packed, int64_t pieces,
                                                           int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    int64_t i, c0;
    split(b, pieces, i, c0);
    if (c0 + kBlock <= i) continue;  // piece lies wholly left of the diagonal
    int64_t j = c0 + threadIdx.x;
    if (j >= i && j < n) packed[tri_row_start(n, i) + (j - i)] = dense[i * ld + j];
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void unpack_triu_kernel(int64_t n, const T *__restrict__ packed,
                                                             T *__restrict__ dense, int64_t ld, int64_t pieces,
                                                             int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    int64_t i, c0;
    split(b, pieces, i, c0);
    int64_t j = c0 + threadIdx.x;
    if (j < n) dense[i * ld + j] = (j >= i) ? packed[tri_row_start(n, i) + (j - i)] : T(0);
  }
}

// lower triangle: row i holds columns 0..i, starting at i(i+1)/2 (Section 4, worked example)
template <bool PACK, typename T>
__global__ __launch_bounds__(kBlock) void tril_copy_kernel(int64_t n, const T *__restrict__ src,
                                                           T *__restrict__ dst, int64_t ld, int64_t pieces,
                                                           int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    int64_t i, c0;
    split(b, pieces, i, c0);
    const int64_t j = c0 + threadIdx.x;
    if (j >= n) continue;
    const int64_t at = (i * (i + 1)) / 2 + j;
    if (PACK) {
      if (j <= i) dst[at] = src[i * ld + j];
    } else {
      dst[i * ld + j] = (j <= i) ? src[at] : T(0);
    }
  }
}

// rows of the cube are (i,j) pairs, flattened as i*n+j
template <typename T>
__global__ __launch_bounds__(kBlock) void pack_tet_kernel(int64_t n, const T *__restrict__ dense,
                                                          T *__restrict__ packed, int64_t pieces,
                                                          int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    int64_t ij, c0;
    split(b, pieces, ij, c0);
    int64_t i = ij / n, j = ij - i * n;
    if (j < i || c0 + kBlock <= j) continue;
    int64_t k = c0 + threadIdx.x;
    if (k >= j && k < n) packed[tet_row_start(n, i, j) + (k - j)] = dense[ij * n + k];
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void unpack_tet_kernel(int64_t n, const T *__restrict__ packed,
                                                            T *__restrict__ dense, int64_t pieces,
                                                            int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    int64_t ij, c0;
    split(b, pieces, ij, c0);
    int64_t i = ij / n, j = ij - i * n;
    int64_t k = c0 + threadIdx.x;
    if (k < n) dense[ij * n + k] = (j >= i && k >= j) ? packed[tet_row_start(n, i, j) + (k - j)] : T(0);
  }
}

// band: rows of the packed block are the diagonals d=-w..w, slot i holds entry (i, i+d)
template <typename T>
__global__ __launch_bounds__(kBlock) void pack_band_kernel(int64_t n, int64_t w, const T *__restrict__ dense,
                                                           int64_t ld, T *__restrict__ diag, int64_t pieces,
                                                           int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    int64_t dd, c0;
    split(b, pieces, dd, c0);
    int64_t d = dd - w, i = c0 + threadIdx.x;
    if (i < n) {
      int64_t j = i + d;
      diag[band_offset(n, w, d, i)] = (j >= 0 && j < n) ? dense[i * ld + j] : T(0);
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void unpack_band_kernel(int64_t n, int64_t w, const T *__restrict__ diag,
                                                             T *__restrict__ dense, int64_t ld, int64_t pieces,
                                                             int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    int64_t i, c0;
    split(b, pieces, i, c0);
    int64_t j = c0 + threadIdx.x;
    if (j < n) {
      int64_t d = j - i;
      dense[i * ld + j] = (d >= -w && d <= w) ? diag[band_offset(n, w, d, i)] : T(0);
    }
  }
}

inline unsigned grid_for(int64_t nblocks) { return (unsigned)(nblocks < (1 << 22) ? nblocks : (1 << 22)); }

// Largest dense extents accepted: the flattened (row, piece) count must stay far inside int64.
constexpr int64_t kDenseMaxN = 1 << 20;   // n*n row-major matrix
constexpr int64_t kCubeMaxN = 1 << 13;    // n*n*n cube

// Element type T: float, or double (the paper's element type).
template <typename T>
int pack_triu(int64_t n, const T *dense, int64_t ld, T *packed, void *stream) {
  if (n < 0 || ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !packed) return DASTAC_ENULL;
  if (overlaps(dense, n * ld * (int64_t)sizeof(T), packed, tri(n) * (int64_t)sizeof(T))) return DASTAC_EALIAS;
  int64_t pieces = ceil_div(n, kBlock), nblocks = n * pieces;
  pack_triu_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, dense, ld, packed, pieces, nblocks);
  return launch_status();
}

template <typename T>
int unpack_triu(int64_t n, const T *packed, T *dense, int64_t ld, void *stream) {
  if (n < 0 || ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !packed) return DASTAC_ENULL;
  if (overlaps(dense, n * ld * (int64_t)sizeof(T), packed, tri(n) * (int64_t)sizeof(T))) return DASTAC_EALIAS;
  int64_t pieces = ceil_div(n, kBlock), nblocks = n * pieces;
  unpack_triu_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, packed, dense, ld, pieces, nblocks);
  return launch_status();
}

template <typename T>
int pack_tet(int64_t n, const T *dense, T *packed, void *stream) {
  if (n < 0) return DASTAC_EINVAL;
  if (n > kCubeMaxN) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !packed) return DASTAC_ENULL;
  if (overlaps(dense, n * n * n * (int64_t)sizeof(T), packed, tet(n) * (int64_t)sizeof(T))) return DASTAC_EALIAS;
  int64_t pieces = ceil_div(n, kBlock), nblocks = n * n * pieces;
  pack_tet_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, dense, packed, pieces, nblocks);
  return launch_status();
}

template <typename T>
int unpack_tet(int64_t n, const T *packed, T *dense, void *stream) {
  if (n < 0) return DASTAC_EINVAL;
  if (n > kCubeMaxN) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !packed) return DASTAC_ENULL;
  if (overlaps(dense, n * n * n * (int64_t)sizeof(T), packed, tet(n) * (int64_t)sizeof(T))) return DASTAC_EALIAS;
  int64_t pieces = ceil_div(n, kBlock), nblocks = n * n * pieces;
  unpack_tet_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, packed, dense, pieces, nblocks);
  return launch_status();
}

template <typename T>
int pack_band(int64_t n, int64_t w, const T *dense, int64_t ld, T *diag_major, void *stream) {
  if (n < 0 || w < 0 || ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN || w > kDenseMaxN) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !diag_major) return DASTAC_ENULL;
  if (overlaps(dense, n * ld * (int64_t)sizeof(T), diag_major, (2 * w + 1) * n * (int64_t)sizeof(T))) return DASTAC_EALIAS;
  int64_t pieces = ceil_div(n, kBlock), nblocks = (2 * w + 1) * pieces;
  pack_band_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, w, dense, ld, diag_major, pieces,
                                                                          nblocks);
  return launch_status();
}

template <typename T>
int unpack_band(int64_t n, int64_t w, const T *diag_major, T *dense, int64_t ld, void *stream) {
  if (n < 0 || w < 0 || ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN || w > kDenseMaxN) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !diag_major) return DASTAC_ENULL;
  if (overlaps(dense, n * ld * (int64_t)sizeof(T), diag_major, (2 * w + 1) * n * (int64_t)sizeof(T))) return DASTAC_EALIAS;
  int64_t pieces = ceil_div(n, kBlock), nblocks = n * pieces;
  unpack_band_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, w, diag_major, dense, ld, pieces,
                                                                            nblocks);
  return launch_status();
}

// PACK: src is the dense matrix (row stride ld), dst the packed lower triangle; else the reverse
template <bool PACK, typename T>
int tril_copy(int64_t n, const T *src, T *dst, int64_t ld, void *stream) {
  if (n < 0 || ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!src || !dst) return DASTAC_ENULL;
  const int64_t dense_bytes = n * ld * (int64_t)sizeof(T), packed_bytes = tri(n) * (int64_t)sizeof(T);
  if (overlaps(src, PACK ? dense_bytes : packed_bytes, dst, PACK ? packed_bytes : dense_bytes)) return DASTAC_EALIAS;
  int64_t pieces = ceil_div(n, kBlock), nblocks = n * pieces;
  tril_copy_kernel<PACK, T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, src, dst, ld, pieces, nblocks);
  return launch_status();
}

}  // namespace

extern "C" {

int dastac_pack_triu_f32(int64_t n, const float *dense, int64_t ld, float *packed, void *stream) {
  return pack_triu<float>(n, dense, ld, packed, stream);
}

int dastac_pack_triu_f64(int64_t n, const double *dense, int64_t ld, double *packed, void *stream) {
  return pack_triu<double>(n, dense, ld, packed, stream);
}

int dastac_unpack_triu_f32(int64_t n, const float *packed, float *dense, int64_t ld, void *stream) {
  return unpack_triu<float>(n, packed, dense, ld, stream);
}

int dastac_unpack_triu_f64(int64_t n, const double *packed, double *dense, int64_t ld, void *stream) {
  return unpack_triu<double>(n, packed, dense, ld, stream);
}

int dastac_pack_tet_f32(int64_t n, const float *dense, float *packed, void *stream) {
  return pack_tet<float>(n, dense, packed, stream);
}

int dastac_pack_tet_f64(int64_t n, const double *dense, double *packed, void *stream) {
  return pack_tet<double>(n, dense, packed, stream);
}

int dastac_unpack_tet_f32(int64_t n, const float *packed, float *dense, void *stream) {
  return unpack_tet<float>(n, packed, dense, stream);
}

int dastac_unpack_tet_f64(int64_t n, const double *packed, double *dense, void *stream) {
  return unpack_tet<double>(n, packed, dense, stream);
}

int dastac_pack_band_f32(int64_t n, int64_t w, const float *dense, int64_t ld, float *diag_major, void *stream) {
  return pack_band<float>(n, w, dense, ld, diag_major, stream);
}

int dastac_pack_band_f64(int64_t n, int64_t w, const double *dense, int64_t ld, double *diag_major, void *stream) {
  return pack_band<double>(n, w, dense, ld, diag_major, stream);
}

int dastac_unpack_band_f32(int64_t n, int64_t w, const float *diag_major, float *dense, int64_t ld, void *stream) {
  return unpack_band<float>(n, w, diag_major, dense, ld, stream);
}

int dastac_unpack_band_f64(int64_t n, int64_t w, const double *diag_major, double *dense, int64_t ld, void *stream) {
  return unpack_band<double>(n, w, diag_major, dense, ld, stream);
}

int dastac_pack_tril_f32(int64_t n, const float *dense, int64_t ld, float *packed, void *stream) {
  return tril_copy<true, float>(n, dense, packed, ld, stream);
}

int dastac_pack_tril_f64(int64_t n, const double *dense, int64_t ld, double *packed, void *stream) {
  return tril_copy<true, double>(n, dense, packed, ld, stream);
}

int dastac_unpack_tril_f32(int64_t n, const float *packed, float *dense, int64_t ld, void *stream) {
  return tril_copy<false, float>(n, packed, dense, ld, stream);
}

int dastac_unpack_tril_f64(int64_t n, const double *packed, double *dense, int64_t ld, void *stream) {
  return tril_copy<false, double>(n, packed, dense, ld, stream);
}

}  // extern "C"
