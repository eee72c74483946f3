// Compression / decompression kernels (Section 3, "Data layout compression": iterate over the
// accessed indices and copy the data in and out of the packed buffer).
//
// Triangles and the tetrahedron: the accessed indices of one dense row are one contiguous piece of
// the packed buffer whose start is the index polynomial of the row, so both kinds of copy are
// copies of contiguous spans.  A wavefront takes one span at a time (a row, or a 2048-element segment
// of a long row): a few scalar elements until the destination is 16-byte aligned, then aligned
// 16-byte non-temporal stores fed by 16-byte loads that only assume element alignment (a packed row
// starts at an arbitrary element), four in flight per lane, then the last few elements.
// Decompression also writes the zeros of the row outside the domain, the same way.
// The band (small matrices only: the dense form has n*n elements) keeps the element-wise kernels.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBlock = 256;
constexpr int64_t kSeg = 2048;  // elements of a dense row per work item

// flattened (row, piece) -> row index and first column of the piece; `pieces` per row
__device__ inline void split(int64_t b, int64_t pieces, int64_t &row, int64_t &col0) {
  row = b / pieces;
  col0 = (b - row * pieces) * kBlock;
}

template <typename T>
struct Piece;
template <>
struct Piece<float> {
  typedef float aligned_t __attribute__((ext_vector_type(4)));
  typedef float loose_t __attribute__((ext_vector_type(4), aligned(4)));
};
template <>
struct Piece<double> {
  typedef double aligned_t __attribute__((ext_vector_type(2)));
  typedef double loose_t __attribute__((ext_vector_type(2), aligned(8)));
};

// One wavefront copies src[0..len) to dst[0..len), or writes zeros when src is null.
template <typename T>
__device__ inline void span(const T *__restrict__ src, T *__restrict__ dst, int64_t len, int lane) {
  typedef typename Piece<T>::aligned_t vec;
  typedef typename Piece<T>::loose_t uvec;
  constexpr int V = 16 / (int)sizeof(T);
  if (len <= 0) return;
  const bool zero = src == nullptr;
  int64_t head = (int64_t)(((16 - ((uintptr_t)dst & 15)) & 15) / sizeof(T));  // elements before dst is 16-byte aligned
  if (head > len) head = len;
  if (lane < head) dst[lane] = zero ? T(0) : src[lane];
  const int64_t nvec = (len - head) / V;
  vec *d = reinterpret_cast<vec *>(dst + head);
  const uvec *q = reinterpret_cast<const uvec *>(src + head);
  int64_t v = lane;
  if (zero) {
    vec z;
    for (int c = 0; c < V; ++c) z[c] = T(0);
    for (; v < nvec; v += 64) __builtin_nontemporal_store(z, d + v);
  } else {
    for (; v + 192 < nvec; v += 256) {
      const vec a0 = __builtin_nontemporal_load(q + v), a1 = __builtin_nontemporal_load(q + v + 64);
      const vec a2 = __builtin_nontemporal_load(q + v + 128), a3 = __builtin_nontemporal_load(q + v + 192);
      __builtin_nontemporal_store(a0, d + v);
      __builtin_nontemporal_store(a1, d + v + 64);
      __builtin_nontemporal_store(a2, d + v + 128);
      __builtin_nontemporal_store(a3, d + v + 192);
    }
    for (; v < nvec; v += 64) {
      const vec a0 = __builtin_nontemporal_load(q + v);
      __builtin_nontemporal_store(a0, d + v);
    }
  }
  const int64_t done = head + nvec * V;
  if (lane < len - done) dst[done + lane] = zero ? T(0) : src[done + lane];
}

// Work items of a wavefront: w, w + nwaves, ...
__device__ inline void my_items(int64_t &first, int64_t &stride, int &lane) {
  lane = threadIdx.x & 63;
  first = (int64_t)blockIdx.x * (kBlock / 64) + uniform32(threadIdx.x >> 6);
  stride = (int64_t)gridDim.x * (kBlock / 64);
}

// Packed triangle <-> dense matrix.  LOWER: row i holds the columns 0..i, starting at i(i+1)/2 (Section 4,
// worked example); else the columns i..n-1, starting at tri_row_start.  A work item is segment `seg` of dense row i.
template <typename T, bool LOWER, bool PACK>
__global__ __launch_bounds__(kBlock) void tri_copy_kernel(int64_t n, const T *__restrict__ src, T *__restrict__ dst,
                                                          int64_t ld, int64_t segs, int64_t items) {
  int64_t it, stride;
  int lane;
  my_items(it, stride, lane);
  for (; it < items; it += stride) {
    const int64_t i = uniform64(it / segs);
    const int64_t s0 = (it - i * segs) * kSeg, s1 = s0 + kSeg < n ? s0 + kSeg : n;
    const int64_t c0 = LOWER ? 0 : i, c1 = LOWER ? i + 1 : n;               // the row's columns inside the domain
    const int64_t at0 = LOWER ? (i * (i + 1)) / 2 : tri_row_start(n, i) - i;  // packed position of column 0 of the row
    const int64_t a = s0 > c0 ? s0 : c0, b = s1 < c1 ? s1 : c1;              // the segment's part of them
    if (PACK) {
      span<T>(src + i * ld + a, dst + at0 + a, b - a, lane);
    } else {
      T *row = dst + i * ld;
      const int64_t z1 = c0 < s1 ? c0 : s1, z2 = c1 > s0 ? c1 : s0;
      span<T>(nullptr, row + s0, z1 - s0, lane);
      span<T>(src + at0 + a, row + a, b - a, lane);
      span<T>(nullptr, row + z2, s1 - z2, lane);
    }
  }
}

// Packed tetrahedron -> dense cube: a work item is dense row (i,j), zeros and all.
template <typename T>
__global__ __launch_bounds__(kBlock) void unpack_tet_kernel(int64_t n, const T *__restrict__ packed,
                                                            T *__restrict__ dense, int64_t items) {
  int64_t it, stride;
  int lane;
  my_items(it, stride, lane);
  for (; it < items; it += stride) {
    const int64_t i = uniform64(it / n), j = it - i * n;
    T *row = dense + it * n;
    if (j < i) {
      span<T>(nullptr, row, n, lane);
    } else {
      span<T>(nullptr, row, j, lane);
      span<T>(packed + tet_row_start(n, i, j), row + j, n - j, lane);
    }
  }
}

// Dense cube -> packed tetrahedron: a work item is the r-th row of the domain, r = tri(n,i,j); its
// elements follow those of row r-1 in the packed buffer.
template <typename T>
__global__ __launch_bounds__(kBlock) void pack_tet_kernel(int64_t n, const T *__restrict__ dense,
                                                          T *__restrict__ packed, int64_t items) {
  int64_t it, stride;
  int lane;
  my_items(it, stride, lane);
  for (; it < items; it += stride) {
    int64_t i, j;
    tri_inverse(n, it, i, j);
    i = uniform64(i);
    j = uniform64(j);
    span<T>(dense + (i * n + j) * n + j, packed + tet_row_start(n, i, j), n - j, lane);
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

// Workgroups for `items` wavefront-sized work items: four wavefronts each, at most what keeps every
// compute unit of a 256-CU part filled several times over (the wavefronts loop over the rest).
inline unsigned grid_for_items(int64_t items) {
  const int64_t wg = ceil_div(items, kBlock / 64);
  return (unsigned)(wg < 256 * 64 ? wg : 256 * 64);
}

// Largest dense extents accepted: the flattened (row, piece) count must stay far inside int64.
constexpr int64_t kDenseMaxN = 1 << 20;   // n*n row-major matrix
constexpr int64_t kCubeMaxN = 1 << 13;    // n*n*n cube

// PACK: src is the dense matrix (row stride ld), dst the packed triangle; else the reverse.
// Element type T: float, or double (the paper's element type).
template <typename T, bool LOWER, bool PACK>
int tri_copy(int64_t n, const T *src, T *dst, int64_t ld, void *stream) {
  if (n < 0 || ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN || ld_too_large(ld)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!src || !dst) return DASTAC_ENULL;
  const int64_t dense_bytes = view_bytes(n, ld, n, sizeof(T)), packed_bytes = tri(n) * (int64_t)sizeof(T);
  if (overlaps(src, PACK ? dense_bytes : packed_bytes, dst, PACK ? packed_bytes : dense_bytes)) return DASTAC_EALIAS;
  const int64_t segs = ceil_div(n, kSeg), items = n * segs;
  tri_copy_kernel<T, LOWER, PACK><<<grid_for_items(items), kBlock, 0, (hipStream_t)stream>>>(n, src, dst, ld, segs, items);
  return launch_status();
}

template <typename T>
int pack_tet(int64_t n, const T *dense, T *packed, void *stream) {
  if (n < 0) return DASTAC_EINVAL;
  if (n > kCubeMaxN) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !packed) return DASTAC_ENULL;
  if (overlaps(dense, n * n * n * (int64_t)sizeof(T), packed, tet(n) * (int64_t)sizeof(T))) return DASTAC_EALIAS;
  pack_tet_kernel<T><<<grid_for_items(tri(n)), kBlock, 0, (hipStream_t)stream>>>(n, dense, packed, tri(n));
  return launch_status();
}

template <typename T>
int unpack_tet(int64_t n, const T *packed, T *dense, void *stream) {
  if (n < 0) return DASTAC_EINVAL;
  if (n > kCubeMaxN) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !packed) return DASTAC_ENULL;
  if (overlaps(dense, n * n * n * (int64_t)sizeof(T), packed, tet(n) * (int64_t)sizeof(T))) return DASTAC_EALIAS;
  unpack_tet_kernel<T><<<grid_for_items(n * n), kBlock, 0, (hipStream_t)stream>>>(n, packed, dense, n * n);
  return launch_status();
}

template <typename T>
int pack_band(int64_t n, int64_t w, const T *dense, int64_t ld, T *diag_major, void *stream) {
  if (n < 0 || w < 0 || ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN || w > kDenseMaxN || ld_too_large(ld)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !diag_major) return DASTAC_ENULL;
  if (overlaps(dense, view_bytes(n, ld, n, sizeof(T)), diag_major, (2 * w + 1) * n * (int64_t)sizeof(T))) return DASTAC_EALIAS;
  int64_t pieces = ceil_div(n, kBlock), nblocks = (2 * w + 1) * pieces;
  pack_band_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, w, dense, ld, diag_major, pieces,
                                                                          nblocks);
  return launch_status();
}

template <typename T>
int unpack_band(int64_t n, int64_t w, const T *diag_major, T *dense, int64_t ld, void *stream) {
  if (n < 0 || w < 0 || ld < n) return DASTAC_EINVAL;
  if (n > kDenseMaxN || w > kDenseMaxN || ld_too_large(ld)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!dense || !diag_major) return DASTAC_ENULL;
  if (overlaps(dense, view_bytes(n, ld, n, sizeof(T)), diag_major, (2 * w + 1) * n * (int64_t)sizeof(T))) return DASTAC_EALIAS;
  int64_t pieces = ceil_div(n, kBlock), nblocks = n * pieces;
  unpack_band_kernel<T><<<grid_for(nblocks), kBlock, 0, (hipStream_t)stream>>>(n, w, diag_major, dense, ld, pieces,
                                                                            nblocks);
  return launch_status();
}

}  // namespace

extern "C" {

int dastac_pack_triu_f32(int64_t n, const float *dense, int64_t ld, float *packed, void *stream) {
  return tri_copy<float, false, true>(n, dense, packed, ld, stream);
}

int dastac_pack_triu_f64(int64_t n, const double *dense, int64_t ld, double *packed, void *stream) {
  return tri_copy<double, false, true>(n, dense, packed, ld, stream);
}

int dastac_unpack_triu_f32(int64_t n, const float *packed, float *dense, int64_t ld, void *stream) {
  return tri_copy<float, false, false>(n, packed, dense, ld, stream);
}

int dastac_unpack_triu_f64(int64_t n, const double *packed, double *dense, int64_t ld, void *stream) {
  return tri_copy<double, false, false>(n, packed, dense, ld, stream);
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
  return tri_copy<float, true, true>(n, dense, packed, ld, stream);
}

int dastac_pack_tril_f64(int64_t n, const double *dense, int64_t ld, double *packed, void *stream) {
  return tri_copy<double, true, true>(n, dense, packed, ld, stream);
}

int dastac_unpack_tril_f32(int64_t n, const float *packed, float *dense, int64_t ld, void *stream) {
  return tri_copy<float, true, false>(n, packed, dense, ld, stream);
}

int dastac_unpack_tril_f64(int64_t n, const double *packed, double *dense, int64_t ld, void *stream) {
  return tri_copy<double, true, false>(n, packed, dense, ld, stream);
}

}  // extern "C"
