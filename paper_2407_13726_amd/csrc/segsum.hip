// TRMV over a packed upper triangle and TTV over a packed upper tetrahedron.
//
//   y(j)    := U(j,k) * x(k),      j<=k        (Table 1/2, SpMV_UT)
//   M(i,j)  := A(i,j,k) * v(k),    i<=j<=k     (same layout rule, one more iterator)
//
// Both are sums over the contiguous rows ("fibres") of the packed buffer: row (i,j) holds the
// elements k=j..n-1 back to back, rows follow one another in iteration order, and the outputs are
// numbered in the same order (M is itself a packed triangle).  Slice i of the tetrahedron is a
// packed triangle of order n-i, so TRMV is exactly the first slice of TTV and one kernel serves
// both.
//
// Work split (Section 5.2, "Parallelization": the index depends only on the current iterators, so
// any partition of the loops is correct).  The packed buffer is cut into equal contiguous shares,
// one per wavefront; a wavefront owns the rows that START inside its share.  The inverse index
// polynomial, evaluated once per wavefront, names the first such row; after that the row start
// advances by the row length (the polynomial's linear term), all in wave-uniform registers.
//
// Inside a share, rows are taken in groups sized to their length so that lanes stay busy when rows
// get short (the tail of every slice): a row of more than 128 elements gets the whole wavefront and
// a loop; shorter rows get 32, 16, ... 1 lanes each and 2, 4, ... 64 rows are summed side by side.
// Lanes read four consecutive packed elements (16 bytes) each, so a wavefront always touches one
// contiguous span of the buffer.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / 64;

// Sum over aligned groups of 2^lg lanes (every lane of a group receives the total).
__device__ inline float group_sum(float v, int lg) {
  for (int s = 0; s < lg; ++s) v += __shfl_xor(v, 1 << s, 64);
  return v;
}

// First row whose first element is at packed position >= q (q < total), and that position.
template <bool TET>
__device__ inline void first_row_from(int64_t n, int64_t q, int64_t &i, int64_t &j, int64_t &p) {
  int64_t a = 0, b, c;
  if (TET)
    tet_inverse(n, q, a, b, c);
  else
    tri_inverse(n, q, b, c);
  if (c == b) {  // q is itself a row start
    i = a; j = b; p = q;
  } else {       // skip the rest of the row that contains q
    p = q + (n - c);
    if (b + 1 < n) { i = a; j = b + 1; }
    else { i = a + 1; j = a + 1; }
  }
}

// Dot product of a row piece: `cnt` (1..4) packed elements at a[0..] with x[0..].
__device__ inline float dot_piece(const float *__restrict__ a, const float *__restrict__ x, int cnt) {
  if (cnt >= 4) {
    f4u av = *reinterpret_cast<const f4u *>(a);
    f4u xv = *reinterpret_cast<const f4u *>(x);
    return av.x * xv.x + av.y * xv.y + av.z * xv.z + av.w * xv.w;
  }
  float s = 0.0f;
  if (cnt > 0) s += a[0] * x[0];
  if (cnt > 1) s += a[1] * x[1];
  if (cnt > 2) s += a[2] * x[2];
  return s;
}

template <bool TET>
__global__ __launch_bounds__(kBlock) void segsum_kernel(int64_t n, const float *__restrict__ A,
                                                        const float *__restrict__ x, float *__restrict__ out,
                                                        int64_t total, int64_t share) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const int64_t lo = wave * share;
  if (lo >= total) return;
  const int64_t hi = lo + share;

  int64_t i, j, p;
  first_row_from<TET>(n, lo, i, j, p);
  int64_t pe = total;  // first position that belongs to the next wavefront's rows
  if (hi < total) {
    int64_t ie, je;
    first_row_from<TET>(n, hi, ie, je, pe);
  }
  i = uniform64(i); j = uniform64(j); p = uniform64(p); pe = uniform64(pe);
  int64_t s = TET ? tri_offset(n, i, j) : j;  // output position of row (i,j)

  while (p < pe) {
    const int len = (int)(n - j);  // row length == rows left in this slice
    if (len <= 0) break;           // cannot happen while p < pe; keeps every wavefront finite
    if (len > 128) {
      const float *a = A + p;
      const float *xv = x + j;
      float acc = 0.0f;
      int t = lane * 4;
      for (; t + 768 + 4 <= len; t += 1024) {
        f4u a0 = *reinterpret_cast<const f4u *>(a + t), a1 = *reinterpret_cast<const f4u *>(a + t + 256);
        f4u a2 = *reinterpret_cast<const f4u *>(a + t + 512), a3 = *reinterpret_cast<const f4u *>(a + t + 768);
        f4u x0 = *reinterpret_cast<const f4u *>(xv + t), x1 = *reinterpret_cast<const f4u *>(xv + t + 256);
        f4u x2 = *reinterpret_cast<const f4u *>(xv + t + 512), x3 = *reinterpret_cast<const f4u *>(xv + t + 768);
        acc += a0.x * x0.x + a0.y * x0.y + a0.z * x0.z + a0.w * x0.w;
        acc += a1.x * x1.x + a1.y * x1.y + a1.z * x1.z + a1.w * x1.w;
        acc += a2.x * x2.x + a2.y * x2.y + a2.z * x2.z + a2.w * x2.w;
        acc += a3.x * x3.x + a3.y * x3.y + a3.z * x3.z + a3.w * x3.w;
      }
      for (; t < len; t += 256) acc += dot_piece(a + t, xv + t, len - t);
      acc = group_sum(acc, 6);
      if (lane == 0) out[s] = acc;
      p += len; s += 1; j += 1;
    } else {
      // 2^lg lanes per row, 64>>lg rows side by side
      const int lg = len > 64 ? 5 : len > 32 ? 4 : len > 16 ? 3 : len > 8 ? 2 : len > 4 ? 1 : 0;
      int rows = 64 >> lg;
      if (rows > len) rows = len;  // stay inside the slice
      const int g = lane >> lg, sub = lane & ((1 << lg) - 1);
      const int len_g = len - g;
      const int64_t start_g = p + (int64_t)g * len - (g * (g - 1)) / 2;
      const bool mine = g < rows && start_g < pe;
      float acc = 0.0f;
      const int pos = sub * 4;
      if (mine && pos < len_g) acc = dot_piece(A + start_g + pos, x + j + g + pos, len_g - pos);
      acc = group_sum(acc, lg);
      const bool writer = mine && sub == 0;
      if (writer) out[s + g] = acc;
      const int used = __popcll(__ballot(writer));
      p += (int64_t)used * len - (used * (used - 1)) / 2;
      s += used; j += used;
    }
    if (j >= n) {  // slice finished
      if (!TET) break;
      i += 1; j = i;
    }
  }
}

// Elements per wavefront share: enough wavefronts to fill 256 CUs several times over, but at
// least a few KB each so the one inverse per wavefront stays negligible.
inline int64_t pick_share(int64_t total) {
  int64_t share = ceil_div(total, (int64_t)256 * 32);
  if (share < 2048) share = 2048;
  return share;
}

template <bool TET>
int launch(int64_t n, const float *A, const float *x, float *out, int64_t total, void *stream) {
  int64_t share = pick_share(total);
  int64_t waves = ceil_div(total, share);
  int64_t blocks = ceil_div(waves, kWavesPerBlock);
  segsum_kernel<TET><<<(unsigned)blocks, kBlock, 0, (hipStream_t)stream>>>(n, A, x, out, total, share);
  return launch_status();
}

}  // namespace

extern "C" {

int dastac_trmv_f32(int64_t n, const float *Up, const float *x, float *y, void *stream) {
  if (n < 0) return DASTAC_EINVAL;
  if (n > DASTAC_TRI_MAX_N || tri(n) > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Up || !x || !y) return DASTAC_ENULL;
  if (overlaps(y, n * 4, Up, tri(n) * 4) || overlaps(y, n * 4, x, n * 4)) return DASTAC_EALIAS;
  return launch<false>(n, Up, x, y, tri(n), stream);
}

int dastac_tet_ttv_f32(int64_t n, const float *Ap, const float *v, float *Mp, void *stream) {
  if (n < 0) return DASTAC_EINVAL;
  if (n > DASTAC_TET_MAX_N || tet(n) > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Ap || !v || !Mp) return DASTAC_ENULL;
  if (overlaps(Mp, tri(n) * 4, Ap, tet(n) * 4) || overlaps(Mp, tri(n) * 4, v, n * 4)) return DASTAC_EALIAS;
  return launch<true>(n, Ap, v, Mp, tet(n), stream);
}

}  // extern "C"
