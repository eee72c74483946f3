// Index polynomials of the three packed domains, forward and inverse, in exact int64
// arithmetic, usable from host and device code.
//
// The packed position of an element is the number of domain points that precede it in
// iteration order (Section 4, "Access domain linearization").  For the domains below that
// count is a single polynomial (no piecewise cases survive, cf. Section 4, "Piecewise
// polynomial simplification"):
//
//   upper triangle  0<=i<=j<n       tri_offset  = i*(2n-i+1)/2 + (j-i)
//       (Section 3's printed P_B with Q=1, l=0: (N-1/2) i - i^2/2 + j)
//   upper tetrahedron 0<=i<=j<=k<n  tet_offset  = [Tet(n)-Tet(n-i)] + [Tri(n-i)-Tri(n-j)] + (k-j)
//   band, diagonal-major            band_offset = (d+w)*n + i
//
// Rational coefficients are never rounded: each product below is formed on a numerator that is
// provably divisible (m(m+1) is even, Tri(m)(m+2) is divisible by 3), the same device the
// paper's generated code uses (Fig. 4: doubled terms, one exact unsigned division).
//
// The inverse maps a packed position back to its index tuple.  It is evaluated once per
// wavefront (to find the row or slice where a contiguous share of the buffer starts), never per
// element.  A floating-point root gives a seed; integer steps make it exact.
#pragma once
#include <stdint.h>
#include <math.h>

#if defined(__HIPCC__)
#define DASTAC_HD __host__ __device__ inline
#else
#define DASTAC_HD inline
#endif

namespace dastac {

// Tri(m) = m(m+1)/2, Tet(m) = m(m+1)(m+2)/6; valid for 0 <= m within the guards of dastac.h.
DASTAC_HD int64_t tri(int64_t m) { return (m * (m + 1)) / 2; }
DASTAC_HD int64_t tet(int64_t m) { return (tri(m) * (m + 2)) / 3; }

// Position of (i,i): rows 0..i-1 hold n, n-1, ..., n-i+1 elements.
DASTAC_HD int64_t tri_row_start(int64_t n, int64_t i) { return (i * (2 * n - i + 1)) / 2; }
DASTAC_HD int64_t tri_offset(int64_t n, int64_t i, int64_t j) { return tri_row_start(n, i) + (j - i); }

// Slice i of the tetrahedron is a packed triangle of order n-i that starts here.
DASTAC_HD int64_t tet_slice_start(int64_t n, int64_t i) { return tet(n) - tet(n - i); }
// Position of (i,j,j): inside slice i, rows i..j-1 hold n-i, ..., n-j+1 elements.
DASTAC_HD int64_t tet_row_start(int64_t n, int64_t i, int64_t j) {
  return tet_slice_start(n, i) + (tri(n - i) - tri(n - j));
}
DASTAC_HD int64_t tet_offset(int64_t n, int64_t i, int64_t j, int64_t k) {
  return tet_row_start(n, i, j) + (k - j);
}

DASTAC_HD int64_t band_offset(int64_t n, int64_t w, int64_t d, int64_t i) { return (d + w) * n + i; }

// Largest r >= 0 with Tri(r) <= q  (q >= 0).
DASTAC_HD int64_t tri_root(int64_t q) {
  int64_t r = (int64_t)((sqrt(8.0 * (double)q + 1.0) - 1.0) * 0.5);
  if (r < 0) r = 0;
  while (tri(r) > q) --r;
  while (tri(r + 1) <= q) ++r;
  return r;
}

// Largest s >= 0 with Tet(s) <= q  (q >= 0).
DASTAC_HD int64_t tet_root(int64_t q) {
  int64_t s = (int64_t)cbrt(6.0 * (double)q);
  if (s < 0) s = 0;
  while (s > 0 && tet(s) > q) --s;
  while (tet(s + 1) <= q) ++s;
  return s;
}

// (i,j) of packed position p, 0 <= p < Tri(n).  The elements from row i to the end number
// Tri(n-i), so p lies in row i exactly when Tri(n-i-1) <= Tri(n)-1-p < Tri(n-i).
DASTAC_HD void tri_inverse(int64_t n, int64_t p, int64_t &i, int64_t &j) {
  int64_t r = tri_root(tri(n) - 1 - p);
  i = n - 1 - r;
  j = i + (p - tri_row_start(n, i));
}

// (i,j,k) of packed position p, 0 <= p < Tet(n): slice by the cubic root, then the triangle
// inverse inside the slice.
DASTAC_HD void tet_inverse(int64_t n, int64_t p, int64_t &i, int64_t &j, int64_t &k) {
  int64_t s = tet_root(tet(n) - 1 - p);
  i = n - 1 - s;
  int64_t jj, kk;
  tri_inverse(n - i, p - tet_slice_start(n, i), jj, kk);
  j = i + jj;
  k = i + kk;
}

}  // namespace dastac
