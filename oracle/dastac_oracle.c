/*
 * CPU oracle for packed structured tensor contractions (DASTAC, "Compressing
 * Structured Tensor Algebra").
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of every
 * result the GPU library produces.  It shares no code with the GPU library and
 * must never be called from the product path; only the tests, the smoke check
 * and the benchmark's CPU-baseline leg may use it.
 *
 * How a result is defined here
 * ----------------------------
 * Section 4 ("Preceding accesses", "Access domain linearization") defines the
 * packed position of a tensor element as the NUMBER OF ACCESSED INDICES THAT
 * PRECEDE IT in iteration order, the order being lexicographic over the
 * iterators taken in the order in which they appear in the rule (Section 4,
 * "Iteration space extraction": output iterators first, the last one
 * contiguous).  Nothing in this file evaluates a closed-form index polynomial:
 * every packed position is obtained by walking the iteration domain in that
 * order with a running counter, or (oracle_count_preceding) by literally
 * counting the preceding domain points.
 *
 * Section 3 ("Data layout compression") defines compression and decompression
 * as copying the accessed indices into and out of the packed buffer; Section
 * 5.2 defines a statement as "load the factors, multiply, add to the output".
 * The contraction routines below are those loop nests, written out, with a
 * double-precision accumulator that is rounded to fp32 once at the end, plus
 * the per-output sum of |products| that the acceptance tolerance is scaled by.
 *
 * Domains (0-based, all bounds inclusive-exclusive as written):
 *   TRIU  (i,j)    0<=i<n, i<=j<n            Table 2, SpMV_UT
 *   TRIL  (i,j)    0<=i<n, 0<=j<=i           Section 4 worked example (Eq. 2)
 *   TET   (i,j,k)  0<=i<=j<=k<n              upper tetrahedron (hyper-triangle of PR3, Table 1)
 *   UHC   (i,j,l)  0<=i<M, i<=j<N, 0<=l<Q    running example, buffer B (Fig. 3, Eq. 1)
 *   BAND  (d,i)    -w<=d<=w, 0<=i<n          one buffer of n slots per diagonal summand
 *                                            (Section 4, per-summand buffers; Section 6.4
 *                                            strided-band structure with unit stride);
 *                                            slot (d,i) holds A[i][i+d], and slots whose
 *                                            column i+d falls outside [0,n) are padding.
 *   SBAND (d,i)    as BAND with slot (d,i) holding A[i][i+d*s]   Section 6.4, strided band, stride s
 *   SUBTRI (i,j)   0<=i<N, 0<=j<N, j-i>=N-k  Section 6.4, sub-triangular structure
 *   LESLIE         (i=0)(0<=j<n) + (1<=i<n)(j=i-1)   Table 2, SpMV_L: two summands, two buffers
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { DOM_TRIU = 0, DOM_TRIL = 1, DOM_TET = 2, DOM_UHC = 3, DOM_BAND = 4 };

/* ---- generic counting definition (tiny sizes only) ----------------------- */

/* Number of iterators of a domain. */
static int dom_rank(int dom) { return (dom == DOM_TET || dom == DOM_UHC) ? 3 : 2; }

/* Bounding box [lo, hi) per iterator, from the domain parameters. */
static void dom_box(int dom, const int64_t *prm, int64_t lo[3], int64_t hi[3]) {
  lo[0] = lo[1] = lo[2] = 0;
  hi[0] = hi[1] = hi[2] = 1;
  switch (dom) {
    case DOM_TRIU: case DOM_TRIL: hi[0] = prm[0]; hi[1] = prm[0]; break;
    case DOM_TET: hi[0] = hi[1] = hi[2] = prm[0]; break;
    case DOM_UHC: hi[0] = prm[0]; hi[1] = prm[1]; hi[2] = prm[2]; break;
    case DOM_BAND: lo[0] = -prm[1]; hi[0] = prm[1] + 1; hi[1] = prm[0]; break;
  }
}

/* Membership predicate: the comparisons of the summand (Section 4, "Iteration space extraction"). */
static int dom_has(int dom, const int64_t *prm, const int64_t x[3]) {
  int64_t lo[3], hi[3];
  dom_box(dom, prm, lo, hi);
  for (int a = 0; a < dom_rank(dom); ++a)
    if (x[a] < lo[a] || x[a] >= hi[a]) return 0;
  switch (dom) {
    case DOM_TRIU: return x[0] <= x[1];
    case DOM_TRIL: return x[1] <= x[0];
    case DOM_TET: return x[0] <= x[1] && x[1] <= x[2];
    case DOM_UHC: return x[0] <= x[1];
    case DOM_BAND: return 1;
  }
  return 0;
}

/* Lexicographic "a strictly before b" over the iterators in rule order. */
static int lex_before(int rank, const int64_t a[3], const int64_t b[3]) {
  for (int t = 0; t < rank; ++t) {
    if (a[t] < b[t]) return 1;
    if (a[t] > b[t]) return 0;
  }
  return 0;
}

/*
 * #P(idx): the number of domain points that precede idx (Section 4, "Access
 * domain linearization": the packed index is the cardinality of the
 * preceding-access set).  Returns -1 if idx itself is not in the domain.
 * Cost is the volume of the bounding box; use for tiny sizes only.
 */
int64_t oracle_count_preceding(int dom, const int64_t *prm, const int64_t *idx) {
  int64_t lo[3], hi[3], x[3], me[3] = {0, 0, 0};
  int rank = dom_rank(dom);
  for (int a = 0; a < rank; ++a) me[a] = idx[a];
  if (!dom_has(dom, prm, me)) return -1;
  dom_box(dom, prm, lo, hi);
  int64_t cnt = 0;
  for (x[0] = lo[0]; x[0] < hi[0]; ++x[0])
    for (x[1] = lo[1]; x[1] < hi[1]; ++x[1])
      for (x[2] = lo[2]; x[2] < hi[2]; ++x[2])
        if (dom_has(dom, prm, x) && lex_before(rank, x, me)) ++cnt;
  return cnt;
}

/* Number of points of the domain (same brute force). */
int64_t oracle_count_domain(int dom, const int64_t *prm) {
  int64_t lo[3], hi[3], x[3];
  dom_box(dom, prm, lo, hi);
  int64_t cnt = 0;
  for (x[0] = lo[0]; x[0] < hi[0]; ++x[0])
    for (x[1] = lo[1]; x[1] < hi[1]; ++x[1])
      for (x[2] = lo[2]; x[2] < hi[2]; ++x[2])
        if (dom_has(dom, prm, x)) ++cnt;
  return cnt;
}

/*
 * The point numbered p when the domain is walked in iteration order (the
 * inverse of oracle_count_preceding, by enumeration).  Returns 0 on success,
 * 1 if p is outside [0, #domain).
 */
int oracle_point_at(int dom, const int64_t *prm, int64_t p, int64_t *out) {
  int64_t lo[3], hi[3], x[3];
  int rank = dom_rank(dom);
  dom_box(dom, prm, lo, hi);
  if (p < 0) return 1;
  int64_t cnt = 0;
  for (x[0] = lo[0]; x[0] < hi[0]; ++x[0])
    for (x[1] = lo[1]; x[1] < hi[1]; ++x[1])
      for (x[2] = lo[2]; x[2] < hi[2]; ++x[2])
        if (dom_has(dom, prm, x)) {
          if (cnt == p) {
            for (int a = 0; a < rank; ++a) out[a] = x[a];
            return 0;
          }
          ++cnt;
        }
  return 1;
}

/* ---- running-counter walks usable at full problem sizes ------------------- */

/*
 * Walk the upper triangle in iteration order and record the running counter at
 * the first element of every row: start[i] = position of (i,i); start[n] = total.
 */
void oracle_triu_row_starts(int64_t n, int64_t *start) {
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i) {
    start[i] = p;
    for (int64_t j = i; j < n; ++j) ++p;
  }
  start[n] = p;
}

/*
 * Walk the upper tetrahedron in iteration order and record the running counter
 * at the first element of every fibre: start[i*n+j] = position of (i,j,j) for
 * i<=j, -1 otherwise.  Returns the total number of points.
 */
int64_t oracle_tet_fibre_starts(int64_t n, int64_t *start) {
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) {
      if (j < i) { start[i * n + j] = -1; continue; }
      start[i * n + j] = p;
      for (int64_t k = j; k < n; ++k) ++p;
    }
  return p;
}

/* Position of (i,j) / (i,j,k) by walking with a running counter; -1 if outside. */
int64_t oracle_triu_position(int64_t n, int64_t i, int64_t j) {
  int64_t p = 0;
  for (int64_t a = 0; a < n; ++a)
    for (int64_t b = a; b < n; ++b) {
      if (a == i && b == j) return p;
      ++p;
    }
  return -1;
}

int64_t oracle_tet_position(int64_t n, int64_t i, int64_t j, int64_t k) {
  int64_t p = 0;
  for (int64_t a = 0; a < n; ++a)
    for (int64_t b = a; b < n; ++b) {
      if (a == i && b == j) {
        for (int64_t c = b; c < n; ++c) {
          if (c == k) return p;
          ++p;
        }
        return -1;
      }
      for (int64_t c = b; c < n; ++c) ++p;
    }
  return -1;
}

/* Inverse by walking: the (i,j) whose running counter equals p.  0 ok, 1 out of range. */
int oracle_triu_point_at(int64_t n, int64_t p, int64_t *i, int64_t *j) {
  if (p < 0) return 1;
  int64_t q = 0;
  for (int64_t a = 0; a < n; ++a) {
    int64_t len = 0;
    for (int64_t b = a; b < n; ++b) ++len;
    if (p < q + len) { *i = a; *j = a + (p - q); return 0; }
    q += len;
  }
  return 1;
}

int oracle_tet_point_at(int64_t n, int64_t p, int64_t *i, int64_t *j, int64_t *k) {
  if (p < 0) return 1;
  int64_t q = 0;
  for (int64_t a = 0; a < n; ++a)
    for (int64_t b = a; b < n; ++b) {
      int64_t len = 0;
      for (int64_t c = b; c < n; ++c) ++len;
      if (p < q + len) { *i = a; *j = b; *k = b + (p - q); return 0; }
      q += len;
    }
  return 1;
}

/* ---- compression / decompression (Section 3, "Data layout compression") --- */

void oracle_pack_triu_f32(int64_t n, const float *dense, int64_t ld, float *packed) {
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = i; j < n; ++j) packed[p++] = dense[i * ld + j];
}

void oracle_unpack_triu_f32(int64_t n, const float *packed, float *dense, int64_t ld) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) dense[i * ld + j] = 0.0f;
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = i; j < n; ++j) dense[i * ld + j] = packed[p++];
}

void oracle_pack_tet_f32(int64_t n, const float *dense, float *packed) {
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = i; j < n; ++j)
      for (int64_t k = j; k < n; ++k) packed[p++] = dense[(i * n + j) * n + k];
}

void oracle_unpack_tet_f32(int64_t n, const float *packed, float *dense) {
  for (int64_t t = 0; t < n * n * n; ++t) dense[t] = 0.0f;
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = i; j < n; ++j)
      for (int64_t k = j; k < n; ++k) dense[(i * n + j) * n + k] = packed[p++];
}

/* Upper half cube (running example, Fig. 3): (i,j,l) with i<=j, all three extents given; the dense
 * tensor is M x N x Q row-major.  The same walk packs the rule's output A(i,j,k), whose last
 * extent is the number of rows of C. */
void oracle_pack_uhc_f32(int64_t M, int64_t N, int64_t Q, const float *dense, float *packed) {
  int64_t p = 0;
  for (int64_t i = 0; i < M; ++i)
    for (int64_t j = i; j < N; ++j)
      for (int64_t l = 0; l < Q; ++l) packed[p++] = dense[(i * N + j) * Q + l];
}

void oracle_unpack_uhc_f32(int64_t M, int64_t N, int64_t Q, const float *packed, float *dense) {
  for (int64_t t = 0; t < M * N * Q; ++t) dense[t] = 0.0f;
  int64_t p = 0;
  for (int64_t i = 0; i < M; ++i)
    for (int64_t j = i; j < N; ++j)
      for (int64_t l = 0; l < Q; ++l) dense[(i * N + j) * Q + l] = packed[p++];
}

/* Band: diagonal d is its own summand with its own n-slot buffer, buffers laid
 * out in summand order d=-w..w; slot i of diagonal d holds A[i][i+d]; padding
 * slots (column outside the matrix) are written as +0. */
void oracle_pack_band_f32(int64_t n, int64_t w, const float *dense, int64_t ld, float *diag) {
  int64_t p = 0;
  for (int64_t d = -w; d <= w; ++d)
    for (int64_t i = 0; i < n; ++i) {
      int64_t j = i + d;
      diag[p++] = (j >= 0 && j < n) ? dense[i * ld + j] : 0.0f;
    }
}

void oracle_unpack_band_f32(int64_t n, int64_t w, const float *diag, float *dense, int64_t ld) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) dense[i * ld + j] = 0.0f;
  int64_t p = 0;
  for (int64_t d = -w; d <= w; ++d)
    for (int64_t i = 0; i < n; ++i) {
      int64_t j = i + d;
      if (j >= 0 && j < n) dense[i * ld + j] = diag[p];
      ++p;
    }
}

/* ---- contractions ---------------------------------------------------------
 * Every routine takes an output-row window [r_lo, r_hi): rows outside it are
 * walked (so the running counter stays right) but not computed and not written.
 * The full result is the window [0, n).  `scale` receives sum |product| per
 * computed output element, in double; it may be NULL.
 */

/* y(i) := U(i,j) * x(j),  i<=j   (Table 1, SpMV with upper-triangular B). */
void oracle_trmv_f32(int64_t n, const float *Up, const float *x, float *y, double *scale,
                     int64_t r_lo, int64_t r_hi) {
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i) {
    int on = (i >= r_lo && i < r_hi);
    double acc = 0.0, mag = 0.0;
    for (int64_t j = i; j < n; ++j) {
      if (on) {
        double t = (double)Up[p] * (double)x[j];
        acc += t;
        mag += fabs(t);
      }
      ++p;
    }
    if (on) {
      y[i] = (float)acc;
      if (scale) scale[i] = mag;
    }
  }
}

/* C(i,c) := U(i,k) * B(k,c),  i<=k   (same layout rule applied to a matrix right-hand side). */
void oracle_trmm_f32(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C,
                     int64_t ldc, double *scale, int64_t r_lo, int64_t r_hi) {
  double *acc = (double *)malloc(sizeof(double) * (size_t)(m > 0 ? m : 1));
  double *mag = (double *)malloc(sizeof(double) * (size_t)(m > 0 ? m : 1));
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i) {
    int on = (i >= r_lo && i < r_hi);
    if (on)
      for (int64_t c = 0; c < m; ++c) acc[c] = mag[c] = 0.0;
    for (int64_t k = i; k < n; ++k) {
      if (on) {
        double u = (double)Up[p];
        for (int64_t c = 0; c < m; ++c) {
          double t = u * (double)B[k * ldb + c];
          acc[c] += t;
          mag[c] += fabs(t);
        }
      }
      ++p;
    }
    if (on)
      for (int64_t c = 0; c < m; ++c) {
        C[i * ldc + c] = (float)acc[c];
        if (scale) scale[i * m + c] = mag[c];
      }
  }
  free(acc);
  free(mag);
}

/* y(i) := sum over diagonal summands d of D_d(i) * x(i+d), column inside the matrix
 * (Section 6.4 strided-band rule with 2w+1 unit-stride summands).  Padding slots
 * are skipped by the predicate, never read for their value. */
void oracle_band_spmv_f32(int64_t n, int64_t w, const float *D, const float *x, float *y,
                          double *scale, int64_t r_lo, int64_t r_hi) {
  for (int64_t i = r_lo; i < r_hi && i < n; ++i) {
    if (i < 0) continue;
    double acc = 0.0, mag = 0.0;
    for (int64_t d = -w; d <= w; ++d) {
      int64_t j = i + d;
      if (j < 0 || j >= n) continue;
      /* slot (d,i) is the i-th slot of the (d+w)-th summand buffer */
      double t = (double)D[(d + w) * n + i] * (double)x[j];
      acc += t;
      mag += fabs(t);
    }
    y[i] = (float)acc;
    if (scale) scale[i] = mag;
  }
}

/* M(i,j) := A(i,j,k) * v(k),  i<=j<=k ; M is itself packed (upper triangle, iteration order).
 * The window [r_lo, r_hi) is over the slice index i. */
void oracle_tet_ttv_f32(int64_t n, const float *Ap, const float *v, float *Mp, double *scale,
                        int64_t r_lo, int64_t r_hi) {
  int64_t p = 0; /* running position in A */
  int64_t q = 0; /* running position in M */
  for (int64_t i = 0; i < n; ++i) {
    int on = (i >= r_lo && i < r_hi);
    for (int64_t j = i; j < n; ++j) {
      double acc = 0.0, mag = 0.0;
      for (int64_t k = j; k < n; ++k) {
        if (on) {
          double t = (double)Ap[p] * (double)v[k];
          acc += t;
          mag += fabs(t);
        }
        ++p;
      }
      if (on) {
        Mp[q] = (float)acc;
        if (scale) scale[q] = mag;
      }
      ++q;
    }
  }
}

/* M(i,r) := A(i,j,k) * B(j,r) * C(k,r),  i<=j<=k   (Table 1 MTTKRP rule on the tetrahedron). */
void oracle_tet_mttkrp_f32(int64_t n, int64_t R, const float *Ap, const float *B, int64_t ldb,
                           const float *C, int64_t ldc, float *M, int64_t ldm, double *scale,
                           int64_t r_lo, int64_t r_hi) {
  double *acc = (double *)malloc(sizeof(double) * (size_t)(R > 0 ? R : 1));
  double *mag = (double *)malloc(sizeof(double) * (size_t)(R > 0 ? R : 1));
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i) {
    int on = (i >= r_lo && i < r_hi);
    if (on)
      for (int64_t r = 0; r < R; ++r) acc[r] = mag[r] = 0.0;
    for (int64_t j = i; j < n; ++j)
      for (int64_t k = j; k < n; ++k) {
        if (on) {
          double a = (double)Ap[p];
          for (int64_t r = 0; r < R; ++r) {
            double t = a * (double)B[j * ldb + r] * (double)C[k * ldc + r];
            acc[r] += t;
            mag[r] += fabs(t);
          }
        }
        ++p;
      }
    if (on)
      for (int64_t r = 0; r < R; ++r) {
        M[i * ldm + r] = (float)acc[r];
        if (scale) scale[i * R + r] = mag[r];
      }
  }
  free(acc);
  free(mag);
}

/* A(i,j,k) := B(i,j,l) * C(k,l),  i<=j   (the running example, Fig. 3; Table 1 TTM with the
 * upper-half-cube structure).  B is packed in iteration order (i,j,l) and the output A, which
 * inherits the structure, in iteration order (i,j,k): both positions come from running counters
 * over the same walk.  C is dense, K x Q row-major with leading dimension ldc.  The window
 * [r_lo, r_hi) selects (i,j) pairs by their number in iteration order. */
void oracle_ttm_ut_f32(int64_t n, int64_t Q, int64_t K, const float *Bp, const float *C, int64_t ldc,
                       float *Ap, double *scale, int64_t r_lo, int64_t r_hi) {
  int64_t pb = 0, pa = 0, pair = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = i; j < n; ++j) {
      if (pair >= r_lo && pair < r_hi) {
        for (int64_t k = 0; k < K; ++k) {
          double acc = 0.0, mag = 0.0;
          for (int64_t l = 0; l < Q; ++l) {
            double t = (double)Bp[pb + l] * (double)C[k * ldc + l];
            acc += t;
            mag += fabs(t);
          }
          Ap[pa + k] = (float)acc;
          if (scale) scale[pa + k] = mag;
        }
      }
      pb += Q;
      pa += K;
      ++pair;
    }
}

/* Lower triangle (Section 4 worked example, Eq. 2): row i holds columns 0..i. */
void oracle_pack_tril_f32(int64_t n, const float *dense, int64_t ld, float *packed) {
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j <= i; ++j) packed[p++] = dense[i * ld + j];
}

void oracle_unpack_tril_f32(int64_t n, const float *packed, float *dense, int64_t ld) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) dense[i * ld + j] = 0.0f;
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j <= i; ++j) dense[i * ld + j] = packed[p++];
}

/* Products of one packed triangle T (upper: row i holds columns i..n-1; lower: columns 0..i) with a
 * vector:  mode 0  y(i) := T(i,j) x(j);  mode 1  y(j) := T(i,j) x(i)  (the transposed product);
 * mode 2  y(i) := S(i,j) x(j) for the symmetric matrix whose unique elements are T (Section 3,
 * "Redundancy map": an index pair outside the unique set is swapped to reach its unique element).
 * Positions come from running-counter row starts. */
void oracle_trimv_f32(int64_t n, int lower, int mode, const float *Tp, const float *x, float *y,
                      double *scale, int64_t r_lo, int64_t r_hi) {
  int64_t *start = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i) { /* walk the rows in iteration order */
    start[i] = p;
    p += lower ? i + 1 : n - i;
  }
  for (int64_t i = 0; i < n; ++i) {
    if (i < r_lo || i >= r_hi) continue;
    double acc = 0.0, mag = 0.0;
    for (int64_t j = 0; j < n; ++j) {
      /* which stored element, if any, is factor (i,j) of output i */
      int64_t a = i, b = j; /* mode 0: T(i,j) */
      if (mode == 1) { a = j; b = i; } /* T^T(i,j) = T(j,i) */
      int inside = lower ? (b <= a) : (a <= b);
      if (mode == 2 && !inside) { int64_t t = a; a = b; b = t; inside = 1; } /* swap to the unique element */
      if (!inside) continue;
      double t = (double)Tp[start[a] + (lower ? b : b - a)] * (double)x[j];
      acc += t;
      mag += fabs(t);
    }
    y[i] = (float)acc;
    if (scale) scale[i] = mag;
  }
  free(start);
}

/* ---- further domains of Section 6.4 and Table 2 ------------------------------------------- */

/* Strided band (Section 6.4, "Distance of Elements and Compression"): summands j-i = d*s for
 * d=-w..w (the paper's experiment is w=1: j=i, j-i=s, i-j=s).  Each summand has its own n-slot
 * buffer, buffers in summand order; slot i of summand d holds A[i][i+d*s]; slots whose column
 * falls outside the matrix are padding (+0 on pack, never used). */
void oracle_pack_sband_f32(int64_t n, int64_t w, int64_t s, const float *dense, int64_t ld, float *diag) {
  int64_t p = 0;
  for (int64_t d = -w; d <= w; ++d)
    for (int64_t i = 0; i < n; ++i) {
      int64_t j = i + d * s;
      diag[p++] = (j >= 0 && j < n) ? dense[i * ld + j] : 0.0f;
    }
}

void oracle_unpack_sband_f32(int64_t n, int64_t w, int64_t s, const float *diag, float *dense, int64_t ld) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) dense[i * ld + j] = 0.0f;
  int64_t p = 0;
  for (int64_t d = -w; d <= w; ++d)
    for (int64_t i = 0; i < n; ++i) {
      int64_t j = i + d * s;
      if (j >= 0 && j < n) dense[i * ld + j] = diag[p];
      ++p;
    }
}

void oracle_sband_spmv_f32(int64_t n, int64_t w, int64_t s, const float *D, const float *x, float *y,
                           double *scale, int64_t r_lo, int64_t r_hi) {
  for (int64_t i = 0; i < n; ++i) {
    if (i < r_lo || i >= r_hi) continue;
    double acc = 0.0, mag = 0.0;
    for (int64_t d = -w; d <= w; ++d) {
      int64_t j = i + d * s;
      if (j < 0 || j >= n) continue;
      double t = (double)D[(d + w) * n + i] * (double)x[j];
      acc += t;
      mag += fabs(t);
    }
    y[i] = (float)acc;
    if (scale) scale[i] = mag;
  }
}

/* Sub-triangular structure (Section 6.4, "Density and Compression"): the unique set is
 * 0<=i<N, 0<=j<N, j-i >= N-k.  Packed in iteration order (i,j) by a running counter. */
void oracle_pack_subtri_f32(int64_t N, int64_t k, const float *dense, int64_t ld, float *packed) {
  int64_t p = 0;
  for (int64_t i = 0; i < N; ++i)
    for (int64_t j = 0; j < N; ++j)
      if (j - i >= N - k) packed[p++] = dense[i * ld + j];
}

void oracle_unpack_subtri_f32(int64_t N, int64_t k, const float *packed, float *dense, int64_t ld) {
  int64_t p = 0;
  for (int64_t i = 0; i < N; ++i)
    for (int64_t j = 0; j < N; ++j) dense[i * ld + j] = (j - i >= N - k) ? packed[p++] : 0.0f;
}

/* y(i) := A(i,j) x(j) over the sub-triangular structure; every one of the N outputs is written
 * (rows without a stored element give 0). */
void oracle_subtri_spmv_f32(int64_t N, int64_t k, const float *Ap, const float *x, float *y, double *scale,
                            int64_t r_lo, int64_t r_hi) {
  int64_t p = 0;
  for (int64_t i = 0; i < N; ++i) {
    double acc = 0.0, mag = 0.0;
    for (int64_t j = 0; j < N; ++j) {
      if (j - i < N - k) continue;
      double t = (double)Ap[p++] * (double)x[j];
      acc += t;
      mag += fabs(t);
    }
    if (i >= r_lo && i < r_hi) {
      y[i] = (float)acc;
      if (scale) scale[i] = mag;
    }
  }
}

/* Leslie structure (Table 2, SpMV_L): (i=0)(0<=j<n) + (1<=i<n)(j=i-1).  Two summands, two
 * buffers: R[n] is the first row in order of j, S[n-1] the sub-diagonal in order of i. */
void oracle_pack_leslie_f32(int64_t n, const float *dense, int64_t ld, float *R, float *S) {
  int64_t p = 0;
  for (int64_t j = 0; j < n; ++j) R[p++] = dense[j];
  p = 0;
  for (int64_t i = 1; i < n; ++i) S[p++] = dense[i * ld + (i - 1)];
}

void oracle_unpack_leslie_f32(int64_t n, const float *R, const float *S, float *dense, int64_t ld) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) dense[i * ld + j] = 0.0f;
  for (int64_t j = 0; j < n; ++j) dense[j] = R[j];
  for (int64_t i = 1; i < n; ++i) dense[i * ld + (i - 1)] = S[i - 1];
}

void oracle_leslie_spmv_f32(int64_t n, const float *R, const float *S, const float *x, float *y, double *scale) {
  if (n <= 0) return;
  double acc = 0.0, mag = 0.0;
  for (int64_t j = 0; j < n; ++j) {
    double t = (double)R[j] * (double)x[j];
    acc += t;
    mag += fabs(t);
  }
  y[0] = (float)acc;
  if (scale) scale[0] = mag;
  for (int64_t i = 1; i < n; ++i) {
    double t = (double)S[i - 1] * (double)x[i - 1];
    y[i] = (float)t;
    if (scale) scale[i] = fabs(t);
  }
}

/* C(i,c) := S(i,j) * B(j,c), S symmetric with its unique elements S(i,j), i<=j, packed as an upper
 * triangle (Section 3, "Redundancy map": a pair with i>j is swapped to reach its unique element).
 * Row starts of the packed triangle come from a running counter. */
void oracle_symm_f32(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C,
                     int64_t ldc, double *scale, int64_t r_lo, int64_t r_hi) {
  int64_t *start = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i) {
    start[i] = p;
    p += n - i;
  }
  for (int64_t i = 0; i < n; ++i) {
    if (i < r_lo || i >= r_hi) continue;
    for (int64_t c = 0; c < m; ++c) {
      double acc = 0.0, mag = 0.0;
      for (int64_t j = 0; j < n; ++j) {
        int64_t a = i, b = j;
        if (a > b) { int64_t t = a; a = b; b = t; } /* the redundancy map */
        double t = (double)Up[start[a] + (b - a)] * (double)B[j * ldb + c];
        acc += t;
        mag += fabs(t);
      }
      C[i * ldc + c] = (float)acc;
      if (scale) scale[i * m + c] = mag;
    }
  }
  free(start);
}

/* Polynomial-regression tensors (Table 1, "Polynomial Regression Degree-D"):
 *   A2(i1,i2)    := B(x,i1) * B(x,i2)            summed over x
 *   A3(i1,i2,i3) := B(x,i1) * B(x,i2) * B(x,i3)  summed over x
 * B is N x d row-major (leading dimension ldb).  Both tensors are symmetric under any permutation
 * of their indices; the unique set is the hyper-triangle i1<=i2(<=i3), stored in iteration order
 * by a running counter.  The window [p_lo, p_hi) selects outputs by packed position. */
void oracle_pr_a2_f32(int64_t N, int64_t d, const float *B, int64_t ldb, float *A2p, double *scale,
                      int64_t p_lo, int64_t p_hi) {
  int64_t p = 0;
  for (int64_t i = 0; i < d; ++i)
    for (int64_t j = i; j < d; ++j, ++p) {
      if (p < p_lo || p >= p_hi) continue;
      double acc = 0.0, mag = 0.0;
      for (int64_t x = 0; x < N; ++x) {
        double t = (double)B[x * ldb + i] * (double)B[x * ldb + j];
        acc += t;
        mag += fabs(t);
      }
      A2p[p] = (float)acc;
      if (scale) scale[p] = mag;
    }
}

void oracle_pr_a3_f32(int64_t N, int64_t d, const float *B, int64_t ldb, float *A3p, double *scale,
                      int64_t p_lo, int64_t p_hi) {
  int64_t p = 0;
  for (int64_t i = 0; i < d; ++i)
    for (int64_t j = i; j < d; ++j)
      for (int64_t k = j; k < d; ++k, ++p) {
        if (p < p_lo || p >= p_hi) continue;
        double acc = 0.0, mag = 0.0;
        for (int64_t x = 0; x < N; ++x) {
          double t = (double)B[x * ldb + i] * (double)B[x * ldb + j] * (double)B[x * ldb + k];
          acc += t;
          mag += fabs(t);
        }
        A3p[p] = (float)acc;
        if (scale) scale[p] = mag;
      }
}

/* ---- double precision (the paper's own element type, Section 6.1) -------------------------
 * The same definitions on double operands.  Accumulation is in long double (64-bit mantissa on
 * this host), rounded to double once at the end, so that the reference stays well below the
 * rounding error of any double-precision summation order it is compared with. */
void oracle_pack_triu_f64(int64_t n, const double *dense, int64_t ld, double *packed) {
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = i; j < n; ++j) packed[p++] = dense[i * ld + j];
}

void oracle_unpack_triu_f64(int64_t n, const double *packed, double *dense, int64_t ld) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) dense[i * ld + j] = 0.0;
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = i; j < n; ++j) dense[i * ld + j] = packed[p++];
}

void oracle_pack_tet_f64(int64_t n, const double *dense, double *packed) {
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = i; j < n; ++j)
      for (int64_t k = j; k < n; ++k) packed[p++] = dense[(i * n + j) * n + k];
}

void oracle_unpack_tet_f64(int64_t n, const double *packed, double *dense) {
  for (int64_t t = 0; t < n * n * n; ++t) dense[t] = 0.0;
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = i; j < n; ++j)
      for (int64_t k = j; k < n; ++k) dense[(i * n + j) * n + k] = packed[p++];
}

void oracle_pack_band_f64(int64_t n, int64_t w, const double *dense, int64_t ld, double *diag) {
  int64_t p = 0;
  for (int64_t d = -w; d <= w; ++d)
    for (int64_t i = 0; i < n; ++i) {
      int64_t j = i + d;
      diag[p++] = (j >= 0 && j < n) ? dense[i * ld + j] : 0.0;
    }
}

void oracle_unpack_band_f64(int64_t n, int64_t w, const double *diag, double *dense, int64_t ld) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) dense[i * ld + j] = 0.0;
  int64_t p = 0;
  for (int64_t d = -w; d <= w; ++d)
    for (int64_t i = 0; i < n; ++i) {
      int64_t j = i + d;
      if (j >= 0 && j < n) dense[i * ld + j] = diag[p];
      ++p;
    }
}

void oracle_trmv_f64(int64_t n, const double *Up, const double *x, double *y, double *scale,
                     int64_t r_lo, int64_t r_hi) {
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i) {
    int on = (i >= r_lo && i < r_hi);
    long double acc = 0.0L, mag = 0.0L;
    for (int64_t j = i; j < n; ++j) {
      if (on) {
        long double t = (long double)Up[p] * (long double)x[j];
        acc += t;
        mag += fabsl(t);
      }
      ++p;
    }
    if (on) {
      y[i] = (double)acc;
      if (scale) scale[i] = (double)mag;
    }
  }
}

void oracle_band_spmv_f64(int64_t n, int64_t w, const double *D, const double *x, double *y,
                          double *scale, int64_t r_lo, int64_t r_hi) {
  for (int64_t i = r_lo; i < r_hi && i < n; ++i) {
    if (i < 0) continue;
    long double acc = 0.0L, mag = 0.0L;
    for (int64_t d = -w; d <= w; ++d) {
      int64_t j = i + d;
      if (j < 0 || j >= n) continue;
      long double t = (long double)D[(d + w) * n + i] * (long double)x[j];
      acc += t;
      mag += fabsl(t);
    }
    y[i] = (double)acc;
    if (scale) scale[i] = (double)mag;
  }
}

void oracle_tet_ttv_f64(int64_t n, const double *Ap, const double *v, double *Mp, double *scale,
                        int64_t r_lo, int64_t r_hi) {
  int64_t p = 0, q = 0;
  for (int64_t i = 0; i < n; ++i) {
    int on = (i >= r_lo && i < r_hi);
    for (int64_t j = i; j < n; ++j) {
      long double acc = 0.0L, mag = 0.0L;
      for (int64_t k = j; k < n; ++k) {
        if (on) {
          long double t = (long double)Ap[p] * (long double)v[k];
          acc += t;
          mag += fabsl(t);
        }
        ++p;
      }
      if (on) {
        Mp[q] = (double)acc;
        if (scale) scale[q] = (double)mag;
      }
      ++q;
    }
  }
}

/* C(i,c) := U(i,k) * B(k,c),  i<=k, on double operands (long-double accumulation). */
void oracle_trmm_f64(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C,
                     int64_t ldc, double *scale, int64_t r_lo, int64_t r_hi) {
  long double *acc = (long double *)malloc(sizeof(long double) * (size_t)(m > 0 ? m : 1));
  long double *mag = (long double *)malloc(sizeof(long double) * (size_t)(m > 0 ? m : 1));
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i) {
    int on = (i >= r_lo && i < r_hi);
    if (on)
      for (int64_t c = 0; c < m; ++c) acc[c] = mag[c] = 0.0L;
    for (int64_t k = i; k < n; ++k) {
      if (on) {
        long double u = (long double)Up[p];
        for (int64_t c = 0; c < m; ++c) {
          long double t = u * (long double)B[k * ldb + c];
          acc[c] += t;
          mag[c] += fabsl(t);
        }
      }
      ++p;
    }
    if (on)
      for (int64_t c = 0; c < m; ++c) {
        C[i * ldc + c] = (double)acc[c];
        if (scale) scale[i * m + c] = (double)mag[c];
      }
  }
  free(acc);
  free(mag);
}

/* C(i,c) := S(i,j) * B(j,c), S symmetric with its unique elements packed as an upper triangle, on double
 * operands (long-double accumulation). */
void oracle_symm_f64(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C,
                     int64_t ldc, double *scale, int64_t r_lo, int64_t r_hi) {
  int64_t *start = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i) {
    start[i] = p;
    p += n - i;
  }
  for (int64_t i = 0; i < n; ++i) {
    if (i < r_lo || i >= r_hi) continue;
    for (int64_t c = 0; c < m; ++c) {
      long double acc = 0.0L, mag = 0.0L;
      for (int64_t j = 0; j < n; ++j) {
        int64_t a = i, b = j;
        if (a > b) { int64_t t = a; a = b; b = t; } /* the redundancy map */
        long double t = (long double)Up[start[a] + (b - a)] * (long double)B[j * ldb + c];
        acc += t;
        mag += fabsl(t);
      }
      C[i * ldc + c] = (double)acc;
      if (scale) scale[i * m + c] = (double)mag;
    }
  }
  free(start);
}

/* The running example on double operands: pack/unpack of the upper half cube and
 * A(i,j,k) := B(i,j,l) * C(k,l), i<=j (long-double accumulation). */
void oracle_pack_uhc_f64(int64_t M, int64_t N, int64_t Q, const double *dense, double *packed) {
  int64_t p = 0;
  for (int64_t i = 0; i < M; ++i)
    for (int64_t j = i; j < N; ++j)
      for (int64_t l = 0; l < Q; ++l) packed[p++] = dense[(i * N + j) * Q + l];
}

void oracle_unpack_uhc_f64(int64_t M, int64_t N, int64_t Q, const double *packed, double *dense) {
  for (int64_t t = 0; t < M * N * Q; ++t) dense[t] = 0.0;
  int64_t p = 0;
  for (int64_t i = 0; i < M; ++i)
    for (int64_t j = i; j < N; ++j)
      for (int64_t l = 0; l < Q; ++l) dense[(i * N + j) * Q + l] = packed[p++];
}

void oracle_ttm_ut_f64(int64_t n, int64_t Q, int64_t K, const double *Bp, const double *C, int64_t ldc,
                       double *Ap, double *scale, int64_t r_lo, int64_t r_hi) {
  int64_t pb = 0, pa = 0, pair = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = i; j < n; ++j) {
      if (pair >= r_lo && pair < r_hi) {
        for (int64_t k = 0; k < K; ++k) {
          long double acc = 0.0L, mag = 0.0L;
          for (int64_t l = 0; l < Q; ++l) {
            long double t = (long double)Bp[pb + l] * (long double)C[k * ldc + l];
            acc += t;
            mag += fabsl(t);
          }
          Ap[pa + k] = (double)acc;
          if (scale) scale[pa + k] = (double)mag;
        }
      }
      pb += Q;
      pa += K;
      ++pair;
    }
}

/* The polynomial-regression tensors on double operands (long-double accumulation). */
void oracle_pr_a2_f64(int64_t N, int64_t d, const double *B, int64_t ldb, double *A2p, double *scale,
                      int64_t p_lo, int64_t p_hi) {
  int64_t p = 0;
  for (int64_t i = 0; i < d; ++i)
    for (int64_t j = i; j < d; ++j, ++p) {
      if (p < p_lo || p >= p_hi) continue;
      long double acc = 0.0L, mag = 0.0L;
      for (int64_t x = 0; x < N; ++x) {
        long double t = (long double)B[x * ldb + i] * (long double)B[x * ldb + j];
        acc += t;
        mag += fabsl(t);
      }
      A2p[p] = (double)acc;
      if (scale) scale[p] = (double)mag;
    }
}

void oracle_pr_a3_f64(int64_t N, int64_t d, const double *B, int64_t ldb, double *A3p, double *scale,
                      int64_t p_lo, int64_t p_hi) {
  int64_t p = 0;
  for (int64_t i = 0; i < d; ++i)
    for (int64_t j = i; j < d; ++j)
      for (int64_t k = j; k < d; ++k, ++p) {
        if (p < p_lo || p >= p_hi) continue;
        long double acc = 0.0L, mag = 0.0L;
        for (int64_t x = 0; x < N; ++x) {
          long double t = (long double)B[x * ldb + i] * (long double)B[x * ldb + j] * (long double)B[x * ldb + k];
          acc += t;
          mag += fabsl(t);
        }
        A3p[p] = (double)acc;
        if (scale) scale[p] = (double)mag;
      }
}

/* M(i,r) := A(i,j,k) * B(j,r) * C(k,r),  i<=j<=k, on double operands (long-double accumulation). */
void oracle_tet_mttkrp_f64(int64_t n, int64_t R, const double *Ap, const double *B, int64_t ldb,
                           const double *C, int64_t ldc, double *M, int64_t ldm, double *scale,
                           int64_t r_lo, int64_t r_hi) {
  long double *acc = (long double *)malloc(sizeof(long double) * (size_t)(R > 0 ? R : 1));
  long double *mag = (long double *)malloc(sizeof(long double) * (size_t)(R > 0 ? R : 1));
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i) {
    int on = (i >= r_lo && i < r_hi);
    if (on)
      for (int64_t r = 0; r < R; ++r) acc[r] = mag[r] = 0.0L;
    for (int64_t j = i; j < n; ++j)
      for (int64_t k = j; k < n; ++k) {
        if (on) {
          long double a = (long double)Ap[p];
          for (int64_t r = 0; r < R; ++r) {
            long double t = a * (long double)B[j * ldb + r] * (long double)C[k * ldc + r];
            acc[r] += t;
            mag[r] += fabsl(t);
          }
        }
        ++p;
      }
    if (on)
      for (int64_t r = 0; r < R; ++r) {
        M[i * ldm + r] = (double)acc[r];
        if (scale) scale[i * R + r] = (double)mag[r];
      }
  }
  free(acc);
  free(mag);
}

/* ---- double precision: the remaining products of one packed triangle and the further domains ---
 * Same definitions as their single-precision namesakes above; long double accumulation, one
 * rounding to double. */
void oracle_pack_tril_f64(int64_t n, const double *dense, int64_t ld, double *packed) {
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j <= i; ++j) packed[p++] = dense[i * ld + j];
}

void oracle_unpack_tril_f64(int64_t n, const double *packed, double *dense, int64_t ld) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) dense[i * ld + j] = 0.0;
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j <= i; ++j) dense[i * ld + j] = packed[p++];
}

/* mode 0: y(i) := T(i,j) x(j); mode 1: y(j) := T(i,j) x(i); mode 2: the symmetric matrix whose
 * unique elements are T (Section 3, "Redundancy map"). */
void oracle_trimv_f64(int64_t n, int lower, int mode, const double *Tp, const double *x, double *y,
                      double *scale, int64_t r_lo, int64_t r_hi) {
  int64_t *start = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
  int64_t p = 0;
  for (int64_t i = 0; i < n; ++i) {
    start[i] = p;
    p += lower ? i + 1 : n - i;
  }
  for (int64_t i = 0; i < n; ++i) {
    if (i < r_lo || i >= r_hi) continue;
    long double acc = 0.0L, mag = 0.0L;
    for (int64_t j = 0; j < n; ++j) {
      int64_t a = i, b = j;
      if (mode == 1) { a = j; b = i; }
      int inside = lower ? (b <= a) : (a <= b);
      if (mode == 2 && !inside) { int64_t t = a; a = b; b = t; inside = 1; }
      if (!inside) continue;
      long double t = (long double)Tp[start[a] + (lower ? b : b - a)] * (long double)x[j];
      acc += t;
      mag += fabsl(t);
    }
    y[i] = (double)acc;
    if (scale) scale[i] = (double)mag;
  }
  free(start);
}

void oracle_pack_sband_f64(int64_t n, int64_t w, int64_t s, const double *dense, int64_t ld, double *diag) {
  int64_t p = 0;
  for (int64_t d = -w; d <= w; ++d)
    for (int64_t i = 0; i < n; ++i) {
      int64_t j = i + d * s;
      diag[p++] = (j >= 0 && j < n) ? dense[i * ld + j] : 0.0;
    }
}

void oracle_unpack_sband_f64(int64_t n, int64_t w, int64_t s, const double *diag, double *dense, int64_t ld) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) dense[i * ld + j] = 0.0;
  int64_t p = 0;
  for (int64_t d = -w; d <= w; ++d)
    for (int64_t i = 0; i < n; ++i) {
      int64_t j = i + d * s;
      if (j >= 0 && j < n) dense[i * ld + j] = diag[p];
      ++p;
    }
}

void oracle_sband_spmv_f64(int64_t n, int64_t w, int64_t s, const double *D, const double *x, double *y,
                           double *scale, int64_t r_lo, int64_t r_hi) {
  for (int64_t i = 0; i < n; ++i) {
    if (i < r_lo || i >= r_hi) continue;
    long double acc = 0.0L, mag = 0.0L;
    for (int64_t d = -w; d <= w; ++d) {
      int64_t j = i + d * s;
      if (j < 0 || j >= n) continue;
      long double t = (long double)D[(d + w) * n + i] * (long double)x[j];
      acc += t;
      mag += fabsl(t);
    }
    y[i] = (double)acc;
    if (scale) scale[i] = (double)mag;
  }
}

void oracle_pack_subtri_f64(int64_t N, int64_t k, const double *dense, int64_t ld, double *packed) {
  int64_t p = 0;
  for (int64_t i = 0; i < N; ++i)
    for (int64_t j = 0; j < N; ++j)
      if (j - i >= N - k) packed[p++] = dense[i * ld + j];
}

void oracle_unpack_subtri_f64(int64_t N, int64_t k, const double *packed, double *dense, int64_t ld) {
  int64_t p = 0;
  for (int64_t i = 0; i < N; ++i)
    for (int64_t j = 0; j < N; ++j) dense[i * ld + j] = (j - i >= N - k) ? packed[p++] : 0.0;
}

void oracle_subtri_spmv_f64(int64_t N, int64_t k, const double *Ap, const double *x, double *y, double *scale,
                            int64_t r_lo, int64_t r_hi) {
  int64_t p = 0;
  for (int64_t i = 0; i < N; ++i) {
    long double acc = 0.0L, mag = 0.0L;
    for (int64_t j = 0; j < N; ++j) {
      if (j - i < N - k) continue;
      long double t = (long double)Ap[p++] * (long double)x[j];
      acc += t;
      mag += fabsl(t);
    }
    if (i >= r_lo && i < r_hi) {
      y[i] = (double)acc;
      if (scale) scale[i] = (double)mag;
    }
  }
}

void oracle_pack_leslie_f64(int64_t n, const double *dense, int64_t ld, double *R, double *S) {
  int64_t p = 0;
  for (int64_t j = 0; j < n; ++j) R[p++] = dense[j];
  p = 0;
  for (int64_t i = 1; i < n; ++i) S[p++] = dense[i * ld + (i - 1)];
}

void oracle_unpack_leslie_f64(int64_t n, const double *R, const double *S, double *dense, int64_t ld) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < n; ++j) dense[i * ld + j] = 0.0;
  for (int64_t j = 0; j < n; ++j) dense[j] = R[j];
  for (int64_t i = 1; i < n; ++i) dense[i * ld + (i - 1)] = S[i - 1];
}

void oracle_leslie_spmv_f64(int64_t n, const double *R, const double *S, const double *x, double *y, double *scale) {
  if (n <= 0) return;
  long double acc = 0.0L, mag = 0.0L;
  for (int64_t j = 0; j < n; ++j) {
    long double t = (long double)R[j] * (long double)x[j];
    acc += t;
    mag += fabsl(t);
  }
  y[0] = (double)acc;
  if (scale) scale[0] = (double)mag;
  for (int64_t i = 1; i < n; ++i) {
    double t = S[i - 1] * x[i - 1]; /* one product: correctly rounded in double already */
    y[i] = t;
    if (scale) scale[i] = fabs(t);
  }
}
