/*
 * dastac.h -- C ABI of libdastac_hip.so: structure-aware contractions over densely
 * packed tensors on AMD gfx950 (MI355X), after "Compressing Structured Tensor
 * Algebra" (DASTAC).
 *
 * Only the elements of a tensor's structure domain are stored, back to back in one
 * buffer, in the iteration order of the rule that reads them (Section 4, "Iteration
 * space extraction": iterators in order of appearance, the last one contiguous).
 * The position of an element is the number of domain points that precede it
 * (Section 4, "Access domain linearization"), which for the domains served
 * here is a closed-form polynomial in the indices and the size:
 *
 *   upper triangle   0<=i<=j<n      tri(n,i,j)   = i*n - i*(i-1)/2 + (j-i)
 *                                   (Section 3's printed P_B with Q=1, l=0)
 *   upper tetrahedron 0<=i<=j<=k<n  tet(n,i,j,k) = [Tet(n)-Tet(n-i)] + [Tri(n-i)-Tri(n-j)] + (k-j)
 *                                   Tri(m)=m(m+1)/2, Tet(m)=m(m+1)(m+2)/6
 *   lower triangle   0<=j<=i<n      tril(n,i,j)  = i*(i+1)/2 + j
 *                                   (Section 4's worked example, Eq. 2)
 *   upper half cube 0<=i<=j<n,      uhc(n,Q,i,j,l) = tri(n,i,j)*Q + l
 *                   0<=l<Q          (Section 3's printed P_B, the running example's buffer B)
 *   band |j-i|<=w                   band(n,w,d,i) = (d+w)*n + i,  d=j-i
 *                                   one n-slot buffer per diagonal summand (Section 4,
 *                                   per-summand buffers), buffers in order d=-w..w;
 *                                   slot i of diagonal d holds A[i][i+d]; the |d| slots of a
 *                                   diagonal whose column falls outside the matrix are padding.
 *   strided band j-i = d*s, |d|<=w  sband(n,w,d,i) = (d+w)*n + i: the same buffers, slot i of summand d
 *                                   holding A[i][i+d*s] (Section 6.4, strided-band structure)
 *   sub-triangle j-i >= N-k         subtri(N,k,i,j) = tri(k, i, j-(N-k)): the upper triangle of the
 *                                   k x k block in the top right corner (Section 6.4, sub-triangular structure)
 *   Leslie (i=0) + (j=i-1)          two summands, two buffers: R[n] with A[0][j] at j, S[n-1] with
 *                                   A[i][i-1] at i-1 (Table 2, SpMV_L)
 *
 * All index arithmetic is exact 64-bit integer arithmetic: the rational coefficients
 * are evaluated on a doubled (or six-fold) numerator that is always divisible
 * (Fig. 4 of the paper does the same: doubled terms, one exact unsigned division).
 *
 * Conventions
 *   - Status codes: DASTAC_OK on success, otherwise one of the codes below.  No
 *     exception or signal crosses this boundary.  dastac_strerror() names a code.
 *   - n == 0 is a successful no-op for every operation.
 *   - "DEVICE" pointers are device memory of the current HIP device, owned by the
 *     caller, at least 4-byte aligned.  The library never allocates, frees or
 *     retains memory.  "HOST" pointers are ordinary host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device
 *     operations are enqueued on it and return without synchronising.  A launch
 *     failure is reported as DASTAC_EHIP.  Every device operation consists of kernel
 *     launches only (outputs that must start at zero are cleared by a fill kernel),
 *     so the calls may be recorded into a HIP graph by stream capture.
 *   - Outputs are overwritten, not accumulated into (the paper's statement adds into
 *     a zero-initialised output, Section 5.2; the result is the same).
 *   - An output buffer that overlaps an input buffer is rejected with DASTAC_EALIAS.  A
 *     matrix with row stride ld occupies the bytes from its first element to the last
 *     used element of its last row, so two column ranges of one row-major buffer that
 *     interleave row by row count as overlapping only if those byte ranges intersect.
 *   - Row strides (ld, ldb, ldc, ldm) above DASTAC_MAX_LD elements are rejected with
 *     DASTAC_EOVERFLOW (rows * ld * element size must stay inside int64).
 *   - The library may be called from several host threads: the only state it keeps is
 *     what it asks of the runtime once per device (how many workgroups of a kernel
 *     the device holds at once).
 */
#ifndef DASTAC_H
#define DASTAC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DASTAC_OK 0
#define DASTAC_EINVAL 1    /* negative size, m/R/w out of range, leading dimension too small, p out of range */
#define DASTAC_ENULL 2     /* a required pointer is NULL */
#define DASTAC_EOVERFLOW 3 /* the element count would leave the guarded int64 range */
#define DASTAC_EALIAS 4    /* an output overlaps an input */
#define DASTAC_EHIP 5      /* the HIP runtime reported an error at launch */

/* Largest sizes accepted: beyond these a count or an intermediate product could overflow int64. */
#define DASTAC_TRI_MAX_N 2147483647LL /* 2*Tri(n) < 2^63 */
#define DASTAC_TET_MAX_N 1048576LL    /* Tri(n)*(n+2) < 2^63 */
#define DASTAC_MAX_LD 268435456LL     /* largest row stride, in elements */

/* Human-readable name of a status code (static storage, never NULL). */
const char *dastac_strerror(int status);

/* ---- index polynomials: HOST, pure, need no device ------------------------------
 * Forward polynomials (Section 4, "Access domain linearization"; the closed forms are
 * listed at the top of this file).  Return the count / offset, or -1 on invalid
 * arguments (n<0, n above the guard, index outside the domain, w<0). */
int64_t dastac_tri_count(int64_t n);
int64_t dastac_tet_count(int64_t n);
int64_t dastac_band_count(int64_t n, int64_t w);
int64_t dastac_tri_offset(int64_t n, int64_t i, int64_t j);
int64_t dastac_tet_offset(int64_t n, int64_t i, int64_t j, int64_t k);
int64_t dastac_band_offset(int64_t n, int64_t w, int64_t d, int64_t i);
/* Lower triangle 0<=j<=i<n (Section 4, worked example): i(i+1)/2 + j; the count is tri_count(n). */
int64_t dastac_tril_offset(int64_t n, int64_t i, int64_t j);
/* Upper half cube of the running example (i<=j<n, 0<=l<Q; Q >= 1): Tri(n)*Q elements. */
int64_t dastac_uhc_count(int64_t n, int64_t Q);
int64_t dastac_uhc_offset(int64_t n, int64_t Q, int64_t i, int64_t j, int64_t l);
/* Sub-triangular structure j-i >= N-k, 0<=k<=N (Section 6.4): tri_count(k) elements. */
int64_t dastac_subtri_offset(int64_t N, int64_t k, int64_t i, int64_t j);

/* Inverse polynomials: the unique domain point whose offset is p.  The paper only
 * mentions inverting a quasi-polynomial as costly when done per iteration (Section 7,
 * "Data layout compression"); here it is evaluated once per wavefront to find the row
 * or slice where a contiguous share of the packed buffer begins.  Exact for every p in
 * [0,count): a floating-point root seeds an integer correction.  Return DASTAC_OK, or
 * DASTAC_EINVAL for p outside [0,count) or an invalid n, DASTAC_ENULL for a NULL output. */
int dastac_tri_inverse(int64_t n, int64_t p, int64_t *i, int64_t *j);
int dastac_tet_inverse(int64_t n, int64_t p, int64_t *i, int64_t *j, int64_t *k);

/* ---- compression / decompression: DEVICE (Section 3, "Data layout compression") --
 * pack copies the domain elements of a dense row-major tensor into the packed buffer;
 * unpack writes the dense tensor back, with +0.0f at every position outside the domain.
 * Bit-exact copies.  `ld` is the dense row stride in elements (ld >= n).
 *   triu : dense n x n (stride ld)      <-> packed[tri_count(n)]
 *   tet  : dense n x n x n, contiguous  <-> packed[tet_count(n)]
 *   band : dense n x n (stride ld)      <-> diag_major[(2w+1)*n]; pack writes +0.0f into padding slots,
 *                                           unpack ignores them.
 *   uhc  : dense n x n x Q, contiguous  <-> packed[uhc_count(n,Q)]
 *   tril : dense n x n (stride ld)      <-> packed[tri_count(n)], row i holding columns 0..i
 *   sband: dense n x n (stride ld)      <-> diag_major[(2w+1)*n], stride s >= 1; padding as for band
 *   subtri: dense N x N (stride ld)     <-> packed[tri_count(k)], 0 <= k <= N
 *   leslie: dense n x n (stride ld)     <-> R[n] and S[n-1] (S may be NULL when n == 1) */
int dastac_pack_triu_f32(int64_t n, const float *dense, int64_t ld, float *packed, void *stream);
int dastac_unpack_triu_f32(int64_t n, const float *packed, float *dense, int64_t ld, void *stream);
int dastac_pack_tet_f32(int64_t n, const float *dense, float *packed, void *stream);
int dastac_unpack_tet_f32(int64_t n, const float *packed, float *dense, void *stream);
int dastac_pack_band_f32(int64_t n, int64_t w, const float *dense, int64_t ld, float *diag_major, void *stream);
int dastac_unpack_band_f32(int64_t n, int64_t w, const float *diag_major, float *dense, int64_t ld, void *stream);
int dastac_pack_tril_f32(int64_t n, const float *dense, int64_t ld, float *packed, void *stream);
int dastac_unpack_tril_f32(int64_t n, const float *packed, float *dense, int64_t ld, void *stream);
int dastac_pack_uhc_f32(int64_t n, int64_t Q, const float *dense, float *packed, void *stream);
int dastac_unpack_uhc_f32(int64_t n, int64_t Q, const float *packed, float *dense, void *stream);
int dastac_pack_sband_f32(int64_t n, int64_t w, int64_t s, const float *dense, int64_t ld, float *diag_major,
                          void *stream);
int dastac_unpack_sband_f32(int64_t n, int64_t w, int64_t s, const float *diag_major, float *dense, int64_t ld,
                            void *stream);
int dastac_pack_subtri_f32(int64_t N, int64_t k, const float *dense, int64_t ld, float *packed, void *stream);
int dastac_unpack_subtri_f32(int64_t N, int64_t k, const float *packed, float *dense, int64_t ld, void *stream);
int dastac_pack_leslie_f32(int64_t n, const float *dense, int64_t ld, float *R, float *S, void *stream);
int dastac_unpack_leslie_f32(int64_t n, const float *R, const float *S, float *dense, int64_t ld, void *stream);

/* ---- contractions: DEVICE, fp32 storage and arithmetic ---------------------------
 * Summation order is unspecified (the paper compiles with fast-math, Section 6.1);
 * each output element is within 1e-4 * sum|products| of the exactly rounded result.
 *
 * Non-finite inputs.  Every contraction propagates Inf and NaN of the elements it multiplies as
 * IEEE arithmetic does, with one exception: in trmv (n <= 8192), tet_ttv and subtri_spmv (k <= 8192)
 * a product with a ZERO factor contributes nothing even if the other factor is Inf or NaN, where
 * IEEE arithmetic and the plain rule give NaN -- in fp32 when either factor is zero, in fp64 when the
 * element of x (of v) is zero.  (These kernels let lanes read past the end of a packed row and pair
 * such elements with zeros; the same multiply serves the elements inside the row.)
 */

/* y(i) := U(i,j) * x(j), i<=j   (Table 1/2, SpMV_UT).  Up[tri_count(n)], x[n], y[n]; n <= 524288.
 * Above n = 8192 the result is accumulated with floating-point atomics (last bits may differ between calls). */
int dastac_trmv_f32(int64_t n, const float *Up, const float *x, float *y, void *stream);

/* y(i) := S(i,j) * x(j), S symmetric with its unique elements S(i,j), i<=j, packed as an upper triangle
 * (Section 3, "Redundancy map": the other half is reached by swapping the two indices).  Every packed
 * element is read once and used twice.  Up[tri_count(n)], x[n], y[n]; n <= 524288 (beyond: DASTAC_EOVERFLOW).
 * The output is accumulated with floating-point atomics, so its last bits may differ between calls. */
int dastac_symv_f32(int64_t n, const float *Up, const float *x, float *y, void *stream);

/* The other products one packed triangle admits, same limits and same atomic accumulation as symv:
 *   trmv_t        y(j) := U(i,j) * x(i), i<=j     the transposed product of the packed upper triangle
 *   trmv_lower    y(i) := L(i,j) * x(j), j<=i     L packed as a LOWER triangle: row i holds columns 0..i, at
 *                                                 tril(n,i,j) = i(i+1)/2 + j (Section 4, worked example, Eq. 2)
 *   trmv_lower_t  y(j) := L(i,j) * x(i), j<=i
 *   symv_lower    y := S x, S symmetric with its unique elements S(i,j), j<=i, packed as a lower triangle
 *                 (the arrangement of Section 3's redundancy-map example). */
int dastac_trmv_t_f32(int64_t n, const float *Up, const float *x, float *y, void *stream);
int dastac_trmv_lower_f32(int64_t n, const float *Lp, const float *x, float *y, void *stream);
int dastac_trmv_lower_t_f32(int64_t n, const float *Lp, const float *x, float *y, void *stream);
int dastac_symv_lower_f32(int64_t n, const float *Lp, const float *x, float *y, void *stream);

/* C(i,c) := U(i,k) * B(k,c), i<=k, 0<=c<m  (the SpMV_UT rule with a matrix right-hand side).
 * B is n x m row-major with row stride ldb >= m, C is n x m with row stride ldc >= m; m >= 1.
 * Only columns 0..m-1 of every row of C are written.  With m <= 64 on n >= 1024 the packed triangle is
 * streamed once per 32 columns and the pieces of C are added with floating-point atomics; otherwise, when
 * m is small against n, the reduction range is shared out over several workgroups that add into a cleared
 * C the same way (in both cases the last bits may differ between calls); at shapes with enough columns
 * every element of C has one writer.
 * (trmm_f64 shares more readily than trmm_f32: also where one workgroup per compute unit is available.) */
int dastac_trmm_f32(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C, int64_t ldc,
                    void *stream);

/* C(i,c) := S(i,k) * B(k,c), S symmetric with its unique elements S(i,k), i<=k, packed as an upper triangle
 * (Section 3, "Redundancy map", with a matrix right-hand side).  Shapes, strides and limits as trmm; no
 * atomics (every tile of C has one owner), each packed element is read twice. */
int dastac_symm_f32(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C, int64_t ldc,
                    void *stream);

/* y(i) := sum_{d=-w..w, 0<=i+d<n} D(d,i) * x(i+d)   (Section 6.4 strided-band rule, unit stride,
 * 2w+1 summands; w=0 is Table 2's SpMV_D).  D[(2w+1)*n] diagonal-major as described above; padding
 * slots are never used for their value.  0 <= w <= 2^20 (beyond: DASTAC_EOVERFLOW); the half-widths
 * 0, 1, 2, 4, 8 and 16 have unrolled kernels. */
int dastac_band_spmv_f32(int64_t n, int64_t w, const float *D, const float *x, float *y, void *stream);

/* y(i) := sum_{d=-w..w, 0<=i+d*s<n} D(d,i) * x(i+d*s)   (Section 6.4, strided band; the paper's experiment
 * is w=1 with s from 1, tridiagonal, to n, diagonal).  D[(2w+1)*n] as for band_spmv with slot (d,i)
 * holding A[i][i+d*s]; 0 <= w <= 2^20, 1 <= s <= 2^40 (s >= n leaves the main diagonal). */
int dastac_sband_spmv_f32(int64_t n, int64_t w, int64_t s, const float *D, const float *x, float *y, void *stream);

/* y(i) := A(i,j) * x(j), j-i >= N-k   (Section 6.4, sub-triangular structure; k = N is SpMV_UT).
 * Ap[tri_count(k)], x[N], y[N]; all N outputs are written, rows k..N-1 with +0.  0 <= k <= N,
 * k <= 524288; above k = 8192 accumulated with atomics like trmv. */
int dastac_subtri_spmv_f32(int64_t N, int64_t k, const float *Ap, const float *x, float *y, void *stream);

/* y(0) := R(j) * x(j);  y(i) := S(i-1) * x(i-1), 1<=i<n   (Table 2, SpMV_L: first row plus sub-diagonal).
 * R[n], S[n-1] (may be NULL when n == 1), x[n], y[n].  y(0) is accumulated with one floating-point
 * atomic per workgroup (last bits may differ between calls); every other output is one exact product. */
int dastac_leslie_spmv_f32(int64_t n, const float *R, const float *S, const float *x, float *y, void *stream);

/* M(i,j) := A(i,j,k) * v(k), i<=j<=k.  Ap[tet_count(n)], v[n]; the output is itself packed:
 * Mp[tri_count(n)] with M(i,j) at tri(n,i,j).  n <= 8192 (a larger tetrahedron
 * exceeds device memory); beyond that DASTAC_EOVERFLOW. */
int dastac_tet_ttv_f32(int64_t n, const float *Ap, const float *v, float *Mp, void *stream);

/* M(i,r) := A(i,j,k) * B(j,r) * C(k,r), i<=j<=k, 0<=r<R  (Table 1 MTTKRP rule on the upper tetrahedron).
 * B, C are n x R row-major with row strides ldb, ldc >= R; M is n x R with row stride ldm >= R.
 * 1 <= R <= 2^20.  The kernel takes 32 columns of the factor
 * matrices at a time: R > 32 runs block by block, each block reading the packed tetrahedron once.  M is
 * cleared first and the blocks of a slice add their parts with floating-point atomics, so the last bits
 * may differ between calls (integer-valued inputs whose partial sums are exact give identical results).
 * The sum is evaluated factored (A with B first, then with C) on blocks padded with zeros, so a non-finite
 * element of B(j,:) or C(k,:), j,k >= i, makes M(i,r) non-finite as the plain rule does, but possibly NaN
 * where the plain rule gives an infinity. */
int dastac_tet_mttkrp_f32(int64_t n, int64_t R, const float *Ap, const float *B, int64_t ldb, const float *C,
                          int64_t ldc, float *M, int64_t ldm, void *stream);

/* A(i,j,k) := B(i,j,l) * C(k,l), i<=j, 0<=l<Q, 0<=k<K   (the running example, Fig. 3; Table 1 TTM with
 * the upper-half-cube structure, TTM_UT).  Bp[uhc_count(n,Q)] is packed; C is K x Q row-major with row
 * stride ldc >= Q; the output inherits the structure and is packed by the same rule:
 * Ap[uhc_count(n,K)] with A(i,j,k) at uhc(n,K,i,j,k).  Q, K >= 1. */
int dastac_ttm_ut_f32(int64_t n, int64_t Q, int64_t K, const float *Bp, const float *C, int64_t ldc, float *Ap,
                      void *stream);

/* The polynomial-regression tensors of Table 1 ("Polynomial Regression Degree-D": A^k(i1..ik) := B(x,i1)*...*B(x,ik),
 * summed over x), orders 2 and 3, written straight into their packed hyper-triangles:
 *   pr_a2   A2(i,j)   := B(x,i) * B(x,j),          i<=j      A2p[tri_count(d)] at tri(d,i,j)
 *   pr_a3   A3(i,j,k) := B(x,i) * B(x,j) * B(x,k), i<=j<=k   A3p[tet_count(d)] at tet(d,i,j,k)
 * B is N x d row-major with row stride ldb >= d.  d == 0 is a no-op; N == 0 writes zeros.  d <= 65536 (a2),
 * d <= 8192 (a3), N <= 2^31.  When the output has few tiles the sample range is split over workgroups that
 * add into the zeroed output with floating-point atomics (last bits may then differ between calls). */
int dastac_pr_a2_f32(int64_t N, int64_t d, const float *B, int64_t ldb, float *A2p, void *stream);
int dastac_pr_a3_f32(int64_t N, int64_t d, const float *B, int64_t ldb, float *A3p, void *stream);

/* Measurement aid, not one of the paper's operations: reads src[count] once (non-temporal 16-byte loads)
 * and writes npartial partial sums, partial[b] = sum of the b-th contiguous chunk of ceil(count/npartial)
 * elements (rounded up to a multiple of 4; chunks past the end give 0).  It is the read-only stream that
 * bench.py times over the same byte count as each bandwidth-bound contraction (Section 6.1 reports run times
 * only; the yardstick is this implementation's).  1 <= npartial <= 2^24, count <= 2^40 (else DASTAC_EINVAL,
 * DASTAC_EOVERFLOW); src and partial are device pointers owned by the caller, 4-byte aligned. */
int dastac_stream_sum_f32(int64_t count, const float *src, float *partial, int64_t npartial, void *stream);

/* ---- double precision (the paper's own element type, Section 6.1) ------------------------------
 * The same layouts, index polynomials, argument rules and error codes as the _f32 entry points of the
 * same name, on double operands (8-byte aligned).  Each output element is within 1e-12 * sum|products|
 * of the exactly rounded result.  tet_ttv_f64 needs n <= 8192 (the vector is kept in LDS), beyond that
 * DASTAC_EOVERFLOW; the products of one packed triangle take n <= 262144.  The matrix-core contractions (TRMM, SYMM, MTTKRP, TTM_UT, the
 * polynomial-regression tensors) run on the fp64 matrix cores; shapes and limits as their _f32 namesakes. */
int dastac_pack_triu_f64(int64_t n, const double *dense, int64_t ld, double *packed, void *stream);
int dastac_unpack_triu_f64(int64_t n, const double *packed, double *dense, int64_t ld, void *stream);
int dastac_pack_tet_f64(int64_t n, const double *dense, double *packed, void *stream);
int dastac_unpack_tet_f64(int64_t n, const double *packed, double *dense, void *stream);
int dastac_pack_band_f64(int64_t n, int64_t w, const double *dense, int64_t ld, double *diag_major, void *stream);
int dastac_unpack_band_f64(int64_t n, int64_t w, const double *diag_major, double *dense, int64_t ld, void *stream);
int dastac_trmv_f64(int64_t n, const double *Up, const double *x, double *y, void *stream);
int dastac_band_spmv_f64(int64_t n, int64_t w, const double *D, const double *x, double *y, void *stream);
int dastac_tet_ttv_f64(int64_t n, const double *Ap, const double *v, double *Mp, void *stream);
int dastac_trmm_f64(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C, int64_t ldc,
                    void *stream);
int dastac_symm_f64(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C, int64_t ldc,
                    void *stream);
int dastac_pack_uhc_f64(int64_t n, int64_t Q, const double *dense, double *packed, void *stream);
int dastac_unpack_uhc_f64(int64_t n, int64_t Q, const double *packed, double *dense, void *stream);
int dastac_ttm_ut_f64(int64_t n, int64_t Q, int64_t K, const double *Bp, const double *C, int64_t ldc, double *Ap,
                      void *stream);
int dastac_tet_mttkrp_f64(int64_t n, int64_t R, const double *Ap, const double *B, int64_t ldb, const double *C,
                          int64_t ldc, double *M, int64_t ldm, void *stream);
int dastac_pr_a2_f64(int64_t N, int64_t d, const double *B, int64_t ldb, double *A2p, void *stream);
int dastac_pr_a3_f64(int64_t N, int64_t d, const double *B, int64_t ldb, double *A3p, void *stream);
int dastac_pack_tril_f64(int64_t n, const double *dense, int64_t ld, double *packed, void *stream);
int dastac_unpack_tril_f64(int64_t n, const double *packed, double *dense, int64_t ld, void *stream);
int dastac_symv_f64(int64_t n, const double *Up, const double *x, double *y, void *stream);
int dastac_trmv_t_f64(int64_t n, const double *Up, const double *x, double *y, void *stream);
int dastac_symv_lower_f64(int64_t n, const double *Lp, const double *x, double *y, void *stream);
int dastac_trmv_lower_f64(int64_t n, const double *Lp, const double *x, double *y, void *stream);
int dastac_trmv_lower_t_f64(int64_t n, const double *Lp, const double *x, double *y, void *stream);
int dastac_pack_sband_f64(int64_t n, int64_t w, int64_t s, const double *dense, int64_t ld, double *diag_major,
                          void *stream);
int dastac_unpack_sband_f64(int64_t n, int64_t w, int64_t s, const double *diag_major, double *dense, int64_t ld,
                            void *stream);
int dastac_sband_spmv_f64(int64_t n, int64_t w, int64_t s, const double *D, const double *x, double *y, void *stream);
int dastac_pack_subtri_f64(int64_t N, int64_t k, const double *dense, int64_t ld, double *packed, void *stream);
int dastac_unpack_subtri_f64(int64_t N, int64_t k, const double *packed, double *dense, int64_t ld, void *stream);
int dastac_subtri_spmv_f64(int64_t N, int64_t k, const double *Ap, const double *x, double *y, void *stream);
int dastac_pack_leslie_f64(int64_t n, const double *dense, int64_t ld, double *R, double *S, void *stream);
int dastac_unpack_leslie_f64(int64_t n, const double *R, const double *S, double *dense, int64_t ld, void *stream);
int dastac_leslie_spmv_f64(int64_t n, const double *R, const double *S, const double *x, double *y, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DASTAC_H */
