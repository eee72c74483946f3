// MTTKRP over a packed upper tetrahedron on the fp32 matrix cores:
//
//   M(i,r) := A(i,j,k) * B(j,r) * C(k,r),   i<=j<=k, 0<=r<R (32 columns r per launch)     (Table 1, MTTKRP rule)
//
// Factored evaluation, contracting over the ROW index first.  Slice i of the packed tetrahedron is a
// packed upper triangle U_i of order m = n-i, so
//
//   M(i,:) = sum_k C(k,:) .* S_i(k,:)   with   S_i = U_i^T * B[i:, :]     (S_i(k,r) = sum_{j<=k} U_i(j,k) B(j,r)).
//
// Contracting over j makes k -- the index that is contiguous in the packed buffer -- the row index of
// the matrix instruction's first operand: v_mfma_f32_32x32x2_f32 takes from lane l the element
// (row l%32, contraction index l/32), so a half-wavefront that loads 32 consecutive 16-byte pieces of
// ONE packed row already holds four operands (one per component: k = k0+4*(l%32)+s) in its registers.
// A load instruction therefore fetches 512 contiguous bytes of each of two neighbouring packed rows, no
// element is moved through LDS, and the instruction stream per two rows is one 16-byte load of A, one
// 4-byte load of B (lane l: row l/32, column l%32 -- the second operand) and four matrix instructions.
//
// Work items.  The slice triangle is cut into blocks of 128 rows x 128 values of k, aligned to its
// lower right corner (so that only the blocks at its top and left edges are ragged).  A block is one
// wavefront's job, in a workgroup of its own: it accumulates the block's part of S_i (128 x 32, four
// accumulators), multiplies it elementwise with C's rows k and adds the 32 column sums into M(i,:)
// with floating-point atomics (the sum over blocks is a sum of partial results: any partition of the
// iteration space is correct, Section 5.2 "Parallelization").  M is cleared by a launch of its own
// first.  Blocks above the diagonal are full and run without any test; blocks on the diagonal (and
// the ragged ones) select away what lies left of the diagonal, past the block's columns or below its
// rows, and aim the loads of wholly dead lanes at the row's first live piece, so nothing outside the
// block is fetched.
//
// Order.  Workgroup ids are dealt to the eight XCDs in turn, so id%8 picks the XCD and id/8 walks that
// XCD's own list: slices of nearly equal order go to the eight XCDs (alternating direction, so the
// totals agree), heaviest first, and a slice's blocks follow each other in memory order -- blocks
// that are neighbours in k, which share the cache lines cut by their common edge, run at the same
// time on the same L2.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kEdge = 128;  // rows and k values per block
constexpr int kDepth = 8;   // two-row steps whose loads are in flight per wavefront
constexpr int kMinOrder = 3;  // slices of order 1 and 2 (4 elements in all) are computed by the clearing launch

typedef float f16v __attribute__((ext_vector_type(16)));

// A wavefront's walk over the two-row steps of its block.  Step t pairs the rows row0+2t (lane half 0)
// and row0+2t+1 (lane half 1); the byte offset of a lane's 16-byte piece grows from step to step by a
// difference that itself shrinks by 16 (a packed row is one element shorter than the one before).
struct Walk {
  const char *As;   // the slice's packed triangle
  unsigned e0;      // byte offset of this lane's piece at step 0
  int delta0;       // growth of that offset from step 0 to step 1
  const float *b0;  // this lane's element of B at step 0 (row of lane half 0 when masked)
  int64_t bstep;    // two rows of B, in elements
  int begin, end;   // first step; one past the last step
  // masked walk only
  int64_t bhalf;    // lane half times one row of B, in elements
  int dd0;          // this lane's row minus the first k of its piece, at step 0
  int row0, rhi;    // this lane's row at step 0; one past the block's last row
  int kspan;        // the block's last k + 1 minus the first k of this lane's piece
  unsigned emax;    // largest byte offset whose 16-byte piece ends inside the packed buffer
};

// Where the walk stands: the state that moves from one request to the next.
struct Cursor {
  unsigned e;
  int delta;
  const float *bp;
  int t;
};

__device__ inline Cursor cursor_at(const Walk &w, int t) {
  Cursor c;
  c.e = w.e0 + (unsigned)(t * w.delta0 - 8 * t * (t - 1));
  c.delta = w.delta0 - 16 * t;
  c.bp = w.b0 + t * w.bstep;
  c.t = t;
  return c;
}

// Requests step c.t: 16 bytes of A and one element of B per lane.
template <bool MASKED>
__device__ inline void request(const Walk &w, const Cursor &c, f4a &a, float &b) {
  if (MASKED) {
    // wholly dead lanes (all four k left of the diagonal) re-aim at the piece that holds the diagonal
    const int dd = w.dd0 + 2 * c.t;
    unsigned e = c.e + (unsigned)(((dd > 0 ? dd : 0) & ~3) << 2);
    e = e < w.emax ? e : w.emax;
    a = *reinterpret_cast<const f4u *>(w.As + e);
    const bool row_ok = w.row0 + 2 * c.t < w.rhi;  // a dead row takes lane half 0's row of B
    b = *(c.bp + (row_ok ? w.bhalf : (int64_t)0));
  } else {
    a = *reinterpret_cast<const f4u *>(w.As + c.e);
    b = c.bp[0];
  }
}

__device__ inline void advance(const Walk &w, Cursor &c) {
  c.e += (unsigned)c.delta;
  c.delta -= 16;
  c.bp += w.bstep;
  ++c.t;
}

template <bool MASKED>
__device__ inline void multiply(const Walk &w, int t, f4a a, float b, f16v (&acc)[4]) {
  if (MASKED) {
    const int lo = w.dd0 + 2 * t;                            // components below lo are left of the diagonal
    const int hi = (w.row0 + 2 * t < w.rhi) ? w.kspan : lo;  // components from hi on are outside the block
    const unsigned span = hi > lo ? (unsigned)(hi - lo) : 0u;
    a.x = ((unsigned)(0 - lo) < span) ? a.x : 0.0f;
    a.y = ((unsigned)(1 - lo) < span) ? a.y : 0.0f;
    a.z = ((unsigned)(2 - lo) < span) ? a.z : 0.0f;
    a.w = ((unsigned)(3 - lo) < span) ? a.w : 0.0f;
  }
  acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b, acc[0], 0, 0, 0);
  acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b, acc[1], 0, 0, 0);
  acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b, acc[2], 0, 0, 0);
  acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b, acc[3], 0, 0, 0);
}

// Steps w.begin .. w.end-1 with the loads of kDepth steps in flight.  The main loop has no control
// flow around its loads, so the compiler keeps exact counts of what is outstanding.
template <bool MASKED>
__device__ inline void sweep(const Walk &w, f16v (&acc)[4]) {
  if (w.begin >= w.end) return;
  f4a a[kDepth];
  float b[kDepth];
  int t = w.begin;
#pragma unroll
  for (int d = 0; d < kDepth; ++d) {  // a block with fewer steps repeats its last one; never multiplied
    const int td = t + d < w.end ? t + d : w.end - 1;
    request<MASKED>(w, cursor_at(w, td), a[d], b[d]);
  }
  Cursor c = cursor_at(w, t + kDepth);
  while (t + 2 * kDepth <= w.end) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      multiply<MASKED>(w, t + d, a[d], b[d], acc);
      request<MASKED>(w, c, a[d], b[d]);
      advance(w, c);
      __builtin_amdgcn_sched_barrier(0);  // keep each request where its registers come free, not at the loop's end
    }
    t += kDepth;
  }
  // fewer than 2*kDepth steps are left; those from t+kDepth on are still to be requested
#pragma unroll
  for (int d = 0; d < kDepth; ++d) {
    if (t + d < w.end) multiply<MASKED>(w, t + d, a[d], b[d], acc);
    if (t + d + kDepth < w.end) request<MASKED>(w, cursor_at(w, t + d + kDepth), a[d], b[d]);
  }
  t += kDepth;
#pragma unroll
  for (int d = 0; d < kDepth; ++d)
    if (t + d < w.end) multiply<MASKED>(w, t + d, a[d], b[d], acc);
}

// Number of blocks of a slice whose triangle is P blocks high.
__host__ __device__ inline int64_t blocks_of(int64_t P) { return P * (P + 1) / 2; }

__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2))) void mttkrp_block_kernel(
    int64_t n, int R, const float *__restrict__ A, const float *__restrict__ Bm, int64_t ldb,
    const float *__restrict__ Cm, int64_t ldc, float *__restrict__ M, int64_t ldm, int64_t total) {
  const int lane = threadIdx.x, l32 = lane & 31, h = lane >> 5;

  // ---- which block: id%8 = XCD, id/8 = position in that XCD's list (slices by descending order m,
  // groups of eight consecutive orders dealt to the XCDs in alternating direction)
  const int x = (int)(blockIdx.x & 7u);
  unsigned seq = blockIdx.x >> 3;
  const int gmax = (int)((n - 1) >> 3);  // group g holds the orders 8g+1 .. 8g+8, all ceil(m/128) = g/16+1 blocks high
  int P = gmax / 16 + 1;
  unsigned cnt = (unsigned)(gmax % 16 + 1);
  unsigned per = (unsigned)blocks_of(P);
  while (P > 1 && seq >= cnt * per) {
    seq -= cnt * per;
    --P;
    cnt = 16;
    per = (unsigned)blocks_of(P);
  }
  if (seq >= cnt * per) return;  // (the grid holds exactly the lists' length: not reached)
  const unsigned s = (unsigned)uniform32((int)(seq / per));
  const int g = 16 * (P - 1) + (int)(cnt - 1 - s);
  const int m = 8 * g + 1 + ((g & 1) ? 7 - x : x);  // order of the slice
  if (m > n || m < kMinOrder) return;
  const int tq = (int)(per - 1 - (seq - s * per));  // blocks in memory order: top block row first
  int a = 0;
  while ((a + 1) * (a + 2) / 2 <= tq) ++a;
  const int p = tq - a * (a + 1) / 2;  // block row a (from the bottom), block column p (from the right), p <= a

  const int64_t i = n - m;
  const int64_t slice0 = tet_slice_start(n, i);
  const int rhi = m - kEdge * a, rlo = rhi > kEdge ? rhi - kEdge : 0;  // rows [rlo, rhi) of the slice triangle
  const int khi = m - kEdge * p;                                      // k values [klo, khi)
  const int klo = khi > kEdge ? khi - kEdge : 0;  // (the top left block is shifted right to start at 0)
  const bool diag = a == p;
  const int nrows = rhi - rlo;

  const int kk0 = klo + 4 * l32;  // first k of this lane's piece
  const int row0 = rlo + h;
  const int cc = l32 < R ? l32 : R - 1;  // lanes past the last column repeat it; their sums are dropped

  Walk w;
  w.As = reinterpret_cast<const char *>(A + slice0);
  // element (row, k) of the slice triangle is at row*m - row(row+1)/2 + k
  w.e0 = 4u * (unsigned)(row0 * m - row0 * (row0 + 1) / 2 + kk0);
  w.delta0 = 4 * (2 * m - 2 * row0 - 3);
  w.bstep = 2 * ldb;
  w.bhalf = h * ldb;
  w.dd0 = row0 - kk0;
  w.row0 = row0;
  w.rhi = rhi;
  w.kspan = khi - kk0;
  {
    const int64_t room = total - 4 - slice0;  // in elements; >= 0 for m >= 3
    w.emax = 4u * (unsigned)(room < 0x3fffffff ? room : 0x3fffffff);
  }
  w.begin = 0;

  f16v acc[4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[q][v] = 0.0f;

  const float *b0 = Bm + (i + rlo) * ldb + cc;  // row of lane half 0 at step 0
  if (!diag) {
    // full width, every row of the block above the diagonal: pairs of rows without any test, then a
    // last odd row (top block row only) through the masked walk
    w.b0 = b0 + w.bhalf;
    w.end = nrows / 2;
    sweep<false>(w, acc);
    if (nrows & 1) {
      w.b0 = b0;
      w.begin = nrows / 2;
      w.end = w.begin + 1;
      sweep<true>(w, acc);
    }
  } else {
    w.b0 = b0;
    w.end = (nrows + 1) / 2;
    sweep<true>(w, acc);
  }

  // ---- fold with C: register v of accumulator q in lane l is S(k, l%32) with
  // k = klo + 4*(8*(v/4) + 4*(l/32) + v%4) + q
  const float *cp = Cm + (i + klo + 16 * h) * ldc + cc;
  float part = 0.0f;
  if (klo + kEdge == khi) {
#pragma unroll
    for (int v = 0; v < 16; ++v)
#pragma unroll
      for (int q = 0; q < 4; ++q) part += acc[q][v] * cp[(int64_t)(32 * (v / 4) + 4 * (v % 4) + q) * ldc];
  } else {
    const int live = khi - klo - 16 * h;  // k offsets below this exist
#pragma unroll
    for (int v = 0; v < 16; ++v)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int off = 32 * (v / 4) + 4 * (v % 4) + q;
        const bool ok = off < live;
        const float cv = cp[ok ? (int64_t)off * ldc : (int64_t)0 - 16 * h * ldc];
        part += ok ? acc[q][v] * cv : 0.0f;
      }
  }
  part += __shfl_xor(part, 32, 64);
  if (h == 0 && l32 < R) unsafeAtomicAdd(&M[i * ldm + l32], part);
}

// Clears M (the block kernel adds into it) and computes the slices of order 1 and 2 -- the last four
// elements of the packed buffer, where a 16-byte load has no room -- directly from the rule.
__global__ __launch_bounds__(256) void mttkrp_clear_kernel(int64_t n, int64_t R, const float *__restrict__ A,
                                                           const float *__restrict__ Bm, int64_t ldb,
                                                           const float *__restrict__ Cm, int64_t ldc,
                                                           float *__restrict__ M, int64_t ldm, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;  // one output element per thread
  if (e >= n * R) return;
  const int64_t i = e / R, r = e - i * R;
  float s = 0.0f;
  if (n - i < kMinOrder) {
    int64_t pos = tet_slice_start(n, i);
    for (int64_t j = i; j < n; ++j)
      for (int64_t k = j; k < n; ++k) s += A[pos++] * Bm[j * ldb + r] * Cm[k * ldc + r];
  }
  M[i * ldm + r] = s;
}

}  // namespace

extern "C" int dastac_tet_mttkrp_f32(int64_t n, int64_t R, const float *Ap, const float *B, int64_t ldb,
                                     const float *C, int64_t ldc, float *M, int64_t ldm, void *stream) {
  if (n < 0 || R < 1 || R > (1 << 20) || ldb < R || ldc < R || ldm < R) return DASTAC_EINVAL;
  if (n > DASTAC_TET_MAX_N || tet(n) > ((int64_t)1 << 40) || ld_too_large(ldb, ldc, ldm))
    return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Ap || !B || !C || !M) return DASTAC_ENULL;
  const int64_t mb = view_bytes(n, ldm, R, 4);
  if (overlaps(M, mb, Ap, tet(n) * 4) || overlaps(M, mb, B, view_bytes(n, ldb, R, 4)) ||
      overlaps(M, mb, C, view_bytes(n, ldc, R, 4)))
    return DASTAC_EALIAS;
  hipStream_t st = (hipStream_t)stream;
  mttkrp_clear_kernel<<<(unsigned)ceil_div(n * R, 256), 256, 0, st>>>(n, R, Ap, B, ldb, C, ldc, M, ldm, tet(n));
  if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  if (n < kMinOrder) return DASTAC_OK;
  // the XCD lists: group g (orders 8g+1..8g+8) gives one slice to each XCD; 16 groups share a height P
  const int64_t gmax = (n - 1) / 8, Ptop = gmax / 16 + 1;
  const int64_t per_xcd = (gmax % 16 + 1) * blocks_of(Ptop) + 16 * tet(Ptop - 1);  // sum of blocks_of(1..Ptop-1) = Tet(Ptop-1)
  if (8 * per_xcd >= ((int64_t)1 << 31)) return DASTAC_EOVERFLOW;
  // the kernel takes up to 32 columns of the factor matrices; wider ones go block by block (each
  // block reads the packed tetrahedron once)
  for (int64_t c0 = 0; c0 < R; c0 += 32) {
    const int Rb = (int)(R - c0 < 32 ? R - c0 : 32);
    mttkrp_block_kernel<<<(unsigned)(8 * per_xcd), 64, 0, st>>>(n, Rb, Ap, B + c0, ldb, C + c0, ldc, M + c0, ldm, tet(n));
    if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  }
  return DASTAC_OK;
}
