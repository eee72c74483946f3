// MTTKRP over a packed upper tetrahedron on the matrix cores, single and double precision:
//
//   M(i,r) := A(i,j,k) * B(j,r) * C(k,r),   i<=j<=k, 0<=r<R (32 columns r per launch)     (Table 1, MTTKRP rule)
//
// Factored evaluation, contracting over the ROW index first.  Slice i of the packed tetrahedron is a
// packed upper triangle U_i of order m = n-i, so
//
//   M(i,:) = sum_k C(k,:) .* S_i(k,:)   with   S_i = U_i^T * B[i:, :]     (S_i(k,r) = sum_{j<=k} U_i(j,k) B(j,r)).
//
// Contracting over j makes k -- the index that is contiguous in the packed buffer -- the row index of
// the matrix instruction's first operand.  v_mfma_f32_32x32x2_f32 takes from lane l the element
// (row l%32, contraction index l/32), so a half-wavefront that loads 32 consecutive 16-byte pieces of
// ONE packed row already holds four operands (one per component: k = k0+4*(l%32)+s) in its registers;
// v_mfma_f64_16x16x4_f64 takes (row l%16, contraction index l/16), so there a quarter-wavefront loads
// 16 consecutive pieces of one row, two operands each (k = k0+2*(l%16)+s), and a lane takes two pieces
// 256 bytes apart.  Either way a step fetches 512 contiguous bytes of each of its packed rows (two
// rows in single, four in double precision), no element is moved through LDS, and the instruction
// stream per step is the 16-byte loads of A, the loads of B (single: lane l holds row l/32, column
// l%32; double: row l/16, columns 2*(l%16) and 2*(l%16)+1 -- the second operands) and the matrix
// instructions.  Shape<T> below holds what differs between the two.
//
// Work items.  The slice triangle is cut into blocks of 128 rows x 512 bytes of k (128 values in
// single, 64 in double precision), aligned to its lower right corner (so that only the blocks at its
// top and left edges are ragged).  A block is one wavefront's job (workgroups are single wavefronts,
// or two independent ones in double precision): it accumulates the block's part of S_i, multiplies it elementwise with C's rows k and adds the 32
// column sums into M(i,:) with floating-point atomics (the sum over blocks is a sum of partial
// results: any partition of the iteration space is correct, Section 5.2 "Parallelization").  M is
// cleared by a launch of its own first.  Rows of a block that lie wholly above the diagonal run
// without any test; where the diagonal crosses (and in the ragged blocks) the walk selects away what
// lies left of the diagonal, past the block's columns or below its rows, and aims the loads of wholly
// dead lanes at the row's first live piece, so nothing outside the block is fetched.
//
// Order.  Workgroup ids are dealt to the eight XCDs in turn, so id%8 picks the XCD and id/8 walks that
// XCD's own list: slices of nearly equal order go to the eight XCDs (alternating direction, so the
// totals agree), heaviest first, and a slice's blocks follow each other in memory order -- blocks
// that are neighbours in k, which share the cache lines cut by their common edge, run at the same
// time on the same L2.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kRows = 128;    // rows per block
constexpr int kMinOrder = 3;  // slices of order 1 and 2 (4 elements in all) are computed by the clearing launch

template <typename T>
struct Shape;

template <>
struct Shape<float> {
  static constexpr int RS = 2;     // packed rows per step (the contraction length of the matrix instruction)
  static constexpr int LPR = 32;   // lanes per row
  static constexpr int V = 4;      // elements per 16-byte piece
  static constexpr int NP = 1;     // pieces per lane and step
  static constexpr int NB = 1;     // columns r per lane
  static constexpr int NV = 16;    // result registers per matrix instruction
  static constexpr int HM = 4;     // result register v of lane group h is row KV(v) + HM*h
  static constexpr int kDepth = 8;  // steps whose loads are in flight per wavefront
  static constexpr int WPB = 1;     // wavefronts (each with a block of its own) per workgroup
  typedef f4a piece;
  typedef f4u upiece;
  typedef f16v accv;
  __device__ static constexpr int KV(int v) { return 8 * (v / 4) + v % 4; }
  __device__ static accv mma(float a, float b, accv c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }
};

template <>
struct Shape<double> {
  static constexpr int RS = 4;
  static constexpr int LPR = 16;
  static constexpr int V = 2;
  static constexpr int NP = 2;
  static constexpr int NB = 2;
  static constexpr int NV = 4;
  static constexpr int HM = 1;
  static constexpr int kDepth = 4;
  static constexpr int WPB = 2;  // the blocks are half as many bytes: launched in pairs (measured 5 % faster; in single precision 3 % slower)
  typedef d2a piece;
  typedef d2u upiece;
  typedef d4v accv;
  __device__ static constexpr int KV(int v) { return 4 * v; }
  __device__ static accv mma(double a, double b, accv c) { return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0); }
};

// k values per block, and block columns per block row height
template <typename T>
constexpr int kCols = Shape<T>::LPR * Shape<T>::V * Shape<T>::NP;
template <typename T>
constexpr int kRatio = kRows / kCols<T>;

// Pins a wave-uniform address to a scalar register pair and hides how it was computed, so that "this address
// plus a 32-bit offset per lane" stays one load with a scalar base instead of 64-bit vector arithmetic per load.
typedef const char __attribute__((address_space(1))) *global_bytes;  // a device-memory address, known as such
__device__ inline global_bytes in_scalar_registers(global_bytes p) {
  asm volatile("" : "+s"(p));
  return p;
}

// A wavefront's walk over the steps of its block.  Step t covers the rows row0 + RS*t of the lane
// groups (lane group h = lane / LPR takes row rlo + RS*t + h); the byte offset of a lane's piece grows
// from step to step by a difference that itself shrinks by RS*RS elements (a packed row is one element
// shorter than the one before).
template <typename T>
struct Walk {
  const char *As;   // the slice's packed triangle
  unsigned e0;      // byte offset of this lane's first piece at step 0
  int delta0;       // growth of that offset from step 0 to step 1
  const T *b0;      // this lane's first element of B at step 0 (row of lane group 0 when masked)
  int bnext;        // distance to its second element of B (NB == 2), in elements
  int64_t bstep;    // RS rows of B, in elements
  int begin, end;   // first step; one past the last step
  // masked walk only
  int64_t bhalf;    // lane group times one row of B, in elements
  int dd0;          // this lane's row minus the first k of its first piece, at step 0
  int row0, rhi;    // this lane's row at step 0; one past the block's last row
  int kspan;        // the block's last k + 1 minus the first k of this lane's first piece
  unsigned emax;    // largest byte offset whose 16-byte piece ends inside the packed buffer
};

// Where the walk stands: the state that moves from one request to the next.
template <typename T>
struct Cursor {
  unsigned e;
  int delta;
  const T *bp;
  int t;
};

template <typename T>
__device__ inline Cursor<T> cursor_at(const Walk<T> &w, int t) {
  constexpr int kSecond = (int)sizeof(T) * Shape<T>::RS * Shape<T>::RS;  // second difference of the offset, bytes
  Cursor<T> c;
  c.e = w.e0 + (unsigned)(t * w.delta0 - (kSecond / 2) * t * (t - 1));
  c.delta = w.delta0 - kSecond * t;
  c.bp = w.b0 + t * w.bstep;
  c.t = t;
  return c;
}

// What one step keeps in registers between its request and its matrix instructions.
template <typename T>
struct Loaded {
  typename Shape<T>::piece a[Shape<T>::NP];
  T b[Shape<T>::NB];
};

// Requests step c.t: NP 16-byte pieces of A and NB elements of B per lane.
template <typename T, bool MASKED>
__device__ inline void request(const Walk<T> &w, const Cursor<T> &c, Loaded<T> &ld) {
  typedef Shape<T> S;
  typedef typename S::upiece upiece;
  constexpr int kPieceBytes = S::LPR * 16;  // from a lane's piece to its next one
  const T *bp = c.bp;
  if (MASKED) {
    // wholly dead lanes (every k left of the diagonal) re-aim at the piece that holds the diagonal
    const int dd = w.dd0 + S::RS * c.t;
#pragma unroll
    for (int p = 0; p < S::NP; ++p) {
      const int ddp = dd - p * S::LPR * S::V;
      unsigned e = c.e + (unsigned)(p * kPieceBytes) + (unsigned)(((ddp > 0 ? ddp : 0) & ~(S::V - 1)) * (int)sizeof(T));
      e = e < w.emax ? e : w.emax;
      ld.a[p] = *reinterpret_cast<const upiece *>(w.As + e);
    }
    const bool row_ok = w.row0 + S::RS * c.t < w.rhi;  // a dead row takes lane group 0's row of B
    bp += row_ok ? w.bhalf : (int64_t)0;
  } else {
#pragma unroll
    for (int p = 0; p < S::NP; ++p) ld.a[p] = *reinterpret_cast<const upiece *>(w.As + c.e + (unsigned)(p * kPieceBytes));
  }
  ld.b[0] = bp[0];
  if (S::NB == 2) ld.b[S::NB - 1] = bp[w.bnext];
}

template <typename T>
__device__ inline void advance(const Walk<T> &w, Cursor<T> &c) {
  c.e += (unsigned)c.delta;
  c.delta -= (int)sizeof(T) * Shape<T>::RS * Shape<T>::RS;
  c.bp += w.bstep;
  ++c.t;
}

// Accumulator (p*V + s)*NB + c holds piece p, component s, column group c.
template <typename T>
struct Acc {
  typename Shape<T>::accv v[Shape<T>::NP * Shape<T>::V * Shape<T>::NB];
};

template <typename T, bool MASKED>
__device__ inline void multiply(const Walk<T> &w, int t, Loaded<T> ld, Acc<T> &acc) {
  typedef Shape<T> S;
  if (MASKED) {
    const int lo0 = w.dd0 + S::RS * t;  // components below lo are left of the diagonal
    const bool row_ok = w.row0 + S::RS * t < w.rhi;
#pragma unroll
    for (int p = 0; p < S::NP; ++p) {
      const int lo = lo0 - p * S::LPR * S::V;
      const int hi = row_ok ? w.kspan - p * S::LPR * S::V : lo;  // components from hi on are outside the block
      const unsigned span = hi > lo ? (unsigned)(hi - lo) : 0u;
#pragma unroll
      for (int s = 0; s < S::V; ++s) ld.a[p][s] = ((unsigned)(s - lo) < span) ? ld.a[p][s] : T(0);
    }
  }
#pragma unroll
  for (int p = 0; p < S::NP; ++p)
#pragma unroll
    for (int s = 0; s < S::V; ++s)
#pragma unroll
      for (int c = 0; c < S::NB; ++c) {
        auto &a = acc.v[(p * S::V + s) * S::NB + c];
        a = S::mma(ld.a[p][s], ld.b[c], a);
      }
}

// Steps w.begin .. w.end-1 with the loads of kDepth steps in flight.  The main loop has no control
// flow around its loads, so the compiler keeps exact counts of what is outstanding.
template <typename T, bool MASKED>
__device__ inline void sweep(const Walk<T> &w, Acc<T> &acc) {
  constexpr int kDepth = Shape<T>::kDepth;
  if (w.begin >= w.end) return;
  Loaded<T> ld[kDepth];
  int t = w.begin;
#pragma unroll
  for (int d = 0; d < kDepth; ++d) {  // a block with fewer steps repeats its last one; never multiplied
    const int td = t + d < w.end ? t + d : w.end - 1;
    request<T, MASKED>(w, cursor_at(w, td), ld[d]);
  }
  Cursor<T> c = cursor_at(w, t + kDepth);
  while (t + 2 * kDepth <= w.end) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      multiply<T, MASKED>(w, t + d, ld[d], acc);
      request<T, MASKED>(w, c, ld[d]);
      advance(w, c);
      __builtin_amdgcn_sched_barrier(0);  // keep each request where its registers come free, not at the loop's end
    }
    t += kDepth;
  }
  // fewer than 2*kDepth steps are left; those from t+kDepth on are still to be requested
#pragma unroll
  for (int d = 0; d < kDepth; ++d) {
    if (t + d < w.end) multiply<T, MASKED>(w, t + d, ld[d], acc);
    if (t + d + kDepth < w.end) request<T, MASKED>(w, cursor_at(w, t + d + kDepth), ld[d]);
  }
  t += kDepth;
#pragma unroll
  for (int d = 0; d < kDepth; ++d)
    if (t + d < w.end) multiply<T, MASKED>(w, t + d, ld[d], acc);
}

// Number of blocks of a slice whose triangle is P block rows high: block row a (from the bottom) has
// ratio*(a+1) block columns that reach the diagonal or lie right of it.
__host__ __device__ inline int64_t blocks_of(int64_t P, int ratio) { return ratio * P * (P + 1) / 2; }

template <typename T>
__global__ __launch_bounds__(64 * Shape<T>::WPB) __attribute__((amdgpu_waves_per_eu(2, 2))) void mttkrp_block_kernel(
    int64_t n, int R, const T *__restrict__ A, const T *__restrict__ Bm, int64_t ldb, const T *__restrict__ Cm,
    int64_t ldc, T *__restrict__ M, int64_t ldm, int64_t total) {
  typedef Shape<T> S;
  constexpr int kC = kCols<T>, kRK = kRatio<T>, kSz = (int)sizeof(T);
  const int lane = threadIdx.x & 63, lr = lane % S::LPR, h = lane / S::LPR;

  // ---- which block: id%8 = XCD, id/8 = position in that XCD's list (slices by descending order m,
  // groups of eight consecutive orders dealt to the XCDs in alternating direction)
  const int x = (int)(blockIdx.x & 7u);
  unsigned seq = (blockIdx.x >> 3) * (unsigned)S::WPB + (unsigned)uniform32((int)(threadIdx.x >> 6));
  const int gmax = (int)((n - 1) >> 3);  // group g holds the orders 8g+1 .. 8g+8, all ceil(m/128) = g/16+1 block rows high
  int P = gmax / 16 + 1;
  unsigned cnt = (unsigned)(gmax % 16 + 1);
  unsigned per = (unsigned)blocks_of(P, kRK);
  while (P > 1 && seq >= cnt * per) {
    seq -= cnt * per;
    --P;
    cnt = 16;
    per = (unsigned)blocks_of(P, kRK);
  }
  if (seq >= cnt * per) return;  // past the end of the list (the grid is rounded up to whole workgroups)
  const unsigned s = (unsigned)uniform32((int)(seq / per));
  const int g = 16 * (P - 1) + (int)(cnt - 1 - s);
  const int m = 8 * g + 1 + ((g & 1) ? 7 - x : x);  // order of the slice
  if (m > n || m < kMinOrder) return;
  const int tq = (int)(per - 1 - (seq - s * per));  // blocks in memory order: top block row first
  int a = 0;
  while (kRK * (a + 1) * (a + 2) / 2 <= tq) ++a;
  const int p = tq - kRK * a * (a + 1) / 2;  // block row a (from the bottom), block column p (from the right), p < ratio*(a+1)
  if (kC * p >= m) return;                   // the top block row of a narrow slice has fewer block columns

  const int64_t i = n - m;
  const int64_t slice0 = tet_slice_start(n, i);
  const int rhi = m - kRows * a, rlo = rhi > kRows ? rhi - kRows : 0;  // rows [rlo, rhi) of the slice triangle
  const int khi = m - kC * p;                                         // k values [klo, khi)
  const int klo = khi > kC ? khi - kC : 0;  // (the leftmost block is shifted right to start at 0)
  // rows [rlo, rfull) lie wholly above the diagonal and span the full width; rows from rdead on are all left of it
  const int rdead = rhi < khi ? rhi : khi;
  const int rfull = khi - klo == kC ? (klo < rdead ? (klo > rlo ? klo : rlo) : rdead) : rlo;

  const int kk0 = klo + S::V * lr;  // first k of this lane's first piece
  const int row0 = rlo + h;
  int cc[S::NB];  // this lane's columns; lanes past the last column repeat it, their sums are dropped
#pragma unroll
  for (int c = 0; c < S::NB; ++c) cc[c] = S::NB * lr + c < R ? S::NB * lr + c : R - 1;

  Walk<T> w;
  w.As = reinterpret_cast<const char *>(A + slice0);
  // element (row, k) of the slice triangle is at row*m - row(row+1)/2 + k
  w.e0 = (unsigned)kSz * (unsigned)(row0 * m - row0 * (row0 + 1) / 2 + kk0);
  w.delta0 = kSz * (S::RS * m - S::RS * row0 - S::RS * (S::RS + 1) / 2);
  w.bstep = S::RS * ldb;
  w.bhalf = h * ldb;
  w.bnext = cc[S::NB - 1] - cc[0];
  w.dd0 = row0 - kk0;
  w.row0 = row0;
  w.rhi = rhi;
  w.kspan = khi - kk0;
  {
    const int64_t room = total - S::V - slice0;  // in elements; >= 0 for m >= 3
    constexpr int64_t kMost = 0xfffffff0 / kSz;
    w.emax = (unsigned)kSz * (unsigned)(room < kMost ? room : kMost);
  }

  Acc<T> acc;
#pragma unroll
  for (int q = 0; q < S::NP * S::V * S::NB; ++q)
#pragma unroll
    for (int v = 0; v < S::NV; ++v) acc.v[q][v] = T(0);

  const T *b0 = Bm + (i + rlo) * ldb + cc[0];  // row of lane group 0 at step 0
  // whole steps of full rows without any test, the rest (a last partial step, the rows the diagonal
  // crosses) through the masked walk
  const int nfull = (rfull - rlo) / S::RS;
  w.b0 = b0 + w.bhalf;
  w.begin = 0;
  w.end = nfull;
  sweep<T, false>(w, acc);
  w.b0 = b0;
  w.begin = nfull;
  w.end = (rdead - rlo + S::RS - 1) / S::RS;
  sweep<T, true>(w, acc);

  // ---- fold with C: register v of accumulator (p*V+s)*NB+c in lane group h is S(k, column c of the lane) with
  // k = klo + LPR*V*p + V*(KV(v) + HM*h) + s
  T part[S::NB];
#pragma unroll
  for (int c = 0; c < S::NB; ++c) part[c] = T(0);
  constexpr int kLaneRows = S::V * S::HM * (64 / S::LPR - 1);  // largest row offset that depends on the lane
  if (m >= kC && ldc <= (int64_t)0x7fffffff / (kLaneRows * kSz + kSz)) {
    // Rows klo .. klo+kC-1 of C all belong to the slice (in the narrow leftmost block the sums of the k values
    // past its last are exact zeros, and those rows exist).  Every address is a wave-uniform row base plus a
    // 32-bit offset that depends on the lane only: one load and one multiply-add per element, nothing else.
    const global_bytes rows = (global_bytes) reinterpret_cast<const char *>(Cm + (i + klo) * ldc);
    unsigned lane_off[S::NB];
#pragma unroll
    for (int c = 0; c < S::NB; ++c) lane_off[c] = (unsigned)kSz * ((unsigned)(S::V * S::HM * h) * (unsigned)ldc + (unsigned)cc[c]);
#pragma unroll
    for (int v = 0; v < S::NV; ++v)
#pragma unroll
      for (int q = 0; q < S::NP * S::V; ++q)
#pragma unroll
        for (int c = 0; c < S::NB; ++c) {
          const int off = S::LPR * S::V * (q / S::V) + S::V * S::KV(v) + q % S::V;
          const global_bytes row = in_scalar_registers(rows + (int64_t)off * ldc * kSz);
          const T cv = *(const T __attribute__((address_space(1))) *)(row + lane_off[c]);
          part[c] += acc.v[q * S::NB + c][v] * cv;
        }
  } else {  // a slice smaller than one block (or a row stride beyond 32-bit offsets): every row tested
    const T *cp[S::NB];
#pragma unroll
    for (int c = 0; c < S::NB; ++c) cp[c] = Cm + (i + klo + S::V * S::HM * h) * ldc + cc[c];
    const int live = khi - klo - S::V * S::HM * h;  // k offsets below this exist
#pragma unroll
    for (int v = 0; v < S::NV; ++v)
#pragma unroll
      for (int q = 0; q < S::NP * S::V; ++q)
#pragma unroll
        for (int c = 0; c < S::NB; ++c) {
          const int off = S::LPR * S::V * (q / S::V) + S::V * S::KV(v) + q % S::V;
          const bool ok = off < live;
          const T cv = cp[c][ok ? (int64_t)off * ldc : (int64_t)0 - S::V * S::HM * h * ldc];
          part[c] += ok ? acc.v[q * S::NB + c][v] * cv : T(0);
        }
  }
#pragma unroll
  for (int c = 0; c < S::NB; ++c) {
#pragma unroll
    for (int d = S::LPR; d < 64; d *= 2) part[c] += __shfl_xor(part[c], d, 64);
    if (h == 0 && S::NB * lr + c < R) unsafeAtomicAdd(&M[i * ldm + S::NB * lr + c], part[c]);
  }
}

// Clears M (the block kernel adds into it) and computes the slices of order 1 and 2 -- the last four
// elements of the packed buffer, where a 16-byte load has no room -- directly from the rule.
template <typename T>
__global__ __launch_bounds__(256) void mttkrp_clear_kernel(int64_t n, int64_t R, const T *__restrict__ A,
                                                           const T *__restrict__ Bm, int64_t ldb,
                                                           const T *__restrict__ Cm, int64_t ldc, T *__restrict__ M,
                                                           int64_t ldm) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;  // one output element per thread
  if (e >= n * R) return;
  const int64_t i = e / R, r = e - i * R;
  T s = T(0);
  if (n - i < kMinOrder) {
    int64_t pos = tet_slice_start(n, i);
    for (int64_t j = i; j < n; ++j)
      for (int64_t k = j; k < n; ++k) s += A[pos++] * Bm[j * ldb + r] * Cm[k * ldc + r];
  }
  M[i * ldm + r] = s;
}

template <typename T>
int run(int64_t n, int64_t R, const T *Ap, const T *B, int64_t ldb, const T *C, int64_t ldc, T *M, int64_t ldm,
        void *stream) {
  constexpr int64_t kSz = (int64_t)sizeof(T);
  if (n < 0 || R < 1 || R > (1 << 20) || ldb < R || ldc < R || ldm < R) return DASTAC_EINVAL;
  if (n > DASTAC_TET_MAX_N || tet(n) > ((int64_t)1 << 40) || ld_too_large(ldb, ldc, ldm))
    return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Ap || !B || !C || !M) return DASTAC_ENULL;
  const int64_t mb = view_bytes(n, ldm, R, kSz);
  if (overlaps(M, mb, Ap, tet(n) * kSz) || overlaps(M, mb, B, view_bytes(n, ldb, R, kSz)) ||
      overlaps(M, mb, C, view_bytes(n, ldc, R, kSz)))
    return DASTAC_EALIAS;
  hipStream_t st = (hipStream_t)stream;
  mttkrp_clear_kernel<T><<<(unsigned)ceil_div(n * R, 256), 256, 0, st>>>(n, R, Ap, B, ldb, C, ldc, M, ldm);
  if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  if (n < kMinOrder) return DASTAC_OK;
  // the XCD lists: group g (orders 8g+1..8g+8) gives one slice to each XCD; 16 groups share a height P
  const int64_t gmax = (n - 1) / 8, Ptop = gmax / 16 + 1;
  // sum of P(P+1)/2 over P = 1..Ptop-1 is Tet(Ptop-1)
  const int64_t per_xcd = (gmax % 16 + 1) * blocks_of(Ptop, kRatio<T>) + 16 * kRatio<T> * tet(Ptop - 1);
  if (8 * per_xcd >= ((int64_t)1 << 31)) return DASTAC_EOVERFLOW;
  // the kernel takes up to 32 columns of the factor matrices; wider ones go block by block (each
  // block reads the packed tetrahedron once)
  for (int64_t c0 = 0; c0 < R; c0 += 32) {
    const int Rb = (int)(R - c0 < 32 ? R - c0 : 32);
    mttkrp_block_kernel<T><<<(unsigned)(8 * ceil_div(per_xcd, Shape<T>::WPB)), 64 * Shape<T>::WPB, 0, st>>>(n, Rb, Ap, B + c0, ldb, C + c0, ldc, M + c0, ldm, tet(n));
    if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  }
  return DASTAC_OK;
}

}  // namespace

extern "C" {

int dastac_tet_mttkrp_f32(int64_t n, int64_t R, const float *Ap, const float *B, int64_t ldb, const float *C,
                          int64_t ldc, float *M, int64_t ldm, void *stream) {
  return run<float>(n, R, Ap, B, ldb, C, ldc, M, ldm, stream);
}

int dastac_tet_mttkrp_f64(int64_t n, int64_t R, const double *Ap, const double *B, int64_t ldb, const double *C,
                          int64_t ldc, double *M, int64_t ldm, void *stream) {
  return run<double>(n, R, Ap, B, ldb, C, ldc, M, ldm, stream);
}

}  // extern "C"
