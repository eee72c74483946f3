// Matrix-vector products over one packed triangle, in every reading the layout allows:
//
//   MODE_ROWS   y := T x           the triangular product itself (lower triangle; the upper one has
//                                  its own kernel next to TTV)
//   MODE_COLS   y := T^T x         the transposed product
//   MODE_SYM    y := S x           S symmetric, T its unique half (Section 3, "Redundancy map": the
//                                  unique set is one triangle, every other element is reached by
//                                  swapping its two indices)
//
// for T packed row by row as an upper triangle (row i holds columns i..n-1, Table 2 SpMV_UT) or as
// a lower triangle (row i holds columns 0..i: the worked example of Section 4, whose polynomial
// i/2 + i^2/2 + j is the row base used here).  The packed buffer is read once; an element U(i,j)
// gives U x(j) to the row sum of i and U x(i) to the column sum of j from the same registers.
//
// Work split.  A lane's load is one 16-byte piece: P = 4 single-precision or 2 double-precision
// elements.  The triangle is cut into column panels of kW = 64*P*NQ columns, and the rows that
// reach a panel into chunks of R consecutive rows; a wavefront owns one (panel, chunk) pair, and the
// four wavefronts of a workgroup own four consecutive chunks of one panel.  Lane l is tied to the same
// P*NQ columns of the panel for the whole chunk (columns c0+P*l+64*P*q .. +P-1), so
//   * the x values of its columns sit in registers (no LDS, no per-row lookup),
//   * the column sums  sum_i T(i,c) x(i)  accumulate in registers; at the end the four wavefronts add
//     theirs up through LDS and the workgroup issues ONE atomic add per column (atomics on one
//     cache line serialise in L2: flushing per wavefront made them the whole run time),
//   * the row sum  sum_c T(i,c) x(c)  is one multiply-add per element and one DPP reduction per
//     row; row sums are parked one per lane and flushed 64 rows at a time,
// all with floating-point atomic adds into an output that is zeroed first (several panels add
// into one row, several workgroups into one column).  A row's piece of a panel is contiguous in the
// packed buffer and starts at row_base(i) + c0, where row_base is the index polynomial of the row
// minus its first column; every load is "scalar row base + fixed lane offset".  Rows that cross a
// panel completely need no masks; inside the panel's diagonal block the elements on the wrong side
// of the diagonal (which belong to a neighbouring row, still inside the buffer) and, in the last
// panel, columns past n-1 are zeroed in registers, and for MODE_SYM the diagonal element is kept
// out of the column sums (it is used once).
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / 64;
constexpr int kMaxPanels = 512;
constexpr int kMaxN = 524288;  // 512 panels of 1024 columns; such a triangle is far larger than device memory

enum { MODE_ROWS = 0, MODE_COLS = 1, MODE_SYM = 2 };


// Per element type: elements in a 16-byte piece, and the piece as a register vector and as a
// load type that only promises the element's own alignment.
template <typename T>
struct Piece;
template <>
struct Piece<float> {
  static constexpr int kPer = 4;
  typedef f4a vec;
  typedef f4u uvec;
};
template <>
struct Piece<double> {
  static constexpr int kPer = 2;
  typedef d2a vec;
  typedef d2u uvec;
};

template <int CTRL>
__device__ inline float dpp_add(float v) {
  int t = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false);
  return v + __builtin_bit_cast(float, t);
}
template <int CTRL>
__device__ inline double dpp_add(double v) {  // the two halves of a double travel separately
  const uint64_t b = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, 0xf, 0xf, false);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, 0xf, 0xf, false);
  return v + __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
// sum over the 64 lanes; every lane receives the total
template <typename T>
__device__ inline T wave_sum(T v) {
  v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
  v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
  v = dpp_add<0x141>(v);  // row_half_mirror
  v = dpp_add<0x140>(v);  // row_mirror
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}

struct Panels {  // first workgroup of every panel (and one past the last)
  int first[kMaxPanels + 1];
};

// rows that reach panel [c0, c0+kW): upper 0 .. min(n, c0+kW)-1, lower c0 .. n-1
template <bool LOWER>
DASTAC_HD void panel_rows(int64_t n, int64_t c0, int64_t kW, int64_t &lo, int64_t &hi) {
  if (LOWER) {
    lo = c0;
    hi = n;
  } else {
    lo = 0;
    hi = c0 + kW < n ? c0 + kW : n;
  }
}

template <typename E, int NQ, bool LOWER, int MODE>
__global__ __launch_bounds__(kBlock) void trimv_kernel(int n, const E *__restrict__ T,
                                                       const E *__restrict__ x, E *__restrict__ y,
                                                       int R, int npanels, Panels pn) {
  constexpr int P = Piece<E>::kPer;
  typedef typename Piece<E>::vec vec;
  typedef typename Piece<E>::uvec uvec;
  constexpr int kW = 64 * P * NQ;
  constexpr bool ROWS = MODE != MODE_COLS, COLS = MODE != MODE_ROWS;
  __shared__ E cs[kWavesPerBlock][kW];  // the wavefronts' column sums
  const int lane = threadIdx.x & 63, wave = uniform32(threadIdx.x >> 6);
  int p = 0;
  while ((int)blockIdx.x >= pn.first[p + 1]) ++p;  // wave-uniform, at most kMaxPanels steps
  const int c0 = p * kW;  // first column of the panel
  int64_t rlo, rhi;
  panel_rows<LOWER>(n, c0, kW, rlo, rhi);
  const int r0 = (int)rlo + ((int)blockIdx.x - pn.first[p]) * (kWavesPerBlock * R) + wave * R;
  const int r1 = r0 + R < (int)rhi ? r0 + R : (int)rhi;
  const bool active = r0 < (int)rhi;  // the panel's last workgroup may be short
  const bool panel_full = c0 + kW <= n;  // every column of the panel exists

  // this lane's columns, their x values, and the load offsets (columns past n-1 are re-aimed at a
  // column every row has -- n-1 in an upper triangle, 0 in a lower one -- and masked)
  int col[NQ];
  unsigned voff[NQ];
  vec xv[NQ], acc[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    col[q] = c0 + P * lane + 64 * P * q;
    voff[q] = (unsigned)sizeof(E) * (unsigned)(col[q] < n ? col[q] : LOWER ? 0 : n - 1);
#pragma unroll
    for (int t = 0; t < P; ++t) {
      xv[q][t] = col[q] + t < n ? x[col[q] + t] : E(0);
      acc[q][t] = E(0);
    }
  }

  struct Row {
    vec a[NQ];
    E xi;
  };
  // element (i,c) of the triangle is at T[row_base(i) + c]
  auto row_base = [&](int i) -> int64_t {
    return LOWER ? ((int64_t)i * (i + 1)) / 2 : tri_row_start((int64_t)n, (int64_t)i) - i;
  };
  // A 16-byte load may start on the last elements of a row and run up to P-1 <= 3 elements past its
  // end, into the next rows.  Only the last two rows of the buffer can have fewer than three elements
  // behind them: they take bounds-tested scalar loads.
  auto load_row = [&](int i, Row &r) {
    const int ii = i < r1 ? i : r1 - 1;  // past the end of the chunk: a repeat that is never used
    const char *base = reinterpret_cast<const char *>(T + row_base(ii));
    r.xi = x[ii];
    if (ii + 2 < n) {
#pragma unroll
      for (int q = 0; q < NQ; ++q) r.a[q] = *reinterpret_cast<const uvec *>(base + voff[q]);
    } else {
      const E *rp = T + row_base(ii);
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
#pragma unroll
        for (int t = 0; t < P; ++t) {
          const int c = col[q] + t;
          r.a[q][t] = (LOWER ? c <= ii : (c >= ii && c < n)) ? rp[c] : E(0);
        }
      }
    }
  };

  E rowacc = E(0);  // lane (i - r0) % 64 parks the sum of row i
  auto flush_rows = [&](int first, int count) {
    if (lane < count) unsafeAtomicAdd(&y[first + lane], rowacc);
    rowacc = E(0);
  };
  auto consume = [&](int i, Row &r) {
    vec ac[NQ];  // what enters the column sums
    const bool crosses = LOWER ? i >= c0 + kW : (panel_full && i < c0);
    if (crosses) {  // the row crosses the whole panel: every element exists, none is diagonal
#pragma unroll
      for (int q = 0; q < NQ; ++q) ac[q] = r.a[q];
    } else {  // diagonal block or last panel: zero what lies outside the triangle
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        const int dg = i - col[q];                        // element dg is the diagonal one
        const int lo = LOWER ? -0x40000000 : dg;          // first element inside
        const int hi = LOWER ? dg + 1 : n - col[q];       // one past the last element inside
#pragma unroll
        for (int t = 0; t < P; ++t) r.a[q][t] = (t >= lo && t < hi) ? r.a[q][t] : E(0);
        if (MODE == MODE_SYM) {  // the diagonal element is used once: the row sum has it
#pragma unroll
          for (int t = 0; t < P; ++t) ac[q][t] = dg == t ? E(0) : r.a[q][t];
        } else {
          ac[q] = r.a[q];
        }
      }
    }
    if (COLS) {
#pragma unroll
      for (int q = 0; q < NQ; ++q) acc[q] += ac[q] * r.xi;
    }
    if (ROWS) {
      E rs = E(0);
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
#pragma unroll
        for (int t = 0; t < P; ++t) rs += r.a[q][t] * xv[q][t];
      }
      rs = wave_sum(rs);
      const int slot = (i - r0) & 63;
      if (lane == slot) rowacc = rs;
      if (slot == 63) flush_rows(i - 63, 64);
    }
  };

  // Two register sets alternate; the loop leaves only at its bottom and every load is issued
  // unconditionally, so the next row's loads are in flight while the current row is summed.
  if (active) {
    Row ra, rb;
    load_row(r0, ra);
    int i = r0;
    do {
      load_row(i + 1, rb);
      consume(i, ra);
      load_row(i + 2, ra);
      if (i + 1 < r1) consume(i + 1, rb);
      i += 2;
    } while (i < r1);
    const int left = (r1 - r0) & 63;
    if (ROWS && left) flush_rows(r1 - left, left);
  }

  if (COLS) {  // column sums: add the wavefronts' up, then one atomic per column
#pragma unroll
    for (int q = 0; q < NQ; ++q) *reinterpret_cast<vec *>(&cs[wave][P * lane + 64 * P * q]) = acc[q];
    __syncthreads();
    for (int c = threadIdx.x; c < kW; c += kBlock) {
      E v = E(0);
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) v += cs[w][c];
      if (c0 + c < n && v != E(0)) unsafeAtomicAdd(&y[c0 + c], v);
    }
  }
}

template <typename E>
__global__ void zero_kernel(E *__restrict__ y, int64_t n) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n) y[t] = E(0);
}

template <typename E, int NQ, bool LOWER, int MODE>
int launch(int64_t n, const E *Tp, const E *x, E *y, hipStream_t st) {
  constexpr int kW = 64 * Piece<E>::kPer * NQ;
  const int npanels = (int)ceil_div(n, kW);
  if (npanels > kMaxPanels) return DASTAC_EOVERFLOW;
  int64_t steps = 0, lo, hi;
  for (int p = 0; p < npanels; ++p) {
    panel_rows<LOWER>(n, (int64_t)p * kW, kW, lo, hi);
    steps += hi - lo;
  }
  // One round of resident workgroups: as many as the device holds at once (occupancy x compute units,
  // asked of the runtime once per device), never more -- a grid a little larger than that leaves most of
  // the chip idle while the stragglers of a second round run (measured for the symmetric product at
  // n=8192, where three workgroups fit a compute unit: 768 workgroups 34 us, 1024 38 us, 2048 46 us).
  // At least 4 rows per wavefront.  Workgroups of 256 threads: 512 measured 42 us, 1024 67 us.
  const int64_t slots = resident_blocks(trimv_kernel<E, NQ, LOWER, MODE>, kBlock);
  if (slots <= 0) return DASTAC_EHIP;
  int64_t R = ceil_div(steps, slots * kWavesPerBlock);
  if (R < 4) R = 4;
  Panels pn;
  int blocks;
  for (;; ++R) {  // the per-panel round-up can push the count past the slots: a few more rows each
    blocks = 0;
    for (int p = 0; p < npanels; ++p) {
      pn.first[p] = blocks;
      panel_rows<LOWER>(n, (int64_t)p * kW, kW, lo, hi);
      blocks += (int)ceil_div(hi - lo, R * kWavesPerBlock);
    }
    if (blocks <= slots || R >= n) break;
  }
  pn.first[npanels] = blocks;
  zero_kernel<E><<<(unsigned)ceil_div(n, 256), 256, 0, st>>>(y, n);
  trimv_kernel<E, NQ, LOWER, MODE><<<(unsigned)blocks, kBlock, 0, st>>>((int)n, Tp, x, y, (int)R, npanels, pn);
  return launch_status();
}

template <typename E, bool LOWER, int MODE>
int run(int64_t n, const E *Tp, const E *x, E *y, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(E);
  if (n < 0) return DASTAC_EINVAL;
  // 512 panels of the widest kind; double-precision panels are half as wide
  if (n > kMaxN / (kB / 4)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Tp || !x || !y) return DASTAC_ENULL;
  if (overlaps(y, n * kB, Tp, tri(n) * kB) || overlaps(y, n * kB, x, n * kB)) return DASTAC_EALIAS;
  if (n <= 2048) return launch<E, 1, LOWER, MODE>(n, Tp, x, y, (hipStream_t)stream);
  return launch<E, 4, LOWER, MODE>(n, Tp, x, y, (hipStream_t)stream);
}

}  // namespace

// y := U x over the packed upper triangle with this file's kernel (no limit on n below kMaxN);
// used by dastac_trmv_f32 for triangles whose vector does not fit in LDS.
int dastac::trmv_upper_by_panels(int64_t n, const float *Up, const float *x, float *y, void *stream) {
  return run<float, false, MODE_ROWS>(n, Up, x, y, stream);
}
int dastac::trmv_upper_by_panels(int64_t n, const double *Up, const double *x, double *y, void *stream) {
  return run<double, false, MODE_ROWS>(n, Up, x, y, stream);
}

extern "C" {

int dastac_symv_f32(int64_t n, const float *Up, const float *x, float *y, void *stream) {
  return run<float, false, MODE_SYM>(n, Up, x, y, stream);
}
int dastac_trmv_t_f32(int64_t n, const float *Up, const float *x, float *y, void *stream) {
  return run<float, false, MODE_COLS>(n, Up, x, y, stream);
}
int dastac_symv_lower_f32(int64_t n, const float *Lp, const float *x, float *y, void *stream) {
  return run<float, true, MODE_SYM>(n, Lp, x, y, stream);
}
int dastac_trmv_lower_f32(int64_t n, const float *Lp, const float *x, float *y, void *stream) {
  return run<float, true, MODE_ROWS>(n, Lp, x, y, stream);
}
int dastac_trmv_lower_t_f32(int64_t n, const float *Lp, const float *x, float *y, void *stream) {
  return run<float, true, MODE_COLS>(n, Lp, x, y, stream);
}

int dastac_symv_f64(int64_t n, const double *Up, const double *x, double *y, void *stream) {
  return run<double, false, MODE_SYM>(n, Up, x, y, stream);
}
int dastac_trmv_t_f64(int64_t n, const double *Up, const double *x, double *y, void *stream) {
  return run<double, false, MODE_COLS>(n, Up, x, y, stream);
}
int dastac_symv_lower_f64(int64_t n, const double *Lp, const double *x, double *y, void *stream) {
  return run<double, true, MODE_SYM>(n, Lp, x, y, stream);
}
int dastac_trmv_lower_f64(int64_t n, const double *Lp, const double *x, double *y, void *stream) {
  return run<double, true, MODE_ROWS>(n, Lp, x, y, stream);
}
int dastac_trmv_lower_t_f64(int64_t n, const double *Lp, const double *x, double *y, void *stream) {
  return run<double, true, MODE_COLS>(n, Lp, x, y, stream);
}

}  // extern "C"
