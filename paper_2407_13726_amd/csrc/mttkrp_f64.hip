// MTTKRP over a packed upper tetrahedron in double precision, on the fp64 matrix cores:
//
//   M(i,r) := A(i,j,k) * B(j,r) * C(k,r),   i<=j<=k, 0<=r<R (32 columns r per launch),   all double     (Table 1, MTTKRP rule)
//
// The plan is the fp32 kernel's.  Slice i of the packed tetrahedron is a packed upper triangle U_i of
// order n-i, so  M(i,:) = sum_j B(j,:) .* T_i(j,:)  with  T_i = U_i * C[i:, :]  -- a TRMM whose result is
// consumed at once and never leaves the registers; A is read exactly once.  One workgroup (8 wavefronts)
// per slice, heaviest slices first, walks k in panels of 256 with the panel's rows of C staged in LDS;
// inside a panel the work items are 32-row blocks of the slice, drawn from an LDS counter.  A wavefront
// streams its 32 packed rows in tiles of 32 rows x 16 values of k (the same 128 contiguous bytes per row
// and 16-byte pieces as in fp32): registers -> private LDS tile -> operands of v_mfma_f64_16x16x4_f64,
// where lane l supplies row (or column) l%16 at k = l/16 of each group of four.  The 32x32 block of T is
// 2x2 tiles of 16x16 with four independent accumulators; it is then multiplied elementwise by B's rows,
// which were requested when the block began, and folded into running sums.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kWaves = 8;
constexpr int kBlock = kWaves * 64;
constexpr int kPanel = 256;  // k values per staged panel of C (64 KB of doubles)
constexpr int kTK = 16;      // k values per tile
constexpr int kTP = kTK + 2;  // pitch (doubles) of a wavefront's private 32 x 16 tile

typedef double d2u __attribute__((ext_vector_type(2), aligned(8)));
typedef double d2a __attribute__((ext_vector_type(2)));
typedef double d4v __attribute__((ext_vector_type(4)));

// Orders LDS traffic between the lanes of ONE wavefront (which executes in lockstep): earlier LDS
// writes are visible to later reads of any lane, and the compiler may not move LDS accesses across.
__device__ inline void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(2, 2))) void mttkrp_f64_kernel(
    int64_t n, int R, const double *__restrict__ A, const double *__restrict__ Bm, int64_t ldb,
    const double *__restrict__ Cm, int64_t ldc, double *__restrict__ M, int64_t ldm, int64_t total) {
  // [k][r]; one tile of zero rows follows the panel: the last tile of a row block may reach past the panel's
  // last row (there its elements of A are masked to zero, and must not meet anything but zeros)
  __shared__ __attribute__((aligned(16))) double Cs[(kPanel + kTK) * 32];
  __shared__ __attribute__((aligned(16))) double At[kWaves][32 * kTP];
  __shared__ double Mred[kWaves][32];
  __shared__ int next_unit;

  const int64_t i = blockIdx.x;
  const int64_t m = n - i;  // order of this slice
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, l4 = lane >> 4;
  const int nblk = (int)ceil_div(m, 32);
  const int npanels = (int)ceil_div(m, kPanel);
  const int64_t slice0 = tet_slice_start(n, i);  // packed position of (i,i,i)
  // a 16-byte load may start up to 15 elements past the end of its row: safe unless the slice is one of
  // the last few of the buffer
  const bool vec_ok = slice0 + tri(m) + kTK <= total;
  const double *__restrict__ As = A + slice0;  // this slice's packed triangle
  const int mi = (int)m;

  // loader role inside a tile: rows lr, lr+8, lr+16, lr+24; two k values from lk
  const int lr = lane >> 3, lk = (lane & 7) * 2;
  double *tile = At[wave];

  double macc[2] = {0.0, 0.0};  // this lane's share of M(i, l16) and M(i, 16 + l16)

  for (int c = 0; c < npanels; ++c) {
    const int64_t kp0 = i + (int64_t)c * kPanel;
    __syncthreads();  // every wavefront is done with the previous panel
    // Stage the panel's rows of C, [k][r] with 32 columns (zeros from column R on and from row n on): all
    // loads are requested before the first is used; a wavefront writes consecutive 16-byte pieces.
    {
      constexpr int kRows = kPanel + kTK, kIter = (kRows * 16 + kBlock - 1) / kBlock;
      d2a v[kIter];
      const int c2 = (tid & 15) * 2;
#pragma unroll
      for (int it = 0; it < kIter; ++it) {
        const int row = (tid >> 4) + it * (kBlock / 16);
        const int64_t k = kp0 + row;
        const double *src = Cm + k * ldc + c2;
        const bool row_ok = row < kPanel && k < n;
        v[it].x = (row_ok && c2 + 0 < R) ? src[0] : 0.0;
        v[it].y = (row_ok && c2 + 1 < R) ? src[1] : 0.0;
      }
#pragma unroll
      for (int it = 0; it < kIter; ++it) {
        const int row = (tid >> 4) + it * (kBlock / 16);
        if (row < kRows) *reinterpret_cast<d2a *>(&Cs[row * 32 + c2]) = v[it];
      }
    }
    if (tid == 0) next_unit = 0;
    __syncthreads();

    const int64_t kp1 = (kp0 + kPanel < n) ? kp0 + kPanel : n;
    const int reach = (kPanel / 32) * (c + 1);
    const int nunits = nblk < reach ? nblk : reach;  // row blocks that reach this panel
    for (;;) {
      int u = 0;
      if (lane == 0) u = atomicAdd(&next_unit, 1);
      u = __builtin_amdgcn_readfirstlane(u);
      if (u >= nunits) break;

      const int64_t j0 = i + 32 * (int64_t)u;          // first row of the block
      const int64_t ks = (j0 > kp0) ? j0 : kp0;        // first k of this block in this panel
      const int ntiles = (int)ceil_div(kp1 - ks, kTK);
      const bool rows_full = j0 + 32 <= n;
      // packed row bases for the rows this lane loads, as 32-bit element offsets from the slice: element
      // (i,j,k) is at As[ro[q] + (k - i)]
      int ro[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        int64_t jj = j0 - i + lr + 8 * q;  // row inside the slice triangle of order m
        if (jj >= m) jj = m - 1;           // keep the address inside the buffer; values are masked below
        ro[q] = (int)(tri_row_start(m, jj) - jj);
      }
      const int kr0 = (int)(ks - i), jr0 = (int)(j0 - i);  // relative to the slice
      const int cs0 = (int)(ks - kp0);                     // relative to the panel
      // byte offsets from the slice of this lane's piece of the block's first tile, row by row; a tile
      // further on is 128 bytes further on
      unsigned vo[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) vo[q] = (unsigned)(ro[q] + kr0 + lk) * 8u;

      // The rows of B this lane will fold with, requested now and used after the last tile: element v of
      // accumulator tile (ra, ca) is row 16 ra + 4 v + l/16 of the block, column 16 ca + l%16.
      double bv[2][2][4];
#pragma unroll
      for (int ra = 0; ra < 2; ++ra)
#pragma unroll
        for (int ca = 0; ca < 2; ++ca)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int64_t j = j0 + 16 * ra + 4 * v + l4;
            const int col = 16 * ca + l16;
            bv[ra][ca][v] = (j < n && col < R) ? Bm[j * ldb + col] : 0.0;
          }

      // Scalar loader with every element bounds-tested; only for the last few slices, where a vector
      // load could reach past the end of the packed buffer.
      auto load_guarded = [&](int t, d2a (&v)[4]) {
        const int64_t k0 = ks + kTK * (int64_t)t;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int64_t j = j0 + lr + 8 * q;
          double e[2];
#pragma unroll
          for (int sidx = 0; sidx < 2; ++sidx) {
            const int64_t k = k0 + lk + sidx;
            e[sidx] = (j < n && k >= j && k < n) ? As[ro[q] + (int)(k - i)] : 0.0;
          }
          v[q] = d2a{e[0], e[1]};
        }
      };
      // Branch-free loader for every other tile, including those cut by the diagonal or by the end of
      // the rows: there the pieces also cover elements of the neighbouring rows (still inside the
      // buffer), which mask_tile() zeroes afterwards.  A tile index at or past `ntiles` loads the last
      // tile again, so that the loop below has no control flow around its loads.
      auto load_vec = [&](int t, d2a (&v)[4]) {
        const unsigned toff = 128u * (unsigned)(t < ntiles ? t : ntiles - 1);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          v[q] = *reinterpret_cast<const d2u *>(reinterpret_cast<const char *>(As) + (vo[q] + toff));
      };
      // Zero what a vector-loaded tile holds outside the domain j<=k<n (and of rows j>=n).  Interior
      // tiles, the great majority, skip this on a wave-uniform test.
      auto mask_tile = [&](int t, d2a (&v)[4]) {
        const int kt = kr0 + kTK * t;
        if (rows_full && kt >= jr0 + 31 && kt + kTK <= mi) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int jr = jr0 + lr + 8 * q;
          const int lo = jr - (kt + lk);                      // elements below lo are left of the diagonal
          const int hi = jr < mi ? mi - (kt + lk) : lo;       // elements from hi on are past the row's end
          const unsigned span = hi > lo ? (unsigned)(hi - lo) : 0u;
          v[q].x = ((unsigned)(0 - lo) < span) ? v[q].x : 0.0;
          v[q].y = ((unsigned)(1 - lo) < span) ? v[q].y : 0.0;
        }
      };

      d4v acc[4];  // 2x2 tiles of 16x16: acc[2*ra + ca]
#pragma unroll
      for (int t = 0; t < 4; ++t) acc[t] = d4v{0.0, 0.0, 0.0, 0.0};

      // one 32 x 16 tile: registers -> private LDS tile -> matrix-core operand layout -> 16 MFMAs
      auto compute = [&](int t, const d2a (&v)[4]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<d2a *>(&tile[(lr + 8 * q) * kTP + lk]) = v[q];
        wave_sync_lds();  // the tile is private to this wavefront: no workgroup barrier needed
        const double *cs = &Cs[(cs0 + kTK * t + l4) * 32 + l16];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const double a0 = tile[l16 * kTP + 4 * g + l4];
          const double a1 = tile[(16 + l16) * kTP + 4 * g + l4];
          const double c0 = cs[(4 * g) * 32];
          const double c1 = cs[(4 * g) * 32 + 16];
          acc[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, c0, acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, c1, acc[1], 0, 0, 0);
          acc[2] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, c0, acc[2], 0, 0, 0);
          acc[3] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, c1, acc[3], 0, 0, 0);
        }
        wave_sync_lds();  // all lanes have read the tile before the next one overwrites it
      };

      d2a s0[4], s1[4], s2[4];
      if (vec_ok) {
        // Three register sets rotate and two tiles are always in flight.  The loop leaves only at its
        // bottom and its loads are unconditional (past the last tile they fetch a dummy), so the
        // compiler keeps exact counts of what is in flight.
        load_vec(0, s0);
        load_vec(1, s1);
        int t = 0;
        do {
          load_vec(t + 2, s2);
          mask_tile(t, s0);
          compute(t, s0);
          load_vec(t + 3, s0);
          if (t + 1 < ntiles) {
            mask_tile(t + 1, s1);
            compute(t + 1, s1);
          }
          load_vec(t + 4, s1);
          if (t + 2 < ntiles) {
            mask_tile(t + 2, s2);
            compute(t + 2, s2);
          }
          t += 3;
        } while (t < ntiles);
      } else {
        for (int t = 0; t < ntiles; ++t) {
          load_guarded(t, s0);
          compute(t, s0);
        }
      }

      // fold the 32x32 block of T with B
#pragma unroll
      for (int ra = 0; ra < 2; ++ra)
#pragma unroll
        for (int ca = 0; ca < 2; ++ca)
#pragma unroll
          for (int v = 0; v < 4; ++v) macc[ca] += acc[2 * ra + ca][v] * bv[ra][ca][v];
    }
  }

  // a column's sum is spread over the four lanes l%16, l%16+16, l%16+32, l%16+48
#pragma unroll
  for (int ca = 0; ca < 2; ++ca) {
    macc[ca] += __shfl_xor(macc[ca], 16, 64);
    macc[ca] += __shfl_xor(macc[ca], 32, 64);
  }
  if (l4 == 0) {
    Mred[wave][l16] = macc[0];
    Mred[wave][16 + l16] = macc[1];
  }
  __syncthreads();
  if (tid < R) {
    double s = 0.0;
#pragma unroll
    for (int q = 0; q < kWaves; ++q) s += Mred[q][tid];
    M[i * ldm + tid] = s;
  }
}

}  // namespace

extern "C" int dastac_tet_mttkrp_f64(int64_t n, int64_t R, const double *Ap, const double *B, int64_t ldb,
                                     const double *C, int64_t ldc, double *M, int64_t ldm, void *stream) {
  if (n < 0 || R < 1 || R > (1 << 20) || ldb < R || ldc < R || ldm < R) return DASTAC_EINVAL;
  if (n > DASTAC_TET_MAX_N || tet(n) > ((int64_t)1 << 40) || ld_too_large(ldb, ldc, ldm)) return DASTAC_EOVERFLOW;
  // packed row bases inside a slice are kept as 32-bit element offsets
  if (tri(n) > ((int64_t)1 << 28)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Ap || !B || !C || !M) return DASTAC_ENULL;
  const int64_t mb = view_bytes(n, ldm, R, 8);
  if (overlaps(M, mb, Ap, tet(n) * 8) || overlaps(M, mb, B, view_bytes(n, ldb, R, 8)) ||
      overlaps(M, mb, C, view_bytes(n, ldc, R, 8)))
    return DASTAC_EALIAS;
  // the kernel takes up to 32 columns of the factor matrices; wider ones go block by block (each
  // block reads the packed tetrahedron once)
  for (int64_t c0 = 0; c0 < R; c0 += 32) {
    const int Rb = (int)(R - c0 < 32 ? R - c0 : 32);
    mttkrp_f64_kernel<<<(unsigned)n, kBlock, 0, (hipStream_t)stream>>>(n, Rb, Ap, B + c0, ldb, C + c0, ldc, M + c0, ldm, tet(n));
    if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  }
  return DASTAC_OK;
}
