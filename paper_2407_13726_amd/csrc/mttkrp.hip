// MTTKRP over a packed upper tetrahedron on the fp32 matrix cores:
//
//   M(i,r) := A(i,j,k) * B(j,r) * C(k,r),   i<=j<=k, 0<=r<R (32 columns r per launch)     (Table 1, MTTKRP rule)
//
// Factored evaluation.  Slice i of the packed tetrahedron is a packed upper triangle U_i of order
// n-i, so   M(i,:) = sum_j B(j,:) .* T_i(j,:)   with   T_i = U_i * C[i:, :]   -- a TRMM whose
// result is consumed at once and never leaves the registers.  A is read exactly once.
//
// One workgroup (8 wavefronts) per slice, heaviest slices first.  The workgroup walks k in panels of
// 512; the panel's rows of C are staged in LDS (the reused dense operand).  Inside a panel the
// work items are 32-row blocks of the slice; wavefronts draw them from an LDS counter, full blocks
// first and the blocks cut by the diagonal (shorter) last, which balances the eight wavefronts.
//
// For one block a wavefront streams its 32 packed rows in 32x32 tiles: coalesced 16-byte loads
// (8 lanes cover 128 contiguous bytes of one row; each row starts at its own element offset, given
// by the index polynomial tet_row_start), a private LDS tile turns them into the operand layout of
// v_mfma_f32_32x32x2_f32 (row = lane%32), and 16 matrix instructions accumulate the 32x32 block of
// T.  As in the TRMM kernel, lane half h takes k values 8t+4h..8t+4h+3 of each group of eight.  Only
// tiles on the diagonal or at the ragged end of a row use predicated loads (zeros for k<j, k>=n).
// The block of T is then multiplied elementwise by B's rows and folded into 32 running sums.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kWaves = 8;
constexpr int kBlock = kWaves * 64;
constexpr int kPanel = 512;  // k values per staged panel of C
constexpr int kTP = 36;      // pitch (floats) of a wavefront's private 32x32 tile

typedef float f16v __attribute__((ext_vector_type(16)));

// Orders LDS traffic between the lanes of ONE wavefront (which executes in lockstep): earlier LDS
// writes are visible to later reads of any lane, and the compiler may not move LDS accesses across.
__device__ inline void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(2, 2))) void mttkrp_mfma_kernel(int64_t n, int R, const float *__restrict__ A,
                                                             const float *__restrict__ Bm, int64_t ldb,
                                                             const float *__restrict__ Cm, int64_t ldc,
                                                             float *__restrict__ M, int64_t ldm, int64_t total) {
  // one tile of zero rows follows the panel: the last tile of a row block may reach past the panel's last row
  // (there its elements of A are masked to zero, and must not meet anything but zeros)
  __shared__ __attribute__((aligned(16))) float Cs[(kPanel + 32) * 32];
  __shared__ __attribute__((aligned(16))) float At[kWaves][32 * kTP];
  __shared__ float Mred[kWaves][32];
  __shared__ int next_unit;

  const int64_t i = blockIdx.x;
  const int64_t m = n - i;  // order of this slice
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  const int nblk = (int)ceil_div(m, 32);
  const int npanels = (int)ceil_div(m, kPanel);
  const int64_t slice0 = tet_slice_start(n, i);  // packed position of (i,i,i)
  // a 16-byte load may start up to 31 elements past the end of its row: safe unless the slice is
  // one of the last few of the buffer
  const bool vec_ok = slice0 + tri(m) + 32 <= total;
  const float *__restrict__ As = A + slice0;  // this slice's packed triangle
  // rows of B can be fetched as 16-byte pieces at 32-bit offsets
  const bool b_vec = R == 32 && n * ldb < ((int64_t)1 << 31);

  // loader role inside a 32x32 tile: rows lr, lr+8, lr+16, lr+24; four k values from lk
  const int lr = lane >> 3, lk = (lane & 7) * 4;
  float *tile = At[wave];

  float macc = 0.0f;  // this lane's share of M(i, l32)

  for (int c = 0; c < npanels; ++c) {
    const int64_t kp0 = i + (int64_t)c * kPanel;
    __syncthreads();  // every wavefront is done with the previous panel
    // Layout [k/4][r][k%4]: the four k values a lane feeds to four consecutive matrix instructions
    // are then one 16-byte read.  A thread stages the same column r of four consecutive rows k, so its
    // LDS write is one 16-byte piece too and the lanes of a wavefront write consecutive pieces (free of
    // bank conflicts); the global loads, 128 contiguous bytes per row and half-wavefront, are all
    // requested before the first is used.
    {
      constexpr int kGroups = (kPanel + 32) / 4, kIter = (kGroups * 32 + kBlock - 1) / kBlock;
      f4a v[kIter];
      const int r = tid & 31;
#pragma unroll
      for (int it = 0; it < kIter; ++it) {
        const int kg = (tid >> 5) + it * (kBlock / 32);
        const int64_t k = kp0 + 4 * (int64_t)kg;
        const float *src = Cm + k * ldc + r;
        const bool ok = r < R && kg < kPanel / 4;
        v[it].x = (ok && k + 0 < n) ? src[0] : 0.0f;
        v[it].y = (ok && k + 1 < n) ? src[ldc] : 0.0f;
        v[it].z = (ok && k + 2 < n) ? src[2 * ldc] : 0.0f;
        v[it].w = (ok && k + 3 < n) ? src[3 * ldc] : 0.0f;
      }
#pragma unroll
      for (int it = 0; it < kIter; ++it) {
        const int kg = (tid >> 5) + it * (kBlock / 32);
        if (kg < kGroups) *reinterpret_cast<f4a *>(&Cs[(kg * 32 + r) * 4]) = v[it];
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
      const int ntiles = (int)ceil_div(kp1 - ks, 32);
      const bool rows_full = j0 + 32 <= n;
      // packed row bases for the rows this lane loads, as 32-bit element offsets from the slice:
      // element (i,j,k) is at As[ro[q] + (k - i)]  (a slice of a buffer that fits in memory has
      // far fewer than 2^30 elements)
      int ro[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        int64_t jj = j0 - i + lr + 8 * q;  // row inside the slice triangle of order m
        if (jj >= m) jj = m - 1;           // keep the address inside the buffer; values are masked below
        ro[q] = (int)(tri_row_start(m, jj) - jj);
      }
      const int kr0 = (int)(ks - i), jr0 = (int)(j0 - i), mi = (int)m;  // relative to the slice
      // Byte offsets from the slice of this lane's piece of the block's first tile, row by row: a tile
      // further on is 128 bytes further on, which keeps the per-tile address arithmetic to one add
      // per load (every VALU instruction here is time taken from the matrix pipe of the same SIMD).
      unsigned vo[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) vo[q] = (unsigned)(ro[q] + kr0 + lk) * 4u;
      // The block's 32 rows of B are requested now and used after the last tile (full row blocks
      // of R = 32 columns only), so the fold below never waits for memory.
      const bool fold_lds = vec_ok && b_vec && rows_full;
      f4a bv[4];
      if (fold_lds) {
        const int bo = (int)((j0 + lr) * ldb) + lk;
#pragma unroll
        for (int q = 0; q < 4; ++q) bv[q] = *reinterpret_cast<const f4u *>(Bm + (bo + q * 8 * (int)ldb));
      }

      // Scalar loader with every element bounds-tested; only for the last few slices, where a
      // vector load could reach past the end of the packed buffer.
      auto load_guarded = [&](int t, f4a (&v)[4]) {
        const int64_t k0 = ks + 32 * (int64_t)t;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int64_t j = j0 + lr + 8 * q;
          float e[4];
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            const int64_t k = k0 + lk + s;
            e[s] = (j < n && k >= j && k < n) ? As[ro[q] + (int)(k - i)] : 0.0f;
          }
          v[q] = f4a{e[0], e[1], e[2], e[3]};
        }
      };
      // Branch-free loader for every other tile, including those cut by the diagonal or by the end
      // of the rows: there the 16-byte pieces also cover elements of the neighbouring rows (still
      // inside the buffer), which mask_tile() zeroes afterwards.  A tile index at or past `ntiles`
      // loads the last tile again, so that the loop below has no control flow around its loads
      // and the compiler can leave them in flight across iterations.  Plain (cached) loads:
      // the 128-byte row pieces are not aligned to cache lines, and the next piece of the same
      // row, requested right behind, uses the other half of the shared line.
      auto load_vec = [&](int t, f4a (&v)[4]) {
        const unsigned toff = 128u * (unsigned)(t < ntiles ? t : ntiles - 1);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          v[q] = *reinterpret_cast<const f4u *>(reinterpret_cast<const char *>(As) + (vo[q] + toff));
      };
      // Zero what a vector-loaded tile holds outside the domain j<=k<n (and of rows j>=n).  Interior
      // tiles, the great majority, skip this on a wave-uniform test.
      auto mask_tile = [&](int t, f4a (&v)[4]) {
        const int kt = kr0 + 32 * t;
        if (rows_full && kt >= jr0 + 31 && kt + 32 <= mi) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int jr = jr0 + lr + 8 * q;
          const int lo = jr - (kt + lk);                      // elements below lo are left of the diagonal
          const int hi = jr < mi ? mi - (kt + lk) : lo;       // elements from hi on are past the row's end
          const unsigned span = hi > lo ? (unsigned)(hi - lo) : 0u;
          v[q].x = ((unsigned)(0 - lo) < span) ? v[q].x : 0.0f;
          v[q].y = ((unsigned)(1 - lo) < span) ? v[q].y : 0.0f;
          v[q].z = ((unsigned)(2 - lo) < span) ? v[q].z : 0.0f;
          v[q].w = ((unsigned)(3 - lo) < span) ? v[q].w : 0.0f;
        }
      };

      f16v acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

      // one 32x32 tile: registers -> private LDS tile -> matrix-core operand layout -> 16 MFMAs
      auto compute = [&](int t, const f4a (&v)[4]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<f4a *>(&tile[(lr + 8 * q) * kTP + lk]) = v[q];
        wave_sync_lds();  // the tile is private to this wavefront: no workgroup barrier needed
        const float *cs = &Cs[((((int)(ks - kp0) + 32 * t) >> 2) + h) * 128 + l32 * 4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f4a a = *reinterpret_cast<const f4a *>(&tile[l32 * kTP + 8 * g + 4 * h]);
          const f4a cv = *reinterpret_cast<const f4a *>(&cs[g * 256]);
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, cv.x, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, cv.y, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, cv.z, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, cv.w, acc, 0, 0, 0);
        }
        wave_sync_lds();  // all lanes have read the tile before the next one overwrites it
      };

      f4a s0[4], s1[4], s2[4];
      if (vec_ok) {
        // Three register sets rotate and two tiles are always in flight.  The loop leaves only at
        // its bottom and its loads are unconditional (past the last tile they fetch a dummy), so
        // the compiler keeps exact counts of what is in flight.
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

      // fold the 32x32 block of T with B: register v of lane l is row 8*(v/4)+4*(l/32)+v%4, column l%32
      if (fold_lds) {
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<f4a *>(&tile[(lr + 8 * q) * kTP + lk]) = bv[q];
        wave_sync_lds();
#pragma unroll
        for (int v = 0; v < 16; ++v) macc += acc[v] * tile[(8 * (v / 4) + 4 * h + (v % 4)) * kTP + l32];
        wave_sync_lds();  // the tile is free again for the next block
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int64_t j = j0 + 8 * (v / 4) + 4 * h + (v % 4);
          if (j < n && l32 < R) macc += acc[v] * Bm[j * ldb + l32];
        }
      }
    }
  }

  macc += __shfl_xor(macc, 32, 64);
  if (h == 0) Mred[wave][l32] = macc;
  __syncthreads();
  if (tid < R) {
    float s = 0.0f;
#pragma unroll
    for (int q = 0; q < kWaves; ++q) s += Mred[q][tid];
    M[i * ldm + tid] = s;
  }
}

}  // namespace

extern "C" int dastac_tet_mttkrp_f32(int64_t n, int64_t R, const float *Ap, const float *B, int64_t ldb,
                                     const float *C, int64_t ldc, float *M, int64_t ldm, void *stream) {
  if (n < 0 || R < 1 || R > (1 << 20) || ldb < R || ldc < R || ldm < R) return DASTAC_EINVAL;
  if (n > DASTAC_TET_MAX_N || tet(n) > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Ap || !B || !C || !M) return DASTAC_ENULL;
  if (overlaps(M, n * ldm * 4, Ap, tet(n) * 4) || overlaps(M, n * ldm * 4, B, n * ldb * 4) ||
      overlaps(M, n * ldm * 4, C, n * ldc * 4))
    return DASTAC_EALIAS;
  // the kernel takes up to 32 columns of the factor matrices; wider ones go block by block (each
  // block reads the packed tetrahedron once)
  for (int64_t c0 = 0; c0 < R; c0 += 32) {
    const int Rb = (int)(R - c0 < 32 ? R - c0 : 32);
    mttkrp_mfma_kernel<<<(unsigned)n, kBlock, 0, (hipStream_t)stream>>>(n, Rb, Ap, B + c0, ldb, C + c0, ldc, M + c0, ldm, tet(n));
    if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  }
  return DASTAC_OK;
}
