// MTTKRP over a packed upper tetrahedron on the fp32 matrix cores:
//
//   M(i,r) := A(i,j,k) * B(j,r) * C(k,r),   i<=j<=k, 0<=r<R<=32     (Table 1, MTTKRP rule)
//
// Factored evaluation.  Slice i of the packed tetrahedron is a packed upper triangle U_i of order
// n-i, so   M(i,:) = sum_j B(j,:) .* T_i(j,:)   with   T_i = U_i * C[i:, :]   -- a TRMM whose
// result is consumed at once and never leaves the registers.  A is read exactly once.
//
// One workgroup (8 wavefronts) per slice, heaviest slices first.  The workgroup walks k in panels of
// 256; the panel's rows of C are staged in LDS (the reused dense operand).  Inside a panel the
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
constexpr int kPanel = 256;  // k values per staged panel of C
constexpr int kTP = 36;      // pitch (floats) of a wavefront's private 32x32 tile

typedef float f16v __attribute__((ext_vector_type(16)));

// Orders LDS traffic between the lanes of ONE wavefront (which executes in lockstep): earlier LDS
// writes are visible to later reads of any lane, and the compiler may not move LDS accesses across.
__device__ inline void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(4, 4))) void mttkrp_mfma_kernel(int64_t n, int R, const float *__restrict__ A,
                                                             const float *__restrict__ Bm, int64_t ldb,
                                                             const float *__restrict__ Cm, int64_t ldc,
                                                             float *__restrict__ M, int64_t ldm) {
  __shared__ __attribute__((aligned(16))) float Cs[kPanel * 32];
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

  // loader role inside a 32x32 tile: rows lr, lr+8, lr+16, lr+24; four k values from lk
  const int lr = lane >> 3, lk = (lane & 7) * 4;
  float *tile = At[wave];

  float macc = 0.0f;  // this lane's share of M(i, l32)

  for (int c = 0; c < npanels; ++c) {
    const int64_t kp0 = i + (int64_t)c * kPanel;
    __syncthreads();  // every wavefront is done with the previous panel
    for (int t = tid; t < kPanel * 8; t += kBlock) {
      const int row = t >> 3, c4 = (t & 7) * 4;
      const int64_t k = kp0 + row;
      f4a v = {0.0f, 0.0f, 0.0f, 0.0f};
      if (k < n) {
        if (R == 32) {
          v = *reinterpret_cast<const f4u *>(Cm + k * ldc + c4);
        } else {
          if (c4 + 0 < R) v.x = Cm[k * ldc + c4 + 0];
          if (c4 + 1 < R) v.y = Cm[k * ldc + c4 + 1];
          if (c4 + 2 < R) v.z = Cm[k * ldc + c4 + 2];
          if (c4 + 3 < R) v.w = Cm[k * ldc + c4 + 3];
        }
      }
      *reinterpret_cast<f4a *>(&Cs[row * 32 + c4]) = v;
    }
    if (tid == 0) next_unit = 0;
    __syncthreads();

    const int64_t kp1 = (kp0 + kPanel < n) ? kp0 + kPanel : n;
    const int nunits = (nblk < 8 * (c + 1)) ? nblk : 8 * (c + 1);  // row blocks that reach this panel
    for (;;) {
      int u = 0;
      if (lane == 0) u = atomicAdd(&next_unit, 1);
      u = __builtin_amdgcn_readfirstlane(u);
      if (u >= nunits) break;

      const int64_t j0 = i + 32 * (int64_t)u;          // first row of the block
      const int64_t ks = (j0 > kp0) ? j0 : kp0;        // first k of this block in this panel
      const int ntiles = (int)ceil_div(kp1 - ks, 32);
      const bool rows_full = j0 + 32 <= n;
      // packed row bases for the rows this lane loads: element (i,j,k) is at rb[q] + k
      const float *rb[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        int64_t j = j0 + lr + 8 * q;
        if (j >= n) j = n - 1;  // keep the address inside the buffer; values are masked below
        const int64_t jj = j - i;  // row inside the slice triangle of order m
        rb[q] = A + slice0 + tri_row_start(m, jj) - j;
      }

      // Guarded loader for tiles cut by the diagonal or by the ragged end of the rows.
      auto load_guarded = [&](int t, f4a (&v)[4]) {
        const int64_t k0 = ks + 32 * (int64_t)t;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int64_t j = j0 + lr + 8 * q;
          float e[4];
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            const int64_t k = k0 + lk + s;
            e[s] = (j < n && k >= j && k < n) ? rb[q][k] : 0.0f;
          }
          v[q] = f4a{e[0], e[1], e[2], e[3]};
        }
      };
      // Branch-free loader for interior tiles; a tile index at or past `fe` loads a harmless dummy
      // address instead, so that the loop below has no control flow around its loads and the
      // compiler can leave them in flight across iterations.  Plain (cached) loads: the 128-byte
      // row pieces are not aligned to cache lines, and the next piece of the same row, requested
      // right behind, uses the other half of the shared line.
      const float *dummy = A + slice0;
      auto load_fast = [&](int t, int fe, f4a (&v)[4]) {
        const int64_t k0 = ks + 32 * (int64_t)t;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float *src = (t < fe) ? rb[q] + k0 + lk : dummy;
          v[q] = *reinterpret_cast<const f4u *>(src);
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
        const float *cs = &Cs[(int)(ks - kp0 + 32 * t + 4 * h) * 32 + l32];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f4a a = *reinterpret_cast<const f4a *>(&tile[l32 * kTP + 8 * g + 4 * h]);
          const float c0 = cs[(8 * g + 0) * 32], c1 = cs[(8 * g + 1) * 32];
          const float c2 = cs[(8 * g + 2) * 32], c3 = cs[(8 * g + 3) * 32];
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, c0, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, c1, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, c2, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, c3, acc, 0, 0, 0);
        }
        wave_sync_lds();  // all lanes have read the tile before the next one overwrites it
      };

      // Tiles [fb, fe) need no predicates: not on the diagonal, all 32 rows exist, all 32 k exist.
      int fb = 0, fe = ntiles;
      if (!rows_full) {
        fe = 0;
      } else {
        if (ks < j0 + 32) fb = 1;                      // the first tile straddles the diagonal
        if (ks + 32 * (int64_t)ntiles > n) fe -= 1;    // the last tile runs past n
        if (fe < fb) fe = fb;
      }
      f4a s0[4], s1[4], s2[4];
      if (fb < fe) {  // three register sets rotate; two tiles are always in flight
        load_fast(fb, fe, s0);
        load_fast(fb + 1, fe, s1);
        for (int t = fb;; t += 3) {
          load_fast(t + 2, fe, s2);
          compute(t, s0);
          if (t + 1 >= fe) break;
          load_fast(t + 3, fe, s0);
          compute(t + 1, s1);
          if (t + 2 >= fe) break;
          load_fast(t + 4, fe, s1);
          compute(t + 2, s2);
          if (t + 3 >= fe) break;
        }
      }
      if (fb == 1) {  // the diagonal tile
        load_guarded(0, s0);
        compute(0, s0);
      }
      for (int t = (fe > fb ? fe : fb); t < ntiles; ++t) {  // the ragged last tile, or all tiles of a ragged row block
        load_guarded(t, s0);
        compute(t, s0);
      }

      // fold the 32x32 block of T with B: register v of lane l is row 8*(v/4)+4*(l/32)+v%4, column l%32
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t j = j0 + 8 * (v / 4) + 4 * h + (v % 4);
        if (j < n && l32 < R) macc += acc[v] * Bm[j * ldb + l32];
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
  if (n < 0 || R < 1 || R > 32 || ldb < R || ldc < R || ldm < R) return DASTAC_EINVAL;
  if (n > DASTAC_TET_MAX_N || tet(n) > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Ap || !B || !C || !M) return DASTAC_ENULL;
  if (overlaps(M, n * ldm * 4, Ap, tet(n) * 4) || overlaps(M, n * ldm * 4, B, n * ldb * 4) ||
      overlaps(M, n * ldm * 4, C, n * ldc * 4))
    return DASTAC_EALIAS;
  mttkrp_mfma_kernel<<<(unsigned)n, kBlock, 0, (hipStream_t)stream>>>(n, (int)R, Ap, B, ldb, C, ldc, M, ldm);
  return launch_status();
}
