// TRMM over a packed upper triangle with few right-hand sides, double precision (m <= 32 per launch):
//
//   C(i,c) := U(i,k) * B(k,c),  i<=k, 0<=c<m,   all double
//
// The single-precision streaming kernel's plan on the fp64 matrix cores: k is cut into panels of 256
// (the panel's rows of B, 64 KB of doubles, are staged in LDS), a wavefront takes one block of 32 packed
// rows through the panel in tiles of 32 rows x 16 values of k (128 contiguous bytes per row, 16-byte
// pieces), a private LDS tile turns them into the operands of v_mfma_f64_16x16x4_f64 (lane l supplies row or
// column l%16 at k = l/16), and the 32x32 piece of C, held as 2x2 tiles of 16x16, is added into a zeroed C
// with floating-point atomics.  A workgroup is eight wavefronts on eight consecutive row blocks of one panel;
// U is read exactly once per 32 columns.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kWaves = 8;
constexpr int kBlock = kWaves * 64;
constexpr int kPanel = 256;  // k values per staged panel of B
constexpr int kRB = 32;      // rows of a block
constexpr int kTK = 16;      // k values per tile
constexpr int kTP = kTK + 2;  // pitch (doubles) of a wavefront's private 32 x 16 tile


// Orders LDS traffic between the lanes of ONE wavefront (which executes in lockstep).
__device__ inline void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroups.  Panel p is reached by the row blocks 0 .. 8(p+1)-1 (fewer in the last panel), eight to a
// workgroup: groups 0 .. p-1 hold blocks that cross the whole panel, group p the blocks cut by the diagonal.
// Ids number the whole groups of all panels first and the cut ones last, so that the last, partly filled
// layer of resident workgroups is made of the short ones.
DASTAC_HD int64_t whole_groups_before(int64_t p) { return p * (p - 1) / 2; }  // sum of q for q < p

__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(2, 2)))
void trmm_skinny_f64_kernel(int64_t n, int m, const double *__restrict__ U, const double *__restrict__ B, int64_t ldb,
                            double *__restrict__ C, int64_t ldc, int64_t total, int npanels) {
  // [k][c]; one tile of zero rows follows the panel
  __shared__ __attribute__((aligned(16))) double Bs[(kPanel + kTK) * 32];
  __shared__ __attribute__((aligned(16))) double At[kWaves][32 * kTP];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, l4 = lane >> 4;
  const int64_t nblk = ceil_div(n, kRB);

  // workgroup id -> (panel, group of eight row blocks)
  int p;
  int64_t g;
  const int64_t whole = whole_groups_before(npanels);
  if ((int64_t)blockIdx.x < whole) {
    p = (int)((1.0f + sqrtf(1.0f + 8.0f * (float)blockIdx.x)) * 0.5f);  // largest p with p(p-1)/2 <= id, about
    while (p > 1 && whole_groups_before(p) > (int64_t)blockIdx.x) --p;
    while (whole_groups_before(p + 1) <= (int64_t)blockIdx.x) ++p;
    g = (int64_t)blockIdx.x - whole_groups_before(p);
  } else {
    p = (int)((int64_t)blockIdx.x - whole);
    g = p;
  }
  p = uniform32(p);
  const int64_t kp0 = (int64_t)p * kPanel;
  const int64_t kp1 = kp0 + kPanel < n ? kp0 + kPanel : n;

  // Stage the panel's rows of B, [k][c] with 32 columns (zeros from column m on and from row n on).
  {
    constexpr int kRows = kPanel + kTK, kIter = (kRows * 16 + kBlock - 1) / kBlock;
    d2a v[kIter];
    const int c2 = (tid & 15) * 2;
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
      const int row = (tid >> 4) + it * (kBlock / 16);
      const int64_t k = kp0 + row;
      const double *src = B + k * ldb + c2;
      const bool row_ok = row < kPanel && k < n;
      v[it].x = (row_ok && c2 + 0 < m) ? src[0] : 0.0;
      v[it].y = (row_ok && c2 + 1 < m) ? src[1] : 0.0;
    }
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
      const int row = (tid >> 4) + it * (kBlock / 16);
      if (row < kRows) *reinterpret_cast<d2a *>(&Bs[row * 32 + c2]) = v[it];
    }
  }
  __syncthreads();

  const int64_t reach = (int64_t)(kPanel / kRB) * (p + 1);
  const int64_t nunits = nblk < reach ? nblk : reach;  // row blocks that reach this panel
  const int64_t u = g * kWaves + wave;                 // this wavefront's row block
  if (u >= nunits) return;                             // (no workgroup barrier below this line)

  // loader role inside a tile: rows lr, lr+8, lr+16, lr+24; two k values from lk
  const int lr = lane >> 3, lk = (lane & 7) * 2;
  double *tile = At[wave];

  const int64_t j0 = kRB * u;                      // first row of the block
  const int64_t ks = j0 > kp0 ? j0 : kp0;          // first k of this block in this panel
  const int ntiles = (int)ceil_div(kp1 - ks, kTK);
  const bool rows_full = j0 + kRB <= n;
  // a 16-byte load may start up to 15 elements past the end of its row
  const int64_t jend = j0 + kRB < n ? j0 + kRB : n;
  const bool vec_ok = tri_row_start(n, jend) + kTK <= total;
  int64_t ro[4];  // element (j,k) of this lane's rows is at U[ro[q] + k]
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    int64_t jj = j0 + lr + 8 * q;
    if (jj >= n) jj = n - 1;  // keep the address inside the buffer; values are masked below
    ro[q] = tri_row_start(n, jj) - jj;
  }
  const double *up[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) up[q] = U + (ro[q] + ks + lk);
  const int cs0 = (int)(ks - kp0);  // relative to the panel

  auto load_guarded = [&](int t, d2a (&v)[4]) {
    const int64_t k0 = ks + kTK * (int64_t)t;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t j = j0 + lr + 8 * q;
      double e[2];
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        const int64_t k = k0 + lk + s;
        e[s] = (j < n && k >= j && k < n) ? U[ro[q] + k] : 0.0;
      }
      v[q] = d2a{e[0], e[1]};
    }
  };
  auto load_vec = [&](int t, d2a (&v)[4]) {
    const int toff = kTK * (t < ntiles ? t : ntiles - 1);
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const d2u *>(up[q] + toff);
  };
  auto mask_tile = [&](int t, d2a (&v)[4]) {
    const int64_t kt = ks + kTK * (int64_t)t;
    if (rows_full && kt >= j0 + 31 && kt + kTK <= n) return;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t j = j0 + lr + 8 * q;
      const int64_t lo = j - (kt + lk);                  // elements below lo are left of the diagonal
      const int64_t hi = j < n ? n - (kt + lk) : lo;     // elements from hi on are past the row's end
      v[q].x = (0 >= lo && 0 < hi) ? v[q].x : 0.0;
      v[q].y = (1 >= lo && 1 < hi) ? v[q].y : 0.0;
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
    const double *bs = &Bs[(cs0 + kTK * t + l4) * 32 + l16];
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const double a0 = tile[l16 * kTP + 4 * gq + l4];
      const double a1 = tile[(16 + l16) * kTP + 4 * gq + l4];
      const double c0 = bs[(4 * gq) * 32];
      const double c1 = bs[(4 * gq) * 32 + 16];
      acc[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, c0, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, c1, acc[1], 0, 0, 0);
      acc[2] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, c0, acc[2], 0, 0, 0);
      acc[3] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, c1, acc[3], 0, 0, 0);
    }
    wave_sync_lds();  // all lanes have read the tile before the next one overwrites it
  };

  d2a s0[4], s1[4], s2[4];
  if (vec_ok) {
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

  // element v of accumulator tile (ra, ca) is row 16 ra + 4 v + l/16 of the block, column 16 ca + l%16
#pragma unroll
  for (int ra = 0; ra < 2; ++ra)
#pragma unroll
    for (int ca = 0; ca < 2; ++ca) {
      const int col = 16 * ca + l16;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int64_t j = j0 + 16 * ra + 4 * v + l4;
        if (j < n && col < m) unsafeAtomicAdd(&C[j * ldc + col], acc[2 * ra + ca][v]);
      }
    }
}

// C(0..n-1, 0..m-1) := 0, leaving the padding columns of every row alone
__global__ __launch_bounds__(256) void zero_rows_kernel(double *__restrict__ C, int64_t n, int64_t m, int64_t ldc) {
  const int64_t total = n * m;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t i = t / m;
    C[i * ldc + (t - i * m)] = 0.0;
  }
}

}  // namespace

// C := U B for m <= 64 columns, 32 at a time (each pass reads the packed triangle once); arguments are
// validated by the caller.
int dastac::trmm_few_columns(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C,
                             int64_t ldc, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  const int64_t zb = ceil_div(n * m, 256);
  zero_rows_kernel<<<(unsigned)(zb < 4096 ? zb : 4096), 256, 0, st>>>(C, n, m, ldc);
  if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  const int64_t npanels = ceil_div(n, kPanel);
  const int64_t groups = whole_groups_before(npanels) + npanels;
  if (groups > 0x7fffffff) return DASTAC_EOVERFLOW;
  for (int64_t c0 = 0; c0 < m; c0 += 32) {
    const int mb = (int)(m - c0 < 32 ? m - c0 : 32);
    trmm_skinny_f64_kernel<<<(unsigned)groups, kBlock, 0, st>>>(n, mb, Up, B + c0, ldb, C + c0, ldc, tri(n), (int)npanels);
    if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  }
  return DASTAC_OK;
}
