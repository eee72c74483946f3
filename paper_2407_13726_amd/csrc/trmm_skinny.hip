// TRMM over a packed upper triangle with few right-hand sides (m <= 32 per launch):
//
//   C(i,c) := U(i,k) * B(k,c),  i<=k, 0<=c<m        (Table 1's SpMV_UT rule with a matrix right-hand side)
//
// With so few columns the product is bound by the one pass over the packed triangle, not by the
// matrix cores, and the tiling of the wide kernel (64x128 tiles of C, half of them empty at m = 64)
// leaves most of the chip idle.  This kernel streams U instead, the way the tetrahedral MTTKRP streams
// a slice: k is cut into panels of 512, the panel's rows of B are staged in LDS (the reused dense
// operand, 64 KB), and a wavefront takes one block of 32 packed rows through the panel in 32x32 tiles:
// coalesced 16-byte loads (8 lanes cover 128 contiguous bytes of a row, each row at its own element
// offset given by the index polynomial), a private LDS tile that turns them into the operand layout
// of v_mfma_f32_32x32x2_f32, 16 matrix instructions per tile.  A workgroup is eight such wavefronts on
// eight consecutive row blocks of one panel; its 32x32 pieces of C are added into a zeroed C with
// floating-point atomics (a row block meets every panel right of its diagonal).  U is read exactly once.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kWaves = 8;
constexpr int kBlock = kWaves * 64;
constexpr int kPanel = 512;  // k values per staged panel of B
constexpr int kRB = 32;      // rows of a block
constexpr int kTP = 36;      // pitch (floats) of a wavefront's private 32x32 tile


// Orders LDS traffic between the lanes of ONE wavefront (which executes in lockstep).
__device__ inline void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroups.  Panel p is reached by the row blocks 0 .. 16(p+1)-1 (fewer in the last panel), eight to a
// workgroup: groups 0 .. 2p-1 hold blocks that cross the whole panel (16 tiles each), groups 2p and 2p+1
// the blocks cut by the diagonal (16 down to 1 tiles).  Ids number the whole groups of all panels first and
// the cut ones last, so that the last, partly filled layer of resident workgroups is made of the short ones.
DASTAC_HD int64_t whole_groups_before(int64_t p) { return p * (p - 1); }  // sum of 2q for q < p

__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(2, 2)))
void trmm_skinny_kernel(int64_t n, int m, const float *__restrict__ U, const float *__restrict__ B, int64_t ldb,
                        float *__restrict__ C, int64_t ldc, int64_t total, int npanels) {
  // one tile of zero rows follows the panel: the last tile of a row block may reach past the panel's last row
  __shared__ __attribute__((aligned(16))) float Bs[(kPanel + 32) * 32];
  __shared__ __attribute__((aligned(16))) float At[kWaves][32 * kTP];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  const int64_t nblk = ceil_div(n, kRB);

  // workgroup id -> (panel, group of eight row blocks)
  int p;
  int64_t g;
  const int64_t whole = whole_groups_before(npanels);
  if ((int64_t)blockIdx.x < whole) {
    p = (int)((1.0f + sqrtf(1.0f + 4.0f * (float)blockIdx.x)) * 0.5f);  // largest p with p(p-1) <= id, about
    while (p > 1 && whole_groups_before(p) > (int64_t)blockIdx.x) --p;
    while (whole_groups_before(p + 1) <= (int64_t)blockIdx.x) ++p;
    g = (int64_t)blockIdx.x - whole_groups_before(p);
  } else {
    const int64_t d = (int64_t)blockIdx.x - whole;
    p = (int)(d >> 1);
    g = 2 * (int64_t)p + (d & 1);
  }
  p = uniform32(p);
  const int64_t kp0 = (int64_t)p * kPanel;
  const int64_t kp1 = kp0 + kPanel < n ? kp0 + kPanel : n;

  // Stage the panel's rows of B.  Layout [k/4][c][k%4]: the four k values a lane feeds to four consecutive
  // matrix instructions are then one 16-byte read; a thread stages the same column of four consecutive rows.
  {
    constexpr int kGroups = (kPanel + 32) / 4, kIter = (kGroups * 32 + kBlock - 1) / kBlock;
    f4a v[kIter];
    const int c = tid & 31;
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
      const int kg = (tid >> 5) + it * (kBlock / 32);
      const int64_t k = kp0 + 4 * (int64_t)kg;
      const float *src = B + k * ldb + c;
      const bool ok = c < m && kg < kPanel / 4;
      v[it].x = (ok && k + 0 < n) ? src[0] : 0.0f;
      v[it].y = (ok && k + 1 < n) ? src[ldb] : 0.0f;
      v[it].z = (ok && k + 2 < n) ? src[2 * ldb] : 0.0f;
      v[it].w = (ok && k + 3 < n) ? src[3 * ldb] : 0.0f;
    }
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
      const int kg = (tid >> 5) + it * (kBlock / 32);
      if (kg < kGroups) *reinterpret_cast<f4a *>(&Bs[(kg * 32 + c) * 4]) = v[it];
    }
  }
  __syncthreads();

  const int64_t reach = (int64_t)(kPanel / kRB) * (p + 1);
  const int64_t nunits = nblk < reach ? nblk : reach;  // row blocks that reach this panel
  const int64_t u = g * kWaves + wave;                 // this wavefront's row block
  if (u >= nunits) return;                             // (no workgroup barrier below this line)

  // loader role inside a 32x32 tile: rows lr, lr+8, lr+16, lr+24; four k values from lk
  const int lr = lane >> 3, lk = (lane & 7) * 4;
  float *tile = At[wave];

  const int64_t j0 = kRB * u;                      // first row of the block
  const int64_t ks = j0 > kp0 ? j0 : kp0;          // first k of this block in this panel
  const int ntiles = (int)ceil_div(kp1 - ks, 32);
  const bool rows_full = j0 + kRB <= n;
  // a 16-byte load may start up to 31 elements past the end of its row: the rows of this block end at
  // tri_row_start(n, j0+32) at the latest, which must leave that much room in the packed buffer
  const int64_t jend = j0 + kRB < n ? j0 + kRB : n;
  const bool vec_ok = tri_row_start(n, jend) + 32 <= total;
  // packed row bases for the rows this lane loads: element (j,k) is at U[ro[q] + k]
  int64_t ro[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    int64_t jj = j0 + lr + 8 * q;
    if (jj >= n) jj = n - 1;  // keep the address inside the buffer; values are masked below
    ro[q] = tri_row_start(n, jj) - jj;
  }
  // this lane's piece of the block's first tile, row by row; a tile further on is 32 elements further on
  const float *up[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) up[q] = U + (ro[q] + ks + lk);

  // Scalar loader with every element bounds-tested: only for the last row blocks of the triangle.
  auto load_guarded = [&](int t, f4a (&v)[4]) {
    const int64_t k0 = ks + 32 * (int64_t)t;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t j = j0 + lr + 8 * q;
      float e[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int64_t k = k0 + lk + s;
        e[s] = (j < n && k >= j && k < n) ? U[ro[q] + k] : 0.0f;
      }
      v[q] = f4a{e[0], e[1], e[2], e[3]};
    }
  };
  // Branch-free loader for every other tile; a tile index at or past `ntiles` loads the last tile again.
  auto load_vec = [&](int t, f4a (&v)[4]) {
    const int toff = 32 * (t < ntiles ? t : ntiles - 1);
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const f4u *>(up[q] + toff);
  };
  // Zero what a vector-loaded tile holds outside the domain j<=k<n (and of rows j>=n).
  auto mask_tile = [&](int t, f4a (&v)[4]) {
    const int64_t kt = ks + 32 * (int64_t)t;
    if (rows_full && kt >= j0 + 31 && kt + 32 <= n) return;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t j = j0 + lr + 8 * q;
      const int64_t lo = j - (kt + lk);                  // elements below lo are left of the diagonal
      const int64_t hi = j < n ? n - (kt + lk) : lo;     // elements from hi on are past the row's end
      v[q].x = (0 >= lo && 0 < hi) ? v[q].x : 0.0f;
      v[q].y = (1 >= lo && 1 < hi) ? v[q].y : 0.0f;
      v[q].z = (2 >= lo && 2 < hi) ? v[q].z : 0.0f;
      v[q].w = (3 >= lo && 3 < hi) ? v[q].w : 0.0f;
    }
  };

  f16v acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

  // one 32x32 tile: registers -> private LDS tile -> matrix-core operand layout -> 16 MFMAs; lane half h
  // takes k values 8g+4h..8g+4h+3 of each group of eight (a sum over k may be taken in any order)
  auto compute = [&](int t, const f4a (&v)[4]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) *reinterpret_cast<f4a *>(&tile[(lr + 8 * q) * kTP + lk]) = v[q];
    wave_sync_lds();  // the tile is private to this wavefront: no workgroup barrier needed
    const float *bs = &Bs[((((int)(ks - kp0) + 32 * t) >> 2) + h) * 128 + l32 * 4];
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const f4a a = *reinterpret_cast<const f4a *>(&tile[l32 * kTP + 8 * gq + 4 * h]);
      const f4a bv = *reinterpret_cast<const f4a *>(&bs[gq * 256]);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, bv.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, bv.y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, bv.z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, bv.w, acc, 0, 0, 0);
    }
    wave_sync_lds();  // all lanes have read the tile before the next one overwrites it
  };

  f4a s0[4], s1[4], s2[4];
  if (vec_ok) {
    // Three register sets rotate and two tiles are always in flight; the loop leaves only at its bottom
    // and its loads are unconditional (past the last tile they fetch a dummy).
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

  // register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32 of the block's piece of C
  if (l32 < m) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t j = j0 + 8 * (v / 4) + 4 * h + (v % 4);
      if (j < n) unsafeAtomicAdd(&C[j * ldc + l32], acc[v]);
    }
  }
}

// C(0..n-1, 0..m-1) := 0, leaving the padding columns of every row alone
__global__ __launch_bounds__(256) void zero_rows_kernel(float *__restrict__ C, int64_t n, int64_t m, int64_t ldc) {
  const int64_t total = n * m;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t i = t / m;
    C[i * ldc + (t - i * m)] = 0.0f;
  }
}

}  // namespace

// C := U B for m <= 64 columns, 32 at a time (each pass reads the packed triangle once); arguments are
// validated by the caller.
int dastac::trmm_few_columns(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C,
                             int64_t ldc, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  const int64_t zb = ceil_div(n * m, 256);
  zero_rows_kernel<<<(unsigned)(zb < 4096 ? zb : 4096), 256, 0, st>>>(C, n, m, ldc);
  if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  const int64_t npanels = ceil_div(n, kPanel);
  const int64_t groups = whole_groups_before(npanels) + 2 * npanels;  // the last panel's second cut group may be empty
  if (groups > 0x7fffffff) return DASTAC_EOVERFLOW;
  for (int64_t c0 = 0; c0 < m; c0 += 32) {
    const int mb = (int)(m - c0 < 32 ? m - c0 : 32);
    trmm_skinny_kernel<<<(unsigned)groups, kBlock, 0, st>>>(n, mb, Up, B + c0, ldb, C + c0, ldc, tri(n), (int)npanels);
    if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  }
  return DASTAC_OK;
}
