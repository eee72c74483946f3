// TRMM over a packed upper triangle with few right-hand sides (m <= 32 per launch), single and double precision:
//
//   C(i,c) := U(i,k) * B(k,c),  i<=k, 0<=c<m        (Table 1's SpMV_UT rule with a matrix right-hand side)
//
// With so few columns the product is bound by the one pass over the packed triangle, not by the
// matrix cores, and the tiling of the wide kernel (64x128 tiles of C, half of them empty at m = 64)
// leaves most of the chip idle.  This kernel streams U instead: k is cut into panels (64 KB of B's rows,
// the reused dense operand, staged in LDS: 512 values of k in single, 256 in double precision), and a
// wavefront takes one block of 32 packed rows through the panel in tiles of 32 rows x 128 bytes:
// coalesced 16-byte loads (8 lanes cover 128 contiguous bytes of a row, each row at its own element
// offset given by the index polynomial), a private LDS tile that turns them into the operand layout of
// the matrix instruction, 16 matrix instructions per tile.  A workgroup is eight such wavefronts on
// eight consecutive row blocks of one panel; its 32x32 pieces of C are added into a zeroed C with
// floating-point atomics (a row block meets every panel right of its diagonal).  U is read exactly once
// per 32 columns.  Skinny<T> holds what differs between the two precisions: the staged layout of B,
// the matrix instructions, and where a result element lives.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kWaves = 8;
constexpr int kBlock = kWaves * 64;
constexpr int kRB = 32;  // rows of a block

// Orders LDS traffic between the lanes of ONE wavefront (which executes in lockstep).
__device__ inline void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <typename T>
struct Skinny;

// v_mfma_f32_32x32x2_f32.  B is staged [k/4][c][k%4]: the four k values a lane feeds to four consecutive
// matrix instructions are one 16-byte read (lane half h takes k values 8g+4h..8g+4h+3 of each group of
// eight -- a sum over k may be taken in any order).
template <>
struct Skinny<float> {
  static constexpr int kPanel = 512;  // k values per staged panel of B
  static constexpr int kTK = 32;      // k values per tile
  static constexpr int kV = 4;        // elements per 16-byte piece
  static constexpr int kTP = 36;      // pitch of a wavefront's private tile
  typedef f4a vec;
  typedef f4u uvec;
  struct Acc {
    f16v v;
  };
  __device__ static void clear(Acc &a) {
#pragma unroll
    for (int v = 0; v < 16; ++v) a.v[v] = 0.0f;
  }
  // stages rows kp0 .. kp0+kPanel-1 of B (zeros from column m on, from row n on, and in the kTK rows after the panel)
  __device__ static void stage(float *Bs, const float *__restrict__ B, int64_t ldb, int64_t kp0, int64_t n, int m, int tid) {
    constexpr int kGroups = (kPanel + kTK) / 4, kIter = (kGroups * 32 + kBlock - 1) / kBlock;
    f4a v[kIter];
    const int c = tid & 31;  // a thread stages the same column of four consecutive rows
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
  // the 16 matrix instructions of the tile that starts `koff` rows into the panel
  __device__ static void multiply(const float *tile, const float *Bs, int koff, int lane, Acc &acc) {
    const int l32 = lane & 31, h = lane >> 5;
    const float *bs = &Bs[((koff >> 2) + h) * 128 + l32 * 4];
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const f4a a = *reinterpret_cast<const f4a *>(&tile[l32 * kTP + 8 * gq + 4 * h]);
      const f4a bv = *reinterpret_cast<const f4a *>(&bs[gq * 256]);
      acc.v = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, bv.x, acc.v, 0, 0, 0);
      acc.v = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, bv.y, acc.v, 0, 0, 0);
      acc.v = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, bv.z, acc.v, 0, 0, 0);
      acc.v = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, bv.w, acc.v, 0, 0, 0);
    }
  }
  // f(row, column, value) for every element of the 32 x 32 piece this lane holds:
  // register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32
  template <typename F>
  __device__ static void for_each(const Acc &acc, int lane, F f) {
#pragma unroll
    for (int v = 0; v < 16; ++v) f(8 * (v / 4) + 4 * (lane >> 5) + (v % 4), lane & 31, acc.v[v]);
  }
};

// v_mfma_f64_16x16x4_f64 (lane l supplies row or column l%16 at k = l/16).  B is staged [k][c]; the 32x32
// piece of C is 2x2 tiles of 16x16.
template <>
struct Skinny<double> {
  static constexpr int kPanel = 256;
  static constexpr int kTK = 16;
  static constexpr int kV = 2;
  static constexpr int kTP = kTK + 2;
  typedef d2a vec;
  typedef d2u uvec;
  struct Acc {
    d4v v[4];  // v[2*ra + ca]
  };
  __device__ static void clear(Acc &a) {
#pragma unroll
    for (int t = 0; t < 4; ++t) a.v[t] = d4v{0.0, 0.0, 0.0, 0.0};
  }
  __device__ static void stage(double *Bs, const double *__restrict__ B, int64_t ldb, int64_t kp0, int64_t n, int m, int tid) {
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
  __device__ static void multiply(const double *tile, const double *Bs, int koff, int lane, Acc &acc) {
    const int l16 = lane & 15, l4 = lane >> 4;
    const double *bs = &Bs[(koff + l4) * 32 + l16];
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const double a0 = tile[l16 * kTP + 4 * gq + l4];
      const double a1 = tile[(16 + l16) * kTP + 4 * gq + l4];
      const double c0 = bs[(4 * gq) * 32];
      const double c1 = bs[(4 * gq) * 32 + 16];
      acc.v[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, c0, acc.v[0], 0, 0, 0);
      acc.v[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, c1, acc.v[1], 0, 0, 0);
      acc.v[2] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, c0, acc.v[2], 0, 0, 0);
      acc.v[3] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, c1, acc.v[3], 0, 0, 0);
    }
  }
  // element v of tile (ra, ca) is row 16 ra + 4 v + l/16, column 16 ca + l%16
  template <typename F>
  __device__ static void for_each(const Acc &acc, int lane, F f) {
#pragma unroll
    for (int ra = 0; ra < 2; ++ra)
#pragma unroll
      for (int ca = 0; ca < 2; ++ca)
#pragma unroll
        for (int v = 0; v < 4; ++v) f(16 * ra + 4 * v + (lane >> 4), 16 * ca + (lane & 15), acc.v[2 * ra + ca][v]);
  }
};

// Workgroups.  With G = kPanel/32/8 groups of eight row blocks per panel height, panel p is reached by the
// row blocks 0 .. 8G(p+1)-1 (fewer in the last panel): groups 0 .. Gp-1 hold blocks that cross the whole
// panel, the G groups after them the blocks cut by the diagonal.  Ids number the whole groups of all panels
// first and the cut ones last, so that the last, partly filled layer of resident workgroups is made of the
// short ones.
template <typename T>
DASTAC_HD int64_t whole_groups_before(int64_t p) {  // sum of G*q for q < p
  return (int64_t)(Skinny<T>::kPanel / kRB / kWaves) * p * (p - 1) / 2;
}

template <typename T>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(2, 2)))
void trmm_skinny_kernel(int64_t n, int m, const T *__restrict__ U, const T *__restrict__ B, int64_t ldb,
                        T *__restrict__ C, int64_t ldc, int64_t total, int npanels) {
  typedef Skinny<T> S;
  typedef typename S::vec vec;
  constexpr int kPanel = S::kPanel, kTK = S::kTK, kV = S::kV, kTP = S::kTP, kG = kPanel / kRB / kWaves;
  // one tile of zero rows follows the panel: the last tile of a row block may reach past the panel's last row
  __shared__ __attribute__((aligned(16))) T Bs[(kPanel + kTK) * 32];
  __shared__ __attribute__((aligned(16))) T At[kWaves][32 * kTP];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t nblk = ceil_div(n, kRB);

  // workgroup id -> (panel, group of eight row blocks)
  int p;
  int64_t g;
  const int64_t whole = whole_groups_before<T>(npanels);
  if ((int64_t)blockIdx.x < whole) {
    p = (int)((1.0f + sqrtf(1.0f + (8.0f / kG) * (float)blockIdx.x)) * 0.5f);  // largest p with G p(p-1)/2 <= id, about
    while (p > 1 && whole_groups_before<T>(p) > (int64_t)blockIdx.x) --p;
    while (whole_groups_before<T>(p + 1) <= (int64_t)blockIdx.x) ++p;
    g = (int64_t)blockIdx.x - whole_groups_before<T>(p);
  } else {
    const int64_t d = (int64_t)blockIdx.x - whole;
    p = (int)(d / kG);
    g = (int64_t)kG * p + d % kG;
  }
  p = uniform32(p);
  const int64_t kp0 = (int64_t)p * kPanel;
  const int64_t kp1 = kp0 + kPanel < n ? kp0 + kPanel : n;

  S::stage(Bs, B, ldb, kp0, n, m, tid);
  __syncthreads();

  const int64_t reach = (int64_t)(kPanel / kRB) * (p + 1);
  const int64_t nunits = nblk < reach ? nblk : reach;  // row blocks that reach this panel
  const int64_t u = g * kWaves + wave;                 // this wavefront's row block
  if (u >= nunits) return;                             // (no workgroup barrier below this line)

  // loader role inside a tile: rows lr, lr+8, lr+16, lr+24; one 16-byte piece from column lk
  const int lr = lane >> 3, lk = (lane & 7) * kV;
  T *tile = At[wave];

  const int64_t j0 = kRB * u;              // first row of the block
  const int64_t ks = j0 > kp0 ? j0 : kp0;  // first k of this block in this panel
  const int cs0 = (int)(ks - kp0);         // the same, relative to the panel
  const int ntiles = (int)ceil_div(kp1 - ks, kTK);
  const bool rows_full = j0 + kRB <= n;
  // a 16-byte load may start up to kTK-1 elements past the end of its row: the rows of this block end at
  // tri_row_start(n, j0+32) at the latest, which must leave that much room in the packed buffer
  const int64_t jend = j0 + kRB < n ? j0 + kRB : n;
  const bool vec_ok = tri_row_start(n, jend) + kTK <= total;
  // packed row bases for the rows this lane loads: element (j,k) is at U[ro[q] + k]
  int64_t ro[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    int64_t jj = j0 + lr + 8 * q;
    if (jj >= n) jj = n - 1;  // keep the address inside the buffer; values are masked below
    ro[q] = tri_row_start(n, jj) - jj;
  }
  // this lane's piece of the block's first tile, row by row; a tile further on is kTK elements further on
  const T *up[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) up[q] = U + (ro[q] + ks + lk);

  // Scalar loader with every element bounds-tested: only for the last row blocks of the triangle.
  auto load_guarded = [&](int t, vec (&v)[4]) {
    const int64_t k0 = ks + kTK * (int64_t)t;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t j = j0 + lr + 8 * q;
#pragma unroll
      for (int s = 0; s < kV; ++s) {
        const int64_t k = k0 + lk + s;
        v[q][s] = (j < n && k >= j && k < n) ? U[ro[q] + k] : T(0);
      }
    }
  };
  // Branch-free loader for every other tile; a tile index at or past `ntiles` loads the last tile again.
  auto load_vec = [&](int t, vec (&v)[4]) {
    const int toff = kTK * (t < ntiles ? t : ntiles - 1);
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const typename S::uvec *>(up[q] + toff);
  };
  // Zero what a vector-loaded tile holds outside the domain j<=k<n (and of rows j>=n).
  auto mask_tile = [&](int t, vec (&v)[4]) {
    const int64_t kt = ks + kTK * (int64_t)t;
    if (rows_full && kt >= j0 + 31 && kt + kTK <= n) return;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t j = j0 + lr + 8 * q;
      const int64_t lo = j - (kt + lk);               // elements below lo are left of the diagonal
      const int64_t hi = j < n ? n - (kt + lk) : lo;  // elements from hi on are past the row's end
#pragma unroll
      for (int s = 0; s < kV; ++s) v[q][s] = (s >= lo && s < hi) ? v[q][s] : T(0);
    }
  };

  typename S::Acc acc;
  S::clear(acc);

  // one tile: registers -> private LDS tile -> matrix-core operand layout -> 16 matrix instructions
  auto compute = [&](int t, const vec (&v)[4]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) *reinterpret_cast<vec *>(&tile[(lr + 8 * q) * kTP + lk]) = v[q];
    wave_sync_lds();  // the tile is private to this wavefront: no workgroup barrier needed
    S::multiply(tile, Bs, cs0 + kTK * t, lane, acc);
    wave_sync_lds();  // all lanes have read the tile before the next one overwrites it
  };

  vec s0[4], s1[4], s2[4];
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

  S::for_each(acc, lane, [&](int row, int col, T value) {
    const int64_t j = j0 + row;
    if (j < n && col < m) unsafeAtomicAdd(&C[j * ldc + col], value);
  });
}

// C(0..n-1, 0..m-1) := 0, leaving the padding columns of every row alone
template <typename T>
__global__ __launch_bounds__(256) void zero_rows_kernel(T *__restrict__ C, int64_t n, int64_t m, int64_t ldc) {
  const int64_t total = n * m;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t i = t / m;
    C[i * ldc + (t - i * m)] = T(0);
  }
}

template <typename T>
int few_columns(int64_t n, int64_t m, const T *Up, const T *B, int64_t ldb, T *C, int64_t ldc, void *stream) {
  constexpr int kPanel = Skinny<T>::kPanel, kG = kPanel / kRB / kWaves;
  hipStream_t st = (hipStream_t)stream;
  const int64_t zb = ceil_div(n * m, 256);
  zero_rows_kernel<T><<<(unsigned)(zb < 4096 ? zb : 4096), 256, 0, st>>>(C, n, m, ldc);
  if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  const int64_t npanels = ceil_div(n, kPanel);
  const int64_t groups = whole_groups_before<T>(npanels) + kG * npanels;  // the last panel's cut groups may be partly empty
  if (groups > 0x7fffffff) return DASTAC_EOVERFLOW;
  for (int64_t c0 = 0; c0 < m; c0 += 32) {
    const int mb = (int)(m - c0 < 32 ? m - c0 : 32);
    trmm_skinny_kernel<T><<<(unsigned)groups, kBlock, 0, st>>>(n, mb, Up, B + c0, ldb, C + c0, ldc, tri(n), (int)npanels);
    if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  }
  return DASTAC_OK;
}

}  // namespace

// C := U B for m <= 64 columns, 32 at a time (each pass reads the packed triangle once); arguments are
// validated by the caller.
int dastac::trmm_few_columns(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C,
                             int64_t ldc, void *stream) {
  return few_columns<float>(n, m, Up, B, ldb, C, ldc, stream);
}
int dastac::trmm_few_columns(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C,
                             int64_t ldc, void *stream) {
  return few_columns<double>(n, m, Up, B, ldb, C, ldc, stream);
}
