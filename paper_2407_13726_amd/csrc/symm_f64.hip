// SYMM over a packed upper triangle in double precision, on the fp64 matrix cores:
//
//   C(i,c) := S(i,k) * B(k,c),   S(i,k) = S(k,i) = U(min(i,k), max(i,k)),   all double
//
// The fp32 SYMM kernel's plan (a workgroup owns a 64 x 128 tile of C and sweeps k over the whole range:
// tiles of packed rows i right of the diagonal block, transposed tiles of packed rows k left of it, a
// scalar loader on the diagonal block; Section 3, "Redundancy map") on the tile shapes of the fp64
// TRMM kernel: k-steps of 16, v_mfma_f64_16x16x4_f64, each wavefront's 32x32 sub-tile as 2x2 tiles of
// 16x16 with four independent accumulators, one double per lane and operand.  A transposed tile is 16
// packed rows k, each contributing the 64 contiguous elements i0..i0+63; it stays transposed in LDS and
// the operand read picks element (k = l/16, i = l%16) from it directly.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBM = 64;    // rows of C per workgroup tile
constexpr int kBN = 128;   // columns of C per workgroup tile
constexpr int kKT = 16;    // k-step
constexpr int kUP = kKT + 2;   // LDS pitch of a row tile [i][k] (doubles)
constexpr int kTP = kBM + 2;   // LDS pitch of a transposed tile [k][i] (doubles)
constexpr int kUS = kBM * kUP;  // doubles per S buffer (>= kKT * kTP)
constexpr int kBlock = 512;
static_assert(kKT * kTP <= kUS, "a transposed tile fits the S buffer");

typedef double d2u __attribute__((ext_vector_type(2), aligned(8)));
typedef double d2a __attribute__((ext_vector_type(2)));
typedef double d4v __attribute__((ext_vector_type(4)));

struct Stage {
  d2a u;     // S: two consecutive elements of one packed row
  d2a b[2];  // B: k rows bk and bk+8, two columns each
};

__global__ __launch_bounds__(kBlock) void symm_f64_kernel(int64_t n, int64_t m, const double *__restrict__ U,
                                                          const double *__restrict__ B, int64_t ldb,
                                                          double *__restrict__ C, int64_t ldc, int nb, int ncb) {
  __shared__ __attribute__((aligned(16))) double Ss[2][kUS];
  __shared__ __attribute__((aligned(16))) double Bs[2][kKT * kBN];

  // workgroup id -> (row block, column block); ids equal mod 8 share an XCD
  const int L = blockIdx.x;
  const int xcd = L & 7, slot = L >> 3;
  const int blk = xcd + 8 * (slot / ncb);
  const int cb = slot % ncb;
  if (blk >= nb) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 2, wc = wave & 3;  // 2x4 wavefronts: 32 rows x 32 columns each
  const int l16 = lane & 15, l4 = lane >> 4;

  // staging roles
  const int ur = tid >> 3, uk = (tid & 7) * 2;     // row tile: row ur, k offset uk
  const int tk = tid >> 5, ti = (tid & 31) * 2;    // transposed tile: packed row tk, i offset ti
  const int bk = tid >> 6, bc = (tid & 63) * 2;    // B: k row bk (+8), column offset bc
  const int64_t col0 = (int64_t)cb * kBN;
  const bool cols_full = col0 + kBN <= m;

  const int64_t i0 = (int64_t)blk * kBM;
  const bool rows_full = i0 + kBM <= n;
  const int nk = (int)ceil_div(n, kKT);
  const int nleft = rows_full ? (int)(i0 / kKT) : 0;  // k-steps [0,nleft) lie wholly left of the diagonal block

  // element (i,k), k>=i, of the packed triangle is at rowbase(i) + k with rowbase(i) = tri_row_start(n,i) - i
  const int64_t iu = i0 + ur;
  const bool urow_ok = iu < n;
  const double *ub = U + (urow_ok ? tri_row_start(n, iu) - iu : 0);
  // transposed tiles: this thread's piece of step kt starts at rowbase(16 kt + tk) + i0 + ti; rowbase moves
  // by 8(2n - 2k - 17) from row k to row k+16, and that step shrinks by 256 per k-step
  int64_t tofs = tri_row_start(n, tk) - tk + i0 + ti;
  int64_t tstep = 8 * (2 * n - 2 * (int64_t)tk - 17);

  auto load_stage = [&](int kt, Stage &s) {
    const int64_t k0 = (int64_t)kt * kKT;
    const bool k_full = k0 + kKT <= n;
    if (kt < nleft) {
      s.u = *reinterpret_cast<const d2u *>(U + tofs);
      tofs += tstep;
      tstep -= 16 * kKT;
    } else if (rows_full && k_full && k0 >= i0 + kBM) {
      s.u = *reinterpret_cast<const d2u *>(ub + k0 + uk);
    } else {
      double v[2];
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int64_t k = k0 + uk + e;
        double t = 0.0;
        if (urow_ok && k < n) t = k >= iu ? ub[k] : U[tri_offset(n, k, iu)];
        v[e] = t;
      }
      s.u = d2a{v[0], v[1]};
    }
    if (k_full && cols_full) {
#pragma unroll
      for (int q = 0; q < 2; ++q) s.b[q] = *reinterpret_cast<const d2u *>(B + (k0 + bk + 8 * q) * ldb + col0 + bc);
    } else {
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int64_t k = k0 + bk + 8 * q;
        double v[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) v[e] = (k < n && col0 + bc + e < m) ? B[k * ldb + col0 + bc + e] : 0.0;
        s.b[q] = d2a{v[0], v[1]};
      }
    }
  };
  auto store_stage = [&](int buf, bool left, const Stage &s) {
    if (left)
      *reinterpret_cast<d2a *>(&Ss[buf][tk * kTP + ti]) = s.u;
    else
      *reinterpret_cast<d2a *>(&Ss[buf][ur * kUP + uk]) = s.u;
#pragma unroll
    for (int q = 0; q < 2; ++q) *reinterpret_cast<d2a *>(&Bs[buf][(bk + 8 * q) * kBN + bc]) = s.b[q];
  };

  d4v acc[4];  // 2x2 tiles of 16x16: acc[2*ra + ca]
#pragma unroll
  for (int t = 0; t < 4; ++t) acc[t] = d4v{0.0, 0.0, 0.0, 0.0};

  // Operands of one group of four k values: lane l supplies row (or column) l%16 at k = l/16.
  struct Ops {
    double a[2], b[2];
  };
  auto read_ops = [&](int buf, bool left, int t, Ops &o) {
    if (left) {
      const double *ss = &Ss[buf][(4 * t + l4) * kTP + wr * 32 + l16];
      o.a[0] = ss[0];
      o.a[1] = ss[16];
    } else {
      const double *ss = &Ss[buf][(wr * 32 + l16) * kUP + 4 * t + l4];
      o.a[0] = ss[0];
      o.a[1] = ss[16 * kUP];
    }
    const double *bs = &Bs[buf][(4 * t + l4) * kBN + wc * 32 + l16];
    o.b[0] = bs[0];
    o.b[1] = bs[16];
  };
  auto mma = [&](const Ops &o) {
    acc[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[0], o.b[0], acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[0], o.b[1], acc[1], 0, 0, 0);
    acc[2] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[1], o.b[0], acc[2], 0, 0, 0);
    acc[3] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[1], o.b[1], acc[3], 0, 0, 0);
  };

  Stage st;
  Ops oa, ob;
  load_stage(0, st);
  store_stage(0, 0 < nleft, st);
  __syncthreads();
  read_ops(0, 0 < nleft, 0, oa);

  // One k-step on LDS buffer `buf`: the next step's global loads are in flight throughout; its LDS stores
  // and the barrier sit before the last group's matrix instructions.
  auto step = [&](int kt, int buf) {
    const bool more = kt + 1 < nk;
    const bool left = kt < nleft, next_left = kt + 1 < nleft;
    if (more) load_stage(kt + 1, st);
    read_ops(buf, left, 1, ob);
    mma(oa);
    read_ops(buf, left, 2, oa);
    mma(ob);
    read_ops(buf, left, 3, ob);
    mma(oa);
    if (more) store_stage(buf ^ 1, next_left, st);
    __syncthreads();
    if (more) read_ops(buf ^ 1, next_left, 0, oa);
    mma(ob);
  };
  for (int kt = 0; kt < nk; kt += 2) {
    step(kt, 0);
    if (kt + 1 < nk) step(kt + 1, 1);
  }

  // D layout of a 16x16 tile: element v of lane l is row 4*v + l/16, column l%16
#pragma unroll
  for (int ra = 0; ra < 2; ++ra)
#pragma unroll
    for (int ca = 0; ca < 2; ++ca) {
      const int64_t col = col0 + wc * 32 + 16 * ca + l16;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int64_t i = i0 + wr * 32 + 16 * ra + 4 * v + l4;
        if (i < n && col < m) C[i * ldc + col] = acc[2 * ra + ca][v];
      }
    }
}

}  // namespace

extern "C" int dastac_symm_f64(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C,
                               int64_t ldc, void *stream) {
  if (n < 0 || m < 1 || ldb < m || ldc < m) return DASTAC_EINVAL;
  if (n > (1 << 24) || m > (1 << 24) || ld_too_large(ldb, ldc)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Up || !B || !C) return DASTAC_ENULL;
  const int64_t cb = view_bytes(n, ldc, m, 8);
  if (overlaps(C, cb, Up, tri(n) * 8) || overlaps(C, cb, B, view_bytes(n, ldb, m, 8))) return DASTAC_EALIAS;
  const int nb = (int)ceil_div(n, kBM);
  const int ncb = (int)ceil_div(m, kBN);
  const int64_t grid = (int64_t)8 * ceil_div(nb, 8) * ncb;
  if (grid > 0x7fffffff) return DASTAC_EOVERFLOW;
  symm_f64_kernel<<<(unsigned)grid, kBlock, 0, (hipStream_t)stream>>>(n, m, Up, B, ldb, C, ldc, nb, ncb);
  return launch_status();
}
