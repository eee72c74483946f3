// TRMM over a packed upper triangle in double precision, on the fp64 matrix cores:
//
//   C(i,c) := U(i,k) * B(k,c),  i<=k        U packed row-major, B and C dense row-major, all double
//
// The paper's element type is double (Section 6.1); this is the fp32 TRMM kernel's tiling carried over
// to v_mfma_f64_16x16x4_f64.  A workgroup (8 wavefronts) owns a 64-row x 128-column tile of C and
// sweeps k from the diagonal of its row block to n in steps of 16: the 64x16 tile of U (each packed
// row piece is 128 contiguous bytes at its own 8-byte-aligned offset) and the 16x128 tile of B are
// staged in LDS, double-buffered against the global loads of the next step.  Each wavefront computes a
// 32x32 sub-tile as 2x2 tiles of 16x16 with four independent accumulators; per group of four k values
// it reads two U operands and two B operands (one double per lane each: lane l supplies row or
// column l%16 at k = l/16) and issues four matrix instructions.
//
// Only the four k-steps that touch the diagonal block (and ragged edges) take the masked loader, which
// writes zeros for k<i.  Row blocks are processed in pairs (b, nb-1-b) so that every workgroup does
// the same work, and workgroups sharing a pair sit on one XCD, as in the fp32 kernel.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBM = 64;    // rows of C per workgroup tile
constexpr int kBN = 128;   // columns of C per workgroup tile
constexpr int kKT = 16;    // k-step
constexpr int kUP = kKT + 2;  // LDS pitch of the U tile (doubles): the 16 rows of one operand read fall on distinct banks
constexpr int kBlock = 512;
constexpr int kDiagSteps = kBM / kKT;  // k-steps that overlap the diagonal block

typedef double d2u __attribute__((ext_vector_type(2), aligned(8)));
typedef double d2a __attribute__((ext_vector_type(2)));
typedef double d4v __attribute__((ext_vector_type(4)));

struct Stage {
  d2a u;     // U: row ur of the tile, two k values
  d2a b[2];  // B: k rows bk and bk+8, two columns each
};

__global__ __launch_bounds__(kBlock) void trmm_f64_kernel(int64_t n, int64_t m, const double *__restrict__ U,
                                                          const double *__restrict__ B, int64_t ldb,
                                                          double *__restrict__ C, int64_t ldc, int nb, int npairs,
                                                          int ncb) {
  __shared__ __attribute__((aligned(16))) double Us[2][kBM * kUP];
  __shared__ __attribute__((aligned(16))) double Bs[2][kKT * kBN];

  // workgroup id -> (row-block pair, column block); ids equal mod 8 share an XCD
  const int L = blockIdx.x;
  const int xcd = L & 7, slot = L >> 3;
  const int pair = xcd + 8 * (slot / ncb);
  const int cb = slot % ncb;
  if (pair >= npairs) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 2, wc = wave & 3;  // 2x4 wavefronts: 32 rows x 32 columns each
  const int l16 = lane & 15, l4 = lane >> 4;

  // staging roles
  const int ur = tid >> 3, uk = (tid & 7) * 2;     // U: row ur, k offset uk
  const int bk = tid >> 6, bc = (tid & 63) * 2;    // B: k row bk (+8), column offset bc
  const int64_t col0 = (int64_t)cb * kBN;
  const bool cols_full = col0 + kBN <= m;

  for (int which = 0; which < 2; ++which) {
    const int blk = which == 0 ? pair : nb - 1 - pair;
    if (which == 1 && blk == pair) break;  // odd number of row blocks: the middle one is alone
    const int64_t i0 = (int64_t)blk * kBM;
    const bool rows_full = i0 + kBM <= n;
    const int nk = (int)ceil_div(n - i0, kKT);

    // element (i,k) of U is at ub + k for this thread's row i
    const int64_t iu = i0 + ur;
    const bool urow_ok = iu < n;
    const double *ub = U + (urow_ok ? tri_row_start(n, iu) - iu : 0);

    auto load_stage = [&](int kt, Stage &s) {
      const int64_t k0 = i0 + (int64_t)kt * kKT;
      const bool k_full = k0 + kKT <= n;
      if (kt >= kDiagSteps && k_full && rows_full) {
        s.u = *reinterpret_cast<const d2u *>(ub + k0 + uk);
      } else {
        double v[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int64_t k = k0 + uk + e;
          v[e] = (urow_ok && k >= iu && k < n) ? ub[k] : 0.0;
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
    auto store_stage = [&](int buf, const Stage &s) {
      *reinterpret_cast<d2a *>(&Us[buf][ur * kUP + uk]) = s.u;
#pragma unroll
      for (int q = 0; q < 2; ++q) *reinterpret_cast<d2a *>(&Bs[buf][(bk + 8 * q) * kBN + bc]) = s.b[q];
    };

    d4v acc[4];  // 2x2 tiles of 16x16: acc[2*ra + ca]
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = d4v{0.0, 0.0, 0.0, 0.0};

    // Operands of one group of four k values.
    struct Ops {
      double a[2], b[2];
    };
    auto read_ops = [&](int buf, int t, Ops &o) {
      const double *us = &Us[buf][(wr * 32 + l16) * kUP + 4 * t + l4];
      const double *bs = &Bs[buf][(4 * t + l4) * kBN + wc * 32 + l16];
      o.a[0] = us[0];
      o.a[1] = us[16 * kUP];
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
    __syncthreads();  // the previous row block's last reads of buffer 0 are done
    store_stage(0, st);
    __syncthreads();
    read_ops(0, 0, oa);

    // One k-step on LDS buffer `buf`: the next step's global loads are in flight throughout; its LDS
    // stores and the barrier sit before the last group's matrix instructions, whose operands are
    // already in registers.
    auto step = [&](int kt, int buf) {
      const bool more = kt + 1 < nk;
      if (more) load_stage(kt + 1, st);
      read_ops(buf, 1, ob);
      mma(oa);
      read_ops(buf, 2, oa);
      mma(ob);
      read_ops(buf, 3, ob);
      mma(oa);
      if (more) store_stage(buf ^ 1, st);
      __syncthreads();
      if (more) read_ops(buf ^ 1, 0, oa);
      mma(ob);
    };
    for (int kt = 0; kt < nk; kt += 2) {
      step(kt, 0);
      if (kt + 1 < nk) step(kt + 1, 1);
    }
    __syncthreads();  // all reads of this row block's buffers are done before the next block's stores

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
}

}  // namespace

extern "C" int dastac_trmm_f64(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C,
                               int64_t ldc, void *stream) {
  if (n < 0 || m < 1 || ldb < m || ldc < m) return DASTAC_EINVAL;
  if (n > (1 << 24) || m > (1 << 24)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Up || !B || !C) return DASTAC_ENULL;
  if (overlaps(C, n * ldc * 8, Up, tri(n) * 8) || overlaps(C, n * ldc * 8, B, n * ldb * 8)) return DASTAC_EALIAS;
  const int nb = (int)ceil_div(n, kBM);
  const int npairs = (nb + 1) / 2;
  const int ncb = (int)ceil_div(m, kBN);
  const int64_t grid = (int64_t)8 * ceil_div(npairs, 8) * ncb;
  if (grid > 0x7fffffff) return DASTAC_EOVERFLOW;
  trmm_f64_kernel<<<(unsigned)grid, kBlock, 0, (hipStream_t)stream>>>(n, m, Up, B, ldb, C, ldc, nb, npairs, ncb);
  return launch_status();
}
