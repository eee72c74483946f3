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

template <bool SPLIT>
__global__ __launch_bounds__(kBlock) void trmm_f64_kernel(int64_t n, int64_t m, const double *__restrict__ U,
                                                          const double *__restrict__ B, int64_t ldb,
                                                          double *__restrict__ C, int64_t ldc, int nb, int npairs,
                                                          int ncb, int S) {
  __shared__ __attribute__((aligned(16))) double Us[2][kBM * kUP];
  __shared__ __attribute__((aligned(16))) double Bs[2][kKT * kBN];

  // workgroup id -> (row-block pair, column block); ids equal mod 8 share an XCD
  const int L = blockIdx.x;
  const int xcd = L & 7, slot = L >> 3;
  const int per_pair = SPLIT ? ncb * S : ncb;
  // an XCD gets a run of consecutive pairs: neighbouring sweeps read the same rows of B four k-steps apart,
  // out of that XCD's L2
  const int pair_lo = (int)((int64_t)npairs * xcd / 8), pair_hi = (int)((int64_t)npairs * (xcd + 1) / 8);
  const int pair = pair_lo + slot / per_pair;
  const int cb = SPLIT ? (slot % per_pair) / S : slot % ncb;
  const int share = SPLIT ? slot % S : 0;
  if (pair >= pair_hi) return;
  // this workgroup's share [t_lo, t_hi) of the pair's k-steps, numbered through both row blocks
  const int steps_a = (int)ceil_div(n - (int64_t)pair * kBM, kKT);
  const int steps_b = (nb - 1 - pair != pair) ? (int)ceil_div(n - (int64_t)(nb - 1 - pair) * kBM, kKT) : 0;
  const int t_lo = SPLIT ? (int)((int64_t)(steps_a + steps_b) * share / S) : 0;
  const int t_hi = SPLIT ? (int)((int64_t)(steps_a + steps_b) * (share + 1) / S) : steps_a + steps_b;

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
    // k-steps [kt_lo, nk) of this row block fall into the share (literal bounds without shares, so that
    // the compiler peels the masked diagonal steps off the loop)
    const int first = which == 0 ? 0 : steps_a;  // number of the block's step 0 in the pair's list
    const int steps_blk = which == 0 ? steps_a : steps_b;
    const int kt_lo = SPLIT ? (t_lo > first ? t_lo - first : 0) : 0;
    const int nk = SPLIT ? (t_hi - first < steps_blk ? t_hi - first : steps_blk) : (int)ceil_div(n - i0, kKT);
    if (SPLIT && kt_lo >= nk) continue;

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
    load_stage(kt_lo, st);
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
    for (int kt = kt_lo; kt < nk; kt += 2) {
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
          if (i < n && col < m) {
            if (SPLIT)
              unsafeAtomicAdd(&C[i * ldc + col], acc[2 * ra + ca][v]);
            else
              C[i * ldc + col] = acc[2 * ra + ca][v];
          }
        }
      }
  }
}

// C(0..n-1, 0..m-1) := 0, leaving the padding columns of every row alone
__global__ __launch_bounds__(256) void zero_rows_kernel(double *__restrict__ C, int64_t n, int64_t m, int64_t ldc) {
  const int64_t pairs = (m + 1) / 2, total = n * pairs;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t i = t / pairs, c = (t - i * pairs) * 2;
    double *row = C + i * ldc;
    for (int64_t e = c; e < c + 2 && e < m; ++e) row[e] = 0.0;
  }
}

}  // namespace

extern "C" int dastac_trmm_f64(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C,
                               int64_t ldc, void *stream) {
  if (n < 0 || m < 1 || ldb < m || ldc < m) return DASTAC_EINVAL;
  if (n > (1 << 24) || m > (1 << 24) || ld_too_large(ldb, ldc)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Up || !B || !C) return DASTAC_ENULL;
  const int64_t cb = view_bytes(n, ldc, m, 8);
  if (overlaps(C, cb, Up, tri(n) * 8) || overlaps(C, cb, B, view_bytes(n, ldb, m, 8))) return DASTAC_EALIAS;
  // one contiguous right-hand side is the matrix-vector product
  if (m == 1 && ldb == 1 && ldc == 1) return dastac_trmv_f64(n, Up, B, C, stream);
  // few right-hand sides on a tall triangle: the streaming kernel (one pass over U per 32 columns)
  if (m <= 64 && n >= 1024) return trmm_few_columns(n, m, Up, B, ldb, C, ldc, stream);
  const int nb = (int)ceil_div(n, kBM);
  const int npairs = (nb + 1) / 2;
  const int ncb = (int)ceil_div(m, kBN);
  const int64_t base = (int64_t)8 * ceil_div(npairs, 8) * ncb;
  if (base > 0x7fffffff) return DASTAC_EOVERFLOW;
  hipStream_t st = (hipStream_t)stream;
  // Shares of the k range per pair, as in the fp32 entry point: the smallest S <= 16, with at least 32
  // k-steps per share, whose workgroups come in whole layers of two per compute unit.  Unlike fp32 the second
  // layer pays at every shape measured (n = 16384: m = 256 1.19 -> 1.12 ms, m = 128 0.63 -> 0.59; n = 8192,
  // m = 256 0.32 -> 0.29), so there is no single-layer exception; with two shares an element of C still gets
  // at most two addends, whose sum does not depend on their order.
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return DASTAC_EHIP;
  const int64_t layer = 2 * (int64_t)cus, steps = ceil_div(n, kKT) + 4;
  int64_t S = 1;
  double best = 0.0;
  for (int64_t s = 1; s <= 16 && (s == 1 || steps / s >= 32); ++s) {
    const int64_t wgs = base * s;
    const double fill = (double)wgs / (double)(ceil_div(wgs, layer) * layer);
    if (fill > best + 0.02) best = fill, S = s;
    if (fill >= 0.95) break;
  }
  if (S <= 1) {
    trmm_f64_kernel<false><<<(unsigned)base, kBlock, 0, st>>>(n, m, Up, B, ldb, C, ldc, nb, npairs, ncb, 1);
    return launch_status();
  }
  const int64_t zb = ceil_div(n * ((m + 1) / 2), 256);
  zero_rows_kernel<<<(unsigned)(zb < 4096 ? zb : 4096), 256, 0, st>>>(C, n, m, ldc);
  if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  trmm_f64_kernel<true><<<(unsigned)(base * S), kBlock, 0, st>>>(n, m, Up, B, ldb, C, ldc, nb, npairs, ncb, (int)S);
  return launch_status();
}
