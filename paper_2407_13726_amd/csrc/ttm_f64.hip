// TTM over a packed upper half cube (the paper's running example, Fig. 3) in double precision:
//
//   A(i,j,k) := B(i,j,l) * C(k,l),   i<=j, 0<=l<Q, 0<=k<K,   all double
//
// The layout rule is the fp32 kernel's: pair number p = tri(n,i,j) is row p of both packed buffers, so the
// contraction is one dense product  Ap[p,k] = sum_l Bp[p,l] * C[k,l]  over the packed rows.  Here it runs on
// v_mfma_f64_16x16x4_f64: a workgroup (8 wavefronts, 2 x 4) owns 64 packed rows x 128 values of k and
// sweeps l in steps of 16; both tiles keep l contiguous, and a lane supplies row (or column) l%16 at
// l-offset l/16 of each group of four, one double per operand.  Each wavefront's 32x32 sub-tile is 2x2
// tiles of 16x16 with four independent accumulators.  About two workgroups per compute unit each walk a
// strided set of row blocks with one uninterrupted pipeline, as in the fp32 kernel.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBM = 64;    // packed rows per workgroup tile
constexpr int kBN = 128;   // values of k per workgroup tile
constexpr int kKT = 16;    // step along l
constexpr int kP = kKT + 2;  // LDS pitch (doubles)
constexpr int kBlock = 512;

typedef double d2u __attribute__((ext_vector_type(2), aligned(8)));
typedef double d2a __attribute__((ext_vector_type(2)));
typedef double d4v __attribute__((ext_vector_type(4)));

struct Stage {
  d2a a;     // Bp: row ar of the tile, two l values
  d2a c[2];  // C: rows cr and cr+64 of the tile, two l values
};

__global__ __launch_bounds__(kBlock) void ttm_f64_kernel(int64_t rows, int64_t Q, int64_t K,
                                                         const double *__restrict__ Bp,
                                                         const double *__restrict__ C, int64_t ldc,
                                                         double *__restrict__ Ap, int lanes, int ncb) {
  __shared__ __attribute__((aligned(16))) double As[2][kBM * kP];
  __shared__ __attribute__((aligned(16))) double Cs[2][kBN * kP];

  // workgroup id -> (first row block, block of k); ids equal mod 8 share an XCD
  const int L = blockIdx.x;
  const int xcd = L & 7, slot = L >> 3;
  const int cb = slot % ncb;
  const int64_t rstride = (int64_t)kBM * 8 * lanes;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 2, wc = wave & 3;  // 2x4 wavefronts: 32 rows x 32 values of k each
  const int l16 = lane & 15, l4 = lane >> 4;

  // staging role: tile row tid/8 (and +64 for C), l offset 2*(tid%8)
  const int sr = tid >> 3, sl = (tid & 7) * 2;
  const int64_t c0 = (int64_t)cb * kBN;
  const bool full_c = c0 + kBN <= K;
  const int nk = (int)ceil_div(Q, kKT);

  const double *cp0 = C + (c0 + sr < K ? c0 + sr : K - 1) * ldc;
  const double *cp1 = C + (c0 + sr + 64 < K ? c0 + sr + 64 : K - 1) * ldc;

  struct Cur {  // wave-uniform cursor over the steps of this workgroup: row block, step along l
    int64_t r0;
    int kt;
    bool valid;
  };
  auto next = [&](Cur c) -> Cur {
    if (!c.valid) return c;
    if (c.kt + 1 < nk) {
      c.kt += 1;
    } else {
      c.kt = 0;
      c.r0 += rstride;
      c.valid = c.r0 < rows;
    }
    return c;
  };

  auto load_stage = [&](const Cur &cu, Stage &s) {
    const int64_t l0 = (int64_t)cu.kt * kKT + sl;
    const double *ap = Bp + (cu.r0 + sr < rows ? cu.r0 + sr : rows - 1) * Q;
    if (full_c && cu.r0 + kBM <= rows && (int64_t)cu.kt * kKT + kKT <= Q) {
      s.a = *reinterpret_cast<const d2u *>(ap + l0);
      s.c[0] = *reinterpret_cast<const d2u *>(cp0 + l0);
      s.c[1] = *reinterpret_cast<const d2u *>(cp1 + l0);
    } else {  // ragged edge: zeros outside the operands
      double a[2], u[2], v[2];
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const bool lok = l0 + e < Q;
        a[e] = (lok && cu.r0 + sr < rows) ? ap[l0 + e] : 0.0;
        u[e] = (lok && c0 + sr < K) ? cp0[l0 + e] : 0.0;
        v[e] = (lok && c0 + sr + 64 < K) ? cp1[l0 + e] : 0.0;
      }
      s.a = d2a{a[0], a[1]};
      s.c[0] = d2a{u[0], u[1]};
      s.c[1] = d2a{v[0], v[1]};
    }
  };
  auto store_stage = [&](int buf, const Stage &s) {
    *reinterpret_cast<d2a *>(&As[buf][sr * kP + sl]) = s.a;
    *reinterpret_cast<d2a *>(&Cs[buf][sr * kP + sl]) = s.c[0];
    *reinterpret_cast<d2a *>(&Cs[buf][(sr + 64) * kP + sl]) = s.c[1];
  };

  d4v acc[4];  // 2x2 tiles of 16x16: acc[2*ra + ca]
#pragma unroll
  for (int t = 0; t < 4; ++t) acc[t] = d4v{0.0, 0.0, 0.0, 0.0};

  // Operands of one group of four l values.
  struct Ops {
    double a[2], c[2];
  };
  auto read_ops = [&](int buf, int t, Ops &o) {
    const double *as = &As[buf][(wr * 32 + l16) * kP + 4 * t + l4];
    const double *cs = &Cs[buf][(wc * 32 + l16) * kP + 4 * t + l4];
    o.a[0] = as[0];
    o.a[1] = as[16 * kP];
    o.c[0] = cs[0];
    o.c[1] = cs[16 * kP];
  };
  auto mma = [&](const Ops &o) {
    acc[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[0], o.c[0], acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[0], o.c[1], acc[1], 0, 0, 0);
    acc[2] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[1], o.c[0], acc[2], 0, 0, 0);
    acc[3] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[1], o.c[1], acc[3], 0, 0, 0);
  };

  Cur cc{(int64_t)kBM * (xcd + 8 * (slot / ncb)), 0, true};  // the step being multiplied
  cc.valid = cc.r0 < rows;
  if (!cc.valid) return;
  Cur cl = cc;  // the step being loaded: one ahead
  Stage st;
  Ops oa, ob;
  load_stage(cl, st);
  store_stage(0, st);
  __syncthreads();
  read_ops(0, 0, oa);

  // One step on LDS buffer `buf`.  The global loads of the next step -- of the next row block, at a
  // block's last step -- are in flight throughout; its LDS stores and the workgroup barrier sit before the
  // last group's matrix instructions, whose operands are already in registers.
  auto step = [&](int buf) {
    cl = next(cl);
    const bool more = cl.valid;
    if (more) load_stage(cl, st);
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
    if (cc.kt == nk - 1) {
      // D layout of a 16x16 tile: element v of lane l is row 4*v + l/16, column l%16
#pragma unroll
      for (int ra = 0; ra < 2; ++ra)
#pragma unroll
        for (int ca = 0; ca < 2; ++ca) {
          const int64_t col = c0 + wc * 32 + 16 * ca + l16;
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int64_t r = cc.r0 + wr * 32 + 16 * ra + 4 * v + l4;
            if (r < rows && col < K) Ap[r * K + col] = acc[2 * ra + ca][v];
          }
          acc[2 * ra + ca] = d4v{0.0, 0.0, 0.0, 0.0};
        }
    }
    cc = next(cc);
  };
  for (;;) {
    step(0);
    if (!cc.valid) break;
    step(1);
    if (!cc.valid) break;
  }
}

inline bool uhc_ok(int64_t n, int64_t Q) {
  return n >= 0 && Q >= 1 && n <= (1 << 20) && Q <= (1 << 24) && (n == 0 || tri(n) <= ((int64_t)1 << 40) / Q);
}

}  // namespace

extern "C" int dastac_ttm_ut_f64(int64_t n, int64_t Q, int64_t K, const double *Bp, const double *C, int64_t ldc,
                                 double *Ap, void *stream) {
  if (n < 0 || Q < 1 || K < 1 || ldc < Q) return DASTAC_EINVAL;
  if (!uhc_ok(n, Q) || !uhc_ok(n, K) || ld_too_large(ldc) || K > ((int64_t)1 << 40) / ldc) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Bp || !C || !Ap) return DASTAC_ENULL;
  const int64_t rows = tri(n);
  if (overlaps(Ap, rows * K * 8, Bp, rows * Q * 8) || overlaps(Ap, rows * K * 8, C, view_bytes(K, ldc, Q, 8))) return DASTAC_EALIAS;
  const int64_t nrb = ceil_div(rows, kBM), ncb = ceil_div(K, kBN);
  if (ncb > (1 << 20)) return DASTAC_EOVERFLOW;
  // about two workgroups per compute unit (256 of them), each walking a strided set of row blocks
  int64_t lanes = ceil_div(512, 8 * ncb);
  if (lanes > ceil_div(nrb, 8)) lanes = ceil_div(nrb, 8);
  const int64_t grid = 8 * lanes * ncb;
  ttm_f64_kernel<<<(unsigned)grid, kBlock, 0, (hipStream_t)stream>>>(rows, Q, K, Bp, C, ldc, Ap, (int)lanes, (int)ncb);
  return launch_status();
}
