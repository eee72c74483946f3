// SYMM over a packed upper triangle on the fp32 matrix cores:
//
//   C(i,c) := S(i,k) * B(k,c),   S(i,k) = S(k,i) = U(min(i,k), max(i,k))
//
// S is symmetric and only its unique elements are stored, as the packed upper triangle of
// Section 4 (row i holds k=i..n-1 contiguously); an index pair below the diagonal is swapped to
// reach its unique element (Section 3, "Redundancy map").
//
// A workgroup (8 wavefronts) owns a 64-row x 128-column tile of C and sweeps k over the whole
// range 0..n in steps of 32.  Right of its diagonal block the 64x32 tile of S is a tile of packed
// rows i (each piece 128 contiguous bytes), as in the triangular product.  Left of it, S(i,k) is
// U(k,i): the tile is 32 packed rows k, each contributing the 64 contiguous elements i0..i0+63,
// so it arrives transposed, is kept transposed in LDS, and the matrix cores' S operand is read
// from it element by element instead of four at a time.  The two k-steps on the diagonal block
// and every tile of a ragged last row block take a scalar loader that picks U(i,k) or U(k,i)
// element by element.  Each packed element is therefore read twice in total (once as part of a
// row tile, once as part of a column tile), and no atomics are needed: a tile of C has one owner.
//
// Every row block costs the same n/32 k-steps.  Workgroups that share a row block (different
// column blocks) get ids that are equal modulo 8, i.e. land on the same XCD and share its L2.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBM = 64;    // rows of C per workgroup tile
constexpr int kBN = 128;   // columns of C per workgroup tile
constexpr int kKT = 32;    // k-step
constexpr int kUP = kKT + 4;   // LDS pitch of a row tile [i][k]
constexpr int kTP = kBM + 4;   // LDS pitch of a transposed tile [k][i]
constexpr int kUS = kBM * kUP;  // floats per S buffer (>= kKT * kTP)
constexpr int kBlock = 512;
static_assert(kKT * kTP <= kUS, "a transposed tile fits the S buffer");

typedef float f16v __attribute__((ext_vector_type(16)));

struct Stage {
  f4a u;     // S: four consecutive elements of one packed row
  f4a b[2];  // B: k rows bk and bk+16, four columns each
};

__global__ __launch_bounds__(kBlock) void symm_mfma_kernel(int64_t n, int64_t m, const float *__restrict__ U,
                                                           const float *__restrict__ B, int64_t ldb,
                                                           float *__restrict__ C, int64_t ldc, int nb, int ncb) {
  __shared__ __attribute__((aligned(16))) float Ss[2][kUS];
  __shared__ __attribute__((aligned(16))) float Bs[2][kKT * kBN];

  const int L = blockIdx.x;
  const int xcd = L & 7, slot = L >> 3;
  const int blk = xcd + 8 * (slot / ncb);
  const int cb = slot % ncb;
  if (blk >= nb) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 2, wc = wave & 3;  // 2x4 wavefronts: 32 rows x 32 columns each
  const int l32 = lane & 31, h = lane >> 5;

  // staging roles
  const int ur = tid >> 3, uk = (tid & 7) * 4;     // row tile: row ur, k offset uk
  const int tk = tid >> 4, ti = (tid & 15) * 4;    // transposed tile: packed row tk, i offset ti
  const int bk = tid >> 5, bc = (tid & 31) * 4;    // B: k row bk (+16), column offset bc
  const int64_t col0 = (int64_t)cb * kBN;
  const bool cols_full = col0 + kBN <= m;

  const int64_t i0 = (int64_t)blk * kBM;
  const bool rows_full = i0 + kBM <= n;
  const int nk = (int)ceil_div(n, kKT);
  const int nleft = rows_full ? (int)(i0 / kKT) : 0;  // k-steps [0,nleft) lie wholly left of the diagonal block

  // element (i,k), k>=i, of the packed triangle is at rowbase(i) + k with rowbase(i) = tri_row_start(n,i) - i
  const int64_t iu = i0 + ur;
  const bool urow_ok = iu < n;
  const float *ub = U + (urow_ok ? tri_row_start(n, iu) - iu : 0);
  // transposed tiles: this thread's piece of step kt starts at rowbase(32 kt + tk) + i0 + ti; rowbase
  // moves by 16(2n-1) - 32 k - 512 from row k to row k+32
  int64_t tofs = tri_row_start(n, tk) - tk + i0 + ti;
  int64_t tstep = 16 * (2 * n - 1) - 32 * (int64_t)tk - 512;

  auto load_stage = [&](int kt, Stage &s) {
    const int64_t k0 = (int64_t)kt * kKT;
    const bool k_full = k0 + kKT <= n;
    if (kt < nleft) {
      s.u = *reinterpret_cast<const f4u *>(U + tofs);
      tofs += tstep;
      tstep -= 32 * kKT;
    } else if (rows_full && k_full && k0 >= i0 + kBM) {
      s.u = *reinterpret_cast<const f4u *>(ub + k0 + uk);
    } else {
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int64_t k = k0 + uk + e;
        float t = 0.0f;
        if (urow_ok && k < n) t = k >= iu ? ub[k] : U[tri_offset(n, k, iu)];
        v[e] = t;
      }
      s.u = f4a{v[0], v[1], v[2], v[3]};
    }
    if (k_full && cols_full) {
#pragma unroll
      for (int q = 0; q < 2; ++q)
        s.b[q] = *reinterpret_cast<const f4u *>(B + (k0 + bk + 16 * q) * ldb + col0 + bc);
    } else {
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int64_t k = k0 + bk + 16 * q;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (k < n && col0 + bc + e < m) ? B[k * ldb + col0 + bc + e] : 0.0f;
        s.b[q] = f4a{v[0], v[1], v[2], v[3]};
      }
    }
  };
  auto store_stage = [&](int buf, bool left, const Stage &s) {
    if (left)
      *reinterpret_cast<f4a *>(&Ss[buf][tk * kTP + ti]) = s.u;
    else
      *reinterpret_cast<f4a *>(&Ss[buf][ur * kUP + uk]) = s.u;
#pragma unroll
    for (int q = 0; q < 2; ++q) *reinterpret_cast<f4a *>(&Bs[buf][(bk + 16 * q) * kBN + bc]) = s.b[q];
  };

  f16v acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

  // Operands of one group of eight k values: lane half h takes k = 8t+4h .. 8t+4h+3 (a sum over k may
  // be taken in any order), four MFMA steps on the wavefront's 32x32 sub-tile.
  struct Ops {
    float a[4];
    float b0[4];
  };
  auto read_ops = [&](int buf, bool left, int t, Ops &o) {
    if (left) {
      const float *ss = &Ss[buf][(4 * h) * kTP + wr * 32 + l32];
#pragma unroll
      for (int q = 0; q < 4; ++q) o.a[q] = ss[(8 * t + q) * kTP];
    } else {
      const f4a a = *reinterpret_cast<const f4a *>(&Ss[buf][(wr * 32 + l32) * kUP + 4 * h + 8 * t]);
      o.a[0] = a.x, o.a[1] = a.y, o.a[2] = a.z, o.a[3] = a.w;
    }
    const float *bs = &Bs[buf][(4 * h) * kBN + wc * 32 + l32];
#pragma unroll
    for (int q = 0; q < 4; ++q) o.b0[q] = bs[(8 * t + q) * kBN];
  };
  auto mma = [&](const Ops &o) {
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a[q], o.b0[q], acc, 0, 0, 0);
  };

  Stage st;
  Ops oa, ob;
  load_stage(0, st);
  store_stage(0, 0 < nleft, st);
  __syncthreads();
  read_ops(0, 0 < nleft, 0, oa);

  // One k-step on LDS buffer `buf`.  The global loads of the next step are in flight throughout; its
  // LDS stores and the workgroup barrier sit before the last group's matrix instructions, whose
  // operands are already in registers.
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

  // D layout of the 32x32 tile: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32
  const int64_t col = col0 + wc * 32 + l32;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int64_t i = i0 + wr * 32 + 8 * (v / 4) + 4 * h + (v % 4);
    if (i < n && col < m) C[i * ldc + col] = acc[v];
  }
}

}  // namespace

extern "C" int dastac_symm_f32(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C,
                               int64_t ldc, void *stream) {
  if (n < 0 || m < 1 || ldb < m || ldc < m) return DASTAC_EINVAL;
  if (n > (1 << 24) || m > (1 << 24) || ld_too_large(ldb, ldc)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Up || !B || !C) return DASTAC_ENULL;
  const int64_t cb = view_bytes(n, ldc, m, 4);
  if (overlaps(C, cb, Up, tri(n) * 4) || overlaps(C, cb, B, view_bytes(n, ldb, m, 4))) return DASTAC_EALIAS;
  const int nb = (int)ceil_div(n, kBM);
  const int ncb = (int)ceil_div(m, kBN);
  const int64_t grid = (int64_t)8 * ceil_div(nb, 8) * ncb;
  if (grid > 0x7fffffff) return DASTAC_EOVERFLOW;
  symm_mfma_kernel<<<(unsigned)grid, kBlock, 0, (hipStream_t)stream>>>(n, m, Up, B, ldb, C, ldc, nb, ncb);
  return launch_status();
}
