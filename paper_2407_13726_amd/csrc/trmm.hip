// TRMM over a packed upper triangle on the fp32 matrix cores:
//
//   C(i,c) := U(i,k) * B(k,c),  i<=k        U packed row-major, B and C dense row-major
//
// The rule is Table 1's SpMV_UT with a matrix right-hand side; U keeps the packed layout of
// Section 4 (row i holds k=i..n-1 contiguously, starting at tri_row_start(n,i)).
//
// Tiling.  A workgroup (8 wavefronts) owns a 64-row x 128-column tile of C and sweeps k from the
// diagonal of its row block to n in steps of 32.  Per step the 64x32 tile of U (each packed row
// piece is 128 contiguous bytes, at its own 4-byte-aligned offset) and the 32x128 tile of B are
// staged in LDS, double-buffered against the global loads of the next step.  Each wavefront
// computes a 32x32 sub-tile with v_mfma_f32_32x32x2_f32: lanes 0-31 feed k, lanes 32-63 feed k+1.
// Because a sum over k may be taken in any order, lane half h is given the four consecutive k
// values 8t+4h..8t+4h+3 of every group of eight, so its U operand is one 16-byte LDS read.
//
// Only the two k-steps that touch the diagonal (and the ragged last step / last row block) take
// the masked loader, which writes zeros for k<i; every other tile is loaded without predicates.
//
// Load balance: row block b needs (n - 64 b)/32 k-steps, so a workgroup processes the pair
// (b, nb-1-b), and every workgroup does the same amount of work.  Workgroups that share a
// row-block pair (different column blocks) get ids that are equal modulo 8, i.e. land on the
// same XCD, so the packed U rows they both read are fetched from HBM once and hit in that XCD's L2;
// an XCD is given a run of consecutive pairs, which lets its L2 serve the re-reads of B as well.
//
// Few columns give few workgroups (m = 256: one per compute unit), and a compute unit whose only
// workgroup waits at its barrier has nothing else to run.  Then the k-steps of a pair, taken as one
// list (the long block's, then the short block's), are cut into S equal shares, one workgroup each;
// a share covers pieces of at most two row blocks and adds each piece into a zeroed C with
// floating-point atomics.  With S = 1 nothing changes: plain stores, no atomics, no fill.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBM = 64;    // rows of C per workgroup tile
constexpr int kBN = 128;   // columns of C per workgroup tile
constexpr int kKT = 32;    // k-step
constexpr int kUP = kKT + 4;  // LDS pitch of the U tile (floats): 16-byte reads of 8 lanes cover all banks
constexpr int kBlock = 512;

typedef float f16v __attribute__((ext_vector_type(16)));

struct Stage {
  f4a u;     // U: row ur of the tile, four k values
  f4a b[2];  // B: k rows bk and bk+16, four columns each
};

template <bool SPLIT>
__global__ __launch_bounds__(kBlock) void trmm_mfma_kernel(int64_t n, int64_t m, const float *__restrict__ U,
                                                           const float *__restrict__ B, int64_t ldb,
                                                           float *__restrict__ C, int64_t ldc, int nb, int npairs,
                                                           int ncb, int S) {
  __shared__ __attribute__((aligned(16))) float Us[2][kBM * kUP];
  __shared__ __attribute__((aligned(16))) float Bs[2][kKT * kBN];

  // workgroup id -> (row-block pair, column block); ids equal mod 8 share an XCD.  An XCD gets a run of
  // consecutive pairs: their sweeps over k start 64 rows apart and move at the same speed, so the rows
  // of B one of them reads are read again by its neighbour two k-steps later, out of that XCD's L2.
  const int L = blockIdx.x;
  const int xcd = L & 7, slot = L >> 3;
  const int per_pair = SPLIT ? ncb * S : ncb;
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
  const int l32 = lane & 31, h = lane >> 5;

  // staging roles
  const int ur = tid >> 3, uk = (tid & 7) * 4;     // U: row ur, k offset uk
  const int bk = tid >> 5, bc = (tid & 31) * 4;    // B: k row bk (+16), column offset bc
  const int64_t col0 = (int64_t)cb * kBN;
  const bool cols_full = col0 + kBN <= m;

  for (int which = 0; which < 2; ++which) {
    const int blk = which == 0 ? pair : nb - 1 - pair;
    if (which == 1 && blk == pair) break;  // odd number of row blocks: the middle one is alone
    const int64_t i0 = (int64_t)blk * kBM;
    const bool rows_full = i0 + kBM <= n;
    // k-steps [kt_lo, nk) of this row block fall into the share
    const int first = which == 0 ? 0 : steps_a;  // number of the block's step 0 in the pair's list
    const int steps_blk = which == 0 ? steps_a : steps_b;
    // (literal bounds without shares: the compiler then peels the two masked steps off the loop)
    const int kt_lo = SPLIT ? (t_lo > first ? t_lo - first : 0) : 0;
    const int nk = SPLIT ? (t_hi - first < steps_blk ? t_hi - first : steps_blk) : (int)ceil_div(n - i0, kKT);
    if (SPLIT && kt_lo >= nk) continue;

    // per-thread packed row bases: element (i,k) of U is at ubase[i] + k
    const int64_t iu = i0 + ur;
    const bool urow_ok = iu < n;
    const float *ub = U + (urow_ok ? tri_row_start(n, iu) - iu : 0);

    auto load_stage = [&](int kt, Stage &s) {
      const int64_t k0 = i0 + (int64_t)kt * kKT;
      const bool k_full = k0 + kKT <= n;
      if (kt >= 2 && k_full && rows_full) {
        s.u = *reinterpret_cast<const f4u *>(ub + k0 + uk);
      } else {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int64_t k = k0 + uk + e;
          v[e] = (urow_ok && k >= iu && k < n) ? ub[k] : 0.0f;
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
    auto store_stage = [&](int buf, const Stage &s) {
      *reinterpret_cast<f4a *>(&Us[buf][ur * kUP + uk]) = s.u;
#pragma unroll
      for (int q = 0; q < 2; ++q) *reinterpret_cast<f4a *>(&Bs[buf][(bk + 16 * q) * kBN + bc]) = s.b[q];
    };

    f16v acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    // Operands of one group of eight k values: four MFMA steps on the wavefront's 32x32 sub-tile.
    struct Ops {
      f4a a;
      float b0[4];
    };
    auto read_ops = [&](int buf, int t, Ops &o) {
      const float *us = &Us[buf][(wr * 32 + l32) * kUP + 4 * h];
      const float *bs = &Bs[buf][(4 * h) * kBN + wc * 32 + l32];
      o.a = *reinterpret_cast<const f4a *>(us + 8 * t);
#pragma unroll
      for (int q = 0; q < 4; ++q) o.b0[q] = bs[(8 * t + q) * kBN];
    };
    auto mma = [&](const Ops &o) {
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a.x, o.b0[0], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a.y, o.b0[1], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a.z, o.b0[2], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a.w, o.b0[3], acc, 0, 0, 0);
    };

    Stage st;
    Ops oa, ob;
    load_stage(kt_lo, st);
    __syncthreads();  // the previous row block's last reads of buffer 0 are done
    store_stage(0, st);
    __syncthreads();
    read_ops(0, 0, oa);

    // One k-step on LDS buffer `buf` (a literal at both call sites, so every LDS address is a
    // compile-time offset).  The global loads of the next step are in flight throughout; its LDS
    // stores and the workgroup barrier sit BEFORE the last group's matrix instructions, whose
    // operands are already in registers, so the matrix pipe has work while the barrier settles and
    // while the first operands of the next step come back from LDS.
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

    // D layout of the 32x32 tile: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32
    const int64_t col = col0 + wc * 32 + l32;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t i = i0 + wr * 32 + 8 * (v / 4) + 4 * h + (v % 4);
      if (i < n && col < m) {
        if (SPLIT)
          unsafeAtomicAdd(&C[i * ldc + col], acc[v]);
        else
          C[i * ldc + col] = acc[v];
      }
    }
  }
}

// C(0..n-1, 0..m-1) := 0, leaving the padding columns of every row alone
__global__ __launch_bounds__(256) void zero_rows_kernel(float *__restrict__ C, int64_t n, int64_t m, int64_t ldc) {
  const int64_t quads = (m + 3) / 4, total = n * quads;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t i = t / quads, c = (t - i * quads) * 4;
    float *row = C + i * ldc;
    for (int64_t e = c; e < c + 4 && e < m; ++e) row[e] = 0.0f;
  }
}

}  // namespace

extern "C" int dastac_trmm_f32(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C,
                               int64_t ldc, void *stream) {
  if (n < 0 || m < 1 || ldb < m || ldc < m) return DASTAC_EINVAL;
  if (n > (1 << 24) || m > (1 << 24) || ld_too_large(ldb, ldc)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Up || !B || !C) return DASTAC_ENULL;
  const int64_t cb = view_bytes(n, ldc, m, 4);
  if (overlaps(C, cb, Up, tri(n) * 4) || overlaps(C, cb, B, view_bytes(n, ldb, m, 4))) return DASTAC_EALIAS;
  // one contiguous right-hand side is the matrix-vector product
  if (m == 1 && ldb == 1 && ldc == 1) return dastac_trmv_f32(n, Up, B, C, stream);
  // few right-hand sides on a tall triangle: the streaming kernel (one pass over U per 32 columns)
  if (m <= 64 && n >= 1024) return trmm_few_columns(n, m, Up, B, ldb, C, ldc, stream);
  const int nb = (int)ceil_div(n, kBM);
  const int npairs = (nb + 1) / 2;
  const int ncb = (int)ceil_div(m, kBN);
  const int64_t base = (int64_t)8 * ceil_div(npairs, 8) * ncb;
  if (base > 0x7fffffff) return DASTAC_EOVERFLOW;
  hipStream_t st = (hipStream_t)stream;
  // Shares of the k range per pair: the smallest S <= 16, with at least 32 k-steps per share, whose
  // workgroups come in whole layers of two per compute unit (n = 16384: m = 128 58 -> 111 TFLOP/s, m = 384
  // 93 -> 120; n = 8192, m = 256 114).  Where the column blocks alone give one full layer of one workgroup
  // per compute unit (m = 256 at n = 16384) a second layer gains 1 % (0.589 -> 0.582 ms with the clearing
  // of C): not worth giving up plain stores and one writer per element, so S = 1 there.
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return DASTAC_EHIP;
  const int64_t steps = ceil_div(n, kKT) + 2;  // k-steps of a pair, about
  int64_t S = 1;
  if ((double)base / (double)(ceil_div(base, cus) * cus) < 0.95) {
    const int64_t layer = 2 * (int64_t)cus;
    double best = 0.0;
    for (int64_t s = 1; s <= 16 && (s == 1 || steps / s >= 32); ++s) {
      const int64_t wgs = base * s;
      const double fill = (double)wgs / (double)(ceil_div(wgs, layer) * layer);
      if (fill > best + 0.02) best = fill, S = s;
      if (fill >= 0.95) break;
    }
  }
  if (S <= 1) {
    trmm_mfma_kernel<false><<<(unsigned)base, kBlock, 0, st>>>(n, m, Up, B, ldb, C, ldc, nb, npairs, ncb, 1);
    return launch_status();
  }
  const int64_t zb = ceil_div(n * ((m + 3) / 4), 256);
  zero_rows_kernel<<<(unsigned)(zb < 4096 ? zb : 4096), 256, 0, st>>>(C, n, m, ldc);
  if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  trmm_mfma_kernel<true><<<(unsigned)(base * S), kBlock, 0, st>>>(n, m, Up, B, ldb, C, ldc, nb, npairs, ncb, (int)S);
  return launch_status();
}
