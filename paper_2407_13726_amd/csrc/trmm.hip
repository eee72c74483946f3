// TRMM over a packed upper triangle on the matrix cores, single and double precision:
//
//   C(i,c) := U(i,k) * B(k,c),  i<=k        U packed row-major, B and C dense row-major
//
// The rule is Table 1's SpMV_UT with a matrix right-hand side; U keeps the packed layout of
// Section 4 (row i holds k=i..n-1 contiguously, starting at tri_row_start(n,i)).
//
// Tiling.  A workgroup (8 wavefronts) owns a 64-row x 128-column tile of C and sweeps k from the
// diagonal of its row block to n in steps of 32 (fp32) or 16 (fp64: the paper's element type, Section
// 6.1).  Per step the 64 x kKT tile of U (each packed row piece is 128 contiguous bytes, at its own
// element-aligned offset) and the kKT x 128 tile of B are staged in LDS, double-buffered against the
// global loads of the next step, and each wavefront multiplies its 32x32 sub-tile.  The sweep and the
// per-type matrix-core pieces are those of mfma_tile.h (v_mfma_f32_32x32x2_f32, with the k values dealt
// to the lane halves so that the U operand is one 16-byte LDS read; v_mfma_f64_16x16x4_f64 on 2x2 tiles
// of 16x16); this file adds what is TRMM's own: the packed row bases, the masked diagonal steps, the
// pairing of row blocks, the XCD numbering and the shares.
//
// Only the k-steps that touch the diagonal block (and the ragged last step / last row block) take
// the masked loader, which writes zeros for k<i; every other tile is loaded without predicates, and those
// steps run as a sweep of their own whose loop holds no test of the kind of step (benchmark shape: 585 -> 565 us).
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
#include "mfma_tile.h"

using namespace dastac;

namespace {

template <typename T>
struct Stage {
  typename Core<T>::vec u;     // U: row ur of the tile, one 16-byte piece of k values
  typename Core<T>::vec b[2];  // B: k rows bk and bk + kKT/2, one 16-byte piece of columns each
};

// PIN: the sweep's instructions stay in the written order (mfma_tile.h); chosen where two workgroups share a CU.
// The three sweeps of a whole tile (below) take the kernel past 128 registers.  Every launch but the one with a
// single workgroup per CU (fp32, no shares, unpinned) wants two workgroups on a CU, so those instantiations are
// held to the 128 registers of four wavefronts per SIMD; the few spilled values cost less than the second
// workgroup brings (fp32 with shares, which had silently been running one workgroup per CU at 134 registers:
// n=16384, m=384 0.92 -> 0.83 ms).
template <typename T, bool SPLIT, bool PIN>
__global__ __launch_bounds__(kTileThreads) __attribute__((amdgpu_waves_per_eu((SPLIT || PIN || sizeof(T) == 8) ? 4 : 1)))
void trmm_mfma_kernel(int64_t n, int64_t m, const T *__restrict__ U,
                                                                 const T *__restrict__ B, int64_t ldb,
                                                                 T *__restrict__ C, int64_t ldc, int nb, int npairs,
                                                                 int ncb, int S) {
  typedef Core<T> K;
  typedef typename K::vec vec;
  typedef typename K::uvec uvec;
  constexpr int kBM = kTileM, kBN = kTileN, kKT = K::kKT, kV = K::kVec, kUP = K::kRowPitch;
  constexpr int kDiagSteps = kBM / kKT;  // k-steps that overlap the diagonal block
  __shared__ __attribute__((aligned(16))) T Us[2][kBM * kUP];
  __shared__ __attribute__((aligned(16))) T Bs[2][kKT * kBN];

  // workgroup id -> (row-block pair, column block); ids equal mod 8 share an XCD.  An XCD gets a run of
  // consecutive pairs: their sweeps over k start 64 rows apart and move at the same speed, so the rows
  // of B one of them reads are read again by its neighbour a few k-steps later, out of that XCD's L2.
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

  // staging roles: eight threads per row of the U tile, 128/kV per row of the B tile
  const int ur = tid >> 3, uk = (tid & 7) * kV;                       // U: row ur, k offset uk
  const int bk = tid / (kBN / kV), bc = (tid % (kBN / kV)) * kV;      // B: k row bk (and bk + kKT/2), column offset bc
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
    // (literal bounds without shares: the first sweep below then has a compile-time trip count)
    const int kt_lo = SPLIT ? (t_lo > first ? t_lo - first : 0) : 0;
    const int nk = SPLIT ? (t_hi - first < steps_blk ? t_hi - first : steps_blk) : (int)ceil_div(n - i0, kKT);
    if (SPLIT && kt_lo >= nk) continue;

    // per-thread packed row base: element (i,k) of U is at ub + k for this thread's row i
    const int64_t iu = i0 + ur;
    const bool urow_ok = iu < n;
    const T *ub = U + (urow_ok ? tri_row_start(n, iu) - iu : 0);

    auto load_stage = [&](int kt, Stage<T> &s) {
      const int64_t k0 = i0 + (int64_t)kt * kKT;
      const bool k_full = k0 + kKT <= n;
      if (kt >= kDiagSteps && k_full && rows_full) {
        s.u = *reinterpret_cast<const uvec *>(ub + k0 + uk);
      } else {
#pragma unroll
        for (int e = 0; e < kV; ++e) {
          const int64_t k = k0 + uk + e;
          s.u[e] = (urow_ok && k >= iu && k < n) ? ub[k] : T(0);
        }
      }
      if (k_full && cols_full) {
#pragma unroll
        for (int q = 0; q < 2; ++q)
          s.b[q] = *reinterpret_cast<const uvec *>(B + (k0 + bk + (kKT / 2) * q) * ldb + col0 + bc);
      } else {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int64_t k = k0 + bk + (kKT / 2) * q;
#pragma unroll
          for (int e = 0; e < kV; ++e) s.b[q][e] = (k < n && col0 + bc + e < m) ? B[k * ldb + col0 + bc + e] : T(0);
        }
      }
    };
    auto store_stage = [&](int buf, int, const Stage<T> &s) {
      *reinterpret_cast<vec *>(&Us[buf][ur * kUP + uk]) = s.u;
#pragma unroll
      for (int q = 0; q < 2; ++q) *reinterpret_cast<vec *>(&Bs[buf][(bk + (kKT / 2) * q) * kBN + bc]) = s.b[q];
    };
    auto read_ops = [&](int buf, int, int t, typename K::Ops &o) {
      K::read_a(&Us[buf][wr * 32 * kUP], lane, t, o);
      K::read_b(&Bs[buf][wc * 32], kBN, lane, t, o);
    };

    typename K::Acc acc;
    K::clear(acc);
    __syncthreads();  // the previous row block's last reads of buffer 0 are done
    if (rows_full && cols_full) {
      // A whole tile: the masked steps on the diagonal block, the whole steps behind it and a ragged last step are
      // three sweeps, so that the long one carries no test of which kind of step it is on.
      const int nfull = (int)((n - i0) / kKT);
      const int a_hi = nk < kDiagSteps ? nk : kDiagSteps;
      const int b_lo = kt_lo > kDiagSteps ? kt_lo : kDiagSteps, b_hi = nk < nfull ? nk : nfull;
      const int c_lo = kt_lo > nfull ? kt_lo : nfull;
      bool between = false;  // a sweep has run: barrier before the next one reuses the buffers
      if (kt_lo < a_hi) {
        sweep_steps<T, Stage<T>, PIN>(kt_lo, a_hi, acc, load_stage, store_stage, read_ops);
        between = true;
      }
      if (b_lo < b_hi) {
        if (between) __syncthreads();
        sweep_steps<T, Stage<T>, PIN>(
            b_lo, b_hi, acc,
            [&](int kt, Stage<T> &s) {
              const int64_t k0 = i0 + (int64_t)kt * kKT;
              s.u = *reinterpret_cast<const uvec *>(ub + k0 + uk);
#pragma unroll
              for (int q = 0; q < 2; ++q)
                s.b[q] = *reinterpret_cast<const uvec *>(B + (k0 + bk + (kKT / 2) * q) * ldb + col0 + bc);
            },
            store_stage, read_ops);
        between = true;
      }
      if (c_lo < nk) {
        if (between) __syncthreads();
        sweep_steps<T, Stage<T>, PIN>(c_lo, nk, acc, load_stage, store_stage, read_ops);
      }
    } else {
      sweep_steps<T, Stage<T>, PIN>(kt_lo, nk, acc, load_stage, store_stage, read_ops);
    }
    __syncthreads();  // all reads of this row block's buffers are done before the next block's stores

    K::for_each(acc, lane, [&](int r, int c, T v) {
      const int64_t i = i0 + wr * 32 + r, col = col0 + wc * 32 + c;
      if (i < n && col < m) {
        if (SPLIT)
          unsafeAtomicAdd(&C[i * ldc + col], v);
        else
          C[i * ldc + col] = v;
      }
    });
  }
}

inline int trmv_contiguous(int64_t n, const float *Up, const float *x, float *y, void *stream) {
  return dastac_trmv_f32(n, Up, x, y, stream);
}
inline int trmv_contiguous(int64_t n, const double *Up, const double *x, double *y, void *stream) {
  return dastac_trmv_f64(n, Up, x, y, stream);
}

template <typename T>
int run(int64_t n, int64_t m, const T *Up, const T *B, int64_t ldb, T *C, int64_t ldc, void *stream) {
  constexpr int kBM = kTileM, kBN = kTileN, kKT = Core<T>::kKT, kBlock = kTileThreads;
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (n < 0 || m < 1 || ldb < m || ldc < m) return DASTAC_EINVAL;
  if (n > (1 << 24) || m > (1 << 24) || ld_too_large(ldb, ldc)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Up || !B || !C) return DASTAC_ENULL;
  const int64_t cb = view_bytes(n, ldc, m, kB);
  if (overlaps(C, cb, Up, tri(n) * kB) || overlaps(C, cb, B, view_bytes(n, ldb, m, kB))) return DASTAC_EALIAS;
  // one contiguous right-hand side is the matrix-vector product
  if (m == 1 && ldb == 1 && ldc == 1) return trmv_contiguous(n, Up, B, C, stream);
  // few right-hand sides on a tall triangle: the streaming kernel (one pass over U per 32 columns)
  if (m <= 64 && n >= 1024) return trmm_few_columns(n, m, Up, B, ldb, C, ldc, stream);
  const int nb = (int)ceil_div(n, kBM);
  const int npairs = (nb + 1) / 2;
  const int ncb = (int)ceil_div(m, kBN);
  const int64_t base = (int64_t)8 * ceil_div(npairs, 8) * ncb;
  if (base > 0x7fffffff) return DASTAC_EOVERFLOW;
  hipStream_t st = (hipStream_t)stream;
  // Shares of the k range per pair: the smallest S <= 16, with at least 32 k-steps per share, whose
  // workgroups come in whole layers of two per compute unit (fp32, n = 16384: m = 128 58 -> 111 TFLOP/s, m = 384
  // 93 -> 120; n = 8192, m = 256 114).  In fp32, where the column blocks alone give one full layer of one
  // workgroup per compute unit (m = 256 at n = 16384), a second layer gains nothing (0.57 ms either way, the
  // clearing of C included): no reason to give up plain stores and one writer per element, so S = 1 there.  In fp64 the
  // second layer pays at every shape measured (n = 16384: m = 256 1.19 -> 1.12 ms, m = 128 0.63 -> 0.59;
  // n = 8192, m = 256 0.32 -> 0.29), so there is no such exception; with two shares an element of C still gets
  // at most two addends, whose sum does not depend on their order.
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return DASTAC_EHIP;
  const int64_t steps = ceil_div(n, kKT) + kBM / kKT;  // k-steps of a pair, about
  const bool one_layer_is_enough = sizeof(T) == 4 && (double)base / (double)(ceil_div(base, cus) * cus) >= 0.95;
  int64_t S = 1;
  if (!one_layer_is_enough) {
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
    // workgroups that share a compute unit (n = 16384: m >= 512): the pinned schedule, 0.76 -> 0.82 of peak there
    if (sizeof(T) == 4 && base > cus)
      trmm_mfma_kernel<T, false, true><<<(unsigned)base, kBlock, 0, st>>>(n, m, Up, B, ldb, C, ldc, nb, npairs, ncb, 1);
    else
      trmm_mfma_kernel<T, false, false><<<(unsigned)base, kBlock, 0, st>>>(n, m, Up, B, ldb, C, ldc, nb, npairs, ncb, 1);
    return launch_status();
  }
  const int64_t zb = ceil_div(n * ceil_div(m, 16 / kB), 256);
  zero_matrix_kernel<T><<<(unsigned)(zb < 4096 ? zb : 4096), 256, 0, st>>>(C, n, m, ldc);
  if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
  trmm_mfma_kernel<T, true, false><<<(unsigned)(base * S), kBlock, 0, st>>>(n, m, Up, B, ldb, C, ldc, nb, npairs, ncb, (int)S);
  return launch_status();
}

}  // namespace

extern "C" int dastac_trmm_f32(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C,
                               int64_t ldc, void *stream) {
  return run<float>(n, m, Up, B, ldb, C, ldc, stream);
}

// Double precision (the paper's element type): the same kernel on the fp64 matrix cores.
extern "C" int dastac_trmm_f64(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C,
                               int64_t ldc, void *stream) {
  return run<double>(n, m, Up, B, ldb, C, ldc, stream);
}
