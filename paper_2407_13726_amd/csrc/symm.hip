// SYMM over a packed upper triangle on the matrix cores, single and double precision:
//
//   C(i,c) := S(i,k) * B(k,c),   S(i,k) = S(k,i) = U(min(i,k), max(i,k))
//
// S is symmetric and only its unique elements are stored, as the packed upper triangle of
// Section 4 (row i holds k=i..n-1 contiguously); an index pair below the diagonal is swapped to
// reach its unique element (Section 3, "Redundancy map").
//
// A workgroup (8 wavefronts) owns a 64-row x 128-column tile of C and sweeps k over the whole
// range 0..n in steps of kKT = 32 (fp32) or 16 (fp64), with the sweep and the per-type matrix-core
// pieces of mfma_tile.h.  Right of its diagonal block the 64 x kKT tile of S is a tile of packed
// rows i (each piece 128 contiguous bytes), as in the triangular product.  Left of it, S(i,k) is
// U(k,i): the tile is kKT packed rows k, each contributing the 64 contiguous elements i0..i0+63,
// so it arrives transposed, is kept transposed in LDS, and the matrix cores' S operand is read
// from it element by element (in fp32: instead of four at a time).  The k-steps on the diagonal block
// and every tile of a ragged last row block take a scalar loader that picks U(i,k) or U(k,i)
// element by element.  The steps left of the diagonal block, those right of it and the few in between
// run as three sweeps with their own loaders, so neither long sweep tests which kind of tile it is on
// (fp32 +7 %, fp64 +16 % against one sweep with the tests inside).  Each packed element is therefore read twice in total (once as part of a
// row tile, once as part of a column tile), and no atomics are needed: a tile of C has one owner.
//
// Every row block costs the same n/kKT k-steps.  Workgroups that share a row block (different
// column blocks) get ids that are equal modulo 8, i.e. land on the same XCD and share its L2.
#include "mfma_tile.h"

using namespace dastac;

namespace {

template <typename T>
struct Stage {
  typename Core<T>::vec u;     // S: one 16-byte piece of one packed row
  typename Core<T>::vec b[2];  // B: k rows bk and bk + kKT/2, one 16-byte piece of columns each
};

// (In double the three sweeps want 142 registers, which would leave a CU one workgroup; capped at the 128 of
// two workgroups per CU the kernel is 8 % faster, 23 spilled registers included.)
template <typename T>
__global__ __launch_bounds__(kTileThreads) __attribute__((amdgpu_waves_per_eu(sizeof(T) == 8 ? 4 : 1)))
void symm_mfma_kernel(int64_t n, int64_t m, const T *__restrict__ U,
                                                                 const T *__restrict__ B, int64_t ldb,
                                                                 T *__restrict__ C, int64_t ldc, int nb, int ncb) {
  typedef Core<T> K;
  typedef typename K::vec vec;
  typedef typename K::uvec uvec;
  constexpr int kBM = kTileM, kBN = kTileN, kKT = K::kKT, kV = K::kVec;
  constexpr int kUP = K::kRowPitch;  // pitch of a row tile [i][k]
  constexpr int kTP = K::kColPitch;  // pitch of a transposed tile [k][i]
  constexpr int kUS = kBM * kUP;     // elements per S buffer
  static_assert(kKT * kTP <= kUS, "a transposed tile fits the S buffer");
  __shared__ __attribute__((aligned(16))) T Ss[2][kUS];
  __shared__ __attribute__((aligned(16))) T Bs[2][kKT * kBN];

  const int L = blockIdx.x;
  const int xcd = L & 7, slot = L >> 3;
  const int blk = xcd + 8 * (slot / ncb);
  const int cb = slot % ncb;
  if (blk >= nb) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 2, wc = wave & 3;  // 2x4 wavefronts: 32 rows x 32 columns each

  // staging roles
  const int ur = tid >> 3, uk = (tid & 7) * kV;                     // row tile: row ur, k offset uk
  const int tk = tid / (kBM / kV), ti = (tid % (kBM / kV)) * kV;    // transposed tile: packed row tk, i offset ti
  const int bk = tid / (kBN / kV), bc = (tid % (kBN / kV)) * kV;    // B: k row bk (and bk + kKT/2), column offset bc
  const int64_t col0 = (int64_t)cb * kBN;
  const bool cols_full = col0 + kBN <= m;

  const int64_t i0 = (int64_t)blk * kBM;
  const bool rows_full = i0 + kBM <= n;
  const int nk = (int)ceil_div(n, kKT);
  const int nleft = rows_full ? (int)(i0 / kKT) : 0;  // k-steps [0,nleft) lie wholly left of the diagonal block

  // element (i,k), k>=i, of the packed triangle is at rowbase(i) + k with rowbase(i) = tri_row_start(n,i) - i
  const int64_t iu = i0 + ur;
  const bool urow_ok = iu < n;
  const T *ub = U + (urow_ok ? tri_row_start(n, iu) - iu : 0);
  // transposed tiles: this thread's piece of step kt starts at rowbase(kKT kt + tk) + i0 + ti; rowbase moves
  // by kKT (2n - 2k - 1 - kKT) / 2 from row k to row k + kKT, and that step shrinks by kKT^2 per k-step
  int64_t tofs = tri_row_start(n, tk) - tk + i0 + ti;
  int64_t tstep = (kKT / 2) * (2 * n - 2 * (int64_t)tk - 1 - kKT);

  auto load_stage = [&](int kt, Stage<T> &s) {
    const int64_t k0 = (int64_t)kt * kKT;
    const bool k_full = k0 + kKT <= n;
    if (kt < nleft) {
      s.u = *reinterpret_cast<const uvec *>(U + tofs);
      tofs += tstep;
      tstep -= kKT * kKT;
    } else if (rows_full && k_full && k0 >= i0 + kBM) {
      s.u = *reinterpret_cast<const uvec *>(ub + k0 + uk);
    } else {
#pragma unroll
      for (int e = 0; e < kV; ++e) {
        const int64_t k = k0 + uk + e;
        T t = T(0);
        if (urow_ok && k < n) t = k >= iu ? ub[k] : U[tri_offset(n, k, iu)];
        s.u[e] = t;
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
  auto store_stage = [&](int buf, int kt, const Stage<T> &s) {
    if (kt < nleft)
      *reinterpret_cast<vec *>(&Ss[buf][tk * kTP + ti]) = s.u;
    else
      *reinterpret_cast<vec *>(&Ss[buf][ur * kUP + uk]) = s.u;
#pragma unroll
    for (int q = 0; q < 2; ++q) *reinterpret_cast<vec *>(&Bs[buf][(bk + (kKT / 2) * q) * kBN + bc]) = s.b[q];
  };
  auto read_ops = [&](int buf, int kt, int t, typename K::Ops &o) {
    if (kt < nleft)
      K::read_a_t(&Ss[buf][wr * 32], kTP, lane, t, o);
    else
      K::read_a(&Ss[buf][wr * 32 * kUP], lane, t, o);
    K::read_b(&Bs[buf][wc * 32], kBN, lane, t, o);
  };

  typename K::Acc acc;
  K::clear(acc);
  if (rows_full && cols_full) {
    // A whole tile away from the ragged edges: the steps left of the diagonal block, the steps right of it and
    // the few in between are three sweeps, so that the two long ones carry one kind of tile each and none of
    // the tests that tell the kinds apart.
    const int nmid = (int)((i0 + kBM) / kKT);  // first step wholly right of the diagonal block
    const int nfull = (int)(n / kKT);           // steps [nmid, nfull) are whole
    auto load_b = [&](int64_t k0, Stage<T> &s) {
#pragma unroll
      for (int q = 0; q < 2; ++q)
        s.b[q] = *reinterpret_cast<const uvec *>(B + (k0 + bk + (kKT / 2) * q) * ldb + col0 + bc);
    };
    auto store_b = [&](int buf, const Stage<T> &s) {
#pragma unroll
      for (int q = 0; q < 2; ++q) *reinterpret_cast<vec *>(&Bs[buf][(bk + (kKT / 2) * q) * kBN + bc]) = s.b[q];
    };
    if (nleft > 0) {
      sweep_steps<T, Stage<T>>(
          0, nleft, acc,
          [&](int kt, Stage<T> &s) {
            s.u = *reinterpret_cast<const uvec *>(U + tofs);
            tofs += tstep;
            tstep -= kKT * kKT;
            load_b((int64_t)kt * kKT, s);
          },
          [&](int buf, int, const Stage<T> &s) {
            *reinterpret_cast<vec *>(&Ss[buf][tk * kTP + ti]) = s.u;
            store_b(buf, s);
          },
          [&](int buf, int, int t, typename K::Ops &o) {
            K::read_a_t(&Ss[buf][wr * 32], kTP, lane, t, o);
            K::read_b(&Bs[buf][wc * 32], kBN, lane, t, o);
          });
      __syncthreads();
    }
    sweep_steps<T, Stage<T>>(nleft, nmid, acc, load_stage, store_stage, read_ops);
    if (nfull > nmid) {
      __syncthreads();
      sweep_steps<T, Stage<T>>(
          nmid, nfull, acc,
          [&](int kt, Stage<T> &s) {
            const int64_t k0 = (int64_t)kt * kKT;
            s.u = *reinterpret_cast<const uvec *>(ub + k0 + uk);
            load_b(k0, s);
          },
          [&](int buf, int, const Stage<T> &s) {
            *reinterpret_cast<vec *>(&Ss[buf][ur * kUP + uk]) = s.u;
            store_b(buf, s);
          },
          [&](int buf, int, int t, typename K::Ops &o) {
            K::read_a(&Ss[buf][wr * 32 * kUP], lane, t, o);
            K::read_b(&Bs[buf][wc * 32], kBN, lane, t, o);
          });
    }
    if (nk > (nfull > nmid ? nfull : nmid)) {
      __syncthreads();
      sweep_steps<T, Stage<T>>(nfull > nmid ? nfull : nmid, nk, acc, load_stage, store_stage, read_ops);
    }
  } else {
    sweep_steps<T, Stage<T>>(0, nk, acc, load_stage, store_stage, read_ops);
  }

  K::for_each(acc, lane, [&](int r, int c, T v) {
    const int64_t i = i0 + wr * 32 + r, col = col0 + wc * 32 + c;
    if (i < n && col < m) C[i * ldc + col] = v;
  });
}

template <typename T>
int run(int64_t n, int64_t m, const T *Up, const T *B, int64_t ldb, T *C, int64_t ldc, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (n < 0 || m < 1 || ldb < m || ldc < m) return DASTAC_EINVAL;
  if (n > (1 << 24) || m > (1 << 24) || ld_too_large(ldb, ldc)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Up || !B || !C) return DASTAC_ENULL;
  const int64_t cb = view_bytes(n, ldc, m, kB);
  if (overlaps(C, cb, Up, tri(n) * kB) || overlaps(C, cb, B, view_bytes(n, ldb, m, kB))) return DASTAC_EALIAS;
  const int nb = (int)ceil_div(n, kTileM);
  const int ncb = (int)ceil_div(m, kTileN);
  const int64_t grid = (int64_t)8 * ceil_div(nb, 8) * ncb;
  if (grid > 0x7fffffff) return DASTAC_EOVERFLOW;
  symm_mfma_kernel<T><<<(unsigned)grid, kTileThreads, 0, (hipStream_t)stream>>>(n, m, Up, B, ldb, C, ldc, nb, ncb);
  return launch_status();
}

}  // namespace

extern "C" int dastac_symm_f32(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C,
                               int64_t ldc, void *stream) {
  return run<float>(n, m, Up, B, ldb, C, ldc, stream);
}

// Double precision (the paper's element type): the same kernel on the fp64 matrix cores.
extern "C" int dastac_symm_f64(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C,
                               int64_t ldc, void *stream) {
  return run<double>(n, m, Up, B, ldb, C, ldc, stream);
}
