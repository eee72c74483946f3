// TTM over a packed upper half cube, the paper's running example (Fig. 3):
//
//   A(i,j,k) := B(i,j,l) * C(k,l),   i<=j, 0<=l<Q, 0<=k<K
//
// B stores only the pairs i<=j, each with its Q values of l back to back, at the position given
// by the printed index polynomial P_B(i,j,l) = tri(n,i,j)*Q + l (Section 3).  The output inherits
// the structure and is packed by the same rule with k in place of l (Section 3, "Data layout
// compression": input and output compression).  Pair number p = tri(n,i,j) is therefore row p of
// both buffers, and the whole contraction is ONE dense product over the packed rows,
//
//   Ap[p, k] = sum_l Bp[p, l] * C[k, l],      p = 0 .. Tri(n)-1
//
// with no structural zero left to skip and no index arithmetic beyond the row number: that is
// the point of the layout.  It runs on the matrix cores, in single and in double precision.
//
// Tiling.  A workgroup (8 wavefronts, 2 x 4) owns 64 packed rows x 128 values of k and sweeps l in
// steps of kKT = 32 (fp32) or 16 (fp64); the 64 x kKT tile of Bp and the 128 x kKT tile of C are staged
// in LDS, double-buffered against the global loads of the next step.  Both tiles keep l contiguous, so
// in fp32 -- with lane half h taking the four consecutive l values 8t+4h..8t+4h+3 of every group of
// eight, as in the TRMM kernel -- both operands of v_mfma_f32_32x32x2_f32 are single 16-byte LDS reads
// (the per-type matrix-core pieces are those of mfma_tile.h).  Workgroups
// that share a row block (different blocks of k) get ids that are equal modulo 8, i.e. the same
// XCD, so the rows of Bp they both read come from HBM once.  About two workgroups per compute unit
// are launched; each walks a strided set of row blocks with one uninterrupted pipeline, so the
// first loads of a row block are in flight while the previous block's last step is multiplied.
#include "mfma_tile.h"

using namespace dastac;

namespace {

// tags that pick a step's flavour at compile time
struct Whole {
  static constexpr bool value = true;
};
struct Any {
  static constexpr bool value = false;
};

template <typename T>
struct Stage {
  typename Core<T>::vec a;     // Bp: row sr of the tile, one 16-byte piece of l values
  typename Core<T>::vec c[2];  // C: rows sr and sr+64 of the tile, one 16-byte piece of l values each
};

template <typename T>
__global__ __launch_bounds__(kTileThreads) void ttm_mfma_kernel(int64_t rows, int64_t Q, int64_t K,
                                                                const T *__restrict__ Bp, const T *__restrict__ C,
                                                                int64_t ldc, T *__restrict__ Ap, int lanes, int ncb) {
  typedef Core<T> Kc;
  typedef typename Kc::vec vec;
  typedef typename Kc::uvec uvec;
  constexpr int kBM = kTileM, kBN = kTileN, kKT = Kc::kKT, kV = Kc::kVec, kP = Kc::kRowPitch;
  __shared__ __attribute__((aligned(16))) T As[2][kBM * kP];
  __shared__ __attribute__((aligned(16))) T Cs[2][kBN * kP];

  // workgroup id -> (first row block, block of k); ids equal mod 8 share an XCD.  A workgroup
  // then walks every (8*lanes)-th row block, keeping its pipeline full across blocks.
  const int L = blockIdx.x;
  const int xcd = L & 7, slot = L >> 3;
  const int cb = slot % ncb;
  const int64_t rstride = (int64_t)kBM * 8 * lanes;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 2, wc = wave & 3;  // 2x4 wavefronts: 32 rows x 32 values of k each

  // staging role: tile row tid/8 (and +64 for C), l offset kV*(tid%8)
  const int sr = tid >> 3, sl = (tid & 7) * kV;
  const int64_t c0 = (int64_t)cb * kBN;
  const bool full_c = c0 + kBN <= K;
  const int nk = (int)ceil_div(Q, kKT);

  const T *cp0 = C + (c0 + sr < K ? c0 + sr : K - 1) * ldc;
  const T *cp1 = C + (c0 + sr + 64 < K ? c0 + sr + 64 : K - 1) * ldc;

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

  auto load_stage = [&](const Cur &cu, Stage<T> &s) {
    const int64_t l0 = (int64_t)cu.kt * kKT + sl;
    const T *ap = Bp + (cu.r0 + sr < rows ? cu.r0 + sr : rows - 1) * Q;
    if (full_c && cu.r0 + kBM <= rows && (int64_t)cu.kt * kKT + kKT <= Q) {
      s.a = *reinterpret_cast<const uvec *>(ap + l0);
      s.c[0] = *reinterpret_cast<const uvec *>(cp0 + l0);
      s.c[1] = *reinterpret_cast<const uvec *>(cp1 + l0);
    } else {  // ragged edge: zeros outside the operands
#pragma unroll
      for (int e = 0; e < kV; ++e) {
        const bool lok = l0 + e < Q;
        s.a[e] = (lok && cu.r0 + sr < rows) ? ap[l0 + e] : T(0);
        s.c[0][e] = (lok && c0 + sr < K) ? cp0[l0 + e] : T(0);
        s.c[1][e] = (lok && c0 + sr + 64 < K) ? cp1[l0 + e] : T(0);
      }
    }
  };
  auto store_stage = [&](int buf, const Stage<T> &s) {
    *reinterpret_cast<vec *>(&As[buf][sr * kP + sl]) = s.a;
    *reinterpret_cast<vec *>(&Cs[buf][sr * kP + sl]) = s.c[0];
    *reinterpret_cast<vec *>(&Cs[buf][(sr + 64) * kP + sl]) = s.c[1];
  };

  typename Kc::Acc acc;
  Kc::clear(acc);
  auto read_ops = [&](int buf, int t, typename Kc::Ops &o) {
    Kc::read_a(&As[buf][wr * 32 * kP], lane, t, o);
    Kc::read_b_rows(&Cs[buf][wc * 32 * kP], lane, t, o);
  };

  Cur cc{(int64_t)kBM * (xcd + 8 * (slot / ncb)), 0, true};  // the step being multiplied
  cc.valid = cc.r0 < rows;
  if (!cc.valid) return;
  Cur cl = cc;  // the step being loaded: one ahead
  Stage<T> st;
  typename Kc::Ops oa, ob;
  load_stage(cl, st);
  store_stage(0, st);
  __syncthreads();
  read_ops(0, 0, oa);

  // One step on LDS buffer `buf` (a literal at every call site).  The global loads of the next
  // step -- of the next row block, at a block's last step -- are in flight throughout; its LDS
  // stores and the workgroup barrier sit before the last group's matrix instructions, whose
  // operands are already in registers.  (The schedule of mfma_tile.h's sweep, run as ONE pipeline over
  // all the workgroup's row blocks.)
  // WHOLE: the step being loaded exists and lies in a whole row block of a whole column block, with Q a
  // multiple of the step (so does the step being multiplied, which comes before it): loads and the stores of
  // a finished tile then need no test and no clamped row, and the loop made of such steps holds none.
  const int64_t aoff = (int64_t)sr * Q + sl;
  auto step = [&](int buf, auto whole_tag) {
    constexpr bool WHOLE = decltype(whole_tag)::value;
    cl = next(cl);
    const bool more = WHOLE || cl.valid;
    if (WHOLE) {
      const int64_t l0 = (int64_t)cl.kt * kKT;
      st.a = *reinterpret_cast<const uvec *>(Bp + (cl.r0 * Q + l0) + aoff);
      st.c[0] = *reinterpret_cast<const uvec *>(cp0 + l0 + sl);
      st.c[1] = *reinterpret_cast<const uvec *>(cp1 + l0 + sl);
    } else if (more) {
      load_stage(cl, st);
    }
    // (Scheduling barriers keep the written order: left alone, the compiler merges the two operand register
    // sets and issues a group's LDS reads after the previous group's matrix instructions instead of before
    // them.  With two workgroups per CU and no shares, as here, the written order is 2.5 % faster.)
    read_ops(buf, 1, ob);
    __builtin_amdgcn_sched_barrier(0);
    Kc::mma(oa, acc);
    __builtin_amdgcn_sched_barrier(0);
    read_ops(buf, 2, oa);
    __builtin_amdgcn_sched_barrier(0);
    Kc::mma(ob, acc);
    __builtin_amdgcn_sched_barrier(0);
    read_ops(buf, 3, ob);
    __builtin_amdgcn_sched_barrier(0);
    Kc::mma(oa, acc);
    __builtin_amdgcn_sched_barrier(0);
    if (more) store_stage(buf ^ 1, st);
    __syncthreads();
    if (more) read_ops(buf ^ 1, 0, oa);
    __builtin_amdgcn_sched_barrier(0);
    Kc::mma(ob, acc);
    __builtin_amdgcn_sched_barrier(0);
    if (cc.kt == nk - 1) {
      Kc::for_each(acc, lane, [&](int r, int c, T v) {
        const int64_t row = cc.r0 + wr * 32 + r, col = c0 + wc * 32 + c;
        if (WHOLE || (row < rows && col < K)) Ap[row * K + col] = v;
      });
      Kc::clear(acc);
    }
    cc = next(cc);
  };
  // whole steps two at a time (all whole row blocks come before the ragged one), then the rest
  if (full_c && Q % kKT == 0) {
    auto whole = [&](const Cur &c) { return c.valid && c.r0 + kBM <= rows; };
    for (;;) {
      const Cur n1 = next(cl);
      if (!whole(n1) || !whole(next(n1))) break;
      step(0, Whole{});
      step(1, Whole{});
    }
  }
  for (;;) {
    step(0, Any{});
    if (!cc.valid) break;
    step(1, Any{});
    if (!cc.valid) break;
  }
}

// ---- compression / decompression of the upper half cube ---------------------------------------
// One workgroup per 256-element piece of one (i,j) row of the dense n x n x Q tensor.
constexpr int kCopy = 256;

template <bool PACK, typename T>
__global__ __launch_bounds__(kCopy) void uhc_copy_kernel(int64_t n, int64_t Q, const T *__restrict__ src,
                                                         T *__restrict__ dst, int64_t pieces,
                                                         int64_t nblocks) {
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
    const int64_t ij = b / pieces, l = (b - ij * pieces) * kCopy + threadIdx.x;
    const int64_t i = ij / n, j = ij - i * n;
    if (l >= Q) continue;
    if (PACK) {
      if (j >= i) dst[tri_offset(n, i, j) * Q + l] = src[ij * Q + l];
    } else {
      dst[ij * Q + l] = (j >= i) ? src[tri_offset(n, i, j) * Q + l] : T(0);
    }
  }
}

inline bool uhc_ok(int64_t n, int64_t Q) {
  return n >= 0 && Q >= 1 && n <= (1 << 20) && Q <= (1 << 24) && (n == 0 || tri(n) <= ((int64_t)1 << 40) / Q);
}

// pack (dense -> packed) or unpack (packed -> dense) of the upper half cube, float or double
template <bool PACK, typename T>
int uhc_copy(int64_t n, int64_t Q, const T *src, T *dst, void *stream) {
  if (n < 0 || Q < 1) return DASTAC_EINVAL;
  if (!uhc_ok(n, Q) || n * n > ((int64_t)1 << 40) / Q) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!src || !dst) return DASTAC_ENULL;
  const int64_t sz = (int64_t)sizeof(T), nd = n * n * Q * sz, np = tri(n) * Q * sz;
  if (overlaps(dst, PACK ? np : nd, src, PACK ? nd : np)) return DASTAC_EALIAS;
  const int64_t pieces = ceil_div(Q, kCopy), nblocks = n * n * pieces;
  const unsigned grid = (unsigned)(nblocks < (1 << 20) ? nblocks : (1 << 20));
  uhc_copy_kernel<PACK, T><<<grid, kCopy, 0, (hipStream_t)stream>>>(n, Q, src, dst, pieces, nblocks);
  return launch_status();
}

template <typename T>
int ttm_ut(int64_t n, int64_t Q, int64_t K, const T *Bp, const T *C, int64_t ldc, T *Ap, void *stream) {
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (n < 0 || Q < 1 || K < 1 || ldc < Q) return DASTAC_EINVAL;
  if (!uhc_ok(n, Q) || !uhc_ok(n, K) || ld_too_large(ldc) || K > ((int64_t)1 << 40) / ldc) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Bp || !C || !Ap) return DASTAC_ENULL;
  const int64_t rows = tri(n);
  if (overlaps(Ap, rows * K * kB, Bp, rows * Q * kB) || overlaps(Ap, rows * K * kB, C, view_bytes(K, ldc, Q, kB)))
    return DASTAC_EALIAS;
  const int64_t nrb = ceil_div(rows, kTileM), ncb = ceil_div(K, kTileN);
  if (ncb > (1 << 20)) return DASTAC_EOVERFLOW;
  // about two workgroups per compute unit (256 of them), each walking a strided set of row blocks
  int64_t lanes = ceil_div(512, 8 * ncb);
  if (lanes > ceil_div(nrb, 8)) lanes = ceil_div(nrb, 8);
  const int64_t grid = 8 * lanes * ncb;
  ttm_mfma_kernel<T><<<(unsigned)grid, kTileThreads, 0, (hipStream_t)stream>>>(rows, Q, K, Bp, C, ldc, Ap, (int)lanes,
                                                                             (int)ncb);
  return launch_status();
}

}  // namespace

extern "C" {

int64_t dastac_uhc_count(int64_t n, int64_t Q) {
  if (!uhc_ok(n, Q)) return -1;
  return tri(n) * Q;
}

int64_t dastac_uhc_offset(int64_t n, int64_t Q, int64_t i, int64_t j, int64_t l) {
  if (!uhc_ok(n, Q) || i < 0 || j < i || j >= n || l < 0 || l >= Q) return -1;
  return tri_offset(n, i, j) * Q + l;
}

int dastac_pack_uhc_f32(int64_t n, int64_t Q, const float *dense, float *packed, void *stream) {
  return uhc_copy<true, float>(n, Q, dense, packed, stream);
}

int dastac_unpack_uhc_f32(int64_t n, int64_t Q, const float *packed, float *dense, void *stream) {
  return uhc_copy<false, float>(n, Q, packed, dense, stream);
}

int dastac_pack_uhc_f64(int64_t n, int64_t Q, const double *dense, double *packed, void *stream) {
  return uhc_copy<true, double>(n, Q, dense, packed, stream);
}

int dastac_unpack_uhc_f64(int64_t n, int64_t Q, const double *packed, double *dense, void *stream) {
  return uhc_copy<false, double>(n, Q, packed, dense, stream);
}

int dastac_ttm_ut_f32(int64_t n, int64_t Q, int64_t K, const float *Bp, const float *C, int64_t ldc, float *Ap,
                      void *stream) {
  return ttm_ut<float>(n, Q, K, Bp, C, ldc, Ap, stream);
}

// Double precision (the paper's element type): the same kernel on the fp64 matrix cores.
int dastac_ttm_ut_f64(int64_t n, int64_t Q, int64_t K, const double *Bp, const double *C, int64_t ldc, double *Ap,
                      void *stream) {
  return ttm_ut<double>(n, Q, K, Bp, C, ldc, Ap, stream);
}

}  // extern "C"
