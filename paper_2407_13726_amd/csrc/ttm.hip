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
// the point of the layout.  It runs on the fp32 matrix cores.
//
// Tiling.  A workgroup (8 wavefronts, 2 x 4) owns 64 packed rows x 128 values of k and sweeps l in
// steps of 32; the 64x32 tile of Bp and the 128x32 tile of C are staged in LDS, double-buffered
// against the global loads of the next step.  Both tiles keep l contiguous, so -- with lane half h
// taking the four consecutive l values 8t+4h..8t+4h+3 of every group of eight, as in the TRMM
// kernel -- both operands of v_mfma_f32_32x32x2_f32 are single 16-byte LDS reads.  Workgroups
// that share a row block (different blocks of k) get ids that are equal modulo 8, i.e. the same
// XCD, so the rows of Bp they both read come from HBM once.  About two workgroups per compute unit
// are launched; each walks a strided set of row blocks with one uninterrupted pipeline, so the
// first loads of a row block are in flight while the previous block's last step is multiplied.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBM = 64;    // packed rows per workgroup tile
constexpr int kBN = 128;   // values of k per workgroup tile
constexpr int kKT = 32;    // step along l
constexpr int kP = kKT + 4;  // LDS pitch (floats): 16-byte reads of 8 lanes cover all banks
constexpr int kBlock = 512;

typedef float f16v __attribute__((ext_vector_type(16)));

struct Stage {
  f4a a;     // Bp: row ar of the tile, four l values
  f4a c[2];  // C: rows cr and cr+64 of the tile, four l values
};

__global__ __launch_bounds__(kBlock) void ttm_mfma_kernel(int64_t rows, int64_t Q, int64_t K,
                                                          const float *__restrict__ Bp,
                                                          const float *__restrict__ C, int64_t ldc,
                                                          float *__restrict__ Ap, int lanes, int ncb) {
  __shared__ __attribute__((aligned(16))) float As[2][kBM * kP];
  __shared__ __attribute__((aligned(16))) float Cs[2][kBN * kP];

  // workgroup id -> (first row block, block of k); ids equal mod 8 share an XCD.  A workgroup
  // then walks every (8*lanes)-th row block, keeping its pipeline full across blocks.
  const int L = blockIdx.x;
  const int xcd = L & 7, slot = L >> 3;
  const int cb = slot % ncb;
  const int64_t rstride = (int64_t)kBM * 8 * lanes;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 2, wc = wave & 3;  // 2x4 wavefronts: 32 rows x 32 values of k each
  const int l32 = lane & 31, h = lane >> 5;

  // staging role: tile row tid/8 (and +64 for C), l offset 4*(tid%8)
  const int sr = tid >> 3, sl = (tid & 7) * 4;
  const int64_t c0 = (int64_t)cb * kBN;
  const bool full_c = c0 + kBN <= K;
  const int nk = (int)ceil_div(Q, kKT);

  const float *cp0 = C + (c0 + sr < K ? c0 + sr : K - 1) * ldc;
  const float *cp1 = C + (c0 + sr + 64 < K ? c0 + sr + 64 : K - 1) * ldc;

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
    const float *ap = Bp + (cu.r0 + sr < rows ? cu.r0 + sr : rows - 1) * Q;
    if (full_c && cu.r0 + kBM <= rows && (int64_t)cu.kt * kKT + kKT <= Q) {
      s.a = *reinterpret_cast<const f4u *>(ap + l0);
      s.c[0] = *reinterpret_cast<const f4u *>(cp0 + l0);
      s.c[1] = *reinterpret_cast<const f4u *>(cp1 + l0);
    } else {  // ragged edge: zeros outside the operands
      float a[4], u[4], v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool lok = l0 + e < Q;
        a[e] = (lok && cu.r0 + sr < rows) ? ap[l0 + e] : 0.0f;
        u[e] = (lok && c0 + sr < K) ? cp0[l0 + e] : 0.0f;
        v[e] = (lok && c0 + sr + 64 < K) ? cp1[l0 + e] : 0.0f;
      }
      s.a = f4a{a[0], a[1], a[2], a[3]};
      s.c[0] = f4a{u[0], u[1], u[2], u[3]};
      s.c[1] = f4a{v[0], v[1], v[2], v[3]};
    }
  };
  auto store_stage = [&](int buf, const Stage &s) {
    *reinterpret_cast<f4a *>(&As[buf][sr * kP + sl]) = s.a;
    *reinterpret_cast<f4a *>(&Cs[buf][sr * kP + sl]) = s.c[0];
    *reinterpret_cast<f4a *>(&Cs[buf][(sr + 64) * kP + sl]) = s.c[1];
  };

  f16v acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

  // Operands of one group of eight l values: four MFMA steps on the wavefront's 32x32 sub-tile.
  struct Ops {
    f4a a, c;
  };
  auto read_ops = [&](int buf, int t, Ops &o) {
    o.a = *reinterpret_cast<const f4a *>(&As[buf][(wr * 32 + l32) * kP + 4 * h + 8 * t]);
    o.c = *reinterpret_cast<const f4a *>(&Cs[buf][(wc * 32 + l32) * kP + 4 * h + 8 * t]);
  };
  auto mma = [&](const Ops &o) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a.x, o.c.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a.y, o.c.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a.z, o.c.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a.w, o.c.w, acc, 0, 0, 0);
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

  // One step on LDS buffer `buf` (a literal at both call sites).  The global loads of the next
  // step -- of the next row block, at a block's last step -- are in flight throughout; its LDS
  // stores and the workgroup barrier sit before the last group's matrix instructions, whose
  // operands are already in registers.
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
      // D layout of the 32x32 tile: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32
      const int64_t col = c0 + wc * 32 + l32;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t r = cc.r0 + wr * 32 + 8 * (v / 4) + 4 * h + (v % 4);
        if (r < rows && col < K) Ap[r * K + col] = acc[v];
        acc[v] = 0.0f;
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
  if (n < 0 || Q < 1 || K < 1 || ldc < Q) return DASTAC_EINVAL;
  if (!uhc_ok(n, Q) || !uhc_ok(n, K) || ld_too_large(ldc) || K > ((int64_t)1 << 40) / ldc) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Bp || !C || !Ap) return DASTAC_ENULL;
  const int64_t rows = tri(n);
  if (overlaps(Ap, rows * K * 4, Bp, rows * Q * 4) || overlaps(Ap, rows * K * 4, C, view_bytes(K, ldc, Q, 4))) return DASTAC_EALIAS;
  const int64_t nrb = ceil_div(rows, kBM), ncb = ceil_div(K, kBN);
  if (ncb > (1 << 20)) return DASTAC_EOVERFLOW;
  // about two workgroups per compute unit (256 of them), each walking a strided set of row blocks
  int64_t lanes = ceil_div(512, 8 * ncb);
  if (lanes > ceil_div(nrb, 8)) lanes = ceil_div(nrb, 8);
  const int64_t grid = 8 * lanes * ncb;
  ttm_mfma_kernel<<<(unsigned)grid, kBlock, 0, (hipStream_t)stream>>>(rows, Q, K, Bp, C, ldc, Ap, (int)lanes, (int)ncb);
  return launch_status();
}

}  // extern "C"
