// Polynomial-regression tensors (Table 1) in double precision, written straight into packed
// hyper-triangles on the fp64 matrix cores:
//
//   A2(i,j)   := B(x,i) * B(x,j)            i<=j        packed upper triangle,   tri(d,i,j)
//   A3(i,j,k) := B(x,i) * B(x,j) * B(x,k)   i<=j<=k     packed upper tetrahedron, tet(d,i,j,k)
//
// The plan is the fp32 kernel's: slice i of A3 is the upper triangle of a weighted Gram matrix (A2: one
// slice, weight 1); a workgroup owns a 64 (j) x BK (k) tile of one slice and a range of samples x (the
// reduction index); dense tile numbering; wavefronts whose sub-tile lies below the diagonal issue no
// matrix instructions; the sample range is split, with float atomics into a zeroed output, when the tiles
// alone cannot fill the chip.  Here a step is 16 samples, the matrix instruction is
// v_mfma_f64_16x16x4_f64, and a wavefront's 32x32 sub-tile is 2x2 tiles of 16x16 with four independent
// accumulators (lane l supplies column l%16 at sample l/16 of each group of four).
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBJ = 64;    // j extent of a workgroup tile
// k extent of a workgroup tile: BK = 128 (eight wavefronts) or BK = 64 (four), a template parameter
constexpr int kXT = 16;    // samples per step
constexpr int kJP = kBJ + 2;  // LDS pitch of the j tile [x][j] (doubles)
constexpr int64_t kMaxD2 = 1 << 16;  // A2: tile grid and tri(d) stay small
constexpr int64_t kMaxD3 = 1 << 13;  // A3: the tile count stays inside gridDim.x
constexpr int64_t kMaxN = (int64_t)1 << 31;
// Up to these d the 64 x 64 tile is used (the fp32 kernel's measured thresholds).
constexpr int64_t kNarrowMaxD2 = 768, kNarrowMaxD3 = 2048;

typedef double d2u __attribute__((ext_vector_type(2), aligned(8)));
typedef double d2a __attribute__((ext_vector_type(2)));
typedef double d4v __attribute__((ext_vector_type(4)));

struct Stage {
  d2a a[2];  // j tile: one or two sample rows, two columns each
  d2a b[2];  // k tile: sample rows bk and bk+8, two columns each
};

// Tiles with work.  A slice of order q has m = ceil(q/64) blocks of rows j and ceil(m/2) blocks of columns k;
// tile (J,K) holds an element with j<=k exactly when K >= J/2 (integer division), so row block J has
// ceil(m/2) - J/2 tiles and the slice has tiles_of(m) in all.  Tiles are numbered densely, slice after slice,
// row block after row block, so that consecutive workgroup ids (which the hardware deals out to the XCDs in
// turn) all carry work: numbering the whole J x K rectangle and letting the empty tiles exit would leave
// the XCDs with very different loads, because the id modulo 8 would select the column block.
// (With BK = 64 the condition is K >= J: row block J has m - J tiles, a slice m(m+1)/2.)
DASTAC_HD int64_t tiles_of(int64_t m, int BK) {
  if (BK == 64) return m * (m + 1) / 2;
  const int64_t p = m / 2;
  return (m & 1) ? p * p + 3 * p + 1 : p * (p + 1);
}

DASTAC_HD int64_t total_tiles(int64_t d, bool cube, int BK) {
  const int64_t m0 = ceil_div(d, kBJ);
  if (!cube) return tiles_of(m0, BK);
  int64_t total = (d - kBJ * (m0 - 1)) * tiles_of(m0, BK);  // slices whose order needs m0 row blocks
  for (int64_t m = m0 - 1; m >= 1; --m) total += kBJ * tiles_of(m, BK);
  return total;
}

// Dense tile number -> slice i and tile (J,K).
__device__ inline void decode_tile(int64_t d, bool cube, int BK, int64_t t, int64_t &i, int &J, int &K) {
  int64_t m = ceil_div(d, kBJ);
  i = 0;
  if (cube) {
    int64_t first = 0, count = d - kBJ * (m - 1);  // slices first .. first+count-1 need m row blocks
    while (t >= count * tiles_of(m, BK)) {
      t -= count * tiles_of(m, BK);
      first += count;
      count = kBJ;
      --m;
    }
    i = first + t / tiles_of(m, BK);
    t = t % tiles_of(m, BK);
  }
  const int64_t nK = BK == 64 ? m : (m + 1) / 2;  // column blocks of the slice
  int64_t Jr = 0;
  while (t >= nK - Jr * kBJ / BK) {  // row block Jr has column blocks Jr*64/BK .. nK-1
    t -= nK - Jr * kBJ / BK;
    ++Jr;
  }
  J = (int)Jr;
  K = (int)(Jr * kBJ / BK + t);
}

template <bool CUBE, bool ATOMIC, int BK>
__global__ __launch_bounds__(4 * BK) void pr_f64_kernel(int64_t N, int64_t d, const double *__restrict__ B,
                                                         int64_t ldb, double *__restrict__ out, int64_t chunk) {
  __shared__ __attribute__((aligned(16))) double As[2][kXT * kJP];
  __shared__ __attribute__((aligned(16))) double Bs[2][kXT * BK];
  constexpr int kThreads = 4 * BK, kWC = BK / 32;  // wavefronts: 2 rows of kWC

  int64_t i;  // slice: every column index of this workgroup is >= i
  int J, K;
  decode_tile(d, CUBE, BK, uniform64((int64_t)blockIdx.x), i, J, K);
  const int64_t q = d - i;  // order of the slice's triangle
  const int64_t xbeg = (int64_t)blockIdx.y * chunk;
  const int64_t xend = xbeg + chunk < N ? xbeg + chunk : N;
  if (xbeg >= xend) return;
  const int nk = (int)ceil_div(xend - xbeg, kXT);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / kWC, wc = wave % kWC;  // 2 x kWC wavefronts: 32 (j) x 32 (k) each
  const int l16 = lane & 15, l4 = lane >> 4;
  // A wavefront whose 32x32 sub-tile lies wholly below the diagonal (largest k < smallest j) still helps
  // to stage the tiles but issues no matrix instructions, which leaves the SIMD's matrix pipe to the
  // wavefronts of the other workgroups resident on it.
  const bool live = uniform32(K * BK + wc * 32 + 31 >= J * kBJ + wr * 32) != 0;

  // j tile: sample rows tk + kJRows*r (r < kJRep), column offset ti; k tile: sample rows bk and bk+8, column offset bc
  constexpr int kJRows = kThreads / 32, kJRep = kXT / kJRows;
  const int tk = tid >> 5, ti = (tid & 31) * 2;
  const int bk = tid / (BK / 2), bc = (tid % (BK / 2)) * 2;
  const int64_t j0 = i + (int64_t)J * kBJ, k0 = i + (int64_t)K * BK;  // absolute first columns
  const bool j_full = j0 + kBJ <= d, k_full = k0 + BK <= d;

  // Columns c, c+1 of one row of B, zero from column d on, with one vector load whose address is pulled
  // back inside the row (needs d >= 2): a lane that straddles the end shifts what it fetched.
  auto load2_clamped = [&](const double *row, int64_t c) -> d2a {
    const int64_t cc = c + 2 <= d ? c : d - 2;
    const d2a v = *reinterpret_cast<const d2u *>(row + cc);
    const int64_t sh = c - cc;  // 0: both inside; 1: the second is beyond the end; >= 2: both beyond
    d2a r;
    r.x = sh == 0 ? v.x : sh == 1 ? v.y : 0.0;
    r.y = sh == 0 ? v.y : 0.0;
    return r;
  };
  const bool wide = d >= 2;

  auto load_stage = [&](int kt, Stage &s) {
    const int64_t x0 = xbeg + (int64_t)kt * kXT;
    const bool x_full = x0 + kXT <= xend;
#pragma unroll
    for (int r = 0; r < kJRep; ++r) {
      const int64_t xa = x0 + tk + kJRows * r;
      if (x_full && j_full) {
        s.a[r] = *reinterpret_cast<const d2u *>(B + xa * ldb + j0 + ti);
      } else if (x_full && wide) {
        s.a[r] = load2_clamped(B + xa * ldb, j0 + ti);
      } else {
        double v[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) v[e] = (xa < xend && j0 + ti + e < d) ? B[xa * ldb + j0 + ti + e] : 0.0;
        s.a[r] = d2a{v[0], v[1]};
      }
      if (CUBE) {
        const double w = xa < xend ? B[xa * ldb + i] : 0.0;
        s.a[r] *= w;
      }
    }
    if (x_full && k_full) {
#pragma unroll
      for (int r = 0; r < 2; ++r) s.b[r] = *reinterpret_cast<const d2u *>(B + (x0 + bk + 8 * r) * ldb + k0 + bc);
    } else if (x_full && wide) {
#pragma unroll
      for (int r = 0; r < 2; ++r) s.b[r] = load2_clamped(B + (x0 + bk + 8 * r) * ldb, k0 + bc);
    } else {
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const int64_t x = x0 + bk + 8 * r;
        double v[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) v[e] = (x < xend && k0 + bc + e < d) ? B[x * ldb + k0 + bc + e] : 0.0;
        s.b[r] = d2a{v[0], v[1]};
      }
    }
  };
  auto store_stage = [&](int buf, const Stage &s) {
#pragma unroll
    for (int r = 0; r < kJRep; ++r) *reinterpret_cast<d2a *>(&As[buf][(tk + kJRows * r) * kJP + ti]) = s.a[r];
#pragma unroll
    for (int r = 0; r < 2; ++r) *reinterpret_cast<d2a *>(&Bs[buf][(bk + 8 * r) * BK + bc]) = s.b[r];
  };

  d4v acc[4];  // 2x2 tiles of 16x16: acc[2*ra + ca]
#pragma unroll
  for (int t = 0; t < 4; ++t) acc[t] = d4v{0.0, 0.0, 0.0, 0.0};

  // Operands of one group of four samples (the sum over x may be taken in any order).
  struct Ops {
    double a[2], b[2];
  };
  auto read_ops = [&](int buf, int t, Ops &o) {
    if (!live) return;
    const double *as = &As[buf][(4 * t + l4) * kJP + wr * 32 + l16];
    const double *bs = &Bs[buf][(4 * t + l4) * BK + wc * 32 + l16];
    o.a[0] = as[0];
    o.a[1] = as[16];
    o.b[0] = bs[0];
    o.b[1] = bs[16];
  };
  auto mma = [&](const Ops &o) {
    if (!live) return;
    acc[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[0], o.b[0], acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[0], o.b[1], acc[1], 0, 0, 0);
    acc[2] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[1], o.b[0], acc[2], 0, 0, 0);
    acc[3] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[1], o.b[1], acc[3], 0, 0, 0);
  };

  Stage st;
  Ops oa = {}, ob = {};
  load_stage(0, st);
  store_stage(0, st);
  __syncthreads();
  read_ops(0, 0, oa);

  // One step on LDS buffer `buf`: the next step's global loads are in flight throughout; its LDS
  // stores and the barrier sit before the last group's matrix instructions.
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

  // D layout of a 16x16 tile: element v of lane l is row 4*v + l/16, column l%16.  Rows are j, columns are k;
  // both relative to the slice's first column i.
  double *slice = out + (CUBE ? tet_slice_start(d, i) : 0);
#pragma unroll
  for (int ra = 0; ra < 2; ++ra)
#pragma unroll
    for (int ca = 0; ca < 2; ++ca) {
      const int64_t kr = (int64_t)K * BK + wc * 32 + 16 * ca + l16;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int64_t jr = (int64_t)J * kBJ + wr * 32 + 16 * ra + 4 * v + l4;
        if (jr <= kr && kr < q) {
          double *p = slice + tri_offset(q, jr, kr);
          if (ATOMIC)
            unsafeAtomicAdd(p, acc[2 * ra + ca][v]);
          else
            *p = acc[2 * ra + ca][v];
        }
      }
    }
}

__global__ void fill_zero_kernel(double *__restrict__ y, int64_t count) {
  for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < count; t += (int64_t)gridDim.x * blockDim.x)
    y[t] = 0.0;
}

template <bool CUBE, int BK>
int run(int64_t N, int64_t d, const double *B, int64_t ldb, double *out, void *stream) {
  constexpr int kBlock = 4 * BK;
  if (N < 0 || d < 0 || ldb < d) return DASTAC_EINVAL;
  if (d > (CUBE ? kMaxD3 : kMaxD2) || N > kMaxN || ld_too_large(ldb)) return DASTAC_EOVERFLOW;
  if (d == 0) return DASTAC_OK;
  if (!out || (N > 0 && !B)) return DASTAC_ENULL;
  const int64_t count = CUBE ? tet(d) : tri(d);
  if (overlaps(out, count * 8, B, view_bytes(N, ldb, d, 8))) return DASTAC_EALIAS;
  hipStream_t st = (hipStream_t)stream;

  const int64_t tiles = total_tiles(d, CUBE, BK);
  if (tiles > 0x7fffffff) return DASTAC_EOVERFLOW;
  // Split the samples when the tiles alone cannot fill the chip.  All workgroups cost the same, so the
  // launch runs in rounds of `slots` resident workgroups: take the smallest split that fills its last
  // round to 90 %, or else the best one found; every share is a multiple of a step and at least 8 steps.
  int64_t split = 1, chunk = kXT;
  if (N > 0) {
    const int64_t slots = resident_blocks(pr_f64_kernel<CUBE, true, BK>, kBlock);
    if (slots <= 0) return DASTAC_EHIP;
    const int64_t max_split = N / (8 * kXT) > 1 ? N / (8 * kXT) : 1;
    double best = -1.0;
    for (int64_t s = 1; s <= max_split && s <= 4096; ++s) {
      const int64_t blocks = tiles * s, rounds = ceil_div(blocks, slots);
      const double fill = (double)blocks / (double)(rounds * slots);
      if (fill > best + 1e-9) best = fill, split = s;
      if (fill >= 0.9 || blocks >= 16 * slots) {
        split = s;
        break;
      }
    }
    chunk = ceil_div(ceil_div(N, split), kXT) * kXT;
    split = ceil_div(N, chunk);
  }
  if (split > 65535) return DASTAC_EOVERFLOW;

  const bool atomic = split > 1;
  if (atomic || N == 0) {
    const int64_t zb = ceil_div(count, 256);
    fill_zero_kernel<<<(unsigned)(zb < 8192 ? zb : 8192), 256, 0, st>>>(out, count);
    if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
    if (N == 0) return DASTAC_OK;
  }
  const dim3 grid((unsigned)tiles, (unsigned)split);
  if (atomic)
    pr_f64_kernel<CUBE, true, BK><<<grid, kBlock, 0, st>>>(N, d, B, ldb, out, chunk);
  else
    pr_f64_kernel<CUBE, false, BK><<<grid, kBlock, 0, st>>>(N, d, B, ldb, out, chunk);
  return launch_status();
}

}  // namespace

extern "C" {

int dastac_pr_a2_f64(int64_t N, int64_t d, const double *B, int64_t ldb, double *A2p, void *stream) {
  return d <= kNarrowMaxD2 ? run<false, 64>(N, d, B, ldb, A2p, stream) : run<false, 128>(N, d, B, ldb, A2p, stream);
}

int dastac_pr_a3_f64(int64_t N, int64_t d, const double *B, int64_t ldb, double *A3p, void *stream) {
  return d <= kNarrowMaxD3 ? run<true, 64>(N, d, B, ldb, A3p, stream) : run<true, 128>(N, d, B, ldb, A3p, stream);
}

}  // extern "C"
