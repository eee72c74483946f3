// Polynomial-regression tensors (Table 1, "Polynomial Regression Degree-D") written straight
// into packed hyper-triangles on the matrix cores, single and double precision:
//
//   A2(i,j)   := B(x,i) * B(x,j)            i<=j        packed upper triangle,   tri(d,i,j)
//   A3(i,j,k) := B(x,i) * B(x,j) * B(x,k)   i<=j<=k     packed upper tetrahedron, tet(d,i,j,k)
//
// B is the dense N x d sample matrix; both outputs are symmetric under any permutation of their
// indices and only the unique elements are computed and stored (the output inherits the structure,
// Section 3).  Slice i of A3 is a weighted Gram matrix, sum_x w(x) B(x,j) B(x,k) with w = B(.,i),
// restricted to j,k >= i, whose upper triangle of order d-i is stored contiguously at
// tet_slice_start(d,i); A2 is the same with w = 1 and a single slice.  One kernel serves both.
//
// A workgroup owns a 64 (j) x 128 (k) tile of one slice (eight wavefronts; for small d a 64 x 64 tile and
// four wavefronts) and a range of samples x, which is the reduction index: per step of kXT samples (32 in
// fp32, 16 in fp64), the kXT x 64 tile of B columns j (multiplied by w on the way in) and the tile of B
// columns k are staged in LDS, double-buffered against the global loads of the next step, and each
// wavefront multiplies its 32x32 sub-tile (sweep and per-type matrix-core pieces: mfma_tile.h; both tiles
// keep the sample index first, so both operands are read element by element).  Tiles that lie wholly below the diagonal are never
// launched; tiles on the diagonal stage their full rectangle, wavefronts whose sub-tile lies below it
// skip their matrix instructions, and only j<=k is stored.  When the tile count alone cannot fill the
// chip the sample range is split over several workgroups, which then add into a pre-zeroed output with
// floating-point atomics.
#include "mfma_tile.h"

using namespace dastac;

namespace {

constexpr int kBJ = kTileM;  // j extent of a workgroup tile
// k extent of a workgroup tile: BK = 128 (eight wavefronts) or BK = 64 (four), a template parameter
constexpr int64_t kMaxD2 = 1 << 16;  // A2: tile grid and tri(d) stay small
constexpr int64_t kMaxD3 = 1 << 13;  // A3: the tile count stays inside gridDim.x
constexpr int64_t kMaxN = (int64_t)1 << 31;
// Up to these d the 64 x 64 tile is used: it wastes less on the diagonal and leaves more workgroups per CU,
// which outweighs its lower operand reuse while diagonal tiles are a large share of all tiles (measured in fp32,
// N=100000 resp. 10000: A2 d=512 73 against 49 TFLOP/s, d=1024 91 against 103; A3 d=256 46 against 36, d=1024 78 against 72).
constexpr int64_t kNarrowMaxD2 = 768, kNarrowMaxD3 = 2048;

template <typename T>
struct Stage {
  typename Core<T>::vec a[2];  // j tile: one or two sample rows, one 16-byte piece of columns each
  typename Core<T>::vec b[2];  // k tile: sample rows bk and bk + kXT/2, one 16-byte piece of columns each
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

template <typename T, bool CUBE, bool ATOMIC, int BK>
__global__ __launch_bounds__(4 * BK) void pr_mfma_kernel(int64_t N, int64_t d, const T *__restrict__ B, int64_t ldb,
                                                         T *__restrict__ out, int64_t chunk, int64_t tiles,
                                                         int64_t split) {
  typedef Core<T> K;
  typedef typename K::vec vec;
  typedef typename K::uvec uvec;
  constexpr int kXT = K::kKT, kV = K::kVec, kJP = K::kColPitch;  // samples per step; pitch of the j tile [x][j]
  __shared__ __attribute__((aligned(16))) T As[2][kXT * kJP];
  __shared__ __attribute__((aligned(16))) T Bs[2][kXT * BK];
  constexpr int kThreads = 4 * BK, kWC = BK / 32;  // wavefronts: 2 rows of kWC

  // Work items are (sample share, tile) pairs, share-major.  Workgroup ids are dealt to the eight XCDs in turn,
  // so id%8 picks the XCD and id/8 the position in that XCD's run of CONSECUTIVE items: the tiles of one share
  // read the same rows of B (each its own columns) and sweep them at the same pace, so on one XCD a row is
  // fetched from memory once and served to the other tiles by that L2.
  const int64_t items = tiles * split, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int64_t item = items * xcd / 8 + slot;
  if (item >= items * (xcd + 1) / 8) return;
  const int64_t share = uniform64(item / tiles);
  int64_t i;  // slice: every column index of this workgroup is >= i
  int J, Kb;
  decode_tile(d, CUBE, BK, uniform64(item - share * tiles), i, J, Kb);
  const int64_t q = d - i;  // order of the slice's triangle
  const int64_t xbeg = share * chunk;
  const int64_t xend = xbeg + chunk < N ? xbeg + chunk : N;
  if (xbeg >= xend) return;
  const int nk = (int)ceil_div(xend - xbeg, kXT);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / kWC, wc = wave % kWC;  // 2 x kWC wavefronts: 32 (j) x 32 (k) each
  // A wavefront whose 32x32 sub-tile lies wholly below the diagonal (largest k < smallest j) still helps
  // to stage the tiles but issues no matrix instructions, which leaves the SIMD's matrix pipe to the
  // wavefronts of the other workgroups resident on it.
  const bool live = uniform32(Kb * BK + wc * 32 + 31 >= J * kBJ + wr * 32) != 0;

  // j tile: sample rows tk + kJRows*r (r < kJRep), column offset ti; k tile: sample rows bk and bk + kXT/2, column offset bc
  constexpr int kJRows = kThreads / (kBJ / kV), kJRep = kXT / kJRows;
  static_assert(kJRep == 1 || kJRep == 2, "a thread stages one or two pieces of the j tile");
  const int tk = tid / (kBJ / kV), ti = (tid % (kBJ / kV)) * kV;
  const int bk = tid / (BK / kV), bc = (tid % (BK / kV)) * kV;
  const int64_t j0 = i + (int64_t)J * kBJ, k0 = i + (int64_t)Kb * BK;  // absolute first columns
  const bool j_full = j0 + kBJ <= d, k_full = k0 + BK <= d;

  // Columns c..c+kV-1 of one row of B, zero from column d on, with one vector load whose address is pulled
  // back inside the row (needs d >= kV): a lane that straddles the end shifts what it fetched.
  auto load_clamped = [&](const T *row, int64_t c) -> vec {
    const int64_t cc = c + kV <= d ? c : d - kV;
    const vec v = *reinterpret_cast<const uvec *>(row + cc);
    const int64_t sh = c - cc;  // 0: all inside; 1..kV-1: that many beyond the end; >= kV: all beyond
    vec r;
#pragma unroll
    for (int e = 0; e < kV; ++e) {
      T t = T(0);
#pragma unroll
      for (int f = e; f < kV; ++f) t = sh == f - e ? v[f] : t;
      r[e] = t;
    }
    return r;
  };
  const bool wide = d >= kV;

  auto load_stage = [&](int kt, Stage<T> &s) {
    const int64_t x0 = xbeg + (int64_t)kt * kXT;
    const bool x_full = x0 + kXT <= xend;
#pragma unroll
    for (int r = 0; r < kJRep; ++r) {
      const int64_t xa = x0 + tk + kJRows * r;
      if (x_full && j_full) {
        s.a[r] = *reinterpret_cast<const uvec *>(B + xa * ldb + j0 + ti);
      } else if (x_full && wide) {
        s.a[r] = load_clamped(B + xa * ldb, j0 + ti);
      } else {
#pragma unroll
        for (int e = 0; e < kV; ++e) s.a[r][e] = (xa < xend && j0 + ti + e < d) ? B[xa * ldb + j0 + ti + e] : T(0);
      }
      if (CUBE) {
        const T w = xa < xend ? B[xa * ldb + i] : T(0);
        s.a[r] *= w;
      }
    }
    if (x_full && k_full) {
#pragma unroll
      for (int r = 0; r < 2; ++r)
        s.b[r] = *reinterpret_cast<const uvec *>(B + (x0 + bk + (kXT / 2) * r) * ldb + k0 + bc);
    } else if (x_full && wide) {
#pragma unroll
      for (int r = 0; r < 2; ++r) s.b[r] = load_clamped(B + (x0 + bk + (kXT / 2) * r) * ldb, k0 + bc);
    } else {
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const int64_t x = x0 + bk + (kXT / 2) * r;
#pragma unroll
        for (int e = 0; e < kV; ++e) s.b[r][e] = (x < xend && k0 + bc + e < d) ? B[x * ldb + k0 + bc + e] : T(0);
      }
    }
  };
  auto store_stage = [&](int buf, int, const Stage<T> &s) {
#pragma unroll
    for (int r = 0; r < kJRep; ++r) *reinterpret_cast<vec *>(&As[buf][(tk + kJRows * r) * kJP + ti]) = s.a[r];
#pragma unroll
    for (int r = 0; r < 2; ++r) *reinterpret_cast<vec *>(&Bs[buf][(bk + (kXT / 2) * r) * BK + bc]) = s.b[r];
  };
  auto read_ops = [&](int buf, int, int t, typename K::Ops &o) {
    K::read_a_t(&As[buf][wr * 32], kJP, lane, t, o);
    K::read_b(&Bs[buf][wc * 32], BK, lane, t, o);
  };

  typename K::Acc acc;
  K::clear(acc);
  sweep_steps<T, Stage<T>>(0, nk, acc, load_stage, store_stage, read_ops, live);

  // Rows are j, columns are k; both relative to the slice's first column i.
  T *slice = out + (CUBE ? tet_slice_start(d, i) : 0);
  K::for_each(acc, lane, [&](int r, int c, T v) {
    const int64_t jr = (int64_t)J * kBJ + wr * 32 + r, kr = (int64_t)Kb * BK + wc * 32 + c;
    if (jr <= kr && kr < q) {
      T *p = slice + tri_offset(q, jr, kr);
      if (ATOMIC)
        unsafeAtomicAdd(p, v);
      else
        *p = v;
    }
  });
}

template <typename T>
__global__ void fill_zero_kernel(T *__restrict__ y, int64_t count) {
  for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < count; t += (int64_t)gridDim.x * blockDim.x)
    y[t] = T(0);
}

template <typename T, bool CUBE, int BK>
int run(int64_t N, int64_t d, const T *B, int64_t ldb, T *out, void *stream) {
  constexpr int kBlock = 4 * BK, kXT = Core<T>::kKT;
  constexpr int64_t kB = (int64_t)sizeof(T);
  if (N < 0 || d < 0 || ldb < d) return DASTAC_EINVAL;
  if (d > (CUBE ? kMaxD3 : kMaxD2) || N > kMaxN || ld_too_large(ldb)) return DASTAC_EOVERFLOW;
  if (d == 0) return DASTAC_OK;
  if (!out || (N > 0 && !B)) return DASTAC_ENULL;
  const int64_t count = CUBE ? tet(d) : tri(d);
  if (overlaps(out, count * kB, B, view_bytes(N, ldb, d, kB))) return DASTAC_EALIAS;
  hipStream_t st = (hipStream_t)stream;

  const int64_t tiles = total_tiles(d, CUBE, BK);
  if (tiles > 0x7fffffff) return DASTAC_EOVERFLOW;
  // Split the samples when the tiles alone cannot fill the chip.  All workgroups cost the same, so the
  // launch runs in rounds of `slots` resident workgroups: take the smallest split that fills its last
  // round to 90 %, or else the best one found; every share is a multiple of a step and at least 8 steps.
  int64_t split = 1, chunk = kXT;
  if (N > 0) {
    const int64_t slots = resident_blocks(pr_mfma_kernel<T, CUBE, true, BK>, kBlock);
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
  // one-dimensional grid: every XCD gets ceil(items / 8) ids, of which it uses its share of the items
  const int64_t per_xcd = ceil_div(tiles * split, 8);
  if (8 * per_xcd > 0x7fffffff) return DASTAC_EOVERFLOW;

  const bool atomic = split > 1;
  if (atomic || N == 0) {
    const int64_t zb = ceil_div(count, 256);
    fill_zero_kernel<T><<<(unsigned)(zb < 8192 ? zb : 8192), 256, 0, st>>>(out, count);
    if (hipGetLastError() != hipSuccess) return DASTAC_EHIP;
    if (N == 0) return DASTAC_OK;
  }
  const unsigned grid = (unsigned)(8 * per_xcd);
  if (atomic)
    pr_mfma_kernel<T, CUBE, true, BK><<<grid, kBlock, 0, st>>>(N, d, B, ldb, out, chunk, tiles, split);
  else
    pr_mfma_kernel<T, CUBE, false, BK><<<grid, kBlock, 0, st>>>(N, d, B, ldb, out, chunk, tiles, split);
  return launch_status();
}

}  // namespace

extern "C" {

int dastac_pr_a2_f32(int64_t N, int64_t d, const float *B, int64_t ldb, float *A2p, void *stream) {
  return d <= kNarrowMaxD2 ? run<float, false, 64>(N, d, B, ldb, A2p, stream)
                           : run<float, false, 128>(N, d, B, ldb, A2p, stream);
}

int dastac_pr_a3_f32(int64_t N, int64_t d, const float *B, int64_t ldb, float *A3p, void *stream) {
  return d <= kNarrowMaxD3 ? run<float, true, 64>(N, d, B, ldb, A3p, stream)
                           : run<float, true, 128>(N, d, B, ldb, A3p, stream);
}

// Double precision (the paper's element type): the same kernel on the fp64 matrix cores.
int dastac_pr_a2_f64(int64_t N, int64_t d, const double *B, int64_t ldb, double *A2p, void *stream) {
  return d <= kNarrowMaxD2 ? run<double, false, 64>(N, d, B, ldb, A2p, stream)
                           : run<double, false, 128>(N, d, B, ldb, A2p, stream);
}

int dastac_pr_a3_f64(int64_t N, int64_t d, const double *B, int64_t ldb, double *A3p, void *stream) {
  return d <= kNarrowMaxD3 ? run<double, true, 64>(N, d, B, ldb, A3p, stream)
                           : run<double, true, 128>(N, d, B, ldb, A3p, stream);
}

}  // extern "C"
