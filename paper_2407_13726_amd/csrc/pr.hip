// Polynomial-regression tensors (Table 1, "Polynomial Regression Degree-D") written straight
// into packed hyper-triangles on the matrix cores, single and double precision:
//
//   A2(i,j)   := B(x,i) * B(x,j)            i<=j        packed upper triangle,   tri(d,i,j)
//   A3(i,j,k) := B(x,i) * B(x,j) * B(x,k)   i<=j<=k     packed upper tetrahedron, tet(d,i,j,k)
//
// B is the dense N x d sample matrix; both outputs are symmetric under any permutation of their
// indices and only the unique elements are computed and stored (the output inherits the structure,
// Section 3).  A2 is the upper triangle of the Gram matrix; slice i of A3 is a weighted Gram matrix,
// sum_x w(x) B(x,j) B(x,k) with w = B(.,i), restricted to i <= j <= k, stored contiguously at
// tet_slice_start(d,i).
//
// A workgroup owns a 64 (j) x 128 (k) tile of the (j,k) plane (eight wavefronts; for small d a 64 x 64
// tile and four wavefronts) and a range of samples x, which is the reduction index: per step of kXT
// samples (32 in fp32, 16 in fp64) the kXT x 64 tile of B's columns j and the tile of B's columns k are
// staged in LDS, double-buffered against the global loads of the next step, and each wavefront
// multiplies its 32x32 sub-tile (sweep and per-type matrix-core pieces: mfma_tile.h; both tiles keep the
// sample index first, so both operands are read element by element).  Tiles that lie wholly below the
// diagonal are never launched; tiles on the diagonal stage their full rectangle, wavefronts whose
// sub-tile lies below it skip their matrix instructions, and only j<=k is stored.
//
// For A3 the tiles are cut on a grid that is the same for every slice, and a workgroup takes its tile
// for several consecutive slices i at once (two or four in fp32, two in fp64): the two staged tiles are shared
// by those slices, whose weights B(x,i) are staged beside them and multiplied onto the first operand in
// registers, one accumulator per slice.  The global loads, LDS traffic and barriers of a step are thus
// spent once per 64 (fp32) matrix instructions of a wavefront instead of once per 16.  A tile serves
// the slices i <= its last row; a wavefront whose rows all lie above the slices of the workgroup
// (j < i) has nothing to compute.
//
// When the work items alone cannot fill the chip the sample range is split over several workgroups,
// which then add into a pre-zeroed output with floating-point atomics.
#include "mfma_tile.h"

using namespace dastac;

namespace {

constexpr int kBJ = kTileM;  // j extent of a workgroup tile
// k extent of a workgroup tile: BK = 128 (eight wavefronts) or BK = 64 (four), a template parameter
constexpr int64_t kMaxD2 = 1 << 16;  // A2: tile grid and tri(d) stay small
constexpr int64_t kMaxD3 = 1 << 13;  // A3: the item count stays inside gridDim.x
constexpr int64_t kMaxN = (int64_t)1 << 31;
// Up to these d the 64 x 64 tile is used: it wastes less on the diagonal and leaves more workgroups per CU,
// which outweighs its lower operand reuse while diagonal tiles are a large share of all tiles.
constexpr int64_t kNarrowMaxD2 = 768, kNarrowMaxD3 = 2048;
constexpr int64_t kFewSlicesMaxD3 = 768;  // fp32 A3: two slices per workgroup up to here, four beyond

// Slices of A3 that share a workgroup's staged tiles, and how their weights reach the first operand.
template <typename T>
struct Slices;
template <>
struct Slices<float> {
  // group t of a step: this lane's samples are 8t + 4*(lane/32) + q, q < 4; ws is [slice][sample]
  template <int kNI, typename Ops3>
  __device__ static void scale(const Core<float>::Ops &r, const float *ws, int lane, int t, Ops3 &o) {
#pragma unroll
    for (int ii = 0; ii < kNI; ++ii) {
      const f4a w = *reinterpret_cast<const f4a *>(ws + ii * Core<float>::kKT + 8 * t + 4 * (lane >> 5));
#pragma unroll
      for (int q = 0; q < 4; ++q) o.a[ii][q] = r.a[q] * w[q];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) o.b[q] = r.b[q];
  }
};
template <>
struct Slices<double> {
  // group t of a step: this lane's sample is 4t + lane/16
  template <int kNI, typename Ops3>
  __device__ static void scale(const Core<double>::Ops &r, const double *ws, int lane, int t, Ops3 &o) {
#pragma unroll
    for (int ii = 0; ii < kNI; ++ii) {
      const double w = ws[ii * Core<double>::kKT + 4 * t + (lane >> 4)];
      o.a[ii][0] = r.a[0] * w;
      o.a[ii][1] = r.a[1] * w;
    }
    o.b[0] = r.b[0];
    o.b[1] = r.b[1];
  }
};

template <typename T>
struct Stage {
  typename Core<T>::vec a[2];  // j tile: one or two sample rows, one 16-byte piece of columns each
  typename Core<T>::vec b[2];  // k tile: sample rows bk and bk + kXT/2, one 16-byte piece of columns each
  T w;                         // A3: one weight (first threads only)
};

// Staging of the two column tiles of B, the same for both kernels: columns j0.. (64 of them) and k0.. (BK),
// sample rows x0 .. x0+kXT-1, zeros from column d and from sample xend on.
template <typename T, int BK>
struct Tiles {
  typedef Core<T> K;
  typedef typename K::vec vec;
  typedef typename K::uvec uvec;
  static constexpr int kXT = K::kKT, kV = K::kVec, kJP = K::kColPitch, kThreads = 4 * BK;
  static constexpr int kJRows = kThreads / (kBJ / kV), kJRep = kXT / kJRows;
  static_assert(kJRep == 1 || kJRep == 2, "a thread stages one or two pieces of the j tile");
  const T *B;
  int64_t ldb, d, j0, k0;
  int tk, ti, bk, bc;  // j tile: sample rows tk + kJRows*r, column offset ti; k tile: rows bk, bk + kXT/2, offset bc
  bool j_full, k_full, wide;

  __device__ Tiles(const T *B_, int64_t ldb_, int64_t d_, int64_t j0_, int64_t k0_, int tid)
      : B(B_), ldb(ldb_), d(d_), j0(j0_), k0(k0_) {
    tk = tid / (kBJ / kV), ti = (tid % (kBJ / kV)) * kV;
    bk = tid / (BK / kV), bc = (tid % (BK / kV)) * kV;
    j_full = j0 + kBJ <= d, k_full = k0 + BK <= d, wide = d >= kV;
  }
  // Columns c..c+kV-1 of one row of B, zero from column d on, with one vector load whose address is pulled
  // back inside the row (needs d >= kV): a lane that straddles the end shifts what it fetched.
  __device__ vec load_clamped(const T *row, int64_t c) const {
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
  }
  __device__ void load(int64_t x0, int64_t xend, Stage<T> &s) const {
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
  }
  // the same for a step that lies wholly inside the samples and the columns: no tests
  __device__ void load_whole(int64_t x0, Stage<T> &s) const {
#pragma unroll
    for (int r = 0; r < kJRep; ++r)
      s.a[r] = *reinterpret_cast<const uvec *>(B + (x0 + tk + kJRows * r) * ldb + j0 + ti);
#pragma unroll
    for (int r = 0; r < 2; ++r)
      s.b[r] = *reinterpret_cast<const uvec *>(B + (x0 + bk + (kXT / 2) * r) * ldb + k0 + bc);
  }
  __device__ void store(T *As, T *Bs, const Stage<T> &s) const {
#pragma unroll
    for (int r = 0; r < kJRep; ++r) *reinterpret_cast<vec *>(&As[(tk + kJRows * r) * kJP + ti]) = s.a[r];
#pragma unroll
    for (int r = 0; r < 2; ++r) *reinterpret_cast<vec *>(&Bs[(bk + (kXT / 2) * r) * BK + bc]) = s.b[r];
  }
};

// Work items are (sample share, unit) pairs, share-major.  Workgroup ids are dealt to the eight XCDs in turn,
// so id%8 picks the XCD and id/8 the position in that XCD's run of CONSECUTIVE items: the units of one share
// read the same rows of B (each its own columns) and sweep them at the same pace, so on one XCD a row is
// fetched from memory once and served to the other units by that L2.  False: this workgroup has no item.
__device__ inline bool my_item(int64_t units, int64_t split, int64_t &share, int64_t &unit) {
  const int64_t items = units * split, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int64_t item = items * xcd / 8 + slot;
  if (item >= items * (xcd + 1) / 8) return false;
  share = uniform64(item / units);
  unit = uniform64(item - share * units);
  return true;
}

// ---- A2 ----------------------------------------------------------------------------------------------

// Tiles with work.  With m = ceil(d/64) blocks of rows j there are ceil(m/2) blocks of 128 columns k; tile
// (J,K) holds an element with j<=k exactly when K >= J/2 (integer division), so row block J has
// ceil(m/2) - J/2 tiles.  Tiles are numbered densely, row block after row block, so that consecutive
// workgroup ids (which the hardware deals out to the XCDs in turn) all carry work: numbering the whole
// J x K rectangle and letting the empty tiles exit would leave the XCDs with very different loads,
// because the id modulo 8 would select the column block.  (With BK = 64 the condition is K >= J: row
// block J has m - J tiles, m(m+1)/2 in all.)
DASTAC_HD int64_t tiles_of(int64_t m, int BK) {
  if (BK == 64) return m * (m + 1) / 2;
  const int64_t p = m / 2;
  return (m & 1) ? p * p + 3 * p + 1 : p * (p + 1);
}

__device__ inline void decode_tile(int64_t d, int BK, int64_t t, int &J, int &K) {
  const int64_t m = ceil_div(d, kBJ);
  const int64_t nK = BK == 64 ? m : (m + 1) / 2;  // column blocks
  int64_t Jr = 0;
  while (t >= nK - Jr * kBJ / BK) {  // row block Jr has column blocks Jr*64/BK .. nK-1
    t -= nK - Jr * kBJ / BK;
    ++Jr;
  }
  J = (int)Jr;
  K = (int)(Jr * kBJ / BK + t);
}

template <typename T, bool ATOMIC, int BK>
__global__ __launch_bounds__(4 * BK) void pr2_mfma_kernel(int64_t N, int64_t d, const T *__restrict__ B, int64_t ldb,
                                                          T *__restrict__ out, int64_t chunk, int64_t tiles,
                                                          int64_t split) {
  typedef Core<T> K;
  constexpr int kXT = K::kKT, kJP = K::kColPitch, kWC = BK / 32;  // wavefronts: 2 rows of kWC
  __shared__ __attribute__((aligned(16))) T As[2][kXT * kJP];
  __shared__ __attribute__((aligned(16))) T Bs[2][kXT * BK];

  int64_t share, unit;
  if (!my_item(tiles, split, share, unit)) return;
  int J, Kb;
  decode_tile(d, BK, unit, J, Kb);
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
  const Tiles<T, BK> tiles_io(B, ldb, d, (int64_t)J * kBJ, (int64_t)Kb * BK, tid);

  auto load_stage = [&](int kt, Stage<T> &s) { tiles_io.load(xbeg + (int64_t)kt * kXT, xend, s); };
  auto store_stage = [&](int buf, int, const Stage<T> &s) { tiles_io.store(As[buf], Bs[buf], s); };
  auto read_ops = [&](int buf, int, int t, typename K::Ops &o) {
    K::read_a_t(&As[buf][wr * 32], kJP, lane, t, o);
    K::read_b(&Bs[buf][wc * 32], BK, lane, t, o);
  };

  typename K::Acc acc;
  K::clear(acc);
  // The whole steps of a whole tile run as a sweep of their own, whose loop holds none of the edge tests; the
  // ragged last step follows.  (Pinned order in double precision: 6 % faster there, no gain in single.)
  const int nwhole = (tiles_io.j_full && tiles_io.k_full) ? (int)((xend - xbeg) / kXT) : 0;
  if (nwhole > 0) {
    sweep_steps<T, Stage<T>, sizeof(T) == 8>(
        0, nwhole, acc, [&](int kt, Stage<T> &s) { tiles_io.load_whole(xbeg + (int64_t)kt * kXT, s); }, store_stage,
        read_ops, live);
    if (nk > nwhole) __syncthreads();
  }
  if (nk > nwhole) sweep_steps<T, Stage<T>, sizeof(T) == 8>(nwhole, nk, acc, load_stage, store_stage, read_ops, live);

  K::for_each(acc, lane, [&](int r, int c, T v) {
    const int64_t j = (int64_t)J * kBJ + wr * 32 + r, k = (int64_t)Kb * BK + wc * 32 + c;
    if (j <= k && k < d) {
      T *p = out + tri_offset(d, j, k);
      if (ATOMIC)
        unsafeAtomicAdd(p, v);
      else
        *p = v;
    }
  });
}

// ---- A3 ----------------------------------------------------------------------------------------------

// Units of A3: tile (J,K) of the (j,k) plane -- the same grid for every slice -- times a group of NI
// consecutive slices.  Row block J serves the slices 0 .. min(64(J+1), d)-1 (a slice needs i <= j), in
// ceil(that / NI) groups, and has as many tiles as in A2; units are numbered densely: row block after row
// block, slice group after slice group, column block after column block.
DASTAC_HD int64_t units_of_row_block(int64_t d, int BK, int NI, int64_t J) {
  const int64_t m = ceil_div(d, kBJ), nK = BK == 64 ? m : (m + 1) / 2;
  const int64_t slices = kBJ * (J + 1) < d ? kBJ * (J + 1) : d;
  return (nK - J * kBJ / BK) * ceil_div(slices, NI);
}

DASTAC_HD int64_t total_units(int64_t d, int BK, int NI) {
  int64_t total = 0;
  for (int64_t J = 0; J < ceil_div(d, kBJ); ++J) total += units_of_row_block(d, BK, NI, J);
  return total;
}

// One operand group of a step for NI slices: the first operand scaled by each slice's weights, the second shared.
template <typename T, int NI>
struct Ops3 {
  static constexpr int kNA = (int)(sizeof(typename Core<T>::Ops) / sizeof(T)) / 2;
  T a[NI][kNA];
  T b[kNA];
};

// NI slices per workgroup: four in fp32 (two up to d = 768, where a third wavefront per SIMD is worth more than the
// reuse: d=256 61 -> 63 TFLOP/s, d=512 82 -> 86, d=1024 104 -> 102), two in fp64.  Three wavefronts per SIMD with two
// slices (in fp64 the register allocator reaches that with a few spilled dwords and the third wavefront gains 15 %);
// the accumulators of four slices leave room for two.
template <typename T, bool ATOMIC, int BK, int NI>
__global__ __launch_bounds__(4 * BK) __attribute__((amdgpu_waves_per_eu(NI == 2 ? 3 : 2, NI == 2 ? 3 : 2)))
void pr3_mfma_kernel(int64_t N, int64_t d, const T *__restrict__ B, int64_t ldb, T *__restrict__ out, int64_t chunk,
                     int64_t units, int64_t split) {
  typedef Core<T> K;
  constexpr int kXT = K::kKT, kJP = K::kColPitch, kWC = BK / 32, kNI = NI;
  constexpr int kWThreads = kXT * kNI;  // threads that stage one weight each
  static_assert(32 % kNI == 0 && kWThreads <= 4 * BK, "slice groups never straddle a sub-tile's first row");
  __shared__ __attribute__((aligned(16))) T As[2][kXT * kJP];
  __shared__ __attribute__((aligned(16))) T Bs[2][kXT * BK];
  __shared__ __attribute__((aligned(16))) T Ws[2][kNI * kXT];  // [slice][sample]

  int64_t share, unit;
  if (!my_item(units, split, share, unit)) return;
  int64_t J = 0;
  while (unit >= units_of_row_block(d, BK, kNI, J)) unit -= units_of_row_block(d, BK, kNI, J), ++J;
  const int64_t m = ceil_div(d, kBJ), nK = BK == 64 ? m : (m + 1) / 2, firstK = J * kBJ / BK;
  const int64_t i0 = kNI * (unit / (nK - firstK));  // first slice of the group
  const int64_t Kb = firstK + unit % (nK - firstK);
  const int64_t xbeg = share * chunk;
  const int64_t xend = xbeg + chunk < N ? xbeg + chunk : N;
  if (xbeg >= xend) return;
  const int nk = (int)ceil_div(xend - xbeg, kXT);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / kWC, wc = wave % kWC;  // 2 x kWC wavefronts: 32 (j) x 32 (k) each
  const int64_t jw = J * kBJ + wr * 32, kw = Kb * BK + wc * 32;  // first row and column of this wavefront's sub-tile
  // Nothing to compute where the sub-tile lies wholly below the diagonal (largest k < smallest j) or wholly
  // above the group's slices (largest j < i0; i0 and the sub-tile's first row are both multiples of kNI, so
  // the group's slices are then all above it or all not).
  const bool live = uniform32((kw + 31 >= jw && jw + 31 >= i0) ? 1 : 0) != 0;
  const Tiles<T, BK> tiles_io(B, ldb, d, J * kBJ, Kb * BK, tid);
  const int wx = tid % kXT, wi = tid / kXT;  // weights: sample wx of slice i0 + wi (threads below kWThreads)

  auto load_stage = [&](int kt, Stage<T> &s) {
    const int64_t x0 = xbeg + (int64_t)kt * kXT;
    tiles_io.load(x0, xend, s);
    if (tid < kWThreads) {
      const int64_t xw = x0 + wx, iw = i0 + wi;
      s.w = (xw < xend && iw < d) ? B[xw * ldb + iw] : T(0);
    }
  };
  auto store_stage = [&](int buf, int, const Stage<T> &s) {
    tiles_io.store(As[buf], Bs[buf], s);
    if (tid < kWThreads) Ws[buf][wi * kXT + wx] = s.w;
  };
  auto read_ops = [&](int buf, int, int t, Ops3<T, NI> &o) {
    typename K::Ops r;
    K::read_a_t(&As[buf][wr * 32], kJP, lane, t, r);
    K::read_b(&Bs[buf][wc * 32], BK, lane, t, r);
    Slices<T>::template scale<NI>(r, Ws[buf], lane, t, o);
  };
  typename K::Acc acc[kNI];
#pragma unroll
  for (int ii = 0; ii < kNI; ++ii) K::clear(acc[ii]);
  auto mma = [&](const Ops3<T, NI> &o) {
#pragma unroll
    for (int ii = 0; ii < kNI; ++ii) {
      typename K::Ops r;
#pragma unroll
      for (int q = 0; q < Ops3<T, NI>::kNA; ++q) r.a[q] = o.a[ii][q], r.b[q] = o.b[q];
      K::mma(r, acc[ii]);
    }
  };
  // whole steps of a whole tile first, in a sweep without edge tests, then the ragged last step
  const int nwhole = (tiles_io.j_full && tiles_io.k_full) ? (int)((xend - xbeg) / kXT) : 0;
  if (nwhole > 0) {
    const bool w_mine = tid < kWThreads && i0 + wi < d;
    sweep_groups<Ops3<T, NI>, Stage<T>>(
        0, nwhole,
        [&](int kt, Stage<T> &s) {
          const int64_t x0 = xbeg + (int64_t)kt * kXT;
          tiles_io.load_whole(x0, s);
          if (tid < kWThreads) s.w = w_mine ? B[(x0 + wx) * ldb + i0 + wi] : T(0);
        },
        store_stage, read_ops, mma, live);
    if (nk > nwhole) __syncthreads();
  }
  if (nk > nwhole) sweep_groups<Ops3<T, NI>, Stage<T>>(nwhole, nk, load_stage, store_stage, read_ops, mma, live);
  if (!live) return;

#pragma unroll
  for (int ii = 0; ii < kNI; ++ii) {
    const int64_t i = i0 + ii, q = d - i;  // slice and the order of its triangle
    if (i >= d) break;
    T *slice = out + tet_slice_start(d, i);
    K::for_each(acc[ii], lane, [&](int r, int c, T v) {
      const int64_t j = jw + r, k = kw + c;
      if (i <= j && j <= k && k < d) {
        T *p = slice + tri_offset(q, j - i, k - i);
        if (ATOMIC)
          unsafeAtomicAdd(p, v);
        else
          *p = v;
      }
    });
  }
}

template <typename T>
__global__ void fill_zero_kernel(T *__restrict__ y, int64_t count) {
  for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < count; t += (int64_t)gridDim.x * blockDim.x)
    y[t] = T(0);
}

template <typename T, bool CUBE, bool ATOMIC, int BK, int NI>
void launch(unsigned grid, hipStream_t st, int64_t N, int64_t d, const T *B, int64_t ldb, T *out, int64_t chunk,
            int64_t units, int64_t split) {
  if (CUBE)
    pr3_mfma_kernel<T, ATOMIC, BK, NI><<<grid, 4 * BK, 0, st>>>(N, d, B, ldb, out, chunk, units, split);
  else
    pr2_mfma_kernel<T, ATOMIC, BK><<<grid, 4 * BK, 0, st>>>(N, d, B, ldb, out, chunk, units, split);
}

// NI: slices per workgroup of the A3 kernel (not used for A2)
template <typename T, bool CUBE, int BK, int NI = 2>
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

  const int64_t units = CUBE ? total_units(d, BK, NI) : tiles_of(ceil_div(d, kBJ), BK);
  if (units > 0x7fffffff) return DASTAC_EOVERFLOW;
  // Split the samples when the units alone cannot fill the chip.  All workgroups cost the same, so the
  // launch runs in rounds of `slots` resident workgroups: take the smallest split that fills its last
  // round to 90 %, or else the best one found; every share is a multiple of a step and at least 8 steps.
  int64_t split = 1, chunk = kXT;
  if (N > 0) {
    const int64_t slots = CUBE ? resident_blocks(pr3_mfma_kernel<T, true, BK, NI>, kBlock)
                               : resident_blocks(pr2_mfma_kernel<T, true, BK>, kBlock);
    if (slots <= 0) return DASTAC_EHIP;
    const int64_t max_split = N / (8 * kXT) > 1 ? N / (8 * kXT) : 1;
    double best = -1.0;
    for (int64_t s = 1; s <= max_split && s <= 4096; ++s) {
      const int64_t blocks = units * s, rounds = ceil_div(blocks, slots);
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
  const int64_t per_xcd = ceil_div(units * split, 8);
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
    launch<T, CUBE, true, BK, NI>(grid, st, N, d, B, ldb, out, chunk, units, split);
  else
    launch<T, CUBE, false, BK, NI>(grid, st, N, d, B, ldb, out, chunk, units, split);
  return launch_status();
}

}  // namespace

extern "C" {

int dastac_pr_a2_f32(int64_t N, int64_t d, const float *B, int64_t ldb, float *A2p, void *stream) {
  return d <= kNarrowMaxD2 ? run<float, false, 64>(N, d, B, ldb, A2p, stream)
                           : run<float, false, 128>(N, d, B, ldb, A2p, stream);
}

int dastac_pr_a3_f32(int64_t N, int64_t d, const float *B, int64_t ldb, float *A3p, void *stream) {
  return d <= kFewSlicesMaxD3 ? run<float, true, 64, 2>(N, d, B, ldb, A3p, stream)
         : d <= kNarrowMaxD3  ? run<float, true, 64, 4>(N, d, B, ldb, A3p, stream)
                              : run<float, true, 128, 4>(N, d, B, ldb, A3p, stream);
}

// Double precision (the paper's element type): the same kernel on the fp64 matrix cores.
int dastac_pr_a2_f64(int64_t N, int64_t d, const double *B, int64_t ldb, double *A2p, void *stream) {
  return d <= kNarrowMaxD2 ? run<double, false, 64>(N, d, B, ldb, A2p, stream)
                           : run<double, false, 128>(N, d, B, ldb, A2p, stream);
}

int dastac_pr_a3_f64(int64_t N, int64_t d, const double *B, int64_t ldb, double *A3p, void *stream) {
  return d <= kNarrowMaxD3 ? run<double, true, 64, 2>(N, d, B, ldb, A3p, stream)
                           : run<double, true, 128, 2>(N, d, B, ldb, A3p, stream);
}

}  // extern "C"
