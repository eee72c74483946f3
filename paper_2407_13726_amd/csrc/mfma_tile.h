// What the matrix-core kernels with a 64 x 128 workgroup tile share, per element type.
//
// TRMM, SYMM, TTM_UT and the polynomial-regression tensors all let a workgroup of eight wavefronts own a
// 64 x 128 tile of the result and sweep the reduction index in steps: per step a 64 x kKT tile of the
// first operand and a kKT x 128 tile of the second are staged in LDS (double-buffered against the global
// loads of the next step) and each wavefront multiplies its 32 x 32 sub-tile.  The schedule of such a
// sweep is written once (sweep_steps below); what depends on the element type -- the step length, the
// 16-byte piece a thread stages, the operand registers of one group of matrix instructions, how they are
// read from the staged tiles, the instructions themselves and where a result element lives -- is one
// Core<T> each:
//
//   float   v_mfma_f32_32x32x2_f32: lane l feeds row (or column) l%32 at reduction index l/32.  A sum may be
//           taken in any order, so lane half h is given the four consecutive indices 8t+4h..8t+4h+3 of each
//           group of eight: a first operand staged [row][k] is then ONE 16-byte LDS read per group.
//   double  v_mfma_f64_16x16x4_f64: lane l feeds row (or column) l%16 at reduction index l/16; the 32 x 32
//           sub-tile is 2 x 2 tiles of 16 x 16 with four independent accumulators.
#pragma once
#include "common.h"

namespace dastac {

constexpr int kTileM = 64;    // rows of the result per workgroup tile
constexpr int kTileN = 128;   // columns of the result per workgroup tile
constexpr int kTileThreads = 512;


template <typename T>
struct Core;

template <>
struct Core<float> {
  static constexpr int kKT = 32;   // reduction indices per staged step
  static constexpr int kVec = 4;   // elements of a 16-byte piece
  static constexpr int kGroups = 4;  // operand groups per step (eight indices, four matrix instructions each)
  static constexpr int kRowPitch = kKT + 4;     // pitch of a first-operand tile staged [row][k]: 16-byte reads of 8 lanes cover all banks
  static constexpr int kColPitch = kTileM + 4;  // pitch of a first-operand tile staged transposed, [k][row]
  typedef f4a vec;
  typedef f4u uvec;
  struct Acc {
    f16v v;
  };
  struct Ops {
    float a[4], b[4];
  };
  __device__ static void clear(Acc &c) {
#pragma unroll
    for (int v = 0; v < 16; ++v) c.v[v] = 0.0f;
  }
  // first operand, staged [row][k] with pitch kRowPitch; `rows` points at the wavefront's first row
  __device__ static void read_a(const float *rows, int lane, int t, Ops &o) {
    const f4a a = *reinterpret_cast<const f4a *>(rows + (lane & 31) * kRowPitch + 4 * (lane >> 5) + 8 * t);
    o.a[0] = a.x, o.a[1] = a.y, o.a[2] = a.z, o.a[3] = a.w;
  }
  // first operand, staged transposed [k][row] with pitch `pitch`; `cols` points at the wavefront's first row
  __device__ static void read_a_t(const float *cols, int pitch, int lane, int t, Ops &o) {
    const float *p = cols + (4 * (lane >> 5) + 8 * t) * pitch + (lane & 31);
#pragma unroll
    for (int q = 0; q < 4; ++q) o.a[q] = p[q * pitch];
  }
  // second operand, staged [k][column] with pitch `pitch`; `cols` points at the wavefront's first column
  __device__ static void read_b(const float *cols, int pitch, int lane, int t, Ops &o) {
    const float *p = cols + (4 * (lane >> 5) + 8 * t) * pitch + (lane & 31);
#pragma unroll
    for (int q = 0; q < 4; ++q) o.b[q] = p[q * pitch];
  }
  // second operand, staged [column][k] with pitch kRowPitch (k contiguous, like the first): one 16-byte read
  __device__ static void read_b_rows(const float *rows, int lane, int t, Ops &o) {
    const f4a b = *reinterpret_cast<const f4a *>(rows + (lane & 31) * kRowPitch + 4 * (lane >> 5) + 8 * t);
    o.b[0] = b.x, o.b[1] = b.y, o.b[2] = b.z, o.b[3] = b.w;
  }
  __device__ static void mma(const Ops &o, Acc &c) {
#pragma unroll
    for (int q = 0; q < 4; ++q) c.v = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a[q], o.b[q], c.v, 0, 0, 0);
  }
  // f(row, column, value) for every element of the wavefront's 32 x 32 sub-tile this lane holds:
  // register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32
  template <typename F>
  __device__ static void for_each(const Acc &c, int lane, F f) {
#pragma unroll
    for (int v = 0; v < 16; ++v) f(8 * (v / 4) + 4 * (lane >> 5) + (v % 4), lane & 31, c.v[v]);
  }
};

template <>
struct Core<double> {
  static constexpr int kKT = 16;
  static constexpr int kVec = 2;
  static constexpr int kGroups = 4;  // four indices, four matrix instructions each
  static constexpr int kRowPitch = kKT + 2;     // the 16 rows of one operand read fall on distinct banks
  static constexpr int kColPitch = kTileM + 2;
  typedef d2a vec;
  typedef d2u uvec;
  struct Acc {
    d4v v[4];  // 2 x 2 tiles of 16 x 16: v[2*ra + ca]
  };
  struct Ops {
    double a[2], b[2];
  };
  __device__ static void clear(Acc &c) {
#pragma unroll
    for (int t = 0; t < 4; ++t) c.v[t] = d4v{0.0, 0.0, 0.0, 0.0};
  }
  __device__ static void read_a(const double *rows, int lane, int t, Ops &o) {
    const double *p = rows + (lane & 15) * kRowPitch + 4 * t + (lane >> 4);
    o.a[0] = p[0];
    o.a[1] = p[16 * kRowPitch];
  }
  __device__ static void read_a_t(const double *cols, int pitch, int lane, int t, Ops &o) {
    const double *p = cols + (4 * t + (lane >> 4)) * pitch + (lane & 15);
    o.a[0] = p[0];
    o.a[1] = p[16];
  }
  __device__ static void read_b(const double *cols, int pitch, int lane, int t, Ops &o) {
    const double *p = cols + (4 * t + (lane >> 4)) * pitch + (lane & 15);
    o.b[0] = p[0];
    o.b[1] = p[16];
  }
  __device__ static void read_b_rows(const double *rows, int lane, int t, Ops &o) {
    const double *p = rows + (lane & 15) * kRowPitch + 4 * t + (lane >> 4);
    o.b[0] = p[0];
    o.b[1] = p[16 * kRowPitch];
  }
  __device__ static void mma(const Ops &o, Acc &c) {
    c.v[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[0], o.b[0], c.v[0], 0, 0, 0);
    c.v[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[0], o.b[1], c.v[1], 0, 0, 0);
    c.v[2] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[1], o.b[0], c.v[2], 0, 0, 0);
    c.v[3] = __builtin_amdgcn_mfma_f64_16x16x4f64(o.a[1], o.b[1], c.v[3], 0, 0, 0);
  }
  // element v of lane l of a 16 x 16 tile is row 4*v + l/16, column l%16
  template <typename F>
  __device__ static void for_each(const Acc &c, int lane, F f) {
#pragma unroll
    for (int ra = 0; ra < 2; ++ra)
#pragma unroll
      for (int ca = 0; ca < 2; ++ca)
#pragma unroll
        for (int v = 0; v < 4; ++v) f(16 * ra + 4 * v + (lane >> 4), 16 * ca + (lane & 15), c.v[2 * ra + ca][v]);
  }
};

// The sweep over k-steps [lo, hi) of one workgroup tile, written once for every kernel and element type.
//   load(kt, stage)       requests the global pieces of step kt into registers
//   store(buf, kt, stage) writes them to LDS buffer buf
//   read(buf, kt, t, ops) reads the operands of group t of step kt from LDS buffer buf
//   mma(ops)              issues the matrix instructions of one group
// Step kt computes on buffer (kt - lo) & 1.  The global loads of the next step are in flight throughout a
// step; its LDS stores and the workgroup barrier sit BEFORE the last group's matrix instructions, whose
// operands are already in registers, so the matrix pipe has work while the barrier settles and while the
// first operands of the next step come back from LDS.  (Everything a group needs from LDS therefore has to
// be part of `ops`: after the barrier the other wavefronts may already be overwriting the buffer.)  Both
// buffers appear as literals (the loop is unrolled by two), so every LDS address is a compile-time offset.
// The caller places a barrier between two sweeps that use the same buffers.  A wavefront with `active`
// false stages and synchronises like the others but reads no operands and issues no matrix instructions
// (its sub-tile holds nothing to compute).
// PIN: scheduling barriers keep the order as written.  Left alone, the compiler merges the two operand register
// sets and issues a group's LDS reads after the previous group's matrix instructions instead of before them;
// that is the faster code with one workgroup per CU or with run-time step bounds, the written order is faster
// (by up to 8 %) where two workgroups share a CU and the bounds are literals, so the kernels choose.
template <typename Ops, typename Stage, bool PIN = false, typename Load, typename Store, typename Read, typename Mma>
__device__ inline void sweep_groups(int lo, int hi, Load load, Store store, Read read, Mma mma, bool active = true) {
  Stage st;
  Ops oa, ob;
  load(lo, st);
  store(0, lo, st);
  __syncthreads();
  if (active) read(0, lo, 0, oa);
  auto step = [&](int kt, int buf) {
    const bool more = kt + 1 < hi;
    if (more) load(kt + 1, st);
    auto pin = [] {
      if (PIN) __builtin_amdgcn_sched_barrier(0);
    };
    if (active) {
      read(buf, kt, 1, ob);
      pin();
      mma(oa);
      pin();
      read(buf, kt, 2, oa);
      pin();
      mma(ob);
      pin();
      read(buf, kt, 3, ob);
      pin();
      mma(oa);
      pin();
    }
    if (more) store(buf ^ 1, kt + 1, st);
    __syncthreads();
    if (active) {
      if (more) read(buf ^ 1, kt + 1, 0, oa);
      pin();
      mma(ob);
      pin();
    }
  };
  for (int kt = lo; kt < hi; kt += 2) {
    step(kt, 0);
    if (kt + 1 < hi) step(kt + 1, 1);
  }
}

// The common case: one accumulator per wavefront, the operand groups and matrix instructions of Core<T>.
template <typename T, typename Stage, bool PIN = false, typename Load, typename Store, typename Read>
__device__ inline void sweep_steps(int lo, int hi, typename Core<T>::Acc &acc, Load load, Store store, Read read,
                                   bool active = true) {
  typedef Core<T> K;
  static_assert(K::kGroups == 4, "the step schedule is written for four operand groups");
  sweep_groups<typename K::Ops, Stage, PIN>(
      lo, hi, load, store, read, [&](const typename K::Ops &o) { K::mma(o, acc); }, active);
}

// Zero-fills the n x m matrix C (row stride ldc), leaving the padding columns of every row alone.
template <typename T>
__global__ __launch_bounds__(256) void zero_matrix_kernel(T *__restrict__ C, int64_t n, int64_t m, int64_t ldc) {
  constexpr int V = 16 / (int)sizeof(T);
  const int64_t pieces = (m + V - 1) / V, total = n * pieces;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t i = t / pieces, c = (t - i * pieces) * V;
    T *row = C + i * ldc;
    for (int64_t e = c; e < c + V && e < m; ++e) row[e] = T(0);
  }
}

}  // namespace dastac
