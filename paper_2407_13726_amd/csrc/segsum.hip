// TRMV over a packed upper triangle and TTV over a packed upper tetrahedron.
//
//   y(j)    := U(j,k) * x(k),      j<=k        (Table 1/2, SpMV_UT)
//   M(i,j)  := A(i,j,k) * v(k),    i<=j<=k     (same layout rule, one more iterator)
//
// Both are sums over the contiguous rows ("fibres") of the packed buffer: row (i,j) holds the
// elements k=j..n-1 back to back, rows follow one another in iteration order, and the outputs are
// numbered in the same order (M is itself a packed triangle).  Slice i of the tetrahedron is a
// packed triangle of order n-i, so TRMV is exactly the first slice of TTV and one kernel serves
// both.
//
// Work split (Section 5.2, "Parallelization": the index depends only on the current iterators, so
// any partition of the loops is correct).  The packed buffer is cut into equal contiguous shares,
// one per wavefront; a wavefront owns the rows that START inside its share.  The inverse index
// polynomial, evaluated once per wavefront, names the first such row; after that the row start
// advances by the row length (the polynomial's linear term), all in wave-uniform registers.
// The last slices of a tetrahedron are tiny, and a step (below) never spans two slices, so equal
// shares would leave the last wavefront with a long chain of nearly empty steps: instead the last
// `tail_order` slices get one wavefront each, located by the forward polynomial alone.
//
// Inside its rows a wavefront takes "steps" of one contiguous span of the buffer:
//   * a row longer than the span is cut into pieces that accumulate per lane and are reduced once,
//     at the row's last piece;
//   * shorter rows get 64, 32, 16, ... 1 lanes each, and 1, 2, 4, ... 64 consecutive rows are summed
//     side by side, so lanes stay busy on the short rows at the end of every slice.
// The step sequence depends only on wave-uniform integers, so the loads of the next step are issued
// before the current step is reduced; two register sets alternate to keep them in flight.
#include "common.h"

using namespace dastac;

namespace {

template <int CTRL>
__device__ inline float dpp_add(float v) {
  int t = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false);
  return v + __builtin_bit_cast(float, t);
}

template <int CTRL>
__device__ inline double dpp_add(double v) {  // the two halves of a double travel separately
  const uint64_t b = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, 0xf, 0xf, false);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, 0xf, 0xf, false);
  return v + __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// Sum over aligned groups of 2^lg lanes; every lane of a group receives the total.
// Strides 1,2 use quad permutes, 4 and 8 the half-row and row mirrors (all lanes of the mirrored
// unit already hold equal values), 16 and 32 go through the LDS crossbar.
template <typename T>
__device__ inline T group_sum(T v, int lg) {
  if (lg >= 1) v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
  if (lg >= 2) v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
  if (lg >= 3) v = dpp_add<0x141>(v);  // row_half_mirror
  if (lg >= 4) v = dpp_add<0x140>(v);  // row_mirror
  if (lg >= 5) v += __shfl_xor(v, 16, 64);
  if (lg >= 6) v += __shfl_xor(v, 32, 64);
  return v;
}

// First row whose first element is at packed position >= q (q < total): its slice i, row j and
// start position p.  This is the inverse index polynomial, arranged so that the device never
// divides: with Q = total-1-q (elements after q),
//   slice:  the largest s with Tet(s) <= Q, tested as s(s+1)(s+2) <= 6Q; the slice is n-1-s, and
//           Q - Tet(s) elements follow q inside it (Tet(s) by an exact multiply with 3^-1 mod 2^64);
//   row:    the largest r with Tri(r) <= Q', tested as r(r+1) <= 2Q'; the row holds r+1 elements
//           and e = Q' - Tri(r) of them follow q.
// Single-precision roots give the seeds; the integer tests make them exact (the seed is within a
// step or two for every size that fits in memory).
template <bool TET>
__device__ inline void first_row_from(int64_t n, int64_t total, int64_t q, int64_t &i, int64_t &j, int64_t &p) {
  uint64_t Q = (uint64_t)(total - 1 - q);
  int64_t a = 0, m = n;
  if (TET) {
    const uint64_t Q6 = 6 * Q;
    uint64_t s = (uint64_t)cbrtf((float)Q6);
    while (s > 0 && s * (s + 1) * (s + 2) > Q6) --s;
    while ((s + 1) * (s + 2) * (s + 3) <= Q6) ++s;
    a = n - 1 - (int64_t)s;
    m = (int64_t)s + 1;
    Q -= (((s * (s + 1)) >> 1) * (s + 2)) * 0xAAAAAAAAAAAAAAABull;  // Tet(s), exact
  }
  const uint64_t Q2 = 2 * Q;
  uint64_t r = (uint64_t)((sqrtf(4.0f * (float)Q2 + 1.0f) - 1.0f) * 0.5f);
  while (r > 0 && r * (r + 1) > Q2) --r;
  while ((r + 1) * (r + 2) <= Q2) ++r;
  const int64_t e = (int64_t)(Q - ((r * (r + 1)) >> 1));  // elements after q in its row
  const int64_t jj = m - 1 - (int64_t)r;                    // row inside the slice, r+1 elements long
  if (e == (int64_t)r) {  // q is itself a row start
    i = a; j = a + jj; p = q;
  } else {                // skip the rest of the row that contains q
    p = q + e + 1;
    if (jj + 1 < m) { i = a; j = a + jj + 1; }
    else { i = a + 1; j = a + 1; }
  }
}

// ---------------------------------------------------------------------------------------------
// The vector operand fits in LDS (n <= kLdsMaxN).  Serves every TTV, and TRMV up to that order
// (larger triangles go to the column-panel kernel of trimv.hip).
//
// x is staged once per workgroup, followed by kPad zeros.  A lane handles sixteen packed elements
// (eight in double precision) per step (four 16-byte loads, each contiguous across the lanes of a row) without any bounds
// test: elements past the end of its row meet a zero of the pad, and the product is formed with
// v_mul_legacy_f32 (0 * anything = 0), so they contribute exactly nothing even if they are Inf or
// NaN.  A load that would lie wholly past the row's end is aimed at the row's last piece instead,
// which is on its way anyway: rows use 3/4 of their lanes' capacity on average, and fetching the
// unused quarter from memory cost 15 % of the bandwidth.  Only steps within kSpan elements of the
// end of the whole buffer take the guarded loader.
// ---------------------------------------------------------------------------------------------
constexpr int kLdsBlock = 512;
constexpr int kLdsWaves = kLdsBlock / 64;
constexpr int kLdsMaxN = 8192;

__device__ inline float mul0(float a, float b) {  // 0 * x == 0 for every x
  float r;
  asm("v_mul_legacy_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

__device__ inline float dot0(f4a a, f4a x) {
  return (mul0(a.x, x.x) + mul0(a.y, x.y)) + (mul0(a.z, x.z) + mul0(a.w, x.w));
}

// Double precision has no multiply that returns 0 for 0 * Inf: a product with a zero of x is dropped by a
// select instead (the same meaning: a zero of x contributes nothing, whatever it multiplies).
__device__ inline double dot0(d2a a, d2a x) {
  return (x.x == 0.0 ? 0.0 : a.x * x.x) + (x.y == 0.0 ? 0.0 : a.y * x.y);
}

// Per element type: a lane's load is one 16-byte piece of kPer elements, a lane takes four pieces per
// step (2^kLg elements), a step spans kSpan elements.
template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int kPer = 4, kLg = 4;
  typedef f4a vec;
  typedef f4u uvec;
};
template <>
struct Elem<double> {
  static constexpr int kPer = 2, kLg = 3;
  typedef d2a vec;
  typedef d2u uvec;
};

template <typename T>
constexpr int kSpanOf = 64 * 4 * Elem<T>::kPer;  // packed elements per step: 64 lanes x 4 loads x one piece
template <typename T>
constexpr int kPadOf = kSpanOf<T> + 8;  // zeros after x: a lane may look up to a span and a piece past the row end

template <typename T>
struct Piece16 {
  typename Elem<T>::vec a[4], x[4];
};

// A step of the LDS variant in 32-bit arithmetic: positions are relative to the wavefront's first
// row (packed position p0, output position s0), which keeps every per-step update to single
// scalar instructions.
struct Step32 {
  int p;    // packed position of the step's first row, minus p0
  int s;    // output position of that row, minus s0
  int j;    // its first column
  int len;  // its length (== rows left in the slice)
  int t0;   // long rows: offset of this piece inside the row; else 0
  int slice;  // slice of the tetrahedron the row belongs to
  bool valid;
};

// STREAM: the packed buffer is larger than the memory-side cache, so its loads are non-temporal
// (measured 10 % faster there); a smaller buffer is read through the caches, where the lines
// shared by two neighbouring rows are fetched once (measured 9 % faster at 90 MB).
// PAD: the output vector goes on for `zeros` entries behind the n sums, and they are zeros of the product (the
// sub-triangular domain of Section 6.4 has no element in those rows); the launch clears them on its way.
template <typename T, bool TET, bool STREAM, bool PAD = false>
__global__ __launch_bounds__(kLdsBlock) void segsum_lds_kernel(int n, const T *__restrict__ A,
                                                               const T *__restrict__ x,
                                                               T *__restrict__ out, int64_t total,
                                                               int64_t total_a, int64_t share, int64_t waves_a,
                                                               int tail_order, int64_t zeros) {
  constexpr int kPer = Elem<T>::kPer, kLg = Elem<T>::kLg, kSpan = kSpanOf<T>, kPad = kPadOf<T>;
  typedef typename Elem<T>::vec vec;
  typedef typename Elem<T>::uvec uvec;
  extern __shared__ __attribute__((aligned(16))) unsigned char xs_bytes[];
  T *xs = reinterpret_cast<T *>(xs_bytes);  // x[0..n), then kPad zeros
  // Request this thread's first four values of x right away; they arrive while the wavefront
  // works out which rows it owns.
  T xr[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int t = threadIdx.x + q * kLdsBlock;
    xr[q] = t < n ? x[t] : T(0);
  }
  if (PAD)
    for (int64_t t = (int64_t)blockIdx.x * kLdsBlock + threadIdx.x; t < zeros; t += (int64_t)gridDim.x * kLdsBlock)
      out[n + t] = T(0);
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * kLdsWaves + uniform32(threadIdx.x >> 6);

  // Which rows are mine: those starting in [first row at or after lo, hi).
  int64_t hi64 = 0, sp = 0, sj = 0;
  int slice = 0;
  bool active = true;
  if (wave < waves_a) {  // an equal share of the first total_a elements
    const int64_t lo = wave * share;
    hi64 = (lo + share < total_a) ? lo + share : total_a;
    int64_t si;
    first_row_from<TET>(n, total, lo, si, sj, sp);
    slice = (int)si;
  } else if (TET && wave - waves_a < tail_order) {  // one whole slice of the tail
    slice = n - tail_order + (int)(wave - waves_a);
    sp = tet_slice_start(n, slice);
    sj = slice;
    hi64 = sp + tri(n - slice);
  } else {
    active = false;
  }
  slice = uniform32(slice);
  const int64_t p0 = uniform64(sp);
  const int64_t s0 = TET ? tri_offset(n, slice, uniform32((int)sj)) : uniform32((int)sj);
  const T *__restrict__ A0 = A + p0;
  T *__restrict__ out0 = out + s0;
  const int64_t room_hi = uniform64(hi64) - p0, room_total = total - p0;
  const int hi = room_hi > 0x3fffffff ? 0x3fffffff : (int)room_hi;          // rows must start before hi
  const int end = room_total > 0x3fffffff ? 0x3fffffff : (int)room_total;    // one past the last element

  Step32 st;
  st.p = 0;
  st.s = 0;
  st.j = uniform32((int)sj);
  st.len = n - st.j;
  st.t0 = 0;
  st.slice = slice;
  st.valid = active && st.p < hi && st.len > 0;

  // per-lane geometry of a step: row g of the group, `used` rows taken by the step
  auto geometry = [&](const Step32 &d, int &g, int &used, bool &mine, int &off, int &sub4, int &lim, int &xi,
                      int &lw4) {
    const int v = (d.len + (1 << kLg) - 1) >> kLg;            // lanes a row of this length needs
    int lg = v <= 1 ? 0 : 32 - __builtin_clz(v - 1);         // ceil(log2(v))
    if (lg > 6) lg = 6;
    lw4 = kPer << lg;  // elements between two consecutive loads of a lane
    int rows = 64 >> lg;
    if (rows > d.len) rows = d.len;  // stay inside the slice
    g = lane >> lg;
    sub4 = (lane & ((1 << lg) - 1)) * kPer;
    const int goff = g * d.len - ((g * (g - 1)) >> 1);  // start of row g relative to d.p
    mine = g < rows && goff < hi - d.p;
    used = __popcll(__ballot(mine && sub4 == 0));
    // element offset (relative to p0) of the first element this lane may use; lanes without a row
    // (whose goff is meaningless, possibly negative) point at the start of the step instead
    off = d.p + (mine ? goff + d.t0 : 0);
    // last 4-element piece that still holds an element of my row (my row has len - g elements, of
    // which t0 are behind this step)
    lim = mine ? (d.len - g - d.t0 - 1) & ~(kPer - 1) : 0;
    // column of my first element; lanes without a row look at the zero pad
    xi = mine ? d.j + g + d.t0 + sub4 : n;
  };
  // every lane's loads of step d lie inside the buffer
  auto fits = [&](const Step32 &d) -> bool { return d.p + d.t0 + kSpan + kPer <= end; };

  // Loads that would start past the end of the lane's row are pointed at the row's last piece
  // instead: the line is being fetched anyway, so they cost no memory traffic, and whatever they
  // return meets a zero of the pad.
  auto issue_a = [&](const Step32 &d, int &g, int &used, int &xi, int &lw4, Piece16<T> &r) {
    bool mine;
    int off, sub4, lim;
    geometry(d, g, used, mine, off, sub4, lim, xi, lw4);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      int e = sub4 + q * lw4;
      e = e < lim ? e : lim;
      const uvec *src = reinterpret_cast<const uvec *>(A0 + off + e);
      r.a[q] = STREAM ? __builtin_nontemporal_load(src) : *src;
    }
  };
  auto issue_x = [&](int xi, int lw4, Piece16<T> &r) {
#pragma unroll
    for (int q = 0; q < 4; ++q) r.x[q] = *reinterpret_cast<const uvec *>(&xs[xi + q * lw4]);
  };
  auto issue_guarded = [&](const Step32 &d, int &g, int &used, Piece16<T> &r) {
    bool mine;
    int off, sub4, lim, xi, lw4;
    geometry(d, g, used, mine, off, sub4, lim, xi, lw4);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      vec e;
#pragma unroll
      for (int c = 0; c < kPer; ++c) {
        const int o = off + sub4 + q * lw4 + c;
        e[c] = (mine && o < end) ? A0[o] : T(0);
      }
      r.a[q] = e;
    }
    issue_x(xi, lw4, r);
  };
  auto advance = [&](const Step32 &d, int used) -> Step32 {
    Step32 nx = d;
    if (d.len > kSpan && d.t0 + kSpan < d.len) {  // next piece of the same long row
      nx.t0 = d.t0 + kSpan;
      return nx;
    }
    nx.t0 = 0;
    nx.p = d.p + used * d.len - ((used * (used - 1)) >> 1);
    nx.s = d.s + used;
    nx.j = d.j + used;
    if (TET && nx.j >= n) {  // slice finished
      nx.slice = d.slice + 1;
      nx.j = nx.slice;
    }
    nx.len = n - nx.j;
    nx.valid = nx.p < hi && nx.len > 0;
    return nx;
  };

  T racc = T(0);  // running per-lane sum of a long row
  auto consume = [&](const Step32 &d, const Piece16<T> &c, int g, int used) {
    T v = (dot0(c.a[0], c.x[0]) + dot0(c.a[1], c.x[1])) + (dot0(c.a[2], c.x[2]) + dot0(c.a[3], c.x[3]));
    if (d.len > kSpan) {
      racc += v;
      if (d.t0 + kSpan >= d.len) {
        v = group_sum(racc, 6);
        racc = T(0);
        if (lane == 0) out0[d.s] = v;
      }
    } else {
      const int w = (d.len + (1 << kLg) - 1) >> kLg;
      int lg = w <= 1 ? 0 : 32 - __builtin_clz(w - 1);
      v = group_sum(v, lg);
      const int sub = lane & ((1 << lg) - 1);
      if (sub == 0 && g < used) out0[d.s + g] = v;
    }
  };

  // The packed loads of the first step do not depend on LDS: request them before x is staged.
  Piece16<T> pa, pb;
  int ga = 0, ua = 0, gb = 0, ub = 0, xia = 0, lwa = 4, xib = 0, lwb = 4;
  const bool fast = st.valid && fits(st);
  if (fast) issue_a(st, ga, ua, xia, lwa, pa);

#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int t = threadIdx.x + q * kLdsBlock;
    if (t < n + kPad) xs[t] = xr[q];
  }
  for (int t = threadIdx.x + 4 * kLdsBlock; t < n + kPad; t += kLdsBlock) xs[t] = t < n ? x[t] : T(0);
  __syncthreads();

  // Unguarded steps: two register sets alternate, and nothing but the reductions is branched
  // around, so the next step's loads stay in flight while the current step is reduced.  When the
  // next step does not exist (or needs the guarded loader) the last good one is loaded again and
  // ignored.  The loop leaves only at its bottom: an exit between the two halves would make the
  // compiler drain every load at the top of the loop.
  if (fast) {
    issue_x(xia, lwa, pa);
    bool more2;
    do {
      const Step32 n1 = advance(st, ua);
      const bool more1 = n1.valid && fits(n1);
      issue_a(more1 ? n1 : st, gb, ub, xib, lwb, pb);
      issue_x(xib, lwb, pb);
      consume(st, pa, ga, ua);
      const Step32 n2 = advance(n1, ub);  // meaningful only if more1
      more2 = more1 && n2.valid && fits(n2);
      issue_a(more2 ? n2 : more1 ? n1 : st, ga, ua, xia, lwa, pa);
      issue_x(xia, lwa, pa);
      if (more1) consume(n1, pb, gb, ub);
      st = more1 ? n2 : n1;
    } while (more2);
  }
  // Steps that reach into the last kSpan elements of the buffer.
  while (st.valid) {
    Piece16<T> pc;
    int gc, uc;
    issue_guarded(st, gc, uc, pc);
    consume(st, pc, gc, uc);
    st = advance(st, uc);
  }
}

// ---- host side -------------------------------------------------------------------------------

// Wavefront shares: about `per_cu` wavefronts per compute unit on a 256-CU part, at least 2048
// elements each so that the one inverse per wavefront stays negligible.  Problems of a megabyte or
// two are bound by the latency of one wavefront's chain of steps, not by the inverse: there a share is
// one step or half a step (measured, event-bracketed: TRMV n=512 8.4 -> 6.4 us, n=2048 8.7 -> 7.5;
// TTV n=128 9.0 -> 7.4; from about 2.6 million elements on the larger floor is the faster one).
inline int64_t pick_share(int64_t total, int per_cu) {
  const int64_t share = ceil_div(total, (int64_t)256 * per_cu);
  const int64_t least = total < ((int64_t)1 << 20) ? 512 : total < ((int64_t)5 << 19) ? 1024 : 2048;
  return share < least ? least : share;
}

constexpr int64_t kStreamBytes = (int64_t)192 << 20;  // above this a buffer does not stay in the 256 MB memory-side cache

template <typename T, bool TET, bool PAD = false>
int launch_lds(int64_t n, const T *A, const T *x, T *out, int64_t total, void *stream, int64_t zeros = 0) {
  int64_t tail_order = 0, total_a = total;
  if (TET) {  // slices whose triangle is below about half a share get a wavefront of their own
    int64_t m0 = (int64_t)sqrt((double)pick_share(total, 24));
    if (m0 < 64) m0 = 64;
    tail_order = m0 < n ? m0 : n;
    total_a = total - tet(tail_order);
  }
  const int64_t share = pick_share(total_a, 24);
  const int64_t waves_a = ceil_div(total_a, share);
  const int64_t blocks = ceil_div(waves_a + tail_order, kLdsWaves);
  const size_t lds = (size_t)(n + kPadOf<T>) * sizeof(T);
  if (total * (int64_t)sizeof(T) > kStreamBytes)
    segsum_lds_kernel<T, TET, true, PAD><<<(unsigned)blocks, kLdsBlock, lds, (hipStream_t)stream>>>(
        (int)n, A, x, out, total, total_a, share, waves_a, (int)tail_order, zeros);
  else
    segsum_lds_kernel<T, TET, false, PAD><<<(unsigned)blocks, kLdsBlock, lds, (hipStream_t)stream>>>(
        (int)n, A, x, out, total, total_a, share, waves_a, (int)tail_order, zeros);
  return launch_status();
}

template <typename T>
__global__ __launch_bounds__(256) void zero_entries_kernel(T *__restrict__ y, int64_t count) {
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < count; t += (int64_t)gridDim.x * 256) y[t] = T(0);
}

template <typename T>
int padded_trmv(int64_t n, const T *Up, const T *x, T *y, int64_t zeros, void *stream) {
  if (n < 1 || zeros < 0) return DASTAC_EINVAL;
  if (n > DASTAC_TRI_MAX_N || tri(n) > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  // the fill rides in the product's launch while it is small beside the triangle (its workgroups then clear a few
  // entries each); a long tail behind a small triangle gets a launch of its own, sized for it
  if (n <= kLdsMaxN && zeros <= tri(n) / 16) return launch_lds<T, false, true>(n, Up, x, y, tri(n), stream, zeros);
  const int rc = n <= kLdsMaxN ? launch_lds<T, false>(n, Up, x, y, tri(n), stream) : trmv_upper_by_panels(n, Up, x, y, stream);
  if (rc != DASTAC_OK || zeros == 0) return rc;
  const int64_t blocks = ceil_div(zeros, 256);
  zero_entries_kernel<T><<<(unsigned)(blocks < 4096 ? blocks : 4096), 256, 0, (hipStream_t)stream>>>(y + n, zeros);
  return launch_status();
}

}  // namespace

namespace dastac {
int trmv_then_zeros(int64_t n, const float *Up, const float *x, float *y, int64_t zeros, void *stream) {
  return padded_trmv<float>(n, Up, x, y, zeros, stream);
}
int trmv_then_zeros(int64_t n, const double *Up, const double *x, double *y, int64_t zeros, void *stream) {
  return padded_trmv<double>(n, Up, x, y, zeros, stream);
}
}  // namespace dastac

extern "C" {

int dastac_trmv_f32(int64_t n, const float *Up, const float *x, float *y, void *stream) {
  if (n < 0) return DASTAC_EINVAL;
  if (n > DASTAC_TRI_MAX_N || tri(n) > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Up || !x || !y) return DASTAC_ENULL;
  if (overlaps(y, n * 4, Up, tri(n) * 4) || overlaps(y, n * 4, x, n * 4)) return DASTAC_EALIAS;
  if (n <= kLdsMaxN) return launch_lds<float, false>(n, Up, x, y, tri(n), stream);
  // x no longer fits in LDS: the column-panel kernel keeps it in registers
  return trmv_upper_by_panels(n, Up, x, y, stream);
}

int dastac_tet_ttv_f32(int64_t n, const float *Ap, const float *v, float *Mp, void *stream) {
  if (n < 0) return DASTAC_EINVAL;
  // a tetrahedron of order above 8192 would not fit in device memory (and v would not fit in LDS)
  if (n > kLdsMaxN) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Ap || !v || !Mp) return DASTAC_ENULL;
  if (overlaps(Mp, tri(n) * 4, Ap, tet(n) * 4) || overlaps(Mp, tri(n) * 4, v, n * 4)) return DASTAC_EALIAS;
  return launch_lds<float, true>(n, Ap, v, Mp, tet(n), stream);
}

// Double precision (the paper's element type): the same kernel with 16-byte pieces of two elements.
int dastac_trmv_f64(int64_t n, const double *Up, const double *x, double *y, void *stream) {
  if (n < 0) return DASTAC_EINVAL;
  if (n > DASTAC_TRI_MAX_N || tri(n) > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Up || !x || !y) return DASTAC_ENULL;
  if (overlaps(y, n * 8, Up, tri(n) * 8) || overlaps(y, n * 8, x, n * 8)) return DASTAC_EALIAS;
  if (n <= kLdsMaxN) return launch_lds<double, false>(n, Up, x, y, tri(n), stream);
  return trmv_upper_by_panels(n, Up, x, y, stream);  // x no longer fits in LDS
}

int dastac_tet_ttv_f64(int64_t n, const double *Ap, const double *v, double *Mp, void *stream) {
  if (n < 0) return DASTAC_EINVAL;
  if (n > kLdsMaxN) return DASTAC_EOVERFLOW;
  if (n == 0) return DASTAC_OK;
  if (!Ap || !v || !Mp) return DASTAC_ENULL;
  if (overlaps(Mp, tri(n) * 8, Ap, tet(n) * 8) || overlaps(Mp, tri(n) * 8, v, n * 8)) return DASTAC_EALIAS;
  return launch_lds<double, true>(n, Ap, v, Mp, tet(n), stream);
}

}  // extern "C"
