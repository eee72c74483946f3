// Shared host-side helpers of the C-ABI entry points: status codes, overlap test,
// launch-error capture.  Device helpers used by more than one kernel file live here too.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/dastac.h"
#include "index_poly.h"

namespace dastac {

// True when the byte ranges [a, a+na) and [b, b+nb) intersect.
inline bool overlaps(const void *a, int64_t na, const void *b, int64_t nb) {
  if (na <= 0 || nb <= 0) return false;
  uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return a0 < b0 + (uintptr_t)nb && b0 < a0 + (uintptr_t)na;
}

// Largest row stride (in elements) an entry point accepts; keeps rows * ld * sizeof(element) inside int64 for
// every row count the entry points accept.  Above it: DASTAC_EOVERFLOW.
constexpr int64_t kMaxLd = DASTAC_MAX_LD;
inline bool ld_too_large(int64_t a, int64_t b = 0, int64_t c = 0) { return a > kMaxLd || b > kMaxLd || c > kMaxLd; }

// Bytes from the first element to one past the last of a view of `rows` rows with row stride ld of which the
// first `cols` columns are used (the tail of the last row is not part of the view).
inline int64_t view_bytes(int64_t rows, int64_t ld, int64_t cols, int64_t elem) {
  return rows <= 0 ? 0 : ((rows - 1) * ld + cols) * elem;
}

// Status of the launch that was just issued on this thread.
inline int launch_status() { return hipGetLastError() == hipSuccess ? DASTAC_OK : DASTAC_EHIP; }

DASTAC_HD int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

#if defined(__HIPCC__)
// Workgroups of `block` threads of `kernel` (no dynamic LDS) that the current device holds at once:
// occupancy per compute unit x compute units.  Asked of the runtime on the first call per (kernel,
// device) and remembered afterwards in a small table; 0 on a runtime error.
template <typename Kernel>
inline int64_t resident_blocks(Kernel kernel, int block) {
  struct Entry {
    const void *fn;
    int dev;
    int64_t blocks;
  };
  constexpr int kEntries = 256;
  static Entry table[kEntries];
  static int used = 0;
  static std::mutex guard;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  const void *fn = reinterpret_cast<const void *>(kernel);
  {
    std::lock_guard<std::mutex> lock(guard);
    for (int e = 0; e < used; ++e)
      if (table[e].fn == fn && table[e].dev == dev) return table[e].blocks;
  }
  int per_cu = 0, cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, block, 0) != hipSuccess)
    return 0;
  const int64_t v = (int64_t)(per_cu > 0 ? per_cu : 1) * (cus > 0 ? cus : 1);
  std::lock_guard<std::mutex> lock(guard);
  if (used < kEntries) table[used++] = Entry{fn, dev, v};  // a full table only means asking again
  return v;
}
#endif

// defined in segsum.hip: y[0..n) := U x on the packed upper triangle and y[n..n+zeros) := 0, n >= 1, in one launch
// while x fits in LDS (arguments otherwise already validated), both precisions
int trmv_then_zeros(int64_t n, const float *Up, const float *x, float *y, int64_t zeros, void *stream);
int trmv_then_zeros(int64_t n, const double *Up, const double *x, double *y, int64_t zeros, void *stream);
// defined in trimv.hip
int trmv_upper_by_panels(int64_t n, const float *Up, const float *x, float *y, void *stream);
int trmv_upper_by_panels(int64_t n, const double *Up, const double *x, double *y, void *stream);
// defined in trmm_skinny.hip: C := U B for few columns (arguments already validated), both precisions
int trmm_few_columns(int64_t n, int64_t m, const float *Up, const float *B, int64_t ldb, float *C, int64_t ldc,
                     void *stream);
int trmm_few_columns(int64_t n, int64_t m, const double *Up, const double *B, int64_t ldb, double *C, int64_t ldc,
                     void *stream);

#if defined(__HIPCC__)
// 16-byte vector of floats that only promises 4-byte alignment: packed rows start at arbitrary
// element offsets, and gfx950 global loads of four dwords need dword alignment only.
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float f4a __attribute__((ext_vector_type(4)));
// the same for doubles: 16 bytes that only promise 8-byte alignment
typedef double d2u __attribute__((ext_vector_type(2), aligned(8)));
typedef double d2a __attribute__((ext_vector_type(2)));
// result registers of one matrix instruction: v_mfma_f32_32x32x2_f32 and v_mfma_f64_16x16x4_f64
typedef float f16v __attribute__((ext_vector_type(16)));
typedef double d4v __attribute__((ext_vector_type(4)));

// Make a wave-uniform 64-bit value provably scalar for the compiler.
__device__ inline int64_t uniform64(int64_t v) {
  uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)v);
  uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
  return (int64_t)(((uint64_t)hi << 32) | lo);
}
__device__ inline int uniform32(int v) { return __builtin_amdgcn_readfirstlane(v); }
#endif

}  // namespace dastac
