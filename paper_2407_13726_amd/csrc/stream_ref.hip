// Measurement aid (not one of the paper's operations): a plain read-only stream over a buffer, the
// yardstick the HBM-bound contractions are compared with.  Workgroup b adds up its contiguous chunk
// of src with non-temporal 16-byte loads, eight in flight per lane, and writes one partial sum.
#include "common.h"

using namespace dastac;

namespace {

constexpr int kBlock = 256;
constexpr int kUnroll = 8;
constexpr int64_t kTile = (int64_t)kBlock * 4 * kUnroll;  // elements a workgroup takes per round

__global__ __launch_bounds__(kBlock) void stream_sum_kernel(int64_t count, int64_t chunk, const float *__restrict__ src,
                                                            float *__restrict__ partial) {
  __shared__ float red[kBlock / 64];
  const int64_t lo = (int64_t)blockIdx.x * chunk;
  const int64_t hi = lo + chunk < count ? lo + chunk : count;
  f4a acc[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) acc[u] = f4a{0.0f, 0.0f, 0.0f, 0.0f};
  int64_t p = lo + 4 * (int64_t)threadIdx.x;
  for (; p + (kUnroll - 1) * kBlock * 4 + 4 <= hi; p += kTile) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      acc[u] += __builtin_nontemporal_load(reinterpret_cast<const f4u *>(src + p + (int64_t)u * kBlock * 4));
  }
  float s = 0.0f;
  for (; p < hi; p += kBlock * 4)  // ragged end of the chunk, element by element
    for (int c = 0; c < 4; ++c)
      if (p + c < hi) s += src[p + c];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) s += (acc[u].x + acc[u].y) + (acc[u].z + acc[u].w);
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

}  // namespace

extern "C" int dastac_stream_sum_f32(int64_t count, const float *src, float *partial, int64_t npartial,
                                     void *stream) {
  if (count < 0 || npartial < 1 || npartial > ((int64_t)1 << 24)) return DASTAC_EINVAL;
  if (count > ((int64_t)1 << 40)) return DASTAC_EOVERFLOW;
  if (!partial || (count > 0 && !src)) return DASTAC_ENULL;
  if (overlaps(partial, npartial * 4, src, count * 4)) return DASTAC_EALIAS;
  // contiguous chunks, a multiple of 4 elements long so that every chunk starts on the same 16-byte phase
  const int64_t chunk = ceil_div(ceil_div(count, npartial), 4) * 4;
  stream_sum_kernel<<<(unsigned)npartial, kBlock, 0, (hipStream_t)stream>>>(count, chunk > 0 ? chunk : 4, src, partial);
  return launch_status();
}
