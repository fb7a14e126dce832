// Wavefront (64 lanes) and workgroup building blocks used by the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace us {

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }
__device__ __forceinline__ uint64_t lanes_below() { return (1ull << lane_id()) - 1ull; }

// inclusive prefix sum across the 64 lanes of a wavefront
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v) {
  const int lane = lane_id();
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t t = __shfl_up(v, d);
    if (lane >= d) v += t;
  }
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

// Exclusive prefix sum over a workgroup of T threads (T multiple of 64, T <= 1024).
// s_wave: T/64 + 1 words of LDS.  Returns the exclusive prefix; *total = workgroup sum.
// Ends with a barrier, so s_wave may be reused right after.
template <int T>
__device__ __forceinline__ uint32_t block_exclusive_sum(uint32_t v, uint32_t *s_wave, uint32_t *total) {
  constexpr int NW = T / 64;
  const int lane = lane_id(), w = wave_id();
  uint32_t inc = wave_inclusive_sum(v);
  if (lane == 63) s_wave[w] = inc;
  __syncthreads();
  if (w == 0) {
    uint32_t x = lane < NW ? s_wave[lane] : 0u;
    uint32_t xi = wave_inclusive_sum(x);
    if (lane < NW) s_wave[lane] = xi - x;
    if (lane == NW - 1) s_wave[NW] = xi;
  }
  __syncthreads();
  uint32_t res = s_wave[w] + inc - v;
  *total = s_wave[NW];
  __syncthreads();
  return res;
}

// upper_bound(ptr, e) - 1: the parent whose segment [ptr[p], ptr[p+1]) holds child e
__device__ __forceinline__ int64_t parent_of(const int32_t *ptr, int64_t nparents, int64_t e) {
  int64_t lo = 0, hi = nparents;
  while (lo < hi) {
    int64_t mid = (lo + hi) >> 1;
    if ((int64_t)ptr[mid + 1] <= e) lo = mid + 1; else hi = mid;
  }
  return lo;
}

}  // namespace us
