// Wavefront-wide helpers for gfx950 (64 lanes).  All kernels in this library launch 1-D blocks
// whose size is a multiple of 64, so lane = threadIdx.x & 63.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace apex {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Inclusive prefix sum of one uint64 per lane.
__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t v)
{
  const int lane = lane_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    uint64_t t = __shfl_up(v, d, kWave);
    if (lane >= d) v += t;
  }
  return v;
}

// Sum over the wave, result in every lane.
__device__ __forceinline__ uint64_t wave_sum(uint64_t v)
{
#pragma unroll
  for (int d = kWave / 2; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
  return v;
}

__device__ __forceinline__ uint64_t wave_min(uint64_t v)
{
#pragma unroll
  for (int d = kWave / 2; d >= 1; d >>= 1) {
    uint64_t t = __shfl_xor(v, d, kWave);
    v = t < v ? t : v;
  }
  return v;
}

// Device-scope atomics on the tree.  The eight XCDs of the chip have separate L2 caches, so
// these must be (and are) performed at agent scope.
__device__ __forceinline__ void atomic_add_u64(uint64_t *p, uint64_t v)
{
  __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace apex
