// Wavefront-wide helpers for gfx950 (64 lanes).  All kernels in this library launch 1-D blocks
// whose size is a multiple of 64, so lane = threadIdx.x & 63.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace apex {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// One step of a prefix sum with data-parallel primitives (no LDS traffic): every lane adds the
// value that the DPP control word routes to it, and 0 where it routes none.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ uint64_t dpp_add_step(uint64_t v)
{
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, kCtrl, kRowMask, 0xf, false);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), kCtrl, kRowMask, 0xf, false);
  return v + (((uint64_t)hi << 32) | lo);
}

// Inclusive prefix sum of one uint64 per lane: shifts by 1, 2, 4, 8 lanes inside each row of 16
// lanes, then the last lane of row 0 (2) is added to row 1 (3), then lane 31 to rows 2 and 3.
__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t v)
{
  v = dpp_add_step<0x111, 0xf>(v);  // row_shr:1
  v = dpp_add_step<0x112, 0xf>(v);  // row_shr:2
  v = dpp_add_step<0x114, 0xf>(v);  // row_shr:4
  v = dpp_add_step<0x118, 0xf>(v);  // row_shr:8
  v = dpp_add_step<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
  v = dpp_add_step<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
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
