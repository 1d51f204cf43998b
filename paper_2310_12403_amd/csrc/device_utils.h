// Wave64 helpers for gfx950.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace coop {

constexpr int kWave = 64;
constexpr int kBlock = 256;              // 4 waves per workgroup
constexpr int kWavesPerBlock = kBlock / kWave;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_in_block() { return threadIdx.x >> 6; }
// the same value, but known to the compiler to be wave-uniform: addresses and loop bounds derived from it stay scalar
__device__ __forceinline__ int uniform_wave_in_block() { return __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); }

// number of set bits of `mask` strictly below this lane
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ uint64_t ballot64(bool p) { return __ballot(p); }

// wave-wide inclusive sum of a uint32 (all lanes get their prefix)
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    uint32_t o = __shfl_up(v, off, kWave);
    if (lane_id() >= off) v += o;
  }
  return v;
}

__device__ __forceinline__ int64_t wave_sum_i64(int64_t v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

}  // namespace coop
