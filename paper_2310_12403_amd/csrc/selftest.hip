// Self-checks of device arithmetic that the bit-exactness of the blended variates (App. A.7, c > 0) leans on.
//
// The filters in front of the exact blend trust approx_phi_inv_f32 (Acklam's Phi^-1 in fp32 with the hardware's
// logarithm, square root and reciprocal) to stay within kPhiInvF32Gap of kit_phi_inv_u32 (the binary64 definition).
// That is a property of this GPU's instructions, so it is measured on the GPU, for every one of the 2^32 inputs.
#include "blend_filters.h"
#include "coop_internal.h"
#include "device_utils.h"

namespace coop {

__device__ __forceinline__ double phi_inv_gap(uint32_t U) {
  const double gap = __builtin_fabs((double)approx_phi_inv_f32(U) - kit_phi_inv_u32(U));
  return gap == gap ? gap : __builtin_inf();  // (a NaN on either side counts as an unbounded distance)
}

// *max_bits = max over U in [first, first + count) of |approx_phi_inv_f32(U) - kit_phi_inv_u32(U)|, by atomicMax on the bit
// pattern (nonnegative doubles order like their bit patterns)
__global__ __launch_bounds__(kBlock) void k_phi_inv_gap(uint64_t first, uint64_t count, unsigned long long* max_bits) {
  double worst = 0.0;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += stride) {
    const double gap = phi_inv_gap((uint32_t)(first + i));
    worst = gap > worst ? gap : worst;
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) {  // wave maximum, then one atomic per wave
    const double o = __shfl_xor(worst, off, kWave);
    worst = o > worst ? o : worst;
  }
  if (lane_id() == 0) atomicMax(max_bits, (unsigned long long)__double_as_longlong(worst));
}

// second pass: *arg_u = the smallest U of the range whose distance equals the maximum found by the first pass
__global__ __launch_bounds__(kBlock) void k_phi_inv_gap_where(uint64_t first, uint64_t count, const unsigned long long* max_bits,
                                                              unsigned long long* arg_u) {
  const unsigned long long want = *max_bits;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += stride) {
    const uint32_t U = (uint32_t)(first + i);
    if ((unsigned long long)__double_as_longlong(phi_inv_gap(U)) == want) atomicMin(arg_u, (unsigned long long)U);
  }
}

}  // namespace coop

using namespace coop;

extern "C" int coop_selftest_phi_inv_gap(uint64_t first, uint64_t count, double* max_gap_out, uint32_t* arg_out, void* workspace,
                                         void* stream) {
  if (!max_gap_out || !workspace) return COOP_E_NULL;
  if (((uintptr_t)workspace & 7) != 0 || count > ((uint64_t)1 << 32) || first > 0xFFFFFFFFull ||
      first + count > ((uint64_t)1 << 32))
    return COOP_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  unsigned long long* d = (unsigned long long*)workspace;  // [0] the maximum's bit pattern, [1] the first input that reaches it
  fill_u64((uint64_t*)d, 1, 0, s);
  fill_u64((uint64_t*)d + 1, 1, ~0ull, s);
  if (count > 0) {
    uint64_t blocks = (count + kBlock - 1) / kBlock;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(k_phi_inv_gap, dim3((unsigned)blocks), dim3(kBlock), 0, s, first, count, d);
    hipLaunchKernelGGL(k_phi_inv_gap_where, dim3((unsigned)blocks), dim3(kBlock), 0, s, first, count, (const unsigned long long*)d, d + 1);
  }
  unsigned long long h[2] = {0, 0};
  COOP_HIP_TRY(hipMemcpyAsync(h, d, sizeof(h), hipMemcpyDeviceToHost, s));
  COOP_HIP_TRY(hipStreamSynchronize(s));
  double gap;
  static_assert(sizeof(gap) == sizeof(h[0]), "bit copy");
  __builtin_memcpy(&gap, &h[0], sizeof(gap));
  *max_gap_out = gap;
  if (arg_out) *arg_out = (uint32_t)h[1];
  return COOP_OK;
}
