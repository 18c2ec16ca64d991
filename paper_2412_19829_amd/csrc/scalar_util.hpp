// Small device helpers shared by the plain-FMA kernels (forward and backward).
#pragma once

#include <hip/hip_runtime.h>

namespace gformer {

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float lane_bcast(float x, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane));
}

// Feature map of section II-B: phi(x) = elu(x) + 1.
__device__ __forceinline__ float feature_map(float x, int phi) {
  if (phi != 0) return x;
  return x > 0.f ? x + 1.f : expf(x);
}
// Its slope, from the mapped value f = phi(x): 1 where x > 0 (f > 1), exp(x) = f elsewhere.
__device__ __forceinline__ float feature_map_slope(float f, int phi) {
  if (phi != 0) return 1.f;
  return f > 1.f ? 1.f : f;
}

}  // namespace gformer
