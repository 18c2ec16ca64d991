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

// Eight consecutive elements of a row as floats, through 16-byte loads (rows are 16-byte aligned
// and `i` is a multiple of 8).
template <typename T> struct Row8;
template <> struct Row8<float> {
  static __device__ __forceinline__ void load(const void* p, int64_t i, float (&f)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p) + i);
    const float4 b = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p) + i + 4);
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
    f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  }
};
template <> struct Row8<uint16_t> {  // bf16 bit patterns
  static __device__ __forceinline__ void load(const void* p, int64_t i, float (&f)[8]) {
    const uint4 w = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(p) + i);
    const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      f[2 * t] = __uint_as_float(u[t] << 16);
      f[2 * t + 1] = __uint_as_float(u[t] & 0xffff0000u);
    }
  }
};

// dot of a row (read by this lane, 16 bytes at a time) with a vector that the wave holds spread
// over its lanes: element c of the vector sits in lane c % 64 of reg[c / 64]
template <typename T, int D>
__device__ __forceinline__ float dot_row_with_spread(const void* base, int64_t row_off,
                                                     const float (&reg)[D / 64]) {
  float s = 0.f;
#pragma unroll
  for (int c0 = 0; c0 < D; c0 += 8) {
    float f[8];
    Row8<T>::load(base, row_off + c0, f);
#pragma unroll
    for (int t = 0; t < 8; ++t) s = fmaf(lane_bcast(reg[(c0 + t) / 64], (c0 + t) % 64), f[t], s);
  }
  return s;
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
