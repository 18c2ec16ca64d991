// gfx950 matrix-core helpers shared by the bf16 kernels.
//
// Lane layout of v_mfma_f32_32x32x16_bf16 (D = A*B + C, A is 32x16, B is 16x32), lane l:
//   A operand: row m = l % 32, k = 8*(l/32) .. 8*(l/32)+7          (8 bf16, 4 VGPRs)
//   B operand: col n = l % 32, k = 8*(l/32) .. 8*(l/32)+7
//   C/D:       col n = l % 32, register r holds row m = 8*(r/4) + 4*(l/32) + r%4
// A fp32 accumulator tile therefore keeps, per lane, one column and 16 of its rows; the rows a
// lane owns in registers [8*kb, 8*kb+8) are exactly the 8 k-indices it must supply as a B
// operand when the contraction index is permuted as
//   pos(k) = 16*(k/16) + 8*((k/4)%2) + 4*((k/8)%2) + k%4          (within a 32-row tile)
// so a score tile can feed the next MFMA straight from registers if the other operand is
// stored in LDS in the same permuted order.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gformer {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ u32x4 as_u32x4(bf16x8 v) { return __builtin_bit_cast(u32x4, v); }

// Two fp32 -> packed bf16 pair (round to nearest even), low half = a.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  bf16x2 v;
  v[0] = (__bf16)a;
  v[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Position of contraction index k (0..31) inside a permuted 32-group (see the top comment).
__host__ __device__ constexpr int kperm32(int k) {
  return 16 * (k / 16) + 8 * ((k / 4) % 2) + 4 * ((k / 8) % 2) + k % 4;
}

// In-register transpose of a 4 (rows) x 8 (cols) bf16 block held as 4 x u32x4 (one row each)
// into 8 x u32x2 (one column each: 4 consecutive rows).
__device__ __forceinline__ void transpose_4x8_bf16(const u32x4 (&r)[4], u32x2 (&c)[8]) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {  // dword w holds columns 2w (low half) and 2w+1 (high half)
    c[2 * w][0] = __builtin_amdgcn_perm(r[1][w], r[0][w], 0x05040100u);
    c[2 * w][1] = __builtin_amdgcn_perm(r[3][w], r[2][w], 0x05040100u);
    c[2 * w + 1][0] = __builtin_amdgcn_perm(r[1][w], r[0][w], 0x07060302u);
    c[2 * w + 1][1] = __builtin_amdgcn_perm(r[3][w], r[2][w], 0x07060302u);
  }
}

}  // namespace gformer
