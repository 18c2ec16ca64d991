// gfx950 matrix-core and LDS helpers shared by the bf16 kernels.
//
// Lane layout of v_mfma_f32_32x32x16_bf16 (D = A*B + C, A is 32x16, B is 16x32), lane l:
//   A operand: row m = l % 32, k-slots 8*(l/32) .. 8*(l/32)+7      (8 bf16, 4 VGPRs)
//   B operand: col n = l % 32, k-slots 8*(l/32) .. 8*(l/32)+7
//   C/D:       col n = l % 32, register r holds row m = 8*(r/4) + 4*(l/32) + r%4
// A fp32 accumulator tile therefore keeps, per lane, one column and 16 of its rows.  Registers
// [8*kb, 8*kb+8) of a lane are rows 16*kb + 8*g + 4*(l/32) + j (g = 0..1, j = 0..3): fed back
// as an MFMA operand they occupy k-slots 8*(l/32) + 4*g + j, i.e. the contraction index is
// permuted inside each group of 32 by
//   kperm32(k) = 16*(k/16) + 8*((k/4)%2) + 4*((k/8)%2) + k%4        (an involution)
// An accumulator tile can thus feed the next MFMA straight from registers as long as the other
// operand supplies its k-index in the same permuted order.
//
// LDS on this chip, measured with eight waves issuing independent accesses, in cycles per wave
// instruction: ds_read_b128 4.5 when 16 consecutive lanes touch 64 distinct banks (lane = row,
// row stride 4 or 12 dwords mod 64) and 8 when the 16 lanes read one contiguous 256-byte row;
// ds_read_b64 2.7 contiguous, 4.2 with lane = row at stride 4 or 12 dwords mod 64, 8 at stride 8,
// 16 at stride 16; ds_read_b64_tr_b16 2.4 at row stride 16 dwords mod 64, 4.5 at 8 or 12, 8 at 4;
// ds_write_b64 8 (16 at row stride 8 dwords mod 64, 32 at 16), ds_write_b128 13.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gformer {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
typedef short v4i16_t __attribute__((ext_vector_type(4)));

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

// acc + a.lo*b.lo + a.hi*b.hi on packed bf16 pairs (v_dot2c_f32_bf16)
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                         __builtin_bit_cast(bf16x2_t, b), acc, false);
}
constexpr uint32_t kOnesBf16x2 = 0x3f803f80u;
// acc + lo + hi of a packed bf16 pair
__device__ __forceinline__ float dot2_ones_bf16(uint32_t a, float acc) {
  return dot2_bf16(a, kOnesBf16x2, acc);
}

// max(a, b, c) / min(a, b, c) in one instruction.  The library forms never see a NaN here (scores
// are finite or the infinity a mask put there), and written this way the compiler does not add
// the quieting moves it puts in front of every fmaxf / fminf.
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float min3(float a, float b, float c) {
  float r;
  asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Lanes l and l^32 exchange a value (v_permlane32_swap): `a` and `b` come back as the lane's own
// x and its partner's, in an order that depends on the half of the wave, so only symmetric
// combinations (max, sum) of the two are meaningful.
__device__ __forceinline__ void exchange_halves(float x, float& a, float& b) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  a = __uint_as_float(r[0]);
  b = __uint_as_float(r[1]);
}
__device__ __forceinline__ float max_over_halves(float x) {
  float a, b;
  exchange_halves(x, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float sum_over_halves(float x) {
  float a, b;
  exchange_halves(x, a, b);
  return a + b;
}

__host__ __device__ constexpr int kperm32(int k) {
  return 16 * (k / 16) + 8 * ((k / 4) % 2) + 4 * ((k / 8) % 2) + k % 4;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load and store (vmcnt(0)), which would expose the full memory latency of
// prefetches that are deliberately left in flight across the barrier.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ bf16x8 lds_read16(const uint16_t* p) {
  return as_bf16x8(*reinterpret_cast<const u32x4*>(p));
}

// LDS transpose read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane p passes the
// address of 4 consecutive bf16; lane i of the group receives element (i % 4) of the values
// addressed by lanes 4*j + i/4, j = 0..3.  With lane p pointing at row (row0 + p/4), columns
// col0 + 4*(p%4) .. +3 of a row-major tile, lane i gets column col0 + i of rows row0 .. row0+3.
__device__ __forceinline__ u32x2 lds_tr4(const uint16_t* p) {
  const v4i16_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) v4i16_t*)(p));
  return __builtin_bit_cast(u32x2, v);
}

// MFMA operand (lane l: row/col index l%32 of the operand = tile column col0 + l%32; 8 k-slots)
// gathered from a ROW-MAJOR tile whose rows are the contraction index: slots 0..3 come from
// tile rows rowA .. rowA+3 and slots 4..7 from rows rowB .. rowB+3 (callers add their own
// dependence on l/32).  `stride` is the tile's row stride in elements.
// The lane-dependent part of lds_operand_tr's addresses, in elements: what is left is uniform.
__device__ __forceinline__ int lds_operand_tr_lane_offset(int stride, int lane) {
  const int p = lane & 15;
  return (p >> 2) * stride + 16 * ((lane >> 4) & 1) + 4 * (p & 3);
}
// lds_operand_tr with the lane-dependent part precomputed: tile + lane_off points at this
// lane's element of (row 0, column 0); rowA, rowB and col0 are uniform.
__device__ __forceinline__ bf16x8 lds_operand_tr_at(const uint16_t* tile_lane, int stride, int rowA,
                                                    int rowB, int col0) {
  const u32x2 a = lds_tr4(tile_lane + rowA * stride + col0);
  const u32x2 b = lds_tr4(tile_lane + rowB * stride + col0);
  u32x4 r;
  r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
  return as_bf16x8(r);
}

__device__ __forceinline__ bf16x8 lds_operand_tr(const uint16_t* tile, int stride, int rowA,
                                                 int rowB, int col0, int lane) {
  const int p = lane & 15;
  const int col = col0 + 16 * ((lane >> 4) & 1) + 4 * (p & 3);
  const u32x2 a = lds_tr4(tile + (rowA + (p >> 2)) * stride + col);
  const u32x2 b = lds_tr4(tile + (rowB + (p >> 2)) * stride + col);
  u32x4 r;
  r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
  return as_bf16x8(r);
}

}  // namespace gformer
