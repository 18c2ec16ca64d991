// Pieces shared by the matrix-core backward kernels of the linear heads (causal scans and
// bidirectional sweeps): tile geometry, the feature map and its slope, MFMA operand fetches from
// row-major LDS tiles, and head addressing.  Internal to one translation unit at a time.
#pragma once

#include "common.hpp"
#include "mfma.hpp"

namespace gformer {
namespace {

constexpr int CH = 64;        // tokens per chunk
constexpr int SR = CH + 8;    // row stride of the 64 x 64 weight tiles
constexpr float kLog2e = 1.4426950408889634f;

template <int D> struct LbCfg {
  static constexpr int MT = D / 32, KS = D / 16;
  static constexpr int NW = 2 * MT, NT = 64 * NW;      // one 32 x 32 output tile per wave and product
  static constexpr int R = D == 128 ? D + 24 : D + 8;  // 12 / 36 dwords mod 64: row and transpose reads
  static constexpr int TPW = MT * MT / NW;             // tiles of the carried sum per wave
  static constexpr int C8 = D / 8;
  static constexpr int PCS = CH * C8 / NT;             // 16-byte pieces per thread and tensor
  static constexpr int ZP = NT / D;                    // threads per column in the column sums
};

__device__ __forceinline__ float phi_elu1(float x) {
  return x > 0.f ? x + 1.f : __builtin_amdgcn_exp2f(x * kLog2e);
}
template <bool ELU1> __device__ __forceinline__ u32x4 map8(u32x4 v) {
  if (!ELU1) return v;
  u32x4 o;
#pragma unroll
  for (int w = 0; w < 4; ++w) o[w] = pack_bf16(phi_elu1(bf16_lo(v[w])), phi_elu1(bf16_hi(v[w])));
  return o;
}
// slope of the feature map from the mapped value
template <bool ELU1> __device__ __forceinline__ float slope_of(float f) {
  if (!ELU1) return 1.f;
  return f > 1.f ? 1.f : f;
}
__device__ __forceinline__ u32x4 scale8(u32x4 v, float s) {
  u32x4 o;
#pragma unroll
  for (int w = 0; w < 4; ++w) o[w] = pack_bf16(bf16_lo(v[w]) * s, bf16_hi(v[w]) * s);
  return o;
}
constexpr u32x4 kZero4 = {0u, 0u, 0u, 0u};

// MFMA operand from a row-major tile, contraction index along the row: lane l takes row
// row0 + l%32, columns 16*ks + 8*(l/32) .. +7
__device__ __forceinline__ bf16x8 row_op(const uint16_t* tile, int stride, int row0, int ks, int ln, int lh) {
  return lds_read16(&tile[(row0 + ln) * stride + 16 * ks + 8 * lh]);
}
// MFMA operand from a row-major tile, contraction index down the rows: lane l takes column
// col0 + l%32, rows k0 + 8*(l/32) .. +7 (tile_lane carries the lane-dependent part)
__device__ __forceinline__ bf16x8 col_op(const uint16_t* tile_lane, int stride, int k0, int col0) {
  return lds_operand_tr_at(tile_lane, stride, k0, k0 + 4, col0);
}
// 4 accumulator registers (rows 4*lh .. +3 of an 8-row group) -> 4 consecutive bf16 of a tile row
__device__ __forceinline__ void put4(uint16_t* p, float a, float b, float c, float d) {
  u32x2 pk;
  pk[0] = pack_bf16(a, b);
  pk[1] = pack_bf16(c, d);
  *reinterpret_cast<u32x2*>(p) = pk;
}
// the same four values as a bf16 pair: high halves to `hi`, bf16(x - bf16(x)) to `lo`
__device__ __forceinline__ void put4_split(uint16_t* hi, uint16_t* lo, float a, float b, float c, float d) {
  u32x2 ph, pl;
  ph[0] = pack_bf16(a, b);
  ph[1] = pack_bf16(c, d);
  pl[0] = pack_bf16(a - bf16_lo(ph[0]), b - bf16_hi(ph[0]));
  pl[1] = pack_bf16(c - bf16_lo(ph[1]), d - bf16_hi(ph[1]));
  *reinterpret_cast<u32x2*>(hi) = ph;
  *reinterpret_cast<u32x2*>(lo) = pl;
}
__device__ __forceinline__ void get4(const uint16_t* p, float (&f)[4]) {
  const u32x2 pk = *reinterpret_cast<const u32x2*>(p);
  f[0] = bf16_lo(pk[0]); f[1] = bf16_hi(pk[0]); f[2] = bf16_lo(pk[1]); f[3] = bf16_hi(pk[1]);
}

template <int D> struct HeadCtx {
  const uint16_t *q, *k, *v, *dout;
  float* ws;
};
template <int D> __device__ __forceinline__ HeadCtx<D> head_ctx(const BwdArgs& a, int b, int h) {
  HeadCtx<D> c;
  c.q = reinterpret_cast<const uint16_t*>(a.q.base) + b * a.q.sb + h * a.q.sh;
  c.k = reinterpret_cast<const uint16_t*>(a.k.base) + b * a.k.sb + h * a.k.sh;
  c.v = reinterpret_cast<const uint16_t*>(a.v.base) + b * a.v.sb + h * a.v.sh;
  c.dout = reinterpret_cast<const uint16_t*>(a.dout.base) + b * a.dout.sb + h * a.dout.sh;
  c.ws = a.ws + ((int64_t)b * a.H + h) * a.N * 2;
  return c;
}


}  // namespace
}  // namespace gformer
