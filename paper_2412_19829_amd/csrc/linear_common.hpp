// Pieces shared by the linear-attention kernels (section III-C, Algorithm 1 by chunks): tile
// geometry, the feature map, head addressing, the layout of a carried (A, Z) state in the
// workspace, and the producers' clamped loads.  Everything here is internal to one translation
// unit at a time (anonymous namespace).
#pragma once

#include "common.hpp"
#include "mfma.hpp"

namespace gformer {
namespace {

constexpr int CH = 64;  // tokens per chunk
constexpr float kLog2e = 1.4426950408889634f;

template <int D> struct LinCfg {
  static constexpr int ET = D / 32;           // 32-wide tiles along a feature / value axis
  static constexpr int NWC = ET;              // compute waves: one per value-column tile
  static constexpr int NTC = NWC * 64;        // compute threads
  static constexpr int NT = 2 * NTC;          // + as many producer threads
  static constexpr int QROW = D + 8;          // phi(Q): 128-bit row reads   (stride = 4 dw mod 64)
  static constexpr int KROW = D == 64 ? D + 8 : D + 24;  // phi(K): 64-bit row reads + transpose
                                              // reads.  Measured per wave instruction at d = 128: stride
                                              // D+24 (12 dwords mod 64) 4.2 / 4.5 cycles, D+16 8.0 / 4.5,
                                              // D+32 16 / 2.5 (D = 64: 8 keeps two workgroups' LDS under 160 KB)
  static constexpr int VROW = D + 32;         // V: transpose reads only     (stride = 16 dw mod 64)
  static constexpr int PROW = CH + 8;         // masked products, [query][key]
  static constexpr int OROW = D + 8;          // normalised output rows on their way to memory
  static constexpr int C8 = D / 8;            // 16-byte pieces per row
  static constexpr int RP = NTC / C8;         // rows covered by one pass of the producer threads
  static constexpr int PIECES = CH / RP;      // pieces per producer thread per tensor per chunk
  static constexpr int STATE = D * D + D;     // floats per (A, Z) state
};

// phi(x) = elu(x) + 1 = max(x + 1, min(exp(x), 1))   (section II-B); the clamp rides on v_exp
__device__ __forceinline__ float elu1(float x) {
  const float e = __builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(x * kLog2e), 0.0f, 1.0f);
  return fmaxf(x + 1.0f, e);
}

// Feature map on 8 packed bf16 values (ELU1 = true: phi(x) = elu(x)+1; false: identity).
template <bool ELU1> __device__ __forceinline__ u32x4 map_features(u32x4 v) {
  if (!ELU1) return v;
  u32x4 o;
#pragma unroll
  for (int w = 0; w < 4; ++w) o[w] = pack_bf16(elu1(bf16_lo(v[w])), elu1(bf16_hi(v[w])));
  return o;
}

__device__ __forceinline__ float sum8_bf16(bf16x8 x, float acc) {
  const u32x4 u = as_u32x4(x);
#pragma unroll
  for (int w = 0; w < 4; ++w) acc = dot2_bf16(u[w], kOnesBf16x2, acc);
  return acc;
}

template <int D> struct HeadPtrs {
  const uint16_t *q, *k, *v;
  uint16_t* o;
};

template <int D>
__device__ __forceinline__ HeadPtrs<D> head_ptrs(const AttnArgs& a, int head_linear) {
  const int H1 = a.H - a.H0;
  const int b = head_linear / H1, h = a.H0 + head_linear % H1;
  HeadPtrs<D> p;
  p.q = reinterpret_cast<const uint16_t*>(a.q.base) + b * a.q.sb + h * a.q.sh;
  p.k = reinterpret_cast<const uint16_t*>(a.k.base) + b * a.k.sb + h * a.k.sh;
  p.v = reinterpret_cast<const uint16_t*>(a.v.base) + b * a.v.sb + h * a.v.sh;
  p.o = reinterpret_cast<uint16_t*>(a.out) + b * a.osb + h * a.osh;
  return p;
}

// Real chunks of piece p: global chunks [g0, g0 + n).  A piece that would run into a head's
// virtual padding (uniform-segment mode) stops at the head's last real chunk.
__device__ __forceinline__ int piece_chunk_count(const AttnArgs& a, int g0, int n_heads) {
  int n = min(a.piece_chunks, n_heads * a.vcph - g0);
  if (a.vcph != a.cph) n = min(n, a.cph - g0 % a.vcph);
  return n;
}

// State tile (ct, wave) in accumulator layout: lane = value column 32*wave + l%32,
// register r = feature row 32*ct + 8*(r/4) + 4*(l/32) + r%4.  The workspace keeps A in exactly
// this order (tile, lane, register) so that a lane moves its 16 values of a tile as four 16-byte
// accesses; Z follows at offset D*D in natural feature order.
template <int D>
__device__ __forceinline__ int state_tile_offset(int ct, int wave, int lane) {
  return ((ct * LinCfg<D>::NWC + wave) * 64 + lane) * 16;
}
template <int D>
__device__ __forceinline__ void state_store(float* dst, const f32x16 (&sacc)[LinCfg<D>::ET],
                                            int wave, int lane) {
#pragma unroll
  for (int ct = 0; ct < LinCfg<D>::ET; ++ct) {
    float4* p = reinterpret_cast<float4*>(dst + state_tile_offset<D>(ct, wave, lane));
#pragma unroll
    for (int g = 0; g < 4; ++g)
      p[g] = make_float4(sacc[ct][4 * g], sacc[ct][4 * g + 1], sacc[ct][4 * g + 2], sacc[ct][4 * g + 3]);
  }
}
template <int D>
__device__ __forceinline__ void state_add(f32x16 (&sacc)[LinCfg<D>::ET], const float* src,
                                          int wave, int lane) {
#pragma unroll
  for (int ct = 0; ct < LinCfg<D>::ET; ++ct) {
    const float4* p = reinterpret_cast<const float4*>(src + state_tile_offset<D>(ct, wave, lane));
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 x = p[g];
      sacc[ct][4 * g] += x.x; sacc[ct][4 * g + 1] += x.y;
      sacc[ct][4 * g + 2] += x.z; sacc[ct][4 * g + 3] += x.w;
    }
  }
}

// Producer-side view of one chunk: producer thread t moves 16-byte pieces (row r0 + i*RP,
// columns col .. col+7), i = 0..PIECES-1, of each tensor from global memory to LDS.
template <int D> struct Staging {
  using C = LinCfg<D>;
  int r0, col, qcol;
  __device__ __forceinline__ explicit Staging(int ptid) : r0(ptid / C::C8), col(8 * (ptid % C::C8)) {
    // phi(Q) pieces land at permuted feature positions: two groups of 4, 8 apart
    const int c8 = ptid % C::C8;
    qcol = 32 * (c8 / 4) + 16 * ((c8 % 4) / 2) + 4 * (c8 % 2);
  }
};

// One tensor's chunk as seen by a producer thread: piece i is read from a wave-uniform base
// (row t0 + i*RP of the head, kept in scalar registers) plus one per-thread byte offset that
// never changes, so a load costs no vector address arithmetic beyond its clamp.  Rows past N-1
// (a head's last chunk only) re-read row N-1, in bounds.  Streamed once: non-temporal loads
// (measured ~7.1 TB/s vs ~6.1 TB/s for plain loads) unless NT = false asks for plain ones.
template <int D> struct PieceOffsets {
  uint32_t off;   // byte offset of (row r0, columns col..col+7) from the piece's first row
  uint32_t colb;  // byte offset of the thread's columns inside a row
  int sn;         // row stride in elements
  __device__ __forceinline__ PieceOffsets(const Staging<D>& st, int64_t row_stride)
      : off(2u * (uint32_t)(st.r0 * (int)row_stride + st.col)), colb(2u * (uint32_t)st.col),
        sn((int)row_stride) {}
};
template <int D, bool NT = true>
__device__ __forceinline__ void load_chunk(u32x4 (&dst)[LinCfg<D>::PIECES], const uint16_t* head,
                                           int t0, int N, const PieceOffsets<D>& po) {
  using C = LinCfg<D>;
  const int last = min(N - 1 - t0, CH - 1);  // last valid row of the chunk
  const char* chunk = reinterpret_cast<const char*>(head + (int64_t)t0 * po.sn);
#pragma unroll
  for (int i = 0; i < C::PIECES; ++i) {
    const int first = min(i * C::RP, last);  // uniform: the piece's first row, clamped
    const char* base = chunk + 2u * (uint32_t)(first * po.sn);
    const uint32_t lim = 2u * (uint32_t)((last - first) * po.sn) + po.colb;
    const u32x4* src = reinterpret_cast<const u32x4*>(base + (size_t)min(po.off, lim));
    dst[i] = NT ? __builtin_nontemporal_load(src) : *src;
  }
}

constexpr u32x4 kZero4 = {0u, 0u, 0u, 0u};

template <typename K> hipError_t allow_lds(K kern, int smem) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                             hipFuncAttributeMaxDynamicSharedMemorySize, smem);
}

}  // namespace
}  // namespace gformer
