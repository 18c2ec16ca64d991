// Windowed causal softmax attention heads on bf16 matrix cores (section III-B, Eq. 1).
//
// One workgroup (4 waves) owns 128 consecutive queries of one (batch, head); each wave owns 32
// of them.  The band of keys those queries can see is walked in tiles of 64 keys; tiles outside
// the band are never touched.  K and V tiles sit in LDS row-major, shared by the 4 waves; K is
// read with 128-bit loads (contraction over the head dimension), V with the LDS transpose
// read (contraction over keys).
//
// Per tile and wave:  S^T = K Q^T  (keys x queries, so one lane owns one query column and the
// running max / sum / rescale are lane-local apart from one exchange between lane l and l^32),
// online softmax in base 2, then O^T += V^T P^T with P^T taken straight from the score
// registers.  Only tiles cut by the diagonal or the window edge are masked.
#include "common.hpp"
#include "mfma.hpp"

namespace gformer {
namespace {

constexpr int BR = kMfmaWindowRows;  // queries per workgroup
constexpr int BC = 64;               // keys per tile
constexpr int WQ = 32;               // queries per wave
constexpr float kLog2e = 1.4426950408889634f;

template <int D> struct WinSmem {
  static constexpr int KROW = D + 8;    // row stride = 4 dwords mod 64: conflict-free b128 reads
  static constexpr int VROW = D + 32;   // row stride = 16 dwords mod 64: conflict-free tr reads
  uint16_t k[BC * KROW];
  uint16_t v[BC * VROW];
};

template <int D>
__global__ __launch_bounds__(kMfmaWindowThreads, 2) void windowed_mfma_kernel(AttnArgs a) {
  constexpr int KS = D / 16;           // k-steps over the head dimension
  constexpr int MT = D / 32;           // 32-row tiles of O^T
  constexpr int KCH = BC * D / 8 / kMfmaWindowThreads;  // 16-byte K chunks per thread per tile
  using Smem = WinSmem<D>;
  __shared__ __attribute__((aligned(16))) Smem sm;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int ln = lane & 31;   // query column / operand row
  const int lh = lane >> 5;   // which half of the k-slots
  const int h = blockIdx.y, b = blockIdx.z;
  const int i0 = blockIdx.x * BR;
  const int q0 = i0 + wave * WQ;
  const int N = a.N, w = a.window;

  const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q.base) + b * a.q.sb + h * a.q.sh;
  const uint16_t* kp = reinterpret_cast<const uint16_t*>(a.k.base) + b * a.k.sb + h * a.k.sh;
  const uint16_t* vp = reinterpret_cast<const uint16_t*>(a.v.base) + b * a.v.sb + h * a.v.sh;
  uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + b * a.osb + h * a.osh;

  // Q^T as B operands, resident for the whole kernel.  Rows past N re-read row N-1 (in bounds);
  // their columns are computed and dropped.
  bf16x8 qreg[KS];
  {
    const int qi = min(q0 + ln, N - 1);
    const uint16_t* qr = qp + (int64_t)qi * a.q.sn + 8 * lh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qreg[ks] = as_bf16x8(*reinterpret_cast<const u32x4*>(qr + 16 * ks));
  }

  f32x16 oacc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[mt][r] = 0.f;
  float m_run = -INFINITY;  // running max of the scaled base-2 scores of this lane's query
  float l_run = 0.f;        // running sum over the keys this lane holds (half of each tile)

  const int kfirst = max(0, i0 - w + 1) / BC;
  const int klast = min(N - 1, i0 + BR - 1) / BC;
  const float sc = a.scale * kLog2e;

  // register staging of the next tile
  u32x4 kst[KCH];
  u32x4 vst[KCH];
  auto load_tile = [&](int t) {
    const int t0 = t * BC;
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int c = tid + i * kMfmaWindowThreads;
      const int row = min(t0 + c / (D / 8), N - 1);
      kst[i] = *reinterpret_cast<const u32x4*>(kp + (int64_t)row * a.k.sn + 8 * (c % (D / 8)));
      vst[i] = *reinterpret_cast<const u32x4*>(vp + (int64_t)row * a.v.sn + 8 * (c % (D / 8)));
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int c = tid + i * kMfmaWindowThreads;
      *reinterpret_cast<u32x4*>(&sm.k[(c / (D / 8)) * Smem::KROW + 8 * (c % (D / 8))]) = kst[i];
      *reinterpret_cast<u32x4*>(&sm.v[(c / (D / 8)) * Smem::VROW + 8 * (c % (D / 8))]) = vst[i];
    }
  };

  load_tile(kfirst);
  for (int t = kfirst; t <= klast; ++t) {
    lds_barrier();  // every wave is done reading the previous tile
    store_tile();
    lds_barrier();
    if (t < klast) load_tile(t + 1);  // in flight while this tile is computed

    const int t0 = t * BC;
    // keys visible to query i: i - w < j <= i
    if (t0 > q0 + WQ - 1 || t0 + BC - 1 <= q0 - w) continue;  // nothing for this wave's queries
    const bool need_mask = !(t0 + BC - 1 <= q0 && t0 > q0 + WQ - 1 - w);

    // S^T = K Q^T for the two 32-key halves of the tile
    f32x16 s[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
      const uint16_t* krow = &sm.k[(32 * kt + ln) * Smem::KROW + 8 * lh];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 ka = as_bf16x8(*reinterpret_cast<const u32x4*>(krow + 16 * ks));
        s[kt] = mfma32(ka, qreg[ks], s[kt]);
      }
    }
    // scale to base-2 logits, mask, tile max
    float mloc = -INFINITY;
    const int qi = q0 + ln;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float x = s[kt][r] * sc;
        if (need_mask) {
          const int j = t0 + 32 * kt + 8 * (r / 4) + 4 * lh + (r % 4);
          x = (j <= qi && j > qi - w) ? x : -INFINITY;
        }
        s[kt][r] = x;
        mloc = fmaxf(mloc, x);
      }
    }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    const float m_new = fmaxf(m_run, mloc);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;  // a query with no visible key yet
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    m_run = m_new;
    float lsum = 0.f;
    uint32_t pb[2][8];  // P^T as packed bf16: pb[kt][4*kb + i] covers registers 8*kb+2i, +1
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const float p0 = __builtin_amdgcn_exp2f(s[kt][r] - m_use);
        const float p1 = __builtin_amdgcn_exp2f(s[kt][r + 1] - m_use);
        const uint32_t pk = pack_bf16(p0, p1);
        pb[kt][r / 2] = pk;
        // the row sum uses the rounded weights the PV product sees
        lsum += bf16_lo(pk) + bf16_hi(pk);
      }
    }
    l_run = l_run * alpha + lsum;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[mt][r] *= alpha;

    // O^T += V^T P^T
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        u32x4 pw;
        pw[0] = pb[kt][4 * kb + 0]; pw[1] = pb[kt][4 * kb + 1];
        pw[2] = pb[kt][4 * kb + 2]; pw[3] = pb[kt][4 * kb + 3];
        const bf16x8 pbv = as_bf16x8(pw);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          // keys in the order the score registers hold them: 16*kb + 4*lh + j, then + 8
          const int r0 = 32 * kt + 16 * kb + 4 * lh;
          const bf16x8 va_ = lds_operand_tr(sm.v, Smem::VROW, r0, r0 + 8, 32 * mt, lane);
          oacc[mt] = mfma32(va_, pbv, oacc[mt]);
        }
      }
    }
  }

  // normalise and write: lane owns query q0+ln, value columns 32*mt + 8*g + 4*lh + 0..3
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_tot;
  const int qi = q0 + ln;
  if (qi < N) {
    uint16_t* orow = op + (int64_t)qi * a.osn;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(oacc[mt][4 * g + 0] * inv, oacc[mt][4 * g + 1] * inv);
        pk[1] = pack_bf16(oacc[mt][4 * g + 2] * inv, oacc[mt][4 * g + 3] * inv);
        *reinterpret_cast<u32x2*>(orow + 32 * mt + 8 * g + 4 * lh) = pk;
      }
    }
  }
}

}  // namespace

hipError_t launch_windowed_mfma(const AttnArgs& a, hipStream_t s) {
  if (a.H0 <= 0 || a.N <= 0 || a.B <= 0) return hipSuccess;
  dim3 grid((a.N + BR - 1) / BR, a.H0, a.B);
  dim3 block(kMfmaWindowThreads);
  if (a.d == 64) windowed_mfma_kernel<64><<<grid, block, 0, s>>>(a);
  else windowed_mfma_kernel<128><<<grid, block, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace gformer
