// Causal linear attention heads on bf16 matrix cores (section III-C, Algorithm 1), chunked.
//
// Algorithm 1 walks tokens one by one: A += phi(k_i) (x) v_i, Z += phi(k_i), then reads row i.
// Here a head's sequence is cut into segments (one workgroup each) and segments into chunks of
// 64 tokens.  Inside a chunk the read-out is the masked quadratic form
//     num = tril(phiQ phiK^T) V + phiQ A_prev ,   den = rowsum(tril(phiQ phiK^T)) + phiQ.Z_prev
// and the carried state moves once per chunk: A += phiK^T V, Z += colsum(phiK).  Instead of
// materialising one E x E outer product per token, a chunk's 64 outer products are one MFMA
// contraction.  A and Z stay fp32 (accumulator registers / LDS); MFMA operands are bf16.
//
// Work split inside a workgroup: wave w owns value columns 32w..32w+31, i.e. the state tiles
// A[:, 32w..] (fp32 accumulators, lane = value column, registers = feature rows) and the
// output tile num^T[32w.., all 64 queries].  Because a lane's accumulator registers are exactly
// the k-slots an MFMA A operand wants (see mfma.hpp), phiQ A_prev is fed straight from the
// state registers; phi(Q) is stored in LDS with its feature index permuted to match.  phi(K)
// and V sit row-major in LDS and are read through the LDS transpose read wherever the
// contraction runs over tokens.
//
// Segments of one head are stitched in three launches: (1) every segment but the last sums its
// own (A, Z); (2) a tiny kernel turns those into exclusive prefixes; (3) the read-out kernel
// starts each segment from its prefix.
#include "common.hpp"
#include "mfma.hpp"

namespace gformer {
namespace {

constexpr int CH = 64;  // tokens per chunk
constexpr float kLog2e = 1.4426950408889634f;

template <int D> struct LinCfg {
  static constexpr int ET = D / 32;           // 32-wide tiles along a feature / value axis
  static constexpr int NW = ET;               // waves per workgroup: one per value-column tile
  static constexpr int NT = NW * 64;          // threads per workgroup
  static constexpr int QROW = D + 8;          // phi(Q): 128-bit row reads   (stride = 4 dw mod 64)
  static constexpr int KROW = D + 16;         // phi(K): 64-bit row reads + transpose reads
  static constexpr int VROW = D + 32;         // V: transpose reads only     (stride = 16 dw mod 64)
  static constexpr int PROW = CH + 8;         // masked products, [query][key]
  static constexpr int C8 = D / 8;            // 16-byte pieces per row
  static constexpr int PIECES = CH * C8 / NT; // pieces per thread per tensor per chunk (= 4)
  static constexpr int STATE = D * D + D;     // floats per (A, Z) state
};

template <int D> struct LinSmem {
  using C = LinCfg<D>;
  uint16_t fq[CH * C::QROW];   // phi(Q), feature index permuted by kperm32 inside 32-groups
  uint16_t fk[CH * C::KROW];   // phi(K), natural order
  uint16_t v[CH * C::VROW];    // V
  uint16_t pt[CH * C::PROW];   // masked products P^T viewed as [query][key]
  float z[2][D];               // Z in the same permuted feature order as fq; double-buffered
  float den[CH];
};

template <int D> struct StateSmem {
  using C = LinCfg<D>;
  uint16_t fk[CH * C::KROW];
  uint16_t v[CH * C::VROW];
};

// phi(x) = elu(x) + 1 = max(x + 1, min(exp(x), 1))   (section II-B)
__device__ __forceinline__ float elu1(float x) {
  const float e = fminf(__builtin_amdgcn_exp2f(x * kLog2e), 1.0f);
  return fmaxf(x + 1.0f, e);
}

// Feature map on 8 packed bf16 values; invalid rows (past the sequence end) become zeros.
__device__ __forceinline__ u32x4 map_features(u32x4 v, int phi, bool valid) {
  u32x4 o;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    float lo = bf16_lo(v[w]), hi = bf16_hi(v[w]);
    if (phi == 0) { lo = elu1(lo); hi = elu1(hi); }
    o[w] = valid ? pack_bf16(lo, hi) : 0u;
  }
  return o;
}

__device__ __forceinline__ float sum8_bf16(bf16x8 x) {
  const u32x4 u = as_u32x4(x);
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) s += bf16_lo(u[w]) + bf16_hi(u[w]);
  return s;
}

template <int D> struct HeadPtrs {
  const uint16_t *q, *k, *v;
  uint16_t* o;
  float* state;  // this head's [n_segments][STATE] block of the workspace (may be null)
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
  p.state = a.ws_states ? a.ws_states + (int64_t)head_linear * a.n_segments * LinCfg<D>::STATE : nullptr;
  return p;
}

// State tile (ct, wave) in accumulator layout: lane = value column 32*wave + l%32,
// register r = feature row 32*ct + 8*(r/4) + 4*(l/32) + r%4.  Workspace layout is [c][e] fp32.
template <int D>
__device__ __forceinline__ int state_index(int ct, int wave, int r, int ln, int lh) {
  return (32 * ct + 8 * (r / 4) + 4 * lh + (r % 4)) * D + 32 * wave + ln;
}

// A += phiK^T V for this wave's value columns, from the row-major chunk tiles in LDS; returns
// this lane's share of colsum(phiK) for features 32*wave + l%32 (tokens of its k-slot half).
template <int D>
__device__ __forceinline__ float update_state(f32x16 (&sacc)[LinCfg<D>::ET], const uint16_t* fk,
                                              const uint16_t* v, int wave, int lane) {
  using C = LinCfg<D>;
  const int lh = lane >> 5;
  float zs = 0.f;
  bf16x8 vb[CH / 16];
#pragma unroll
  for (int kk = 0; kk < CH / 16; ++kk)
    vb[kk] = lds_operand_tr(v, C::VROW, 16 * kk + 8 * lh, 16 * kk + 8 * lh + 4, 32 * wave, lane);
#pragma unroll
  for (int ct = 0; ct < C::ET; ++ct) {
#pragma unroll
    for (int kk = 0; kk < CH / 16; ++kk) {
      const bf16x8 fa =
          lds_operand_tr(fk, C::KROW, 16 * kk + 8 * lh, 16 * kk + 8 * lh + 4, 32 * ct, lane);
      if (ct == wave) zs += sum8_bf16(fa);
      sacc[ct] = mfma32(fa, vb[kk], sacc[ct]);
    }
  }
  return zs;
}

// -----------------------------------------------------------------------------------------
// (1) per-segment state sums.  Workgroup (head, s) with s < n_segments-1 writes
//     sum_{t in segment s} phi(k_t) (x) v_t  and  sum phi(k_t)  into workspace slot s+1.
// -----------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(LinCfg<D>::NT, 2) void linear_state_kernel(AttnArgs a) {
  using C = LinCfg<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  StateSmem<D>& sm = *reinterpret_cast<StateSmem<D>*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int nsm1 = a.n_segments - 1;
  const int head = blockIdx.x / nsm1, seg = blockIdx.x % nsm1;
  const HeadPtrs<D> hp = head_ptrs<D>(a, head);
  const int N = a.N;
  const int seg_start = seg * a.segment_len;
  const int seg_end = min(N, seg_start + a.segment_len);

  f32x16 sacc[C::ET];
#pragma unroll
  for (int i = 0; i < C::ET; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[i][r] = 0.f;
  float zacc = 0.f;

  u32x4 kst[C::PIECES], vst[C::PIECES];
  auto load_chunk = [&](int t0) {
#pragma unroll
    for (int i = 0; i < C::PIECES; ++i) {
      const int c = tid + i * C::NT;
      const int row = min(t0 + c / C::C8, N - 1);
      kst[i] = *reinterpret_cast<const u32x4*>(hp.k + (int64_t)row * a.k.sn + 8 * (c % C::C8));
      vst[i] = *reinterpret_cast<const u32x4*>(hp.v + (int64_t)row * a.v.sn + 8 * (c % C::C8));
    }
  };
  load_chunk(seg_start);
  for (int t0 = seg_start; t0 < seg_end; t0 += CH) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < C::PIECES; ++i) {
      const int c = tid + i * C::NT;
      const int row = c / C::C8, col = 8 * (c % C::C8);
      const bool valid = t0 + row < N;
      *reinterpret_cast<u32x4*>(&sm.fk[row * C::KROW + col]) = map_features(kst[i], a.phi, valid);
      *reinterpret_cast<u32x4*>(&sm.v[row * C::VROW + col]) = valid ? vst[i] : u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();
    if (t0 + CH < seg_end) load_chunk(t0 + CH);
    zacc += update_state<D>(sacc, sm.fk, sm.v, wave, lane);
  }
  float* dst = hp.state + (int64_t)(seg + 1) * C::STATE;
#pragma unroll
  for (int ct = 0; ct < C::ET; ++ct)
#pragma unroll
    for (int r = 0; r < 16; ++r) dst[state_index<D>(ct, wave, r, ln, lh)] = sacc[ct][r];
  zacc += __shfl_xor(zacc, 32, 64);
  if (lh == 0) dst[D * D + 32 * wave + ln] = zacc;
}

// (2) slots 1..n_segments-1 hold per-segment sums of segments 0..n_segments-2; make slot s the
//     sum of all segments before s.
__global__ __launch_bounds__(256) void linear_prefix_kernel(float* ws, int n_heads, int n_segments,
                                                             int state_floats) {
  const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int head = blockIdx.y;
  if (x >= state_floats || head >= n_heads) return;
  float* p = ws + (int64_t)head * n_segments * state_floats + x;
  float run = p[state_floats];
  for (int s = 2; s < n_segments; ++s) {
    run += p[(int64_t)s * state_floats];
    p[(int64_t)s * state_floats] = run;
  }
}

// -----------------------------------------------------------------------------------------
// (3) read-out.  Workgroup (head, segment) walks its chunks carrying (A, Z).
// -----------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(LinCfg<D>::NT, 2) void linear_main_kernel(AttnArgs a) {
  using C = LinCfg<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  LinSmem<D>& sm = *reinterpret_cast<LinSmem<D>*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int head = blockIdx.x / a.n_segments, seg = blockIdx.x % a.n_segments;
  const HeadPtrs<D> hp = head_ptrs<D>(a, head);
  const int N = a.N;
  const int seg_start = seg * a.segment_len;
  const int seg_end = min(N, seg_start + a.segment_len);
  if (seg_start >= seg_end) return;  // uniform: nothing in this segment

  // carried state
  f32x16 sacc[C::ET];
  const float* src = (seg > 0 && hp.state) ? hp.state + (int64_t)seg * C::STATE : nullptr;
#pragma unroll
  for (int ct = 0; ct < C::ET; ++ct)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      sacc[ct][r] = src ? src[state_index<D>(ct, wave, r, ln, lh)] : 0.f;
  if (lh == 0) sm.z[0][32 * wave + kperm32(ln)] = src ? src[D * D + 32 * wave + ln] : 0.f;

  // global -> register staging, row-major 16-byte pieces
  u32x4 qst[C::PIECES], kst[C::PIECES], vst[C::PIECES];
  auto load_chunk = [&](int t0) {
#pragma unroll
    for (int i = 0; i < C::PIECES; ++i) {
      const int c = tid + i * C::NT;
      const int row = min(t0 + c / C::C8, N - 1);
      const int col = 8 * (c % C::C8);
      qst[i] = *reinterpret_cast<const u32x4*>(hp.q + (int64_t)row * a.q.sn + col);
      kst[i] = *reinterpret_cast<const u32x4*>(hp.k + (int64_t)row * a.k.sn + col);
      vst[i] = *reinterpret_cast<const u32x4*>(hp.v + (int64_t)row * a.v.sn + col);
    }
  };

  constexpr int PPT = C::NT / CH;  // threads per query in the denominator
  load_chunk(seg_start);
  int zc = 0;
  for (int t0 = seg_start; t0 < seg_end; t0 += CH, zc ^= 1) {
    __syncthreads();  // (1) previous chunk fully consumed
#pragma unroll
    for (int i = 0; i < C::PIECES; ++i) {
      const int c = tid + i * C::NT;
      const int row = c / C::C8, c8 = c % C::C8, col = 8 * c8;
      const bool valid = t0 + row < N;
      // phi(Q): features 8*c8 .. +7 go to permuted positions (two groups of 4, 8 apart)
      const u32x4 fqv = map_features(qst[i], a.phi, true);
      const int x = c8 % 4;
      uint16_t* qd = &sm.fq[row * C::QROW + 32 * (c8 / 4) + 16 * (x / 2) + 4 * (x % 2)];
      *reinterpret_cast<u32x2*>(qd) = u32x2{fqv[0], fqv[1]};
      *reinterpret_cast<u32x2*>(qd + 8) = u32x2{fqv[2], fqv[3]};
      *reinterpret_cast<u32x4*>(&sm.fk[row * C::KROW + col]) = map_features(kst[i], a.phi, valid);
      *reinterpret_cast<u32x4*>(&sm.v[row * C::VROW + col]) = valid ? vst[i] : u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();  // (2) chunk tiles (and on the first pass Z) visible
    if (t0 + CH < seg_end) load_chunk(t0 + CH);

    // masked products P^T[key][query] = phi(k_key).phi(q_query), key <= query: three 32x32
    // tiles (the fourth lies above the diagonal), dealt round-robin to the waves
#pragma unroll
    for (int tile = 0; tile < 3; ++tile) {
      if (tile % C::NW != wave) continue;
      const int tk = tile == 2 ? 1 : 0, tqa = tile == 0 ? 0 : 1;
      f32x16 p;
#pragma unroll
      for (int r = 0; r < 16; ++r) p[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        // k-slot 8*lh + 4*g + j of this step is feature 16*ks + 8*g + 4*lh + j
        const uint16_t* kr = &sm.fk[(32 * tk + ln) * C::KROW + 16 * ks + 4 * lh];
        const u32x2 k0 = *reinterpret_cast<const u32x2*>(kr);
        const u32x2 k1 = *reinterpret_cast<const u32x2*>(kr + 8);
        const bf16x8 ka = as_bf16x8(u32x4{k0[0], k0[1], k1[0], k1[1]});
        const bf16x8 qb = lds_read16(&sm.fq[(32 * tqa + ln) * C::QROW + 16 * ks + 8 * lh]);
        p = mfma32(ka, qb, p);
      }
      if (tk == tqa) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (8 * (r / 4) + 4 * lh + (r % 4) > ln) p[r] = 0.f;
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(p[4 * g + 0], p[4 * g + 1]);
        pk[1] = pack_bf16(p[4 * g + 2], p[4 * g + 3]);
        *reinterpret_cast<u32x2*>(&sm.pt[(32 * tqa + ln) * C::PROW + 32 * tk + 8 * g + 4 * lh]) = pk;
      }
    }
    // num^T = A^T phiQ^T with A straight from the state registers
    f32x16 num[2];
#pragma unroll
    for (int tq = 0; tq < 2; ++tq)
#pragma unroll
      for (int r = 0; r < 16; ++r) num[tq][r] = 0.f;
#pragma unroll
    for (int ct = 0; ct < C::ET; ++ct) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        u32x4 sw;
#pragma unroll
        for (int i = 0; i < 4; ++i) sw[i] = pack_bf16(sacc[ct][8 * kb + 2 * i], sacc[ct][8 * kb + 2 * i + 1]);
        const bf16x8 sa = as_bf16x8(sw);
#pragma unroll
        for (int tq = 0; tq < 2; ++tq) {
          const bf16x8 qb = lds_read16(&sm.fq[(32 * tq + ln) * C::QROW + 32 * ct + 16 * kb + 8 * lh]);
          num[tq] = mfma32(sa, qb, num[tq]);
        }
      }
    }
    __syncthreads();  // (3) products visible

    // denominator: rowsum of the (rounded) products + phi(q).Z_prev, PPT threads per query
    {
      const int qrow = tid / PPT, part = tid % PPT;
      constexpr int KW = CH / PPT;  // product slots per thread
      constexpr int CW = D / PPT;   // features per thread
      float s = 0.f;
      const int kvis = qrow < 32 ? 32 : 64;  // keys >= 32 are never visible to the first 32 queries
#pragma unroll
      for (int x = 0; x < KW; x += 8) {
        if (KW * part + x < kvis) {
          const u32x4 pv = *reinterpret_cast<const u32x4*>(&sm.pt[qrow * C::PROW + KW * part + x]);
#pragma unroll
          for (int w = 0; w < 4; ++w) s += bf16_lo(pv[w]) + bf16_hi(pv[w]);
        }
      }
#pragma unroll
      for (int x = 0; x < CW; x += 8) {
        const u32x4 qv = *reinterpret_cast<const u32x4*>(&sm.fq[qrow * C::QROW + CW * part + x]);
        const float* zz = &sm.z[zc][CW * part + x];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          s = fmaf(bf16_lo(qv[w]), zz[2 * w], s);
          s = fmaf(bf16_hi(qv[w]), zz[2 * w + 1], s);
        }
      }
#pragma unroll
      for (int o = 1; o < PPT; o <<= 1) s += __shfl_xor(s, o, 64);
      if (part == 0) sm.den[qrow] = s + a.eps;
    }
    // num^T += V^T P^T (inside the chunk); the first 32 queries see only the first 32 keys
#pragma unroll
    for (int kk = 0; kk < CH / 16; ++kk) {
      const bf16x8 va_ =
          lds_operand_tr(sm.v, C::VROW, 16 * kk + 8 * lh, 16 * kk + 8 * lh + 4, 32 * wave, lane);
#pragma unroll
      for (int tq = 0; tq < 2; ++tq) {
        if (16 * kk < 32 * (tq + 1)) {
          const bf16x8 pb = lds_read16(&sm.pt[(32 * tq + ln) * C::PROW + 16 * kk + 8 * lh]);
          num[tq] = mfma32(va_, pb, num[tq]);
        }
      }
    }
    // state update: A += phiK^T V, Z += colsum(phiK)
    {
      float zs = update_state<D>(sacc, sm.fk, sm.v, wave, lane);
      zs += __shfl_xor(zs, 32, 64);
      const int zi = 32 * wave + kperm32(ln);
      if (lh == 0) sm.z[zc ^ 1][zi] = sm.z[zc][zi] + zs;
    }
    __syncthreads();  // (4) denominators visible
#pragma unroll
    for (int tq = 0; tq < 2; ++tq) {
      const int qi = t0 + 32 * tq + ln;
      if (qi < N) {
        const float inv = 1.f / sm.den[32 * tq + ln];
        uint16_t* orow = hp.o + (int64_t)qi * a.osn + 32 * wave + 4 * lh;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 pk;
          pk[0] = pack_bf16(num[tq][4 * g + 0] * inv, num[tq][4 * g + 1] * inv);
          pk[1] = pack_bf16(num[tq][4 * g + 2] * inv, num[tq][4 * g + 3] * inv);
          *reinterpret_cast<u32x2*>(orow + 8 * g) = pk;
        }
      }
    }
  }
}

template <int D> hipError_t launch_state_t(const AttnArgs& a, hipStream_t s) {
  using C = LinCfg<D>;
  const int heads = a.B * (a.H - a.H0);
  auto kern = linear_state_kernel<D>;
  const int smem = (int)sizeof(StateSmem<D>);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (e != hipSuccess) return e;
  kern<<<dim3(heads * (a.n_segments - 1)), dim3(C::NT), smem, s>>>(a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (a.n_segments > 2) {
    linear_prefix_kernel<<<dim3((C::STATE + 255) / 256, heads), dim3(256), 0, s>>>(
        a.ws_states, heads, a.n_segments, C::STATE);
    e = hipGetLastError();
  }
  return e;
}

template <int D> hipError_t launch_main_t(const AttnArgs& a, hipStream_t s) {
  using C = LinCfg<D>;
  const int heads = a.B * (a.H - a.H0);
  auto kern = linear_main_kernel<D>;
  const int smem = (int)sizeof(LinSmem<D>);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (e != hipSuccess) return e;
  kern<<<dim3(heads * a.n_segments), dim3(C::NT), smem, s>>>(a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_linear_state_mfma(const AttnArgs& a, hipStream_t s) {
  if (a.H - a.H0 <= 0 || a.N <= 0 || a.B <= 0 || a.n_segments <= 1) return hipSuccess;
  return a.d == 64 ? launch_state_t<64>(a, s) : launch_state_t<128>(a, s);
}

hipError_t launch_linear_main_mfma(const AttnArgs& a, hipStream_t s) {
  if (a.H - a.H0 <= 0 || a.N <= 0 || a.B <= 0) return hipSuccess;
  return a.d == 64 ? launch_main_t<64>(a, s) : launch_main_t<128>(a, s);
}

}  // namespace gformer
