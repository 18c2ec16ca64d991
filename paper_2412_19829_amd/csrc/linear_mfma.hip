// Causal linear attention heads on bf16 matrix cores (section III-C, Algorithm 1), chunked.
//
// Algorithm 1 walks tokens one by one: A += phi(k_i) (x) v_i, Z += phi(k_i), then reads row i.
// Here a head's sequence is cut into segments (one workgroup each) and segments into chunks of
// 64 tokens.  Inside a chunk the read-out is the masked quadratic form
//     num = tril(phiQ phiK^T) V + phiQ A_prev ,   den = rowsum(tril(phiQ phiK^T)) + phiQ.Z_prev
// and the carried state moves once per chunk: A += phiK^T V, Z += colsum(phiK).  Instead of
// materialising one E x E outer product per token, a chunk's 64 outer products are one MFMA
// contraction.  A and Z stay fp32 (accumulator registers / LDS); operands are bf16.
//
// Segments of one head are stitched in three launches: (1) every segment but the last sums its
// own (A, Z); (2) a tiny kernel turns those into exclusive prefixes; (3) the read-out kernel
// starts each segment from its prefix.
//
// Everything is computed transposed (num^T = V^T P^T + A^T phiQ^T, value column x query) so one
// lane owns one query column and normalisation is lane-local.
#include "common.hpp"
#include "mfma.hpp"

namespace gformer {
namespace {

constexpr int CH = 64;  // tokens per chunk
constexpr float kLog2e = 1.4426950408889634f;

template <int D> struct LinCfg {
  static constexpr int NW = D / 16;           // waves per workgroup
  static constexpr int NT = NW * 64;          // threads per workgroup
  static constexpr int ROW = D + 8;           // bf16 elements per row of a row-major tile
  static constexpr int TROW = CH + 8;         // bf16 elements per row of a transposed tile
  static constexpr int ET = D / 32;           // 32-wide tiles along a feature / value axis
  static constexpr int STILES = ET * ET / NW; // state tiles per wave
  static constexpr int KS = D / 16;           // k-steps over the feature axis
  static constexpr int C8 = D / 8;            // 16-byte pieces per row
  static constexpr int STATE = D * D + D;     // floats per (A, Z) state
};

template <int D> struct LinSmem {
  using C = LinCfg<D>;
  uint16_t fq[CH * C::ROW];     // phi(Q) chunk, row-major [token][feature]
  uint16_t fk[CH * C::ROW];     // phi(K) chunk, row-major
  uint16_t fkt[D * C::TROW];    // phi(K)^T, [feature][token, permuted]
  uint16_t vt[D * C::TROW];     // V^T, [value column][token, permuted]
  uint16_t at[CH * C::TROW];    // masked products, [query][key, permuted]
  uint16_t sb[D * C::ROW];      // bf16 copy of the state A, [value column][feature]
  float z[2][D];                // Z, double-buffered across chunks
  float den[CH];
};

template <int D> struct StateSmem {
  using C = LinCfg<D>;
  uint16_t fkt[D * C::TROW];
  uint16_t vt[D * C::TROW];
  float z[D];
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

// A 4-token x 8-column block: global rows -> registers.  Rows past N are clamped (in bounds).
__device__ __forceinline__ void load_block(const uint16_t* base, int64_t sn, int row0, int col0,
                                           int N, u32x4 (&r)[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = min(row0 + j, N - 1);
    r[j] = *reinterpret_cast<const u32x4*>(base + (int64_t)row * sn + col0);
  }
}

// Store a 4-token x 8-column block transposed: 8 rows (columns col0..col0+7) of 4 tokens each,
// at the permuted position of token group `tok4` (multiple of 4, < 64).
template <int TROW>
__device__ __forceinline__ void store_block_transposed(uint16_t* dst, const u32x4 (&r)[4],
                                                       int col0, int tok4) {
  u32x2 col[8];
  transpose_4x8_bf16(r, col);
  const int pos = 32 * (tok4 / 32) + kperm32(tok4 % 32);
#pragma unroll
  for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x2*>(&dst[(col0 + i) * TROW + pos]) = col[i];
}

__device__ __forceinline__ bf16x8 lds_operand(const uint16_t* p) {
  return as_bf16x8(*reinterpret_cast<const u32x4*>(p));
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

// Z += column sums of the bf16 phi(K) chunk held transposed in LDS: 4 threads per feature.
template <int D>
__device__ __forceinline__ float chunk_feature_sum(const uint16_t* fkt, int tid) {
  using C = LinCfg<D>;
  const int c = tid >> 2, part = tid & 3;
  const u32x4 x0 = *reinterpret_cast<const u32x4*>(&fkt[c * C::TROW + 16 * part]);
  const u32x4 x1 = *reinterpret_cast<const u32x4*>(&fkt[c * C::TROW + 16 * part + 8]);
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) s += bf16_lo(x0[w]) + bf16_hi(x0[w]);
#pragma unroll
  for (int w = 0; w < 4; ++w) s += bf16_lo(x1[w]) + bf16_hi(x1[w]);
  s += __shfl_xor(s, 1, 64);
  s += __shfl_xor(s, 2, 64);
  return s;
}

// -----------------------------------------------------------------------------------------
// (1) per-segment state sums.  Workgroup (head, s) with s < n_segments-1 writes
//     sum_{t in segment s} phi(k_t) (x) v_t  and  sum phi(k_t)  into workspace slot s+1.
// -----------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(LinCfg<D>::NT) void linear_state_kernel(AttnArgs a) {
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

  f32x16 sacc[C::STILES];
#pragma unroll
  for (int i = 0; i < C::STILES; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[i][r] = 0.f;
  if (tid < D) sm.z[tid] = 0.f;

  const bool k_thread = tid < C::NT / 2;
  const int bt = k_thread ? tid : tid - C::NT / 2;
  const int va = bt / C::C8, vc8 = bt % C::C8;
  u32x4 blk[4];
  auto load_chunk = [&](int t0) {
    load_block(k_thread ? hp.k : hp.v, k_thread ? a.k.sn : a.v.sn, t0 + 4 * va, 8 * vc8, N, blk);
  };
  load_chunk(seg_start);
  for (int t0 = seg_start; t0 < seg_end; t0 += CH) {
    __syncthreads();
    if (k_thread) {
#pragma unroll
      for (int j = 0; j < 4; ++j) blk[j] = map_features(blk[j], a.phi, t0 + 4 * va + j < N);
      store_block_transposed<C::TROW>(sm.fkt, blk, 8 * vc8, 4 * va);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (t0 + 4 * va + j >= N) blk[j] = u32x4{0u, 0u, 0u, 0u};
      store_block_transposed<C::TROW>(sm.vt, blk, 8 * vc8, 4 * va);
    }
    __syncthreads();
    if (t0 + CH < seg_end) load_chunk(t0 + CH);
#pragma unroll
    for (int i = 0; i < C::STILES; ++i) {
      const int ti = wave * C::STILES + i, ct = ti / C::ET, et = ti % C::ET;
#pragma unroll
      for (int kk = 0; kk < CH / 16; ++kk) {
        const bf16x8 fa = lds_operand(&sm.fkt[(32 * ct + ln) * C::TROW + 16 * kk + 8 * lh]);
        const bf16x8 vb = lds_operand(&sm.vt[(32 * et + ln) * C::TROW + 16 * kk + 8 * lh]);
        sacc[i] = mfma32(fa, vb, sacc[i]);
      }
    }
    const float zs = chunk_feature_sum<D>(sm.fkt, tid);
    if ((tid & 3) == 0) sm.z[tid >> 2] += zs;  // each feature has exactly one writer
  }
  __syncthreads();
  float* dst = hp.state + (int64_t)(seg + 1) * C::STATE;
#pragma unroll
  for (int i = 0; i < C::STILES; ++i) {
    const int ti = wave * C::STILES + i, ct = ti / C::ET, et = ti % C::ET;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      dst[(32 * ct + 8 * (r / 4) + 4 * lh + (r % 4)) * D + 32 * et + ln] = sacc[i][r];
  }
  if (tid < D) dst[D * D + tid] = sm.z[tid];
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
__global__ __launch_bounds__(LinCfg<D>::NT) void linear_main_kernel(AttnArgs a) {
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

  // carried state: this wave's tiles of A in accumulator layout (lane = value column,
  // registers = feature rows), Z in LDS
  f32x16 sacc[C::STILES];
  const float* src = (seg > 0 && hp.state) ? hp.state + (int64_t)seg * C::STATE : nullptr;
#pragma unroll
  for (int i = 0; i < C::STILES; ++i) {
    const int ti = wave * C::STILES + i, ct = ti / C::ET, et = ti % C::ET;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      sacc[i][r] = src ? src[(32 * ct + 8 * (r / 4) + 4 * lh + (r % 4)) * D + 32 * et + ln] : 0.f;
  }
  if (tid < D) sm.z[0][tid] = src ? src[D * D + tid] : 0.f;
  auto publish_state = [&]() {  // bf16 copy of A for the phiQ A_prev product
#pragma unroll
    for (int i = 0; i < C::STILES; ++i) {
      const int ti = wave * C::STILES + i, ct = ti / C::ET, et = ti % C::ET;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(sacc[i][4 * g + 0], sacc[i][4 * g + 1]);
        pk[1] = pack_bf16(sacc[i][4 * g + 2], sacc[i][4 * g + 3]);
        *reinterpret_cast<u32x2*>(&sm.sb[(32 * et + ln) * C::ROW + 32 * ct + 8 * g + 4 * lh]) = pk;
      }
    }
  };
  publish_state();

  // global -> register staging: 2 row-major Q pieces per thread, one 4x8 block of K or V
  const bool k_thread = tid < C::NT / 2;
  const int bt = k_thread ? tid : tid - C::NT / 2;
  const int va = bt / C::C8, vc8 = bt % C::C8;
  u32x4 qst[2];
  u32x4 blk[4];
  auto load_chunk = [&](int t0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + i * C::NT;
      const int row = min(t0 + c / C::C8, N - 1);
      qst[i] = *reinterpret_cast<const u32x4*>(hp.q + (int64_t)row * a.q.sn + 8 * (c % C::C8));
    }
    load_block(k_thread ? hp.k : hp.v, k_thread ? a.k.sn : a.v.sn, t0 + 4 * va, 8 * vc8, N, blk);
  };

  const int et_n = wave % C::ET;  // this wave's tile of num^T: value columns 32*et_n ..
  const int tq = wave / C::ET;    // .. by queries 32*tq ..
  constexpr int PPT = C::NT / CH; // threads per query in the denominator
  load_chunk(seg_start);
  int zc = 0;
  for (int t0 = seg_start; t0 < seg_end; t0 += CH, zc ^= 1) {
    __syncthreads();  // (1) previous chunk fully consumed
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + i * C::NT;
      *reinterpret_cast<u32x4*>(&sm.fq[(c / C::C8) * C::ROW + 8 * (c % C::C8)]) =
          map_features(qst[i], a.phi, true);
    }
    if (k_thread) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        blk[j] = map_features(blk[j], a.phi, t0 + 4 * va + j < N);
        *reinterpret_cast<u32x4*>(&sm.fk[(4 * va + j) * C::ROW + 8 * vc8]) = blk[j];
      }
      store_block_transposed<C::TROW>(sm.fkt, blk, 8 * vc8, 4 * va);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (t0 + 4 * va + j >= N) blk[j] = u32x4{0u, 0u, 0u, 0u};
      store_block_transposed<C::TROW>(sm.vt, blk, 8 * vc8, 4 * va);
    }
    __syncthreads();  // (2) chunk tiles (and on the first pass the state copy) visible
    if (t0 + CH < seg_end) load_chunk(t0 + CH);

    // masked products P^T[key][query] = phi(k_key).phi(q_query), key <= query: three 32x32
    // tiles (the fourth lies above the diagonal), one each on waves 0..2
    if (wave < 3) {
      const int tk = wave == 2 ? 1 : 0, tqa = wave == 0 ? 0 : 1;
      f32x16 p;
#pragma unroll
      for (int r = 0; r < 16; ++r) p[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks) {
        const bf16x8 ka = lds_operand(&sm.fk[(32 * tk + ln) * C::ROW + 16 * ks + 8 * lh]);
        const bf16x8 qb = lds_operand(&sm.fq[(32 * tqa + ln) * C::ROW + 16 * ks + 8 * lh]);
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
        *reinterpret_cast<u32x2*>(
            &sm.at[(32 * tqa + ln) * C::TROW + 32 * tk + 16 * (g / 2) + 8 * lh + 4 * (g % 2)]) = pk;
      }
    }
    // num^T = A^T phiQ^T  (carried state part)
    f32x16 num;
#pragma unroll
    for (int r = 0; r < 16; ++r) num[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      const bf16x8 sa = lds_operand(&sm.sb[(32 * et_n + ln) * C::ROW + 16 * ks + 8 * lh]);
      const bf16x8 qb = lds_operand(&sm.fq[(32 * tq + ln) * C::ROW + 16 * ks + 8 * lh]);
      num = mfma32(sa, qb, num);
    }
    __syncthreads();  // (3) products visible; nobody reads the old state copy any more

    // denominator: rowsum of the (rounded) products + phi(q).Z_prev, PPT threads per query
    {
      const int qrow = tid / PPT, part = tid % PPT;
      constexpr int KW = CH / PPT;  // product slots per thread
      constexpr int CW = D / PPT;   // features per thread
      float s = 0.f;
      const int kvis = qrow < 32 ? 32 : 64;  // slots >= 32 of the first 32 queries are unused
#pragma unroll
      for (int x = 0; x < KW; x += 8) {
        if (KW * part + x < kvis) {
          const u32x4 pv = *reinterpret_cast<const u32x4*>(&sm.at[qrow * C::TROW + KW * part + x]);
#pragma unroll
          for (int w = 0; w < 4; ++w) s += bf16_lo(pv[w]) + bf16_hi(pv[w]);
        }
      }
#pragma unroll
      for (int x = 0; x < CW; x += 8) {
        const u32x4 qv = *reinterpret_cast<const u32x4*>(&sm.fq[qrow * C::ROW + CW * part + x]);
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
    // num^T += V^T P^T  (inside the chunk); the first 32 queries see only the first 32 keys
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      if (kt <= tq) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const bf16x8 va_ = lds_operand(&sm.vt[(32 * et_n + ln) * C::TROW + 32 * kt + 16 * kb + 8 * lh]);
          const bf16x8 pb = lds_operand(&sm.at[(32 * tq + ln) * C::TROW + 32 * kt + 16 * kb + 8 * lh]);
          num = mfma32(va_, pb, num);
        }
      }
    }
    // state update: A += phiK^T V, Z += colsum(phiK); then refresh the bf16 copy
#pragma unroll
    for (int i = 0; i < C::STILES; ++i) {
      const int ti = wave * C::STILES + i, ct = ti / C::ET, et = ti % C::ET;
#pragma unroll
      for (int kk = 0; kk < CH / 16; ++kk) {
        const bf16x8 fa = lds_operand(&sm.fkt[(32 * ct + ln) * C::TROW + 16 * kk + 8 * lh]);
        const bf16x8 vb = lds_operand(&sm.vt[(32 * et + ln) * C::TROW + 16 * kk + 8 * lh]);
        sacc[i] = mfma32(fa, vb, sacc[i]);
      }
    }
    publish_state();
    {
      const float zs = chunk_feature_sum<D>(sm.fkt, tid);
      if ((tid & 3) == 0) sm.z[zc ^ 1][tid >> 2] = sm.z[zc][tid >> 2] + zs;
    }
    __syncthreads();  // (4) denominators visible
    const int qi = t0 + 32 * tq + ln;
    if (qi < N) {
      const float inv = 1.f / sm.den[32 * tq + ln];
      uint16_t* orow = hp.o + (int64_t)qi * a.osn + 32 * et_n + 4 * lh;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(num[4 * g + 0] * inv, num[4 * g + 1] * inv);
        pk[1] = pack_bf16(num[4 * g + 2] * inv, num[4 * g + 3] * inv);
        *reinterpret_cast<u32x2*>(orow + 8 * g) = pk;
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
