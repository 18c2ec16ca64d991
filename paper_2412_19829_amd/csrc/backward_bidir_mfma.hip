// Backward pass of the bidirectional linear heads on bf16 matrix cores (section II-B's ratio over
// all keys, differentiated; formulas at the top of backward_bidir_scalar.hip).
//
// With fq = phi(q), fk = phi(k), S = sum_j fk_j v_j^T, z = sum_j fk_j, den_i = fq_i.z + eps,
// g_i = dO_i / den_i, r_i = S g_i, c_i = fq_i.r_i / den_i:
//   dfq_i = r_i - c_i z,   B = sum_i fq_i g_i^T,   Y = sum_i c_i fq_i,
//   dfk_j = B v_j - Y,     dv_j = B^T fk_j.
// Nothing depends on the position: three sweeps, chunks of 64 tokens, every product a 32 x 32
// MFMA tile job handed out over the waves (the tile and operand conventions of the causal scans
// in backward_linear_mfma.hip, without their in-chunk weights):
//   (1) S, z: each workgroup sums its segment of its head and writes the partial sums;
//   (2) dq: the head's S and z (partials added up, bf16 copy of S in LDS as the operand) against
//       every chunk of the segment; B and Y are summed on the way and written as partials;
//   (3) dk, dv from the head's B and Y.
// A head is cut into up to four segments (one workgroup each) when there are fewer heads than
// compute units.  Operands are bf16, sums and vectors fp32.  The d x d sums are operands as bf16
// pairs (high half + rounded remainder) where their product is one side of a difference:
// r_i = S g_i against c_i z, and B v_j against Y.  On a long head a single bf16 would do (worst row
// of a CPU model with these roundings: 0.5 %), but with a handful of tokens the two sides are
// nearly equal (one token: exactly equal, the gradients with respect to q and k vanish) and the
// 2^-9 of a single bf16 is all that is left: 2.6 % of the test's measure.  dv = B^T fk has no such
// difference and takes the high half alone.  g = dO / den is a pair as well (in S g and in the
// sum B): measured on heads of 1 to 30 tokens the worst row is 1.6 % without and under 1 % with it.
#include "backward_linear_common.hpp"

namespace gformer {
namespace {

constexpr int kMaxSeg = kBidirStateSlots;   // segments per head = slots per sum in the workspace

template <int D> struct BbSmem {
  using C = LbCfg<D>;
  uint16_t ta[CH * C::R], tb[CH * C::R];   // the chunk's two tensors: (fk, v) or (fq, dO -> g)
  uint16_t tbl[CH * C::R];                 // low half of g (second sweep)
  uint16_t st[D * C::R];                   // bf16 copy of the head's d x d sum, [feature][value] ...
  uint16_t stl[D * C::R];                  // ... and bf16 of what that copy leaves
  float z[D];                              // its vector (z or Y); sweep 1: the running column sum
  float zpart[C::ZP][D];
  float dz[CH], den[CH], cc[CH], pd[C::MT][CH];
};

template <int D> constexpr int kState = D * D + D;

// slot of (head, which sum, segment) in the workspace
template <int D>
__device__ __forceinline__ float* state_slot(const BwdArgs& a, int head_linear, int which, int seg) {
  return a.ws_state + (((int64_t)head_linear * 2 + which) * kMaxSeg + seg) * kState<D>;
}
// chunks [cb, ce) of segment s when a head of nchunks chunks is cut into nseg equal segments
__device__ __forceinline__ void segment_bounds(int nchunks, int nseg, int s, int& cb, int& ce) {
  cb = (int)((int64_t)nchunks * s / nseg);
  ce = (int)((int64_t)nchunks * (s + 1) / nseg);
}

// the partial sums of a head added up: bf16 copy of the matrix into st, the vector into z
template <int D>
__device__ __forceinline__ void load_total(BbSmem<D>& sm, const BwdArgs& a, int head_linear, int which,
                                           int nseg, int tid) {
  using C = LbCfg<D>;
  const float* base = state_slot<D>(a, head_linear, which, 0);
  for (int x = tid * 4; x < D * D; x += C::NT * 4) {
    float4 s4 = *reinterpret_cast<const float4*>(base + x);
    for (int s = 1; s < nseg; ++s) {
      const float4 t4 = *reinterpret_cast<const float4*>(base + (int64_t)s * kState<D> + x);
      s4.x += t4.x; s4.y += t4.y; s4.z += t4.z; s4.w += t4.w;
    }
    put4_split(&sm.st[(x / D) * C::R + x % D], &sm.stl[(x / D) * C::R + x % D], s4.x, s4.y, s4.z, s4.w);
  }
  if (tid < D) {
    float zz = base[D * D + tid];
    for (int s = 1; s < nseg; ++s) zz += base[(int64_t)s * kState<D> + D * D + tid];
    sm.z[tid] = zz;
  }
}

// accumulator tiles of a d x d sum (value block vt, feature block ft per tile, as in the causal
// scans) -> fp32 [feature][value] in the workspace
template <int D>
__device__ __forceinline__ void store_partial(float* out, const f32x16 (&sacc)[LbCfg<D>::TPW], int wave,
                                              int ln, int lh) {
  using C = LbCfg<D>;
#pragma unroll
  for (int u = 0; u < C::TPW; ++u) {
    const int stile = wave * C::TPW + u, vt = stile / C::MT, ft = stile % C::MT;
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4)
      *reinterpret_cast<float4*>(out + (32 * ft + ln) * D + 32 * vt + 8 * g4 + 4 * lh) =
          make_float4(sacc[u][4 * g4], sacc[u][4 * g4 + 1], sacc[u][4 * g4 + 2], sacc[u][4 * g4 + 3]);
  }
}

// ---------------------------------------------------------------------------------------
// (1) S = sum fk v^T, z = sum fk over the segment.  grid = (H - H0, B, segments)
// ---------------------------------------------------------------------------------------
template <int D, bool ELU1>
__global__ __launch_bounds__(LbCfg<D>::NT, 1) void linear_bidir_sum_mfma_kernel(BwdArgs a) {
  using C = LbCfg<D>;
  constexpr int MT = C::MT, NT = C::NT, R = C::R, TPW = C::TPW, PCS = C::PCS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  BbSmem<D>& sm = *reinterpret_cast<BbSmem<D>*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ln = lane & 31, lh = lane >> 5;
  const int h = a.H0 + blockIdx.x, b = blockIdx.y, seg = blockIdx.z;
  const int head_linear = b * (a.H - a.H0) + blockIdx.x;
  const HeadCtx<D> hc = head_ctx<D>(a, b, h);
  const int N = a.N, nchunks = (N + CH - 1) / CH;
  int cb, ce;
  segment_bounds(nchunks, a.lin_segments, seg, cb, ce);
  const int trl = lds_operand_tr_lane_offset(R, lane) + 8 * lh * R;

  f32x16 sacc[TPW];
#pragma unroll
  for (int u = 0; u < TPW; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[u][r] = 0.f;
  if (tid < D) sm.z[tid] = 0.f;

  u32x4 rk[PCS], rv[PCS];
  auto load_chunk = [&](int n) {
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const int64_t tok = min(n * CH + row, N - 1);
      rk[i] = *reinterpret_cast<const u32x4*>(hc.k + tok * a.k.sn + col);
      rv[i] = *reinterpret_cast<const u32x4*>(hc.v + tok * a.v.sn + col);
    }
  };
  auto stage_chunk = [&](int n) {
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const bool valid = n * CH + row < N;   // rows past the end become zeros: they add nothing
      *reinterpret_cast<u32x4*>(&sm.ta[row * R + col]) = valid ? map8<ELU1>(rk[i]) : kZero4;
      *reinterpret_cast<u32x4*>(&sm.tb[row * R + col]) = valid ? rv[i] : kZero4;
    }
  };
  if (cb < ce) load_chunk(cb);
  for (int n = cb; n < ce; ++n) {
    stage_chunk(n);
    if (n + 1 < ce) load_chunk(n + 1);
    lds_barrier();
#pragma unroll
    for (int u = 0; u < TPW; ++u) {
      const int stile = wave * TPW + u, vt = stile / MT, ft = stile % MT;
#pragma unroll
      for (int kk = 0; kk < CH / 16; ++kk)
        sacc[u] = mfma32(col_op(sm.tb + trl, R, 16 * kk, 32 * vt), col_op(sm.ta + trl, R, 16 * kk, 32 * ft), sacc[u]);
    }
    {
      const int f = tid % D, part = tid / D;
      constexpr int RPP = CH / C::ZP;
      float acc = 0.f;
#pragma unroll
      for (int r = 0; r < RPP; ++r) acc += __uint_as_float((uint32_t)sm.ta[(part * RPP + r) * R + f] << 16);
      sm.zpart[part][f] = acc;
    }
    lds_barrier();   // every read of the tiles is done; the partial column sums are visible
    if (tid < D) {
      float zz = sm.z[tid];
#pragma unroll
      for (int pz = 0; pz < C::ZP; ++pz) zz += sm.zpart[pz][tid];
      sm.z[tid] = zz;
    }
  }
  float* out = state_slot<D>(a, head_linear, 0, seg);
  store_partial<D>(out, sacc, wave, ln, lh);
  if (tid < D) out[D * D + tid] = sm.z[tid];   // written and read by the same thread
}

// ---------------------------------------------------------------------------------------
// (2) dq; B = sum fq g^T and Y = sum c fq over the segment.  grid = (H - H0, B, segments)
// ---------------------------------------------------------------------------------------
template <int D, bool ELU1>
__global__ __launch_bounds__(LbCfg<D>::NT, 1) void linear_bidir_dq_mfma_kernel(BwdArgs a) {
  using C = LbCfg<D>;
  constexpr int MT = C::MT, KS = C::KS, NW = C::NW, NT = C::NT, R = C::R, TPW = C::TPW, PCS = C::PCS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  BbSmem<D>& sm = *reinterpret_cast<BbSmem<D>*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ln = lane & 31, lh = lane >> 5;
  const int h = a.H0 + blockIdx.x, b = blockIdx.y, seg = blockIdx.z;
  const int head_linear = b * (a.H - a.H0) + blockIdx.x;
  const HeadCtx<D> hc = head_ctx<D>(a, b, h);
  uint16_t* dqp = reinterpret_cast<uint16_t*>(a.dq) + b * a.q.sb + h * a.q.sh;
  const int N = a.N, nchunks = (N + CH - 1) / CH;
  int cb, ce;
  segment_bounds(nchunks, a.lin_segments, seg, cb, ce);
  const int trl = lds_operand_tr_lane_offset(R, lane) + 8 * lh * R;
  uint16_t* fq = sm.ta;   // phi(q), later dq
  uint16_t* gt = sm.tb;   // dO, then g = dO / den

  load_total<D>(sm, a, head_linear, 0, a.lin_segments, tid);   // S (bf16 copy) and z
  f32x16 sacc[TPW];   // B^T tiles: value block vt, feature block ft
#pragma unroll
  for (int u = 0; u < TPW; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[u][r] = 0.f;
  float yacc = 0.f;   // Y[tid], tid < D

  u32x4 rq[PCS], rdo[PCS];
  auto load_chunk = [&](int n) {
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const int64_t tok = min(n * CH + row, N - 1);
      rq[i] = *reinterpret_cast<const u32x4*>(hc.q + tok * a.q.sn + col);
      rdo[i] = *reinterpret_cast<const u32x4*>(hc.dout + tok * a.dout.sn + col);
    }
  };
  auto stage_chunk = [&](int n) {
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const bool valid = n * CH + row < N;   // rows past the end: zeros (they add nothing to B, Y)
      *reinterpret_cast<u32x4*>(&fq[row * R + col]) = valid ? map8<ELU1>(rq[i]) : kZero4;
      *reinterpret_cast<u32x4*>(&gt[row * R + col]) = valid ? rdo[i] : kZero4;
    }
  };
  const int ot = wave % MT, it2 = wave / MT;   // output tile of the 64 x d products
  if (cb < ce) {
    load_chunk(cb);
    stage_chunk(cb);
    if (cb + 1 < ce) load_chunk(cb + 1);
  }
  lds_barrier();   // first chunk staged; S, z visible

  for (int n = cb; n < ce; ++n) {
    const int t0 = n * CH;
    // ---- (a) den_i = fq_i . z + eps: NW threads per token, D / NW features each ----
    {
      constexpr int FP = D / NW;
      const int i = tid / NW, part = tid % NW;
      float acc = 0.f;
#pragma unroll
      for (int c = 0; c < FP; c += 8) {
        const u32x4 f8 = *reinterpret_cast<const u32x4*>(&fq[i * R + part * FP + c]);
        const float4 z0 = *reinterpret_cast<const float4*>(&sm.z[part * FP + c]);
        const float4 z1 = *reinterpret_cast<const float4*>(&sm.z[part * FP + c + 4]);
        acc = fmaf(bf16_lo(f8[0]), z0.x, acc); acc = fmaf(bf16_hi(f8[0]), z0.y, acc);
        acc = fmaf(bf16_lo(f8[1]), z0.z, acc); acc = fmaf(bf16_hi(f8[1]), z0.w, acc);
        acc = fmaf(bf16_lo(f8[2]), z1.x, acc); acc = fmaf(bf16_hi(f8[2]), z1.y, acc);
        acc = fmaf(bf16_lo(f8[3]), z1.z, acc); acc = fmaf(bf16_hi(f8[3]), z1.w, acc);
      }
#pragma unroll
      for (int o = 1; o < NW; o <<= 1) acc += __shfl_xor(acc, o, 64);
      if (part == 0) sm.den[i] = (t0 + i < N) ? acc + a.eps : 1.f;   // rows past N: zero dO over 1
    }
    lds_barrier();
    // ---- (b) g = dO / den in place, as a bf16 pair (high half over dO, low half beside it) ----
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      u32x4* gp = reinterpret_cast<u32x4*>(&gt[row * R + col]);
      const u32x4 d8 = *gp;
      const float inv = 1.f / sm.den[row];
      u32x4 hi, lo;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float x0 = bf16_lo(d8[w]) * inv, x1 = bf16_hi(d8[w]) * inv;
        hi[w] = pack_bf16(x0, x1);
        lo[w] = pack_bf16(x0 - bf16_lo(hi[w]), x1 - bf16_hi(hi[w]));
      }
      *gp = hi;
      *reinterpret_cast<u32x4*>(&sm.tbl[row * R + col]) = lo;
    }
    lds_barrier();
    // ---- (c) r^T tile (feature block ot, token block it2) = S g^T, and its part of fq_i . r_i ----
    f32x16 racc;
#pragma unroll
    for (int r = 0; r < 16; ++r) racc[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 gop = row_op(gt, R, 32 * it2, ks, ln, lh);
      const bf16x8 sop = row_op(sm.st, R, 32 * ot, ks, ln, lh);
      racc = mfma32(sop, gop, racc);
      racc = mfma32(row_op(sm.stl, R, 32 * ot, ks, ln, lh), gop, racc);
      racc = mfma32(sop, row_op(sm.tbl, R, 32 * it2, ks, ln, lh), racc);
    }
    const int i = 32 * it2 + ln;   // this lane's token
    {
      float dot = 0.f;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        float f4[4];
        get4(&fq[i * R + 32 * ot + 8 * g4 + 4 * lh], f4);
#pragma unroll
        for (int e = 0; e < 4; ++e) dot = fmaf(f4[e], racc[4 * g4 + e], dot);
      }
      dot = sum_over_halves(dot);
      if (lh == 0) sm.pd[ot][i] = dot;
    }
    // B^T += g^T fq (reads both tiles whole: before dq replaces phi(q))
#pragma unroll
    for (int u = 0; u < TPW; ++u) {
      const int stile = wave * TPW + u, vt = stile / MT, ft = stile % MT;
#pragma unroll
      for (int kk = 0; kk < CH / 16; ++kk) {
        const bf16x8 qop = col_op(fq + trl, R, 16 * kk, 32 * ft);
        sacc[u] = mfma32(col_op(gt + trl, R, 16 * kk, 32 * vt), qop, sacc[u]);
        sacc[u] = mfma32(col_op(sm.tbl + trl, R, 16 * kk, 32 * vt), qop, sacc[u]);
      }
    }
    lds_barrier();
    // ---- (d) c_i; Y += sum_i c_i fq_i (column sums in ZP parts) ----
    if (tid < CH) {
      float dot = 0.f;
#pragma unroll
      for (int m = 0; m < MT; ++m) dot += sm.pd[m][tid];
      sm.cc[tid] = dot / sm.den[tid];
    }
    lds_barrier();
    {
      const int f = tid % D, part = tid / D;
      constexpr int RPP = CH / C::ZP;
      float acc = 0.f;
#pragma unroll
      for (int r = 0; r < RPP; ++r) {
        const int t = part * RPP + r;
        acc = fmaf(sm.cc[t], __uint_as_float((uint32_t)fq[t * R + f] << 16), acc);
      }
      sm.zpart[part][f] = acc;
    }
    lds_barrier();   // every read of phi(q) is done
    // ---- (e) dq_i = (r_i - c_i z) * phi'(q_i) replaces phi(q) in this wave's corner of the tile ----
    {
      const float ci = sm.cc[i];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int f0 = 32 * ot + 8 * g4 + 4 * lh;
        const float4 z4 = *reinterpret_cast<const float4*>(&sm.z[f0]);
        uint16_t* fp = &fq[i * R + f0];
        float fv[4];
        get4(fp, fv);
        put4(fp, (racc[4 * g4 + 0] - ci * z4.x) * slope_of<ELU1>(fv[0]),
             (racc[4 * g4 + 1] - ci * z4.y) * slope_of<ELU1>(fv[1]),
             (racc[4 * g4 + 2] - ci * z4.z) * slope_of<ELU1>(fv[2]),
             (racc[4 * g4 + 3] - ci * z4.w) * slope_of<ELU1>(fv[3]));
      }
    }
    if (tid < D) {
#pragma unroll
      for (int pz = 0; pz < C::ZP; ++pz) yacc += sm.zpart[pz][tid];
    }
    lds_barrier();
    // ---- (f) dq rows out; next chunk in (a thread overwrites the pieces it has just read) ----
#pragma unroll
    for (int x = 0; x < PCS; ++x) {
      const int p = tid + x * NT, row = p / C::C8, col = 8 * (p % C::C8);
      if (t0 + row < N)
        *reinterpret_cast<u32x4*>(dqp + (int64_t)(t0 + row) * a.q.sn + col) =
            *reinterpret_cast<const u32x4*>(&fq[row * R + col]);
    }
    if (n + 1 < ce) stage_chunk(n + 1);
    if (n + 2 < ce) load_chunk(n + 2);
    lds_barrier();
  }
  float* out = state_slot<D>(a, head_linear, 1, seg);
  store_partial<D>(out, sacc, wave, ln, lh);
  if (tid < D) out[D * D + tid] = yacc;
}

// ---------------------------------------------------------------------------------------
// (3) dk = (v B^T - 1 Y^T) * phi'(k), dv = fk B.  grid = (H - H0, B, segments)
// ---------------------------------------------------------------------------------------
template <int D, bool ELU1>
__global__ __launch_bounds__(LbCfg<D>::NT, 1) void linear_bidir_dkv_mfma_kernel(BwdArgs a) {
  using C = LbCfg<D>;
  constexpr int MT = C::MT, KS = C::KS, NT = C::NT, R = C::R, PCS = C::PCS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  BbSmem<D>& sm = *reinterpret_cast<BbSmem<D>*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ln = lane & 31, lh = lane >> 5;
  const int h = a.H0 + blockIdx.x, b = blockIdx.y, seg = blockIdx.z;
  const int head_linear = b * (a.H - a.H0) + blockIdx.x;
  const HeadCtx<D> hc = head_ctx<D>(a, b, h);
  uint16_t* dkp = reinterpret_cast<uint16_t*>(a.dk) + b * a.k.sb + h * a.k.sh;
  uint16_t* dvp = reinterpret_cast<uint16_t*>(a.dv) + b * a.v.sb + h * a.v.sh;
  const int N = a.N, nchunks = (N + CH - 1) / CH;
  int cb, ce;
  segment_bounds(nchunks, a.lin_segments, seg, cb, ce);
  const int trl = lds_operand_tr_lane_offset(R, lane) + 8 * lh * R;
  uint16_t* fk = sm.ta;   // phi(k), later dk
  uint16_t* vt_ = sm.tb;  // v, later dv

  load_total<D>(sm, a, head_linear, 1, a.lin_segments, tid);   // B (bf16 copy) and Y

  u32x4 rk[PCS], rv[PCS];
  auto load_chunk = [&](int n) {
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const int64_t tok = min(n * CH + row, N - 1);
      rk[i] = *reinterpret_cast<const u32x4*>(hc.k + tok * a.k.sn + col);
      rv[i] = *reinterpret_cast<const u32x4*>(hc.v + tok * a.v.sn + col);
    }
  };
  auto stage_chunk = [&](int n) {   // rows past the end repeat the last row: never written out
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      *reinterpret_cast<u32x4*>(&fk[row * R + col]) = map8<ELU1>(rk[i]);
      *reinterpret_cast<u32x4*>(&vt_[row * R + col]) = rv[i];
    }
  };
  const int ot = wave % MT, jt2 = wave / MT;
  if (cb < ce) {
    load_chunk(cb);
    stage_chunk(cb);
    if (cb + 1 < ce) load_chunk(cb + 1);
  }
  lds_barrier();

  for (int n = cb; n < ce; ++n) {
    const int t0 = n * CH;
    f32x16 kacc, vacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) { kacc[r] = 0.f; vacc[r] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      // dfk^T tile (feature block ot, key block jt2) = B v^T;  dv^T tile (value block ot) = B^T fk^T
      const bf16x8 vop = row_op(vt_, R, 32 * jt2, ks, ln, lh);
      kacc = mfma32(row_op(sm.st, R, 32 * ot, ks, ln, lh), vop, kacc);
      kacc = mfma32(row_op(sm.stl, R, 32 * ot, ks, ln, lh), vop, kacc);
      vacc = mfma32(col_op(sm.st + trl, R, 16 * ks, 32 * ot), row_op(fk, R, 32 * jt2, ks, ln, lh), vacc);
    }
    lds_barrier();   // every read of the phi(k) and v tiles is done
    {
      const int j = 32 * jt2 + ln;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int c0 = 32 * ot + 8 * g4 + 4 * lh;
        const float4 y4 = *reinterpret_cast<const float4*>(&sm.z[c0]);
        uint16_t* fp = &fk[j * R + c0];
        float fv[4];
        get4(fp, fv);
        put4(fp, (kacc[4 * g4 + 0] - y4.x) * slope_of<ELU1>(fv[0]), (kacc[4 * g4 + 1] - y4.y) * slope_of<ELU1>(fv[1]),
             (kacc[4 * g4 + 2] - y4.z) * slope_of<ELU1>(fv[2]), (kacc[4 * g4 + 3] - y4.w) * slope_of<ELU1>(fv[3]));
        put4(&vt_[j * R + c0], vacc[4 * g4 + 0], vacc[4 * g4 + 1], vacc[4 * g4 + 2], vacc[4 * g4 + 3]);
      }
    }
    lds_barrier();
#pragma unroll
    for (int x = 0; x < PCS; ++x) {
      const int p = tid + x * NT, row = p / C::C8, col = 8 * (p % C::C8);
      if (t0 + row < N) {
        *reinterpret_cast<u32x4*>(dkp + (int64_t)(t0 + row) * a.k.sn + col) =
            *reinterpret_cast<const u32x4*>(&fk[row * R + col]);
        *reinterpret_cast<u32x4*>(dvp + (int64_t)(t0 + row) * a.v.sn + col) =
            *reinterpret_cast<const u32x4*>(&vt_[row * R + col]);
      }
    }
    if (n + 1 < ce) stage_chunk(n + 1);
    if (n + 2 < ce) load_chunk(n + 2);
    lds_barrier();
  }
}

template <int D, bool ELU1> hipError_t launch_bidir_mfma_t(const BwdArgs& a, hipStream_t s) {
  const dim3 grid(a.H - a.H0, a.B, a.lin_segments), block(LbCfg<D>::NT);
  const int smem = (int)sizeof(BbSmem<D>);
  hipError_t e = hipSuccess;
  auto launch = [&](auto kern) {
    if (e != hipSuccess) return;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e == hipSuccess) kern<<<grid, block, smem, s>>>(a);
  };
  launch(linear_bidir_sum_mfma_kernel<D, ELU1>);
  launch(linear_bidir_dq_mfma_kernel<D, ELU1>);
  launch(linear_bidir_dkv_mfma_kernel<D, ELU1>);
  return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace

// Bidirectional linear heads [H0, H) of a bf16 call.
hipError_t launch_linear_backward_bidir_mfma(const BwdArgs& args, hipStream_t s) {
  if (args.H - args.H0 <= 0 || args.N <= 0 || args.B <= 0 || !args.ws_state) return hipSuccess;
  BwdArgs a = args;
  const int heads = (a.H - a.H0) * a.B, nchunks = (a.N + CH - 1) / CH;
  // one workgroup per head and segment; segments of at least four chunks, as many as fill the chip
  a.lin_segments = std::max(1, std::min(std::min(kMaxSeg, device_compute_units() / heads), nchunks / 4));
  const bool elu1 = a.phi == 0;
  if (a.d == 64) return elu1 ? launch_bidir_mfma_t<64, true>(a, s) : launch_bidir_mfma_t<64, false>(a, s);
  return elu1 ? launch_bidir_mfma_t<128, true>(a, s) : launch_bidir_mfma_t<128, false>(a, s);
}

}  // namespace gformer
