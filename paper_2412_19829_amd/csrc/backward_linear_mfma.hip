// Backward pass of the causal linear-attention heads on bf16 matrix cores (section II-B's ratio
// and Algorithm 1's running sums, differentiated; the formulas are stated at the top of
// backward_scalar.hip).
//
// With fq = phi(q), fk = phi(k), A_i = sum_{j<=i} fk_j v_j^T, Z_i = sum_{j<=i} fk_j,
// den_i = fq_i.Z_i + eps, g_i = dO_i / den_i, c_i = g_i.(fq_i^T A_i) / den_i:
//   dfq_i = A_i g_i - c_i Z_i,
//   dfk_j = B_j v_j - Y_j,  dv_j = B_j^T fk_j,   B_j = sum_{i>=j} fq_i g_i^T,  Y_j = sum_{i>=j} c_i fq_i.
// In chunks of 64 tokens, with S = tril(fq fk^T), T' = tril(g v^T - c 1^T) (row i, column j <= i)
// and the sums (A, Z) over earlier chunks, (B, Y) over later chunks:
//   forward scan:  num = S v + fq A,  den = rowsum(S) + fq.Z + eps,  c = rowdot(dO, num) / den^2,
//                  dfq = T' fk + g A^T - c Z^T;           then A += fk^T v, Z += colsum(fk)
//   reverse scan:  dfk = T'^T fq + v B^T - 1 Y^T,  dv = S^T g + fk B;   then B += fq^T g, Y += fq^T c
// One workgroup per (batch, head), segment and scan: with fewer heads than compute units a head
// is cut into up to four segments, and a workgroup first sums the chunks in front of (behind)
// its segment in light rounds (the update of the carried sums alone) before it scans the segment.
// Every product is a 32x32 MFMA tile job handed out
// over the waves; the chunk's tiles sit in LDS row-major with a row stride that serves both the
// row read (contraction over the feature/value index) and the transpose read (contraction over
// tokens); the carried d x d sum lives in fp32 accumulators spread over the waves, with a bf16
// copy in LDS as the operand of the next chunk's products; Z, Y, den and c stay in fp32.
// The forward scan leaves (den_i, c_i) in the workspace for the reverse scan.
#include "backward_linear_common.hpp"

namespace gformer {
namespace {

// T' is a difference of two nearly equal terms and a gradient row sums it against phi with
// signs: its rounding to one bf16 is the largest single error of these kernels.  It is therefore
// kept as a pair, bf16(T') in `tp` and bf16(T' - bf16(T')) in `tl` (16 mantissa bits), and every
// product with T' runs over both.  The forward scan does the same with S (`sm`, `sl`) for the
// numerator, and sums both halves into the denominator, because c = dO.num / den^2 enters every
// T' of its row; dv = S^T g in the reverse scan takes the one-bf16 S (its rows do not cancel).
template <int D, int RS_> struct LbSmemBase {
  using C = LbCfg<D>;
  static constexpr int RS = RS_;      // row stride of the carried sum's operand copy
  uint16_t fq[CH * C::R], fk[CH * C::R], v[CH * C::R], g[CH * C::R];
  uint16_t st[D * RS];                // bf16 copy of the carried sum, [feature][value]
  uint16_t sm[CH * SR], tp[CH * SR];  // S and T' (forward scan: [i][j]; reverse scan: [j][i])
  uint16_t tl[CH * SR];               // low half of T'
  float z[D];                         // Z (forward scan) or Y (reverse scan)
  float zpart[C::ZP][D];
  float dz[CH], den[CH], cc[CH];
};
template <int D> struct LbSmem : LbSmemBase<D, LbCfg<D>::R> {
  uint16_t sl[CH * SR];               // low half of S
  float rs[2][CH], pd[LbCfg<D>::MT][CH];
};

// the reverse scan also keeps dO itself: T' is formed as (dO.v)/den - c in fp32, exactly as the
// forward scan forms c, so that the two cancel where they must (a token that only sees itself).
// Its tiles fill the LDS of a compute unit at d = 128: the operand copy of the carried sum and
// dO (read by rows only) take the narrower row stride there.
template <int D> struct LbSmemKv : LbSmemBase<D, D + 8> {
  static constexpr int RD = D + 8;
  uint16_t dout[CH * RD];
};
static_assert(sizeof(LbSmemKv<128>) <= 160 * 1024 && sizeof(LbSmem<128>) <= 160 * 1024,
              "one workgroup's tiles must fit the LDS of a compute unit");

// ---------------------------------------------------------------------------------------
// forward scan: dq, and (den_i, c_i) into the workspace.  grid = (H - H0, B)
// ---------------------------------------------------------------------------------------
template <int D, bool ELU1>
__global__ __launch_bounds__(LbCfg<D>::NT, 1) void linear_bwd_q_mfma_kernel(BwdArgs a) {
  using C = LbCfg<D>;
  constexpr int MT = C::MT, KS = C::KS, NW = C::NW, NT = C::NT, R = C::R, TPW = C::TPW, PCS = C::PCS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  LbSmem<D>& sm = *reinterpret_cast<LbSmem<D>*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ln = lane & 31, lh = lane >> 5;
  const int h = a.H0 + blockIdx.x, b = blockIdx.y;
  const HeadCtx<D> hc = head_ctx<D>(a, b, h);
  uint16_t* dqp = reinterpret_cast<uint16_t*>(a.dq) + b * a.q.sb + h * a.q.sh;
  const int N = a.N;
  // this workgroup writes the chunks [cb, ce) of its head; the chunks in front of them are only
  // summed (light rounds: the state update alone)
  const int cb = a.lin_bounds[blockIdx.z], ce = a.lin_bounds[blockIdx.z + 1];
  if (cb >= ce) return;
  const int trl = lds_operand_tr_lane_offset(R, lane) + 8 * lh * R;

  u32x4 rq[PCS], rk[PCS], rv[PCS], rdo[PCS];
  auto load_chunk = [&](int n) {
    const bool full = n >= cb;   // uniform
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const int64_t tok = min(n * CH + row, N - 1);
      rk[i] = *reinterpret_cast<const u32x4*>(hc.k + tok * a.k.sn + col);
      rv[i] = *reinterpret_cast<const u32x4*>(hc.v + tok * a.v.sn + col);
      if (full) {
        rq[i] = *reinterpret_cast<const u32x4*>(hc.q + tok * a.q.sn + col);
        rdo[i] = *reinterpret_cast<const u32x4*>(hc.dout + tok * a.dout.sn + col);
      }
    }
  };
  // the feature map, in place in the staging registers (light rounds: only the tensor they read)
  auto map_chunk = [&](int n) {
    const bool full = n >= cb;
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      rk[i] = map8<ELU1>(rk[i]);
      if (full) rq[i] = map8<ELU1>(rq[i]);
    }
  };
  auto stage_chunk = [&](int n) {
    const bool full = n >= cb;
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const bool valid = n * CH + row < N;   // rows past the end become zeros: they contribute nothing
      *reinterpret_cast<u32x4*>(&sm.fk[row * R + col]) = valid ? rk[i] : kZero4;
      *reinterpret_cast<u32x4*>(&sm.v[row * R + col]) = valid ? rv[i] : kZero4;
      if (full) {
        *reinterpret_cast<u32x4*>(&sm.fq[row * R + col]) = valid ? rq[i] : kZero4;
        *reinterpret_cast<u32x4*>(&sm.g[row * R + col]) = valid ? rdo[i] : kZero4;   // dO until den is known
      }
    }
  };

  // carried sum A^T in accumulators: tile u of this wave is value block vt, feature block ft
  f32x16 sacc[TPW];
#pragma unroll
  for (int u = 0; u < TPW; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[u][r] = 0.f;
  for (int i = tid; i < D * R / 2; i += NT) reinterpret_cast<uint32_t*>(sm.st)[i] = 0u;
  if (tid < D) sm.z[tid] = 0.f;

  // Light rounds, two chunks at a time: the chunks in front of the segment only feed the carried
  // sums, so phi(K) and V of chunk n go to the fk / v tiles and those of chunk n + 1 to the fq / g
  // tiles (and travel in the q / dO staging registers), one barrier pair for both.
  auto load_pair = [&](int n) {
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const int64_t t0 = min(n * CH + row, N - 1), t1 = min((n + 1) * CH + row, N - 1);
      rk[i] = *reinterpret_cast<const u32x4*>(hc.k + t0 * a.k.sn + col);
      rv[i] = *reinterpret_cast<const u32x4*>(hc.v + t0 * a.v.sn + col);
      rq[i] = *reinterpret_cast<const u32x4*>(hc.k + t1 * a.k.sn + col);
      rdo[i] = *reinterpret_cast<const u32x4*>(hc.v + t1 * a.v.sn + col);
    }
  };
  int n0 = 0;   // first chunk of the round-by-round loop below
  if (cb >= 2) {
    load_pair(0);
    for (; n0 + 2 <= cb; n0 += 2) {
      // chunks in front of a segment are whole: no rows past the end here
#pragma unroll
      for (int i = 0; i < PCS; ++i) {
        const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
        *reinterpret_cast<u32x4*>(&sm.fk[row * R + col]) = map8<ELU1>(rk[i]);
        *reinterpret_cast<u32x4*>(&sm.v[row * R + col]) = rv[i];
        *reinterpret_cast<u32x4*>(&sm.fq[row * R + col]) = map8<ELU1>(rq[i]);
        *reinterpret_cast<u32x4*>(&sm.g[row * R + col]) = rdo[i];
      }
      if (n0 + 4 <= cb) load_pair(n0 + 2);
      lds_barrier();
#pragma unroll
      for (int u = 0; u < TPW; ++u) {
        const int stile = wave * TPW + u, vt = stile / MT, ft = stile % MT;
#pragma unroll
        for (int kk = 0; kk < CH / 16; ++kk) {
          sacc[u] = mfma32(col_op(sm.v + trl, R, 16 * kk, 32 * vt), col_op(sm.fk + trl, R, 16 * kk, 32 * ft), sacc[u]);
          sacc[u] = mfma32(col_op(sm.g + trl, R, 16 * kk, 32 * vt), col_op(sm.fq + trl, R, 16 * kk, 32 * ft), sacc[u]);
        }
      }
      {
        const int f = tid % D, part = tid / D;
        constexpr int RPP = CH / C::ZP;
        float acc = 0.f;
#pragma unroll
        for (int r = 0; r < RPP; ++r)
          acc += __uint_as_float((uint32_t)sm.fk[(part * RPP + r) * R + f] << 16) +
                 __uint_as_float((uint32_t)sm.fq[(part * RPP + r) * R + f] << 16);
        sm.zpart[part][f] = acc;
      }
      lds_barrier();
      if (tid < D) {
        float zz = sm.z[tid];
#pragma unroll
        for (int pz = 0; pz < C::ZP; ++pz) zz += sm.zpart[pz][tid];
        sm.z[tid] = zz;
      }
    }
    if (n0 >= cb) {   // the next round scans: it reads the operand copy of the carried sum
#pragma unroll
      for (int u = 0; u < TPW; ++u) {
        const int stile = wave * TPW + u, vt = stile / MT, ft = stile % MT;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
          put4(&sm.st[(32 * ft + ln) * R + 32 * vt + 8 * g4 + 4 * lh], sacc[u][4 * g4 + 0], sacc[u][4 * g4 + 1],
               sacc[u][4 * g4 + 2], sacc[u][4 * g4 + 3]);
      }
    }
  }

  load_chunk(n0);
  map_chunk(n0);
  stage_chunk(n0);
  if (n0 + 1 < ce) load_chunk(n0 + 1);
  lds_barrier();

  const int ti = wave & 3, jt = ti & 1, it = ti >> 1;   // 32 x 32 tile of the 64 x 64 products
  const bool do_s = NW == 4 || wave < 4, do_t = NW == 4 || wave >= 4;
  const int ot = wave % MT, it2 = wave / MT;            // output tile of the 64 x d products

  for (int n = n0; n < ce; ++n) {
    const int t0 = n * CH;
    const bool full = n >= cb;   // uniform over the workgroup
    f32x16 traw;
    if (full) {
    // ---- (a) S^T and (dO v^T)^T tiles: rows j, columns i (a lane owns one token i) ----
    if (do_s) {
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        s = mfma32(row_op(sm.fk, R, 32 * jt, ks, ln, lh), row_op(sm.fq, R, 32 * it, ks, ln, lh), s);
      const int i = 32 * it + ln;
      float rsum = 0.f;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = 32 * jt + 8 * g4 + 4 * lh + e;
          x[e] = j <= i ? s[4 * g4 + e] : 0.f;
        }
        u32x2 pk, pl;
        pk[0] = pack_bf16(x[0], x[1]);
        pk[1] = pack_bf16(x[2], x[3]);
        pl[0] = pack_bf16(x[0] - bf16_lo(pk[0]), x[1] - bf16_hi(pk[0]));
        pl[1] = pack_bf16(x[2] - bf16_lo(pk[1]), x[3] - bf16_hi(pk[1]));
        rsum = dot2_ones_bf16(pk[0], rsum);   // the row sum of the weights the numerator sees:
        rsum = dot2_ones_bf16(pk[1], rsum);   // both halves of the pair
        rsum = dot2_ones_bf16(pl[0], rsum);
        rsum = dot2_ones_bf16(pl[1], rsum);
        *reinterpret_cast<u32x2*>(&sm.sm[i * SR + 32 * jt + 8 * g4 + 4 * lh]) = pk;
        *reinterpret_cast<u32x2*>(&sm.sl[i * SR + 32 * jt + 8 * g4 + 4 * lh]) = pl;
      }
      rsum = sum_over_halves(rsum);
      if (lh == 0) sm.rs[jt][i] = rsum;
    }
    if (do_t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) traw[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        traw = mfma32(row_op(sm.v, R, 32 * jt, ks, ln, lh), row_op(sm.g, R, 32 * it, ks, ln, lh), traw);
    }
    {
      // fq_i . Z: NW threads per token, D / NW features each
      constexpr int FP = D / NW;   // 16
      const int i = tid / NW, part = tid % NW;
      float acc = 0.f;
#pragma unroll
      for (int c = 0; c < FP; c += 8) {
        const u32x4 f8 = *reinterpret_cast<const u32x4*>(&sm.fq[i * R + part * FP + c]);
        const float4 z0 = *reinterpret_cast<const float4*>(&sm.z[part * FP + c]);
        const float4 z1 = *reinterpret_cast<const float4*>(&sm.z[part * FP + c + 4]);
        acc = fmaf(bf16_lo(f8[0]), z0.x, acc); acc = fmaf(bf16_hi(f8[0]), z0.y, acc);
        acc = fmaf(bf16_lo(f8[1]), z0.z, acc); acc = fmaf(bf16_hi(f8[1]), z0.w, acc);
        acc = fmaf(bf16_lo(f8[2]), z1.x, acc); acc = fmaf(bf16_hi(f8[2]), z1.y, acc);
        acc = fmaf(bf16_lo(f8[3]), z1.z, acc); acc = fmaf(bf16_hi(f8[3]), z1.w, acc);
      }
#pragma unroll
      for (int o = 1; o < NW; o <<= 1) acc += __shfl_xor(acc, o, 64);
      if (part == 0) sm.dz[i] = acc;
    }
    lds_barrier();

    // ---- (b) num^T tile (value block ot, token block it2) and its part of dO_i . num_i ----
    {
      f32x16 nacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) nacc[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < CH / 16; ++kk) {
        const bf16x8 vop = col_op(sm.v + trl, R, 16 * kk, 32 * ot);
        nacc = mfma32(vop, row_op(sm.sm, SR, 32 * it2, kk, ln, lh), nacc);
        nacc = mfma32(vop, row_op(sm.sl, SR, 32 * it2, kk, ln, lh), nacc);
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        nacc = mfma32(col_op(sm.st + trl, R, 16 * ks, 32 * ot), row_op(sm.fq, R, 32 * it2, ks, ln, lh), nacc);
      const int i = 32 * it2 + ln;
      float dot = 0.f;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        float d4[4];
        get4(&sm.g[i * R + 32 * ot + 8 * g4 + 4 * lh], d4);
#pragma unroll
        for (int e = 0; e < 4; ++e) dot = fmaf(d4[e], nacc[4 * g4 + e], dot);
      }
      dot = sum_over_halves(dot);
      if (lh == 0) sm.pd[ot][i] = dot;
    }
    lds_barrier();

    // ---- (c) den, c; T' tile; g = dO / den in place ----
    auto den_of = [&](int i, bool valid) {
      return valid ? sm.rs[0][i] + sm.rs[1][i] + sm.dz[i] + a.eps : 1.f;
    };
    auto c_of = [&](int i, float den) {
      float dot = 0.f;
#pragma unroll
      for (int m = 0; m < MT; ++m) dot += sm.pd[m][i];
      return dot / (den * den);
    };
    if (do_t) {
      const int i = 32 * it + ln;
      const float den = den_of(i, t0 + i < N);
      const float ci = c_of(i, den);
      const float inv = 1.f / den;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = 32 * jt + 8 * g4 + 4 * lh + e;
          x[e] = j <= i ? fmaf(traw[4 * g4 + e], inv, -ci) : 0.f;
        }
        put4_split(&sm.tp[i * SR + 32 * jt + 8 * g4 + 4 * lh], &sm.tl[i * SR + 32 * jt + 8 * g4 + 4 * lh],
                   x[0], x[1], x[2], x[3]);
      }
    }
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const float den = den_of(row, t0 + row < N);
      u32x4* gp = reinterpret_cast<u32x4*>(&sm.g[row * R + col]);
      *gp = scale8(*gp, 1.f / den);
    }
    if (tid < CH) {
      const bool valid = t0 + tid < N;
      const float den = den_of(tid, valid);
      const float ci = c_of(tid, den);
      sm.cc[tid] = ci;
      if (valid) {
        float2 o;
        o.x = den;
        o.y = ci;
        *reinterpret_cast<float2*>(&hc.ws[2 * (int64_t)(t0 + tid)]) = o;
      }
    }
    lds_barrier();
    }  // full

    // ---- (d) dfq^T tile (feature block ot, token block it2), then the carried sums ----
    if (full) {
      f32x16 dacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) dacc[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < CH / 16; ++kk) {
        const bf16x8 kop = col_op(sm.fk + trl, R, 16 * kk, 32 * ot);
        dacc = mfma32(kop, row_op(sm.tp, SR, 32 * it2, kk, ln, lh), dacc);
        dacc = mfma32(kop, row_op(sm.tl, SR, 32 * it2, kk, ln, lh), dacc);
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        dacc = mfma32(row_op(sm.st, R, 32 * ot, ks, ln, lh), row_op(sm.g, R, 32 * it2, ks, ln, lh), dacc);
      const int i = 32 * it2 + ln;
      const float ci = sm.cc[i];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int f0 = 32 * ot + 8 * g4 + 4 * lh;
        const float4 z4 = *reinterpret_cast<const float4*>(&sm.z[f0]);
        uint16_t* fp = &sm.fq[i * R + f0];   // this wave's own corner of the tile: dq replaces phi(q)
        float fv[4];
        get4(fp, fv);
        put4(fp, (dacc[4 * g4 + 0] - ci * z4.x) * slope_of<ELU1>(fv[0]),
             (dacc[4 * g4 + 1] - ci * z4.y) * slope_of<ELU1>(fv[1]),
             (dacc[4 * g4 + 2] - ci * z4.z) * slope_of<ELU1>(fv[2]),
             (dacc[4 * g4 + 3] - ci * z4.w) * slope_of<ELU1>(fv[3]));
      }
    }
#pragma unroll
    for (int u = 0; u < TPW; ++u) {
      const int stile = wave * TPW + u, vt = stile / MT, ft = stile % MT;
#pragma unroll
      for (int kk = 0; kk < CH / 16; ++kk)
        sacc[u] = mfma32(col_op(sm.v + trl, R, 16 * kk, 32 * vt), col_op(sm.fk + trl, R, 16 * kk, 32 * ft), sacc[u]);
    }
    {
      const int f = tid % D, part = tid / D;
      constexpr int RPP = CH / C::ZP;
      float acc = 0.f;
#pragma unroll
      for (int r = 0; r < RPP; ++r) acc += __uint_as_float((uint32_t)sm.fk[(part * RPP + r) * R + f] << 16);
      sm.zpart[part][f] = acc;
    }
    lds_barrier();

    // ---- (e) hand the sums to the next chunk; dq rows out; next chunk in ----
    if (n + 1 >= cb) {   // light rounds do not read the operand copy
#pragma unroll
    for (int u = 0; u < TPW; ++u) {
      const int stile = wave * TPW + u, vt = stile / MT, ft = stile % MT;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4)
        put4(&sm.st[(32 * ft + ln) * R + 32 * vt + 8 * g4 + 4 * lh], sacc[u][4 * g4 + 0], sacc[u][4 * g4 + 1],
             sacc[u][4 * g4 + 2], sacc[u][4 * g4 + 3]);
    }
    }
    if (tid < D) {
      float zz = sm.z[tid];
#pragma unroll
      for (int pz = 0; pz < C::ZP; ++pz) zz += sm.zpart[pz][tid];
      sm.z[tid] = zz;
    }
    if (full) {
#pragma unroll
      for (int i = 0; i < PCS; ++i) {
        const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
        if (t0 + row < N)
          *reinterpret_cast<u32x4*>(dqp + (int64_t)(t0 + row) * a.q.sn + col) =
              *reinterpret_cast<const u32x4*>(&sm.fq[row * R + col]);
      }
    }
    if (n + 1 < ce) {
      map_chunk(n + 1);
      stage_chunk(n + 1);   // the same thread overwrites the pieces it has just read
    }
    if (n + 2 < ce) load_chunk(n + 2);
      lds_barrier();
  }
}

// ---------------------------------------------------------------------------------------
// reverse scan: dk, dv from (den_i, c_i) of the workspace.  grid = (H - H0, B)
// ---------------------------------------------------------------------------------------
template <int D, bool ELU1>
__global__ __launch_bounds__(LbCfg<D>::NT, 1) void linear_bwd_kv_mfma_kernel(BwdArgs a) {
  using C = LbCfg<D>;
  constexpr int MT = C::MT, KS = C::KS, NW = C::NW, NT = C::NT, R = C::R, TPW = C::TPW, PCS = C::PCS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  LbSmemKv<D>& sm = *reinterpret_cast<LbSmemKv<D>*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ln = lane & 31, lh = lane >> 5;
  const int h = a.H0 + blockIdx.x, b = blockIdx.y;
  const HeadCtx<D> hc = head_ctx<D>(a, b, h);
  uint16_t* dkp = reinterpret_cast<uint16_t*>(a.dk) + b * a.k.sb + h * a.k.sh;
  uint16_t* dvp = reinterpret_cast<uint16_t*>(a.dv) + b * a.v.sb + h * a.v.sh;
  const int N = a.N, nchunks = (N + CH - 1) / CH;
  // this workgroup writes the chunks [cb, ce) of its head; the chunks behind them are only summed
  const int cb = nchunks - a.lin_bounds[blockIdx.z + 1], ce = nchunks - a.lin_bounds[blockIdx.z];
  if (cb >= ce) return;
  const int trl = lds_operand_tr_lane_offset(R, lane) + 8 * lh * R;
  constexpr int RS = LbSmemKv<D>::RS, RD = LbSmemKv<D>::RD;   // strides of the carried-sum copy and of dO
  const int trl_s = lds_operand_tr_lane_offset(RS, lane) + 8 * lh * RS;

  u32x4 rq[PCS], rk[PCS], rv[PCS], rdo[PCS];
  float rden[PCS];
  float2 rstat = {1.f, 0.f};
  auto load_chunk = [&](int n) {
    const bool full = n < ce;   // uniform
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const int64_t tok = min(n * CH + row, N - 1);
      rq[i] = *reinterpret_cast<const u32x4*>(hc.q + tok * a.q.sn + col);
      rdo[i] = *reinterpret_cast<const u32x4*>(hc.dout + tok * a.dout.sn + col);
      rden[i] = hc.ws[2 * tok];
      if (full) {
        rk[i] = *reinterpret_cast<const u32x4*>(hc.k + tok * a.k.sn + col);
        rv[i] = *reinterpret_cast<const u32x4*>(hc.v + tok * a.v.sn + col);
      }
    }
    if (tid < CH) rstat = *reinterpret_cast<const float2*>(&hc.ws[2 * (int64_t)min(n * CH + tid, N - 1)]);
  };
  auto map_chunk = [&](int n) {
    const bool full = n < ce;
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      rq[i] = map8<ELU1>(rq[i]);
      if (full) rk[i] = map8<ELU1>(rk[i]);
    }
  };
  auto stage_chunk = [&](int n) {
    const bool full = n < ce;
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const bool valid = n * CH + row < N;
      *reinterpret_cast<u32x4*>(&sm.fq[row * R + col]) = valid ? rq[i] : kZero4;
      *reinterpret_cast<u32x4*>(&sm.g[row * R + col]) = valid ? scale8(rdo[i], 1.f / rden[i]) : kZero4;
      if (full) {
        *reinterpret_cast<u32x4*>(&sm.fk[row * R + col]) = valid ? rk[i] : kZero4;
        *reinterpret_cast<u32x4*>(&sm.v[row * R + col]) = valid ? rv[i] : kZero4;
        *reinterpret_cast<u32x4*>(&sm.dout[row * RD + col]) = valid ? rdo[i] : kZero4;
      }
    }
    if (tid < CH) {
      const bool valid = n * CH + tid < N;
      sm.cc[tid] = valid ? rstat.y : 0.f;
      sm.den[tid] = valid ? 1.f / rstat.x : 1.f;   // the reciprocal
    }
  };

  f32x16 sacc[TPW];   // B^T tiles: value block vt, feature block ft
#pragma unroll
  for (int u = 0; u < TPW; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[u][r] = 0.f;
  for (int i = tid; i < D * RS / 2; i += NT) reinterpret_cast<uint32_t*>(sm.st)[i] = 0u;
  if (tid < D) sm.z[tid] = 0.f;

  // Light rounds, two chunks at a time (the chunks behind the segment only feed the carried
  // sums): phi(q), g and c of chunk n go to the fq / g tiles and cc, those of chunk n - 1 to the
  // fk / v tiles and dz (and travel in the k / v staging registers).
  float rden2[PCS];
  float2 rstat2 = {1.f, 0.f};
  auto load_pair = [&](int n) {
#pragma unroll
    for (int i = 0; i < PCS; ++i) {
      const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
      const int64_t t0 = min(n * CH + row, N - 1), t1 = (n - 1) * CH + row;
      rq[i] = *reinterpret_cast<const u32x4*>(hc.q + t0 * a.q.sn + col);
      rdo[i] = *reinterpret_cast<const u32x4*>(hc.dout + t0 * a.dout.sn + col);
      rden[i] = hc.ws[2 * t0];
      rk[i] = *reinterpret_cast<const u32x4*>(hc.q + t1 * a.q.sn + col);
      rv[i] = *reinterpret_cast<const u32x4*>(hc.dout + t1 * a.dout.sn + col);
      rden2[i] = hc.ws[2 * t1];
    }
    if (tid < CH) {
      rstat = *reinterpret_cast<const float2*>(&hc.ws[2 * (int64_t)min(n * CH + tid, N - 1)]);
      rstat2 = *reinterpret_cast<const float2*>(&hc.ws[2 * (int64_t)((n - 1) * CH + tid)]);
    }
  };
  int n1 = nchunks - 1;   // first chunk of the round-by-round loop below
  if (nchunks - ce >= 2) {
    load_pair(n1);
    for (; n1 - 1 >= ce; n1 -= 2) {
#pragma unroll
      for (int i = 0; i < PCS; ++i) {
        const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
        const bool valid = n1 * CH + row < N;   // only the head's last chunk can be ragged
        *reinterpret_cast<u32x4*>(&sm.fq[row * R + col]) = valid ? map8<ELU1>(rq[i]) : kZero4;
        *reinterpret_cast<u32x4*>(&sm.g[row * R + col]) = valid ? scale8(rdo[i], 1.f / rden[i]) : kZero4;
        *reinterpret_cast<u32x4*>(&sm.fk[row * R + col]) = map8<ELU1>(rk[i]);
        *reinterpret_cast<u32x4*>(&sm.v[row * R + col]) = scale8(rv[i], 1.f / rden2[i]);
      }
      if (tid < CH) {
        sm.cc[tid] = (n1 * CH + tid < N) ? rstat.y : 0.f;
        sm.dz[tid] = rstat2.y;
      }
      if (n1 - 3 >= ce) load_pair(n1 - 2);
      lds_barrier();
#pragma unroll
      for (int u = 0; u < TPW; ++u) {
        const int stile = wave * TPW + u, vt = stile / MT, ft = stile % MT;
#pragma unroll
        for (int kk = 0; kk < CH / 16; ++kk) {
          sacc[u] = mfma32(col_op(sm.g + trl, R, 16 * kk, 32 * vt), col_op(sm.fq + trl, R, 16 * kk, 32 * ft), sacc[u]);
          sacc[u] = mfma32(col_op(sm.v + trl, R, 16 * kk, 32 * vt), col_op(sm.fk + trl, R, 16 * kk, 32 * ft), sacc[u]);
        }
      }
      {
        const int f = tid % D, part = tid / D;
        constexpr int RPP = CH / C::ZP;
        float acc = 0.f;
#pragma unroll
        for (int r = 0; r < RPP; ++r) {
          const int i = part * RPP + r;
          acc = fmaf(sm.cc[i], __uint_as_float((uint32_t)sm.fq[i * R + f] << 16), acc);
          acc = fmaf(sm.dz[i], __uint_as_float((uint32_t)sm.fk[i * R + f] << 16), acc);
        }
        sm.zpart[part][f] = acc;
      }
      lds_barrier();
      if (tid < D) {
        float yy = sm.z[tid];
#pragma unroll
        for (int pz = 0; pz < C::ZP; ++pz) yy += sm.zpart[pz][tid];
        sm.z[tid] = yy;
      }
    }
    if (n1 < ce) {   // the next round scans: it reads the operand copy of the carried sum
#pragma unroll
      for (int u = 0; u < TPW; ++u) {
        const int stile = wave * TPW + u, vt = stile / MT, ft = stile % MT;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
          put4(&sm.st[(32 * ft + ln) * RS + 32 * vt + 8 * g4 + 4 * lh], sacc[u][4 * g4 + 0], sacc[u][4 * g4 + 1],
               sacc[u][4 * g4 + 2], sacc[u][4 * g4 + 3]);
      }
    }
  }

  load_chunk(n1);
  map_chunk(n1);
  stage_chunk(n1);
  if (n1 - 1 >= cb) load_chunk(n1 - 1);
  lds_barrier();

  const int ti = wave & 3, it = ti & 1, jt = ti >> 1;   // here rows are i, columns j (a lane owns a key j)
  const bool do_s = NW == 4 || wave < 4, do_t = NW == 4 || wave >= 4;
  const int ot = wave % MT, jt2 = wave / MT;

  for (int n = n1; n >= cb; --n) {
    const int t0 = n * CH;
    const bool full = n < ce;   // uniform over the workgroup
    // ---- (a) S and T' tiles, stored transposed ([j][i]); column sums for Y ----
    if (full && do_s) {
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        s = mfma32(row_op(sm.fq, R, 32 * it, ks, ln, lh), row_op(sm.fk, R, 32 * jt, ks, ln, lh), s);
      const int j = 32 * jt + ln;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 32 * it + 8 * g4 + 4 * lh + e;
          x[e] = j <= i ? s[4 * g4 + e] : 0.f;
        }
        put4(&sm.sm[j * SR + 32 * it + 8 * g4 + 4 * lh], x[0], x[1], x[2], x[3]);
      }
    }
    if (full && do_t) {
      f32x16 tr;
#pragma unroll
      for (int r = 0; r < 16; ++r) tr[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        tr = mfma32(row_op(sm.dout, RD, 32 * it, ks, ln, lh), row_op(sm.v, R, 32 * jt, ks, ln, lh), tr);
      const int j = 32 * jt + ln;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const float4 c4 = *reinterpret_cast<const float4*>(&sm.cc[32 * it + 8 * g4 + 4 * lh]);
        const float4 r4 = *reinterpret_cast<const float4*>(&sm.den[32 * it + 8 * g4 + 4 * lh]);
        const float cv[4] = {c4.x, c4.y, c4.z, c4.w}, rv4[4] = {r4.x, r4.y, r4.z, r4.w};
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 32 * it + 8 * g4 + 4 * lh + e;
          x[e] = j <= i ? fmaf(tr[4 * g4 + e], rv4[e], -cv[e]) : 0.f;
        }
        put4_split(&sm.tp[j * SR + 32 * it + 8 * g4 + 4 * lh], &sm.tl[j * SR + 32 * it + 8 * g4 + 4 * lh],
                   x[0], x[1], x[2], x[3]);
      }
    }
    {
      const int f = tid % D, part = tid / D;
      constexpr int RPP = CH / C::ZP;
      float acc = 0.f;
#pragma unroll
      for (int r = 0; r < RPP; ++r) {
        const int i = part * RPP + r;
        acc = fmaf(sm.cc[i], __uint_as_float((uint32_t)sm.fq[i * R + f] << 16), acc);
      }
      sm.zpart[part][f] = acc;
    }
    lds_barrier();

    // ---- (b) dfk^T tile (feature block ot, key block jt2), dv^T tile (value block ot), B^T ----
    f32x16 kacc, vacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) { kacc[r] = 0.f; vacc[r] = 0.f; }
    if (full) {
#pragma unroll
    for (int kk = 0; kk < CH / 16; ++kk) {
      const bf16x8 qop = col_op(sm.fq + trl, R, 16 * kk, 32 * ot);
      kacc = mfma32(qop, row_op(sm.tp, SR, 32 * jt2, kk, ln, lh), kacc);
      kacc = mfma32(qop, row_op(sm.tl, SR, 32 * jt2, kk, ln, lh), kacc);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      kacc = mfma32(row_op(sm.st, RS, 32 * ot, ks, ln, lh), row_op(sm.v, R, 32 * jt2, ks, ln, lh), kacc);
#pragma unroll
    for (int kk = 0; kk < CH / 16; ++kk)
      vacc = mfma32(col_op(sm.g + trl, R, 16 * kk, 32 * ot), row_op(sm.sm, SR, 32 * jt2, kk, ln, lh), vacc);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      vacc = mfma32(col_op(sm.st + trl_s, RS, 16 * ks, 32 * ot), row_op(sm.fk, R, 32 * jt2, ks, ln, lh), vacc);
    }  // full
#pragma unroll
    for (int u = 0; u < TPW; ++u) {
      const int stile = wave * TPW + u, vt = stile / MT, ft = stile % MT;
#pragma unroll
      for (int kk = 0; kk < CH / 16; ++kk)
        sacc[u] = mfma32(col_op(sm.g + trl, R, 16 * kk, 32 * vt), col_op(sm.fq + trl, R, 16 * kk, 32 * ft), sacc[u]);
    }
    lds_barrier();   // every read of the phi(k) and v tiles is done

    // ---- (c) dk replaces phi(k), dv replaces v ----
    if (full) {
      const int j = 32 * jt2 + ln;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int c0 = 32 * ot + 8 * g4 + 4 * lh;
        const float4 y4 = *reinterpret_cast<const float4*>(&sm.z[c0]);
        uint16_t* fp = &sm.fk[j * R + c0];
        float fv[4];
        get4(fp, fv);
        put4(fp, (kacc[4 * g4 + 0] - y4.x) * slope_of<ELU1>(fv[0]), (kacc[4 * g4 + 1] - y4.y) * slope_of<ELU1>(fv[1]),
             (kacc[4 * g4 + 2] - y4.z) * slope_of<ELU1>(fv[2]), (kacc[4 * g4 + 3] - y4.w) * slope_of<ELU1>(fv[3]));
        put4(&sm.v[j * R + c0], vacc[4 * g4 + 0], vacc[4 * g4 + 1], vacc[4 * g4 + 2], vacc[4 * g4 + 3]);
      }
    }
    lds_barrier();

    // ---- (d) hand the sums on; dk, dv rows out; next (earlier) chunk in ----
    if (n - 1 < ce) {   // light rounds do not read the operand copy
#pragma unroll
    for (int u = 0; u < TPW; ++u) {
      const int stile = wave * TPW + u, vt = stile / MT, ft = stile % MT;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4)
        put4(&sm.st[(32 * ft + ln) * RS + 32 * vt + 8 * g4 + 4 * lh], sacc[u][4 * g4 + 0], sacc[u][4 * g4 + 1],
             sacc[u][4 * g4 + 2], sacc[u][4 * g4 + 3]);
    }
    }
    if (tid < D) {
      float yy = sm.z[tid];
#pragma unroll
      for (int pz = 0; pz < C::ZP; ++pz) yy += sm.zpart[pz][tid];
      sm.z[tid] = yy;
    }
    if (full) {
#pragma unroll
      for (int i = 0; i < PCS; ++i) {
        const int p = tid + i * NT, row = p / C::C8, col = 8 * (p % C::C8);
        if (t0 + row < N) {
          *reinterpret_cast<u32x4*>(dkp + (int64_t)(t0 + row) * a.k.sn + col) =
              *reinterpret_cast<const u32x4*>(&sm.fk[row * R + col]);
          *reinterpret_cast<u32x4*>(dvp + (int64_t)(t0 + row) * a.v.sn + col) =
              *reinterpret_cast<const u32x4*>(&sm.v[row * R + col]);
        }
      }
    }
    if (n - 1 >= cb) {
      map_chunk(n - 1);
      stage_chunk(n - 1);
    }
    if (n - 2 >= cb) load_chunk(n - 2);
      lds_barrier();
  }
}

template <int D, bool ELU1> hipError_t launch_lin_bwd_t(const BwdArgs& a, hipStream_t s) {
  const dim3 grid(a.H - a.H0, a.B, a.lin_segments), block(LbCfg<D>::NT);
  const int smem = (int)sizeof(LbSmem<D>), smem_kv = (int)sizeof(LbSmemKv<D>);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_bwd_q_mfma_kernel<D, ELU1>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_bwd_kv_mfma_kernel<D, ELU1>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, smem_kv);
  if (e != hipSuccess) return e;
  linear_bwd_q_mfma_kernel<D, ELU1><<<grid, block, smem, s>>>(a);
  linear_bwd_kv_mfma_kernel<D, ELU1><<<grid, block, smem_kv, s>>>(a);
  return hipGetLastError();
}

}  // namespace

// Linear heads [H0, H) of a bf16 call; the workspace receives (den_i, c_i) per token.
hipError_t launch_linear_backward_mfma(const BwdArgs& args, hipStream_t s) {
  if (args.H - args.H0 <= 0 || args.N <= 0 || args.B <= 0) return hipSuccess;
  // A head is one sequential scan.  With fewer heads than compute units each head is cut into
  // segments, one workgroup per segment: it first sums the chunks in front of (behind) its
  // segment in light rounds, then scans the segment.
  BwdArgs a = args;
  const int heads = (a.H - a.H0) * a.B, nchunks = (a.N + CH - 1) / CH;
  a.lin_segments = std::max(1, std::min(std::min(4, device_compute_units() / heads), nchunks / 4));
  // A chunk of a light round costs about a quarter of a chunk of a full round (measured: the
  // step is flat between 0.7 and 0.8 below), and segment s runs the light rounds of everything in
  // front of it: lengths in the ratio 0.75^s finish together.  The reverse scan uses the same cut
  // mirrored.
  {
    double wsum = 0.0, w = 1.0;
    for (int sgm = 0; sgm < a.lin_segments; ++sgm, w *= 0.75) wsum += w;
    double acc = 0.0;
    w = 1.0;
    a.lin_bounds[0] = 0;
    for (int sgm = 1; sgm <= a.lin_segments; ++sgm, w *= 0.75) {
      acc += w;
      a.lin_bounds[sgm] = sgm == a.lin_segments ? nchunks : std::min(nchunks, (int)(nchunks * acc / wsum + 0.5));
    }
  }
  const bool elu1 = a.phi == 0;
  if (a.d == 64) return elu1 ? launch_lin_bwd_t<64, true>(a, s) : launch_lin_bwd_t<64, false>(a, s);
  return elu1 ? launch_lin_bwd_t<128, true>(a, s) : launch_lin_bwd_t<128, false>(a, s);
}

}  // namespace gformer
