// Backward pass of the windowed softmax heads on bf16 matrix cores (section III-B, Eq. 1,
// differentiated; the formulas are stated at the top of backward_scalar.hip).
//
// With s_ij = scale q_i.k_j, p_ij the softmax over the causal window, dp_ij = dO_i.v_j,
// D_i = sum_j p_ij dp_ij and ds_ij = p_ij (dp_ij - D_i):
//   dq_i = scale sum_j ds_ij k_j,   dk_j = scale sum_i ds_ij q_i,   dv_j = sum_i p_ij dO_i.
//
// Every one of these is a band product like the forward pass: 32 "resident" rows per wave (their
// operands stay in registers) against the band of "streamed" rows they interact with, walked in
// tiles of 64 rows that pass through LDS.  One kernel template, four passes:
//   kStats  resident queries (q, dO), streamed keys (K, V): log-sum-exp and D_i of every query,
//           left in the workspace;
//   kDq     the same band again: ds from the stored statistics, dq^T += K^T ds^T;
//   kDv     resident keys (k), streamed queries (Q, dO): dv^T += dO^T p;
//   kDk     resident keys (k, v), streamed queries (Q, dO): dk^T += Q^T ds.
// Scores are computed with the streamed rows as MFMA rows and the resident rows as columns, so a
// lane owns one resident row; the weights then feed the output product straight from the score
// registers (the k-index permutation of an accumulator tile used as an operand is matched by the
// order in which the transposed LDS read delivers the streamed tile).
//
// Arithmetic: bf16 products with fp32 accumulation; the softmax statistics, D_i and ds in fp32;
// p and ds are rounded to bf16 as operands of the output product.  Nothing of the forward result
// is an input.
#include "common.hpp"
#include "mfma.hpp"

namespace gformer {
namespace {

constexpr int BR = 128;              // resident rows per workgroup (4 waves of 32)
constexpr int BC = 64;               // streamed rows per tile
constexpr int WR = 32;               // resident rows per wave
constexpr int NT = 256;
constexpr float kLog2e = 1.4426950408889634f;

enum BandPass { kStats = 0, kDq = 1, kDv = 2, kDk = 3 };

// Row stride of a streamed tile that is read both by rows (128-bit reads, 16 consecutive rows
// must start 4 dwords apart mod 64) and through the transpose read (4 consecutive rows must
// start at least 8 dwords apart mod 64): 12 dwords mod 64 at d = 128, 36 at d = 64.
template <int D> struct BandTiles {
  static constexpr int ROW = D == 128 ? D + 24 : D + 8;
  uint16_t x[BC * ROW];   // K (query-resident passes) or Q (key-resident passes)
  uint16_t y[BC * ROW];   // V or dO
  float lse[BC];          // statistics of the streamed queries (key-resident passes)
  float dd[BC];
};
template <int D> struct BandSmem {
  BandTiles<D> buf[2];
};

template <int D, int PASS>
__global__ __launch_bounds__(NT, 2) void windowed_bwd_band_kernel(BwdArgs a) {
  constexpr int KS = D / 16;
  constexpr int MT = D / 32;
  constexpr int KCH = BC * D / 8 / NT;
  constexpr bool RES_Q = PASS == kStats || PASS == kDq;   // resident rows are queries
  constexpr bool HAS_DP = PASS != kDv;
  using Smem = BandSmem<D>;
  using Tiles = BandTiles<D>;
  constexpr int ROW = Tiles::ROW;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int ln = lane & 31;
  const int lh = lane >> 5;
  // the same block order as the forward kernel: each XCD (own L2) gets a contiguous run of
  // resident blocks, neighbours share most of their band
  const int nrb = (a.N + BR - 1) / BR;
  const int total = nrb * a.H0 * a.B;
  constexpr int kXcds = 8;
  int lb = blockIdx.x;
  {
    const int per = total / kXcds, rem = total % kXcds;
    const int xcd = lb % kXcds, slot = lb / kXcds;
    lb = xcd * per + min(xcd, rem) + slot;
  }
  const int rb = lb % nrb;
  const int h = (lb / nrb) % a.H0, b = lb / (nrb * a.H0);
  const int i0 = rb * BR;
  const int r0 = i0 + wave * WR;
  const int N = a.N, wl = a.wleft, wr = a.wright;

  auto head = [&](const TensorView& t) {
    return reinterpret_cast<const uint16_t*>(t.base) + b * t.sb + h * t.sh;
  };
  const TensorView& res1_t = RES_Q ? a.q : a.k;
  const TensorView& res2_t = RES_Q ? a.dout : a.v;
  const TensorView& str1_t = RES_Q ? a.k : a.q;
  const TensorView& str2_t = RES_Q ? a.v : a.dout;
  const uint16_t* res1 = head(res1_t);
  const uint16_t* res2 = head(res2_t);
  const uint16_t* xp = head(str1_t);
  const uint16_t* yp = head(str2_t);
  float* ws = a.ws + ((int64_t)b * a.H + h) * N * 2;

  // resident operands (B operands of the score products); rows past N re-read row N-1
  const int ri = r0 + ln;
  const int ric = min(ri, N - 1);
  bf16x8 reg1[KS], reg2[HAS_DP ? KS : 1];
  {
    const uint16_t* p1 = res1 + (int64_t)ric * res1_t.sn + 8 * lh;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      reg1[ks] = as_bf16x8(*reinterpret_cast<const u32x4*>(p1 + 16 * ks));
    if (HAS_DP) {
      const uint16_t* p2 = res2 + (int64_t)ric * res2_t.sn + 8 * lh;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        reg2[ks] = as_bf16x8(*reinterpret_cast<const u32x4*>(p2 + 16 * ks));
    }
  }
  // statistics of the resident query (kDq)
  float lse_q = 0.f, dd_q = 0.f;
  if (PASS == kDq) {
    lse_q = ws[2 * (int64_t)ric];
    dd_q = ws[2 * (int64_t)ric + 1];
  }
  __builtin_amdgcn_sched_barrier(0);   // keep these loads in front of the tile loads (in-order return)

  // streamed rows this lane's resident row interacts with: [lo, hi]
  //   resident query i: keys i - wl .. min(i + wr, N - 1) (causal: wr = 0);
  //   resident key j: the queries that see it, j - wr .. min(j + wl, N - 1)
  const int back = RES_Q ? wl : wr, ahead = RES_Q ? wr : wl;
  const int lo = ri - back;
  const int hi = min(ri + ahead, N - 1);
  const int span = max(hi - lo + 1, 0);          // rows past N: whatever they gather is never stored
  // over the wave: union [ulo, uhi], intersection [ilo, ihi] of the lanes' intervals
  const int ulo = r0 - back, uhi = r0 + WR - 1 + ahead;
  const int ilo = r0 + WR - 1 - back, ihi = r0 + ahead;
  const int tfirst = max(0, i0 - back) / BC;
  const int tlast = min(N - 1, i0 + BR - 1 + ahead) / BC;
  const float sc = (a.scale == 0.f ? 1e-30f : a.scale) * kLog2e;

  // global -> register -> LDS staging of a tile, as in the forward kernel
  constexpr int C8 = D / 8, RP = NT / C8;
  static_assert(KCH * RP == BC, "tile rows must be covered exactly");
  const int prow = tid / C8, pcol = 8 * (tid % C8);
  const int xsn = (int)str1_t.sn, ysn = (int)str2_t.sn;
  const uint32_t colb = 2u * (uint32_t)pcol;
  const uint32_t xoff = 2u * (uint32_t)(prow * xsn) + colb, yoff = 2u * (uint32_t)(prow * ysn) + colb;
  u32x4 xst[KCH], yst[KCH];
  float st_lse = 0.f, st_dd = 0.f;
  auto load_tile = [&](int t) {
    const int t0 = t * BC;
    const int last = min(N - 1 - t0, BC - 1);
    const char* xbase = reinterpret_cast<const char*>(xp + (int64_t)t0 * xsn);
    const char* ybase = reinterpret_cast<const char*>(yp + (int64_t)t0 * ysn);
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int first = min(i * RP, last);
      const uint32_t xlim = 2u * (uint32_t)((last - first) * xsn) + colb;
      const uint32_t ylim = 2u * (uint32_t)((last - first) * ysn) + colb;
      xst[i] = *reinterpret_cast<const u32x4*>(xbase + 2u * (uint32_t)(first * xsn) + (size_t)min(xoff, xlim));
      yst[i] = *reinterpret_cast<const u32x4*>(ybase + 2u * (uint32_t)(first * ysn) + (size_t)min(yoff, ylim));
    }
    if (!RES_Q && tid < BC) {
      const int row = t0 + min(tid, last);
      st_lse = ws[2 * (int64_t)row];
      st_dd = ws[2 * (int64_t)row + 1];
    }
  };
  auto store_tile = [&](Tiles& bt) {
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      *reinterpret_cast<u32x4*>(&bt.x[(prow + i * RP) * ROW + pcol]) = xst[i];
      *reinterpret_cast<u32x4*>(&bt.y[(prow + i * RP) * ROW + pcol]) = yst[i];
    }
    if (!RES_Q && tid < BC) {
      bt.lse[tid] = st_lse;
      bt.dd[tid] = st_dd;
    }
  };

  f32x16 acc[PASS == kStats ? 1 : MT];
  if (PASS != kStats) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
  }
  float m_run = -INFINITY, l_run = 0.f, d_run = 0.f;   // kStats
  const int trlane = lds_operand_tr_lane_offset(ROW, lane) + 4 * lh * ROW;

  load_tile(tfirst);
  store_tile(sm.buf[0]);
  if (tfirst < tlast) load_tile(tfirst + 1);
  lds_barrier();
  for (int t = tfirst; t <= tlast; ++t) {
    const Tiles& cur = sm.buf[(t - tfirst) & 1];
    if (t < tlast) store_tile(sm.buf[(t - tfirst + 1) & 1]);
    if (t + 1 < tlast) load_tile(t + 2);
    const int t0 = t * BC;
    if (!(t0 > uhi || t0 + BC - 1 < ulo)) {
      const bool need_mask = !(t0 >= ilo && t0 + BC - 1 <= ihi && t0 + BC <= N);
      const int rel = t0 + 4 * lh - lo;    // streamed row of register c, minus lo, is rel + c

#pragma unroll
      for (int half = 0; half < 2; ++half) {
        // scores: streamed rows 32*half .. +31 of the tile against the resident rows
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; if (HAS_DP) dp[r] = 0.f; }
        {
          const uint16_t* xrow = &cur.x[(32 * half + ln) * ROW + 8 * lh];
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) s = mfma32(lds_read16(xrow + 16 * ks), reg1[ks], s);
          if (HAS_DP) {
            const uint16_t* yrow = &cur.y[(32 * half + ln) * ROW + 8 * lh];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) dp = mfma32(lds_read16(yrow + 16 * ks), reg2[ks], dp);
          }
        }
        // base-2 logits, masked rows at -inf
        float x[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = 32 * half + 8 * (r / 4) + (r % 4);
          const bool vis = !need_mask || (unsigned)(rel + c) < (unsigned)span;
          x[r] = vis ? s[r] * sc : -INFINITY;
        }
        if (PASS == kStats) {
          float mloc = -INFINITY;
#pragma unroll
          for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, x[r]);
          mloc = max_over_halves(mloc);
          const float m_new = fmaxf(m_run, mloc);
          const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
          const float alpha = __builtin_amdgcn_exp2f(m_run - m_ref);   // 0 on the first visible rows
          m_run = m_new;
          float lsum = 0.f, dsum = 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(x[r] - m_ref);
            lsum += p;
            dsum = fmaf(p, dp[r], dsum);
          }
          l_run = fmaf(l_run, alpha, lsum);
          d_run = fmaf(d_run, alpha, dsum);
        } else {
          // weights of the output product, packed bf16 in accumulator-register order
          uint32_t wb[8];
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            // statistics of the four streamed queries this group of registers belongs to
            float lse4[4] = {lse_q, lse_q, lse_q, lse_q}, dd4[4] = {dd_q, dd_q, dd_q, dd_q};
            if (!RES_Q) {
              const float4 l4 = *reinterpret_cast<const float4*>(&cur.lse[32 * half + 8 * g + 4 * lh]);
              lse4[0] = l4.x; lse4[1] = l4.y; lse4[2] = l4.z; lse4[3] = l4.w;
              if (HAS_DP) {
                const float4 d4 = *reinterpret_cast<const float4*>(&cur.dd[32 * half + 8 * g + 4 * lh]);
                dd4[0] = d4.x; dd4[1] = d4.y; dd4[2] = d4.z; dd4[3] = d4.w;
              }
            }
            float wv[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float p = __builtin_amdgcn_exp2f(x[4 * g + e] - lse4[e]);
              wv[e] = HAS_DP ? p * (dp[4 * g + e] - dd4[e]) : p;
            }
            wb[2 * g] = pack_bf16(wv[0], wv[1]);
            wb[2 * g + 1] = pack_bf16(wv[2], wv[3]);
          }
          // acc^T[column, resident row] += Y^T[column, streamed row] * weight[streamed row, resident row]
          const uint16_t* ytile = (PASS == kDv) ? cur.y : cur.x;
#pragma unroll
          for (int kb = 0; kb < 2; ++kb) {
            u32x4 pw;
            pw[0] = wb[4 * kb + 0]; pw[1] = wb[4 * kb + 1];
            pw[2] = wb[4 * kb + 2]; pw[3] = wb[4 * kb + 3];
            const bf16x8 wop = as_bf16x8(pw);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
              const int rr = 32 * half + 16 * kb;
              const bf16x8 ya = lds_operand_tr_at(ytile + trlane, ROW, rr, rr + 8, 32 * mt);
              acc[mt] = mfma32(ya, wop, acc[mt]);
            }
          }
        }
      }
    }
    lds_barrier();
  }

  if (PASS == kStats) {
    // both halves of the wave hold the same reference m_run; the sums are over disjoint rows
    const float l_tot = sum_over_halves(l_run);
    const float d_tot = sum_over_halves(d_run);
    if (lh == 0 && ri < N) {
      const float m_ref = (m_run == -INFINITY) ? 0.f : m_run;
      float2 o;
      o.x = m_ref + __builtin_amdgcn_logf(l_tot);   // log2
      o.y = d_tot / l_tot;
      *reinterpret_cast<float2*>(&ws[2 * (int64_t)ri]) = o;
    }
    return;
  }

  // rows leave through LDS as whole rows (the tiles are dead after the loop's last barrier)
  const float f = (PASS == kDv) ? 1.f : a.scale;
  constexpr int OROW = D + 8;
  static_assert(BR * OROW * 2 <= (int)sizeof(Smem), "output staging must fit in the tile memory");
  uint16_t* ot = reinterpret_cast<uint16_t*>(&sm);
  {
    uint16_t* orow = ot + (WR * wave + ln) * OROW + 4 * lh;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(acc[mt][4 * g + 0] * f, acc[mt][4 * g + 1] * f);
        pk[1] = pack_bf16(acc[mt][4 * g + 2] * f, acc[mt][4 * g + 3] * f);
        *reinterpret_cast<u32x2*>(orow + 32 * mt + 8 * g) = pk;
      }
    }
  }
  lds_barrier();
  const TensorView& like = PASS == kDq ? a.q : (PASS == kDk ? a.k : a.v);
  uint16_t* outp = reinterpret_cast<uint16_t*>(PASS == kDq ? a.dq : (PASS == kDk ? a.dk : a.dv)) +
                   b * like.sb + h * like.sh;
  constexpr int OPIECES = BR * (D / 8) / NT;
#pragma unroll
  for (int i = 0; i < OPIECES; ++i) {
    const int c = tid + i * NT;
    const int row = c / (D / 8), col = 8 * (c % (D / 8));
    if (i0 + row < N) {
      const u32x4 o = *reinterpret_cast<const u32x4*>(ot + row * OROW + col);
      *reinterpret_cast<u32x4*>(outp + (int64_t)(i0 + row) * like.sn + col) = o;
    }
  }
}

template <int D> hipError_t launch_windowed_bwd_t(const BwdArgs& a, hipStream_t s) {
  const dim3 grid(((a.N + BR - 1) / BR) * a.H0 * a.B), block(NT);
  const int smem = (int)sizeof(BandSmem<D>);
  hipError_t e = hipSuccess;
  auto launch = [&](auto kern) {
    if (e != hipSuccess) return;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e == hipSuccess) kern<<<grid, block, smem, s>>>(a);
  };
  launch(windowed_bwd_band_kernel<D, kStats>);
  launch(windowed_bwd_band_kernel<D, kDq>);
  launch(windowed_bwd_band_kernel<D, kDv>);
  launch(windowed_bwd_band_kernel<D, kDk>);
  return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace

// Windowed heads [0, H0) of a bf16 call; the workspace receives (log2-sum-exp, D_i) per query.
hipError_t launch_windowed_backward_mfma(const BwdArgs& a, hipStream_t s) {
  if (a.H0 <= 0 || a.N <= 0 || a.B <= 0) return hipSuccess;
  return a.d == 64 ? launch_windowed_bwd_t<64>(a, s) : launch_windowed_bwd_t<128>(a, s);
}

}  // namespace gformer
