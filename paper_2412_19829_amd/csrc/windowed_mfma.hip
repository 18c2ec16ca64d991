// Windowed softmax attention heads on bf16 matrix cores (section III-B, Eq. 1): the causal window
// ending at the token, or (bidirectional variant) the window centred on it.
//
// The query-block kernel: used for windows wider than five key tiles and for small calls (the
// streaming kernel in windowed_stream.hip takes the rest).
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
//
// The K tiles run one step ahead of the V tiles: a step first turns the scores of tile t (made
// at the end of the step before) into weights, which is vector work only, and then issues the
// value products of tile t and the score products of tile t+1 back to back, sixteen and sixteen
// matrix instructions over six independent accumulators with their LDS operands fetched ahead.
// So a wave alternates between a stretch that needs only the vector unit and a stretch that
// needs only the matrix core and LDS, and the two waves a SIMD holds fill each other's gaps.
#include <type_traits>

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
  uint16_t k[2][BC * KROW];   // K tile t in k[(t - first tile) % 2], V tile t in v[...] likewise:
  uint16_t v[2][BC * VROW];   // one of each is filled while the other is read
};

// NEG: the softmax scale is negative, so the largest logit belongs to the smallest raw score
// (a compile-time switch keeps the running-extremum code free of branches).
template <int D, bool NEG>
__global__ __launch_bounds__(kMfmaWindowThreads, 2) void windowed_mfma_kernel(AttnArgs a) {
  constexpr int KS = D / 16;           // k-steps over the head dimension
  constexpr int MT = D / 32;           // 32-row tiles of O^T
  constexpr int KCH = BC * D / 8 / kMfmaWindowThreads;  // 16-byte K chunks per thread per tile
  using Smem = WinSmem<D>;
  constexpr int KROW = Smem::KROW, VROW = Smem::VROW;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int ln = lane & 31;   // query column / operand row
  const int lh = lane >> 5;   // which half of the k-slots
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Neighbouring query
  // blocks of a head share most of their key band, so the logical block order (query block
  // fastest, then head, then batch) is laid out such that each XCD gets one contiguous run of it.
  const int nqb = (a.N + BR - 1) / BR;
  const int total = nqb * a.H0 * a.B;
  constexpr int kXcds = 8;
  int lb = blockIdx.x;
  {
    const int per = total / kXcds, rem = total % kXcds;   // first `rem` XCDs get one more
    const int xcd = lb % kXcds, slot = lb / kXcds;
    lb = xcd * per + min(xcd, rem) + slot;
  }
  const int qb = lb % nqb;
  const int h = (lb / nqb) % a.H0, b = lb / (nqb * a.H0);
  const int i0 = qb * BR;
  const int q0 = i0 + wave * WQ;
  const int N = a.N;

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
      qreg[ks] = as_bf16x8(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(qr + 16 * ks)));
  }
  // Memory loads retire in issue order, so the wait for the first tile below also covers these
  // loads, but only if they stay in front of it: were they to slip behind, every later use of Q
  // would have to wait for whatever tile load is in flight at that point, and the prefetch
  // distance of the loop would be lost.
  __builtin_amdgcn_sched_barrier(0);

  f32x16 oacc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[mt][r] = 0.f;
  float m_run = -INFINITY;  // running max of the scaled base-2 scores of this lane's query
  float l_run = 0.f;        // running sum over the keys this lane holds (half of each tile)

  // token i sees keys i - wl .. i + wr (cut at the ends): wl = w - 1, wr = 0 for the causal window
  // ending at the token, wl = w / 2, wr = w - 1 - wl for the window centred on it
  const int wl = a.wleft, wr = a.wright;
  const int kfirst = max(0, i0 - wl) / BC;
  const int klast = min(N - 1, i0 + BR - 1 + wr) / BC;
  // base-2 logits = raw score * sc; a zero scale is nudged so that masked (infinite) scores
  // still map to weight 0 instead of NaN
  const float sc = (a.scale == 0.f ? 1e-30f : a.scale) * kLog2e;

  // register staging of a tile on its way from global memory to LDS: thread t moves 16-byte
  // pieces (row t/C8 + i*RP, columns 8*(t%C8)..), a uniform row base plus a constant offset
  constexpr int C8 = D / 8, RP = kMfmaWindowThreads / C8;
  static_assert(KCH * RP == BC, "tile rows must be covered exactly");
  const int prow = tid / C8, pcol = 8 * (tid % C8);
  // piece i is read from a wave-uniform base (row t0 + i*RP, in scalar registers) plus one
  // per-thread byte offset that never changes, clamped so that rows past N-1 (last tile of the
  // sequence only) re-read row N-1: in bounds, masked later
  const int ksn = (int)a.k.sn, vsn = (int)a.v.sn;
  const uint32_t colb = 2u * (uint32_t)pcol;
  const uint32_t koff = 2u * (uint32_t)(prow * ksn) + colb, voff = 2u * (uint32_t)(prow * vsn) + colb;
  u32x4 kst[KCH];
  u32x4 vst[KCH];
  auto load_rows = [&](u32x4 (&dst)[KCH], const uint16_t* base, int sn, uint32_t off, int t) {
    const int t0 = t * BC;
    const int last = min(N - 1 - t0, BC - 1);
    const char* rb = reinterpret_cast<const char*>(base + (int64_t)t0 * sn);
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int first = min(i * RP, last);  // uniform
      const uint32_t lim = 2u * (uint32_t)((last - first) * sn) + colb;
      dst[i] = *reinterpret_cast<const u32x4*>(rb + 2u * (uint32_t)(first * sn) + (size_t)min(off, lim));
    }
  };
  auto store_rows = [&](uint16_t* tile, int stride, const u32x4 (&src)[KCH]) {
#pragma unroll
    for (int i = 0; i < KCH; ++i)
      *reinterpret_cast<u32x4*>(&tile[(prow + i * RP) * stride + pcol]) = src[i];
  };

  // S^T = K Q^T for the two 32-key halves of a tile: two accumulator chains taken in turn, the
  // K operands of a k-step fetched while the step before is on the matrix core
  f32x16 s[2];
  auto scores = [&](const uint16_t* ktile) {
    const uint16_t* kr0 = ktile + ln * KROW + 8 * lh;
    const uint16_t* kr1 = kr0 + 32 * KROW;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
    bf16x8 ka[2][2];
    ka[0][0] = lds_read16(kr0);
    ka[0][1] = lds_read16(kr1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) {
        ka[(ks + 1) & 1][0] = lds_read16(kr0 + 16 * (ks + 1));
        ka[(ks + 1) & 1][1] = lds_read16(kr1 + 16 * (ks + 1));
      }
      s[0] = mfma32(ka[ks & 1][0], qreg[ks], s[0]);
      s[1] = mfma32(ka[ks & 1][1], qreg[ks], s[1]);
    }
  };
  // this lane's corner of the V operand reads: row 4*lh of the tile plus the transpose pattern
  const int vlane = 4 * lh * VROW + lds_operand_tr_lane_offset(VROW, lane);

  // One step: tile t's scores (in s) become weights, then the value products of tile t and, unless
  // this is the last tile, the score products of tile t+1.  Tile t+1's keys and tile t's values
  // move from the staging registers to LDS at the top of the step and are waited for at its one
  // barrier, by which time every wave is done reading what they overwrite (read two steps ago);
  // the loads of tile t+2's keys and tile t+1's values are in flight meanwhile.
  // does any query of this wave see any key of tile t?  (wave-uniform)
  auto in_band = [&](int t) {
    const int t0 = t * BC;
    return !(t0 > q0 + WQ - 1 + wr || t0 + BC - 1 < q0 - wl);
  };
  auto step = [&](int t, auto last_tag) {
    constexpr bool LAST = decltype(last_tag)::value;
    const int it = t - kfirst;
    const bool mine = in_band(t);
    if (!LAST) store_rows(sm.k[(it + 1) & 1], KROW, kst);
    store_rows(sm.v[it & 1], VROW, vst);
    if (!LAST) {
      if (t + 1 < klast) load_rows(kst, kp, ksn, koff, t + 2);
      load_rows(vst, vp, vsn, voff, t + 1);
    }
    const int t0 = t * BC;
    bf16x8 pbv[2][2];  // P^T as packed bf16 operands: pbv[kt][kb] covers registers 8*kb .. 8*kb+7
    if (mine) {
      // keys visible to query i: i - wl <= j <= min(i + wr, N - 1); a tile every query of this wave
      // sees in full needs no mask; one it sees nothing of is left out (mine)
      const bool need_mask =
          !(t0 + BC - 1 <= q0 + wr && t0 >= q0 + WQ - 1 - wl && t0 + BC <= N);
      // Online softmax in base 2 on the raw scores: p = 2^(s*sc - m), m a per-query reference.
      // The reference follows the running maximum lazily: accumulators are rescaled only when
      // some query's maximum grows by more than 8 (weights stay <= 2^8, harmless in bf16/fp32),
      // which after the first tile or two is rare.
      constexpr float worst = NEG ? INFINITY : -INFINITY;
      if (need_mask) {
        // register (kt, r) of this lane is key t0 + c + 4*lh, c = 32*kt + 8*(r/4) + r%4;
        // with hi = min(qi + wr, N - 1) the key is visible iff 0 <= hi - key <= hi - (qi - wl)
        const int qi = q0 + ln;
        const int hi = min(qi + wr, N - 1);
        int rel = hi - t0 - 4 * lh;
        // opaque to the optimiser: left to itself it keeps all 32 values of rel - c in registers
        // across the loop and steps each of them on every tile
        asm volatile("" : "+v"(rel));
        const unsigned wv = (unsigned)max(hi - qi + wl + 1, 0);   // visible keys (0: a row past N)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int c = 32 * kt + 8 * (r / 4) + (r % 4);
            s[kt][r] = ((unsigned)(rel - c) >= wv) ? worst : s[kt][r];
          }
      }
      float ext = worst;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; r += 2)
          ext = NEG ? min3(ext, s[kt][r], s[kt][r + 1]) : max3(ext, s[kt][r], s[kt][r + 1]);
      float mloc = (ext == worst) ? -INFINITY : ext * sc;   // no visible key in this lane's half
      mloc = max_over_halves(mloc);
      if (__builtin_amdgcn_ballot_w64(mloc > m_run + 8.f) != 0) {   // wave-uniform
        const float m_new = fmaxf(m_run, mloc);
        const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_ref);  // 0 on the first visible tile
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[mt][r] *= alpha;
      }
      const float m_use = (m_run == -INFINITY) ? 0.f : m_run;  // a query with no visible key yet
      float lsum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          u32x4 pw;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int r = 8 * kb + 2 * i;
            const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kt][r], sc, -m_use));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kt][r + 1], sc, -m_use));
            pw[i] = pack_bf16(p0, p1);
            // the row sum uses the rounded weights the PV product sees
            lsum = dot2_ones_bf16(pw[i], lsum);
          }
          pbv[kt][kb] = as_bf16x8(pw);
        }
      }
      l_run += lsum;
    }

    lds_barrier();   // tile t's values and tile t+1's keys are in place

    // O^T += V^T P^T
    const uint16_t* vt = sm.v[it & 1] + vlane;
    if (mine) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            // keys in the order the score registers hold them: 16*kb + 4*lh + j, then + 8
            const int r0 = 32 * kt + 16 * kb;
            const bf16x8 va_ = lds_operand_tr_at(vt, VROW, r0, r0 + 8, 32 * mt);
            oacc[mt] = mfma32(va_, pbv[kt][kb], oacc[mt]);
          }
        }
      }
    }
    if (!LAST && in_band(t + 1)) scores(sm.k[(it + 1) & 1]);
  };

  load_rows(kst, kp, ksn, koff, kfirst);
  store_rows(sm.k[0], KROW, kst);
  load_rows(vst, vp, vsn, voff, kfirst);
  if (kfirst < klast) load_rows(kst, kp, ksn, koff, kfirst + 1);
  lds_barrier();
  if (in_band(kfirst)) scores(sm.k[0]);
  for (int t = kfirst; t < klast; ++t) step(t, std::false_type{});
  step(klast, std::true_type{});
  lds_barrier();   // every wave is done with the tiles: their memory takes the output rows

  // normalise; rows go through LDS (the K/V tiles are dead by now) so that they leave as whole
  // rows, 16 bytes per lane.  Lane owns query q0+ln, value columns 32*mt + 8*g + 4*lh + 0..3.
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.f / l_tot;
  constexpr int OROW = D + 8;
  static_assert(BR * OROW * 2 <= (int)sizeof(Smem), "output staging must fit in the tile memory");
  uint16_t* ot = reinterpret_cast<uint16_t*>(&sm);
  {
    uint16_t* orow = ot + (WQ * wave + ln) * OROW + 4 * lh;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(oacc[mt][4 * g + 0] * inv, oacc[mt][4 * g + 1] * inv);
        pk[1] = pack_bf16(oacc[mt][4 * g + 2] * inv, oacc[mt][4 * g + 3] * inv);
        *reinterpret_cast<u32x2*>(orow + 32 * mt + 8 * g) = pk;
      }
    }
  }
  lds_barrier();
  constexpr int OPIECES = BR * (D / 8) / kMfmaWindowThreads;
#pragma unroll
  for (int i = 0; i < OPIECES; ++i) {
    const int c = tid + i * kMfmaWindowThreads;
    const int row = c / (D / 8), col = 8 * (c % (D / 8));
    if (i0 + row < N) {
      const u32x4 o = *reinterpret_cast<const u32x4*>(ot + row * OROW + col);
      __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(op + (int64_t)(i0 + row) * a.osn + col));
    }
  }
}

}  // namespace

hipError_t launch_windowed_mfma(const AttnArgs& a, hipStream_t s) {
  if (a.H0 <= 0 || a.N <= 0 || a.B <= 0) return hipSuccess;
  dim3 grid(((a.N + BR - 1) / BR) * a.H0 * a.B);
  dim3 block(kMfmaWindowThreads);
  const bool neg = a.scale < 0.f;
  hipError_t e = hipSuccess;
  auto launch = [&](auto kern, int smem) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e == hipSuccess) kern<<<grid, block, smem, s>>>(a);
  };
  if (a.d == 64) {
    if (neg) launch(windowed_mfma_kernel<64, true>, (int)sizeof(WinSmem<64>));
    else launch(windowed_mfma_kernel<64, false>, (int)sizeof(WinSmem<64>));
  } else {
    if (neg) launch(windowed_mfma_kernel<128, true>, (int)sizeof(WinSmem<128>));
    else launch(windowed_mfma_kernel<128, false>, (int)sizeof(WinSmem<128>));
  }
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

}  // namespace gformer
