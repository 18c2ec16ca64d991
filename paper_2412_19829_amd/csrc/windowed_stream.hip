// Windowed softmax attention heads as a stream of key tiles (section III-B, Eq. 1), for windows
// that span at most 5 tiles of 64 keys per 64 queries (w <= 257 causal or centred).
//
// A pair of 32-query groups (64 consecutive queries) sees the key tiles m - dl .. m + dr, m its
// own tile index: at most 5 of them.  While tile t is in LDS the pairs t - dr .. t + dl need it,
// so with 5 pair slots (pair m in slot m % 5, two waves per slot) EVERY consumer wave has work on
// EVERY tile, each K/V tile is fetched once per workgroup, and a slot's next pair starts on the
// step after its current pair ends.  One workgroup walks one piece of one (batch, head): a run of
// pairs plus the dl + dr tiles of halo around it.
//
// 12 waves: 10 consumers (slot = wave / 2, group of the pair = wave % 2) and 2 producers that
// move the K/V tile of step t+1 and the Q rows of the pair that starts on step t+1 from staging
// registers into LDS while the loads of step t+2 are in flight.  One barrier per step.
//
// Per tile and consumer wave, as in the query-block kernel:  S^T = K Q^T  (keys x queries, one
// lane owns one query column), online softmax in base 2 with lane-local running max / sum, then
// O^T += V^T P^T with P^T taken straight from the score registers.
#include <type_traits>

#include "common.hpp"
#include "mfma.hpp"

namespace gformer {
namespace {

constexpr int BC = 64;            // keys per tile
constexpr int PQ = 64;            // queries per pair
constexpr int WQ = 32;            // queries per consumer wave
constexpr int NS = kStreamSlots;  // pair slots
constexpr int NWC = 2 * NS;       // consumer waves
constexpr int NWP = 2;            // producer waves
constexpr int NT = 64 * (NWC + NWP);
constexpr int NPT = 64 * NWP;     // producer threads
constexpr float kLog2e = 1.4426950408889634f;

template <int D> struct StreamSmem {
  static constexpr int KROW = D + 8;    // row stride = 4 dwords mod 64: conflict-free b128 reads
  static constexpr int VROW = D + 32;   // row stride = 16 dwords mod 64: conflict-free tr reads
  static constexpr int QROW = D + 8;
  static constexpr int OROW = D + 8;
  struct KV {
    uint16_t k[BC * KROW];
    uint16_t v[BC * VROW];
  } kv[2];                     // step s of the piece uses kv[s % 2]
  uint16_t q[2][PQ * QROW];    // Q rows of the pair that starts on step s in q[s % 2]
  uint16_t o[2][WQ * OROW];    // finished rows of the pair that ends on this step, by group
};

// NEG: the softmax scale is negative, so the largest logit belongs to the smallest raw score.
template <int D, bool NEG>
__global__ __launch_bounds__(NT, 1) void windowed_stream_kernel(AttnArgs a) {
  constexpr int KS = D / 16;   // k-steps over the head dimension
  constexpr int MT = D / 32;   // 32-row tiles of O^T
  using Smem = StreamSmem<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int N = a.N;
  const int wl = a.wleft, wr = a.wright;
  const int dl = (wl + BC - 1) / BC;     // tiles a pair reaches to the left of its own
  const int dr = (BC - 1 + wr) / BC;     // ... and to the right
  const int npairs = (N + PQ - 1) / PQ;
  const int pph = a.win_pieces_per_head, ppp = a.win_pairs_per_piece;

  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2; neighbouring pieces of
  // a head share their halo tiles, so each XCD gets one contiguous run of the piece order.
  int pc = blockIdx.x;
  {
    constexpr int kXcds = 8;
    const int total = gridDim.x;
    const int per = total / kXcds, rem = total % kXcds;
    const int xcd = pc % kXcds, slot = pc / kXcds;
    pc = xcd * per + min(xcd, rem) + slot;
  }
  const int piece = pc % pph;
  const int h = (pc / pph) % a.H0, b = pc / (pph * a.H0);
  const int m0 = piece * ppp, m1 = min(npairs, m0 + ppp);
  if (m0 >= m1) return;   // uniform over the workgroup (the host sizes the grid so this never happens)
  // steps of the piece: one per tile index, first pair's first tile .. last pair's last tile.
  // Tile indices outside the sequence (window cut at its ends) are walked but neither loaded
  // nor computed, so that every pair starts and ends on its regular step.
  const int t_begin = m0 - dl, t_end = m1 - 1 + dr;
  const int t_real_max = (N - 1) / BC;

  if (wave >= NWC) {
    // ------------------------------ producers ------------------------------
    const int ptid = tid - 64 * NWC;
    constexpr int C8 = D / 8, RP = NPT / C8, CH = BC / RP;   // 16-byte pieces per thread and tensor
    static_assert(CH * RP == BC && PQ == BC, "tile rows must be covered exactly");
    const int prow = ptid / C8, pcol = 8 * (ptid % C8);
    const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q.base) + b * a.q.sb + h * a.q.sh;
    const uint16_t* kp = reinterpret_cast<const uint16_t*>(a.k.base) + b * a.k.sb + h * a.k.sh;
    const uint16_t* vp = reinterpret_cast<const uint16_t*>(a.v.base) + b * a.v.sb + h * a.v.sh;
    const int qsn = (int)a.q.sn, ksn = (int)a.k.sn, vsn = (int)a.v.sn;
    const uint32_t colb = 2u * (uint32_t)pcol;
    const uint32_t qoff = 2u * (uint32_t)(prow * qsn) + colb;
    const uint32_t koff = 2u * (uint32_t)(prow * ksn) + colb;
    const uint32_t voff = 2u * (uint32_t)(prow * vsn) + colb;
    u32x4 qst[CH], kst[CH], vst[CH];
    // Piece i of a tile is read from a wave-uniform base (first row + i*RP, in scalar registers)
    // plus one per-thread byte offset that never changes, clamped so that rows past N-1 re-read
    // row N-1 (in bounds, masked or dropped later).  Steps whose tile or pair does not exist
    // repeat the nearest one that does: the loads stay unconditional and in bounds, and the
    // waits the compiler derives for them stay exact.
    auto load_rows = [&](u32x4 (&dst)[CH], const uint16_t* base, int sn, uint32_t off, int r0) {
      const int last = min(N - 1 - r0, BC - 1);
      const char* rb = reinterpret_cast<const char*>(base + (int64_t)r0 * sn);
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        const int first = min(i * RP, last);  // uniform
        const uint32_t lim = 2u * (uint32_t)((last - first) * sn) + colb;
        dst[i] = __builtin_nontemporal_load(
            reinterpret_cast<const u32x4*>(rb + 2u * (uint32_t)(first * sn) + (size_t)min(off, lim)));
      }
    };
    auto load_step = [&](int t) {
      const int tc = min(max(t, 0), t_real_max);
      const int mq = min(max(t + dl, m0), m1 - 1);   // the pair that starts on step t
      load_rows(kst, kp, ksn, koff, tc * BC);
      load_rows(vst, vp, vsn, voff, tc * BC);
      load_rows(qst, qp, qsn, qoff, mq * PQ);
    };
    auto store_step = [&](int s) {
      typename Smem::KV& kv = sm.kv[s & 1];
      uint16_t* qd = sm.q[s & 1];
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        *reinterpret_cast<u32x4*>(&kv.k[(prow + i * RP) * Smem::KROW + pcol]) = kst[i];
        *reinterpret_cast<u32x4*>(&kv.v[(prow + i * RP) * Smem::VROW + pcol]) = vst[i];
        *reinterpret_cast<u32x4*>(&qd[(prow + i * RP) * Smem::QROW + pcol]) = qst[i];
      }
    };
    load_step(t_begin);
    store_step(0);
    load_step(t_begin + 1);
    lds_barrier();
    for (int t = t_begin; t <= t_end; ++t) {
      store_step(t - t_begin + 1);
      load_step(t + 2);
      lds_barrier();
    }
    return;
  }

  // ------------------------------ consumers ------------------------------
  const int ln = lane & 31;   // query column / operand row
  const int lh = lane >> 5;   // which half of the k-slots
  const int ps = wave >> 1;   // pair slot
  const int hf = wave & 1;    // group of the pair
  uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + b * a.osb + h * a.osh;
  // base-2 logits = raw score * sc; a zero scale is nudged so that masked (infinite) scores
  // still map to weight 0 instead of NaN
  const float sc = (a.scale == 0.f ? 1e-30f : a.scale) * kLog2e;

  bf16x8 qreg[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) qreg[ks] = as_bf16x8(u32x4{0u, 0u, 0u, 0u});
  // this lane's corner of the V operand reads: row 4*lh of the tile plus the transpose pattern
  const int vlane = 4 * lh * Smem::VROW + lds_operand_tr_lane_offset(Smem::VROW, lane);
  f32x16 oacc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[mt][r] = 0.f;
  float m_run = -INFINITY;  // running max of the scaled base-2 scores of this lane's query
  float l_run = 0.f;        // running sum over the keys this lane holds (half of each tile)

  int m_cur = m0 + ((ps - m0 % NS) + NS) % NS;   // this slot's first pair in the piece
  lds_barrier();
  for (int t = t_begin; t <= t_end; ++t) {
    const int s = t - t_begin;
    const typename Smem::KV& cur = sm.kv[s & 1];
    const bool mine = m_cur < m1;                 // uniform
    if (mine && t == m_cur - dl) {
      // a new pair starts: its Q rows were put in place during the previous step
      const uint16_t* qrow = &sm.q[s & 1][(WQ * hf + ln) * Smem::QROW + 8 * lh];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) qreg[ks] = lds_read16(qrow + 16 * ks);
      // The accumulators are not cleared here: with the running maximum back at -inf, the first
      // visible key of a query triggers the rescale below with a factor of exactly 0, which
      // clears them (they hold the previous pair's finite sums) before anything is added.
      m_run = -INFINITY;
      l_run = 0.f;
    }
    const int q0 = m_cur * PQ + hf * WQ;
    const int t0 = t * BC;
    // keys visible to query i: i - wl <= j <= min(i + wr, N - 1); a tile with none for this
    // wave's queries is skipped, a tile every one of them sees in full needs no mask
    if (mine && t >= m_cur - dl && t >= 0 && t <= t_real_max &&
        !(t0 > q0 + WQ - 1 + wr || t0 + BC - 1 < q0 - wl)) {
      const bool need_mask =
          !(t0 + BC - 1 <= q0 + wr && t0 >= q0 + WQ - 1 - wl && t0 + BC <= N);

      // One copy of the tile body with the window mask and one without: left to itself the
      // compiler turns the mask into selects that run on every tile.
      auto tile_body = [&](auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
      // The two 32-key halves of the tile one after the other (scores of one half live at a
      // time): S^T = K Q^T, online softmax, O^T += V^T P^T.
      constexpr float worst = NEG ? INFINITY : -INFINITY;
      // register r of a half is key t0 + 32*kt + c + 4*lh, c = 8*(r/4) + r%4; with
      // hi = min(qi + wr, N - 1) the key is visible iff 0 <= hi - key <= hi - (qi - wl)
      const int qi = q0 + ln;
      const int hi = min(qi + wr, N - 1);
      const int rel = hi - t0 - 4 * lh;
      const int wv = max(hi - qi + wl + 1, 0);   // visible keys of this query (0: a row past N)
      // both score products are issued before the first softmax, so that the second runs on the
      // matrix core while the vector unit works on the first
      f32x16 sboth[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sboth[kt][r] = 0.f;
        const uint16_t* krow = &cur.k[(32 * kt + ln) * Smem::KROW + 8 * lh];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 ka = lds_read16(krow + 16 * ks);
          sboth[kt] = mfma32(ka, qreg[ks], sboth[kt]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        f32x16& sreg = sboth[kt];
        if (MASKED) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int c = 32 * kt + 8 * (r / 4) + (r % 4);
            sreg[r] = ((unsigned)(rel - c) >= (unsigned)wv) ? worst : sreg[r];
          }
        }
        // Online softmax in base 2 on the raw scores: p = 2^(s*sc - m), m a per-query
        // reference that follows the running maximum lazily: accumulators are rescaled only
        // when some query's maximum grows by more than 8 (weights stay <= 2^8, harmless in
        // bf16/fp32), which after the first tile or two is rare.
        float ext = worst;
#pragma unroll
        for (int r = 0; r < 16; r += 2)
          ext = NEG ? min3(ext, sreg[r], sreg[r + 1]) : max3(ext, sreg[r], sreg[r + 1]);
        float mloc = (ext == worst) ? -INFINITY : ext * sc;   // no visible key in this lane's quarter
        mloc = max_over_halves(mloc);
        if (__builtin_amdgcn_ballot_w64(mloc > m_run + 8.f) != 0) {   // wave-uniform
          const float m_new = fmaxf(m_run, mloc);
          const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
          const float alpha = __builtin_amdgcn_exp2f(m_run - m_ref);  // 0 on the first visible keys
          m_run = m_new;
          l_run *= alpha;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[mt][r] *= alpha;
        }
        const float m_use = (m_run == -INFINITY) ? 0.f : m_run;  // a query with no visible key yet
        uint32_t pb[8];  // P^T as packed bf16: pb[4*kb + i] covers registers 8*kb+2i, +1
        float lsum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(sreg[r], sc, -m_use));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(sreg[r + 1], sc, -m_use));
          const uint32_t pk = pack_bf16(p0, p1);
          pb[r / 2] = pk;
          // the row sum uses the rounded weights the PV product sees
          lsum = dot2_ones_bf16(pk, lsum);
        }
        l_run += lsum;
        // O^T += V^T P^T: 8 products (2 groups of 16 keys x 4 row tiles of O^T); the V operand
        // of product i + PDV is fetched from LDS before product i is issued (two ahead fits the
        // 168-register budget without spills and is 2-3 % faster than one; three spills)
        bf16x8 pbv[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          u32x4 pw;
          pw[0] = pb[4 * kb + 0]; pw[1] = pb[4 * kb + 1];
          pw[2] = pb[4 * kb + 2]; pw[3] = pb[4 * kb + 3];
          pbv[kb] = as_bf16x8(pw);
        }
        constexpr int NPV = 2 * MT, PDV = 2;
        // keys in the order the score registers hold them: 16*kb + 4*lh + j, then + 8
        auto v_operand = [&](int i) {
          const int r0 = 32 * kt + 16 * (i / MT);
          return lds_operand_tr_at(cur.v + vlane, Smem::VROW, r0, r0 + 8, 32 * (i % MT));
        };
        bf16x8 vop[NPV];
#pragma unroll
        for (int i = 0; i < PDV && i < NPV; ++i) vop[i] = v_operand(i);
#pragma unroll
        for (int i = 0; i < NPV; ++i) {
          if (i + PDV < NPV) vop[i + PDV] = v_operand(i + PDV);
          oacc[i % MT] = mfma32(vop[i], pbv[i / MT], oacc[i % MT]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
          };
      if (need_mask) tile_body(std::true_type{});
      else tile_body(std::false_type{});
    }
    if (mine && t == m_cur + dr) {
      // the pair ends: normalise; the 32 rows go through this group's LDS patch (only one pair
      // ends per step, so the patch is this wave's alone until the barrier below) and leave as
      // whole rows, 16 bytes per lane.  Lane owns query q0+ln, value columns
      // 32*mt + 8*g + 4*lh + 0..3.
      const float l_tot = sum_over_halves(l_run);
      const float inv = 1.f / l_tot;
      uint16_t* ot = sm.o[hf];
      {
        uint16_t* orow = ot + ln * Smem::OROW + 4 * lh;
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
      // LDS operations of one wave execute in order; the fence keeps the compiler from moving
      // the reads below above the writes above
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      constexpr int OPIECES = WQ * (D / 8) / 64;
#pragma unroll
      for (int i = 0; i < OPIECES; ++i) {
        const int c = lane + i * 64;
        const int row = c / (D / 8), col = 8 * (c % (D / 8));
        if (q0 + row < N) {
          const u32x4 o = *reinterpret_cast<const u32x4*>(ot + row * Smem::OROW + col);
          __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(op + (int64_t)(q0 + row) * a.osn + col));
        }
      }
      m_cur += NS;
    }
    lds_barrier();  // this step's tile is consumed, the next one is in place
  }
}

}  // namespace

StreamPlan windowed_stream_plan(int64_t heads, int N, int wleft, int wright) {
  StreamPlan sp{};
  const int dl = (wleft + BC - 1) / BC, dr = (BC - 1 + wright) / BC;
  sp.applies = dl + dr + 1 <= NS;
  sp.threads = NT;
  if (!sp.applies || heads <= 0 || N <= 0) return sp;
  // Pieces: one per compute unit where the heads allow it, never shorter than the halo a piece
  // has to walk on top of its own pairs.
  const int npairs = (N + PQ - 1) / PQ;
  const int64_t kComputeUnits = device_compute_units();
  int64_t pph = heads >= kComputeUnits ? 1 : kComputeUnits / heads;
  int ppp = (int)((npairs + pph - 1) / pph);
  ppp = std::max(ppp, std::min(npairs, NS - 1));
  pph = (npairs + ppp - 1) / ppp;
  sp.pairs_per_piece = ppp;
  sp.pieces_per_head = (int)pph;
  sp.blocks = heads * pph;
  // A piece is a serial walk of pairs + halo steps of about 1.5 us each: with little work per
  // compute unit the query-block kernel's many short independent workgroups finish sooner.
  // Measured crossover: about two full rounds of its 128-query workgroups (2 per CU).
  sp.preferred = heads * ((N + 127) / 128) >= 4 * kComputeUnits;
  return sp;
}

hipError_t launch_windowed_stream(const AttnArgs& a0, hipStream_t s) {
  if (a0.H0 <= 0 || a0.N <= 0 || a0.B <= 0) return hipSuccess;
  AttnArgs a = a0;
  const int64_t heads = (int64_t)a.B * a.H0;
  const StreamPlan sp = windowed_stream_plan(heads, a.N, a.wleft, a.wright);
  if (!sp.applies) return hipErrorInvalidValue;   // the caller asks windowed_stream_plan first
  a.win_pairs_per_piece = sp.pairs_per_piece;
  a.win_pieces_per_head = sp.pieces_per_head;
  const int64_t pph = sp.pieces_per_head;
  dim3 grid((unsigned)(heads * pph));
  dim3 block(NT);
  const bool neg = a.scale < 0.f;
  hipError_t e = hipSuccess;
  auto launch = [&](auto kern, int smem) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e == hipSuccess) kern<<<grid, block, smem, s>>>(a);
  };
  if (a.d == 64) {
    if (neg) launch(windowed_stream_kernel<64, true>, (int)sizeof(StreamSmem<64>));
    else launch(windowed_stream_kernel<64, false>, (int)sizeof(StreamSmem<64>));
  } else {
    if (neg) launch(windowed_stream_kernel<128, true>, (int)sizeof(StreamSmem<128>));
    else launch(windowed_stream_kernel<128, false>, (int)sizeof(StreamSmem<128>));
  }
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

}  // namespace gformer
