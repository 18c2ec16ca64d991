// Linear attention heads on bf16 matrix cores, chunked: the causal form of section III-C,
// Algorithm 1 (described first), and the bidirectional form of section II-B (end of this note).
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
// The chunks of all linear heads form one list that is cut into pieces, one workgroup each:
// uniform segments per head (chosen by the planner when a whole number per head fills most of
// the chip, or on request), else equal pieces with no regard to head boundaries.
// Pieces are stitched in stream-ordered launches: (1) for every sub-piece boundary (a piece is
// cut into 1, 2 or 4 sub-pieces) that falls inside a head and is followed by a piece start in
// the same head, sum (A, Z) over the part of that head lying in the sub-piece before it; (2) only when a head holds many such
// sums, a tiny kernel turns them into running sums; (3) the read-out kernel starts each piece
// from the state carried to its first chunk (adding up the few sums itself otherwise) and
// restarts from zero at head boundaries.
//
// Bidirectional form: out_i = phi(q_i)^T S / (phi(q_i).z + eps) with S, z summed over the whole
// head.  Pieces are uniform segments per head, launch (1) sums every piece, and the read-out
// kernel (CAUSAL = false) contracts phi(Q) with the head's total state only: K and V are read
// once, by the state pass.
#include "linear_common.hpp"

#include <type_traits>

// Register sets of the read-out kernel's producers (chunks of loads in flight): 2 or 3.  Three
// were measured and are no faster (178 against 176 us on the headline layer).
#ifndef GF_MAIN_SETS
#define GF_MAIN_SETS 2
#endif

namespace gformer {
namespace {

template <int D> struct ChunkTiles {
  using C = LinCfg<D>;
  uint16_t fq[CH * C::QROW];   // phi(Q), feature index permuted by kperm32 inside 32-groups
  uint16_t fk[CH * C::KROW];   // phi(K), natural order
  uint16_t v[CH * C::VROW];    // V
};

template <int D> struct LinSmem {
  using C = LinCfg<D>;
  ChunkTiles<D> buf[2];        // chunk n in buf[n % 2]: producers fill one while the other is read
  uint16_t pt[CH * C::PROW];   // masked products P^T viewed as [query][key]
  float z[2][D];               // Z in fq's permuted feature order; double-buffered across chunks
  uint16_t zh[2][D];           // bf16(Z) and bf16(Z - bf16(Z)): Z to 16 mantissa bits for the
  uint16_t zl[2][D];           // packed dot products of the denominator
  float den[CH];
  uint16_t ot[CH * C::OROW];   // finished output rows of the previous chunk, [query][value]
};

template <int D> struct StateTiles {
  using C = LinCfg<D>;
  uint16_t fk[CH * C::KROW];
  uint16_t v[CH * C::VROW];
};
template <int D> struct StateSmem {
  StateTiles<D> buf[2];
};

// Walks the chunk list of a piece: (linear head, chunk inside the head), one step at a time.
// All state is wave-uniform; the head's pointers are recomputed only when a head boundary is
// crossed.
template <int D> struct ChunkCursor {
  int head, lc;
  HeadPtrs<D> hp;
  __device__ __forceinline__ ChunkCursor(const AttnArgs& a, int g)
      : head(g / a.vcph), lc(g % a.vcph), hp(head_ptrs<D>(a, g / a.vcph)) {}
  __device__ __forceinline__ void next(const AttnArgs& a, bool more) {
    if (++lc == a.vcph && more) {
      lc = 0;
      ++head;
      hp = head_ptrs<D>(a, head);
    }
  }
  __device__ __forceinline__ int t0() const { return lc * CH; }
};

// One 16-token step of A += phiK^T V for this wave's value columns: `vt` is the V^T operand of
// tokens 16*kk.. (lane = value column 32*wave + l%32), phi(K) comes from its row-major LDS tile
// through the transpose read.  Adds this lane's share of colsum(phiK) for feature
// 32*wave + l%32 (the tokens of its k-slot half) to `zs`.  The ET accumulator tiles take turns,
// so no matrix instruction waits for the one before it.
template <int D>
__device__ __forceinline__ float update_state_step(f32x16 (&sacc)[LinCfg<D>::ET], const uint16_t* fk,
                                                   bf16x8 vt, int kk, int wave, int lane, float zs) {
  using C = LinCfg<D>;
  const int lh = lane >> 5;
#pragma unroll
  for (int ct = 0; ct < C::ET; ++ct) {
    const bf16x8 fa =
        lds_operand_tr(fk, C::KROW, 16 * kk + 8 * lh, 16 * kk + 8 * lh + 4, 32 * ct, lane);
    sacc[ct] = mfma32(fa, vt, sacc[ct]);
  }
  // the wave's own feature tile once more: cheaper than a wave-dependent branch or select
  const bf16x8 fz =
      lds_operand_tr(fk, C::KROW, 16 * kk + 8 * lh, 16 * kk + 8 * lh + 4, 32 * wave, lane);
  return sum8_bf16(fz, zs);
}
// A += phiK^T V over a whole chunk; returns the lane's share of colsum(phiK).
template <int D>
__device__ __forceinline__ float update_state(f32x16 (&sacc)[LinCfg<D>::ET], const uint16_t* fk,
                                              const uint16_t* v, int wave, int lane) {
  using C = LinCfg<D>;
  const int lh = lane >> 5;
  float zs = 0.f;
#pragma unroll
  for (int kk = 0; kk < CH / 16; ++kk) {
    const bf16x8 vt =
        lds_operand_tr(v, C::VROW, 16 * kk + 8 * lh, 16 * kk + 8 * lh + 4, 32 * wave, lane);
    zs = update_state_step<D>(sacc, fk, vt, kk, wave, lane, zs);
  }
  return zs;
}

// -----------------------------------------------------------------------------------------
// (1) state sums.  Every piece is cut into state_sub equal sub-pieces.  Workgroup j-1 serves the
//     sub-piece boundary at global chunk e = j*piece_chunks/state_sub: if e falls inside a head
//     and a piece boundary follows inside the same head, it sums phi(k_t) (x) v_t and phi(k_t)
//     over the chunks of that head lying in sub-piece j-1 and writes them to workspace slot j.
//     Waves [0, NWC) contract; waves [NWC, 2 NWC) load, map and stage the next chunk.
// -----------------------------------------------------------------------------------------
template <int D, bool ELU1>
__global__ __launch_bounds__(LinCfg<D>::NT, 2) void linear_state_kernel(AttnArgs a) {
  using C = LinCfg<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  StateSmem<D>& sm = *reinterpret_cast<StateSmem<D>*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int ls = a.piece_chunks / a.state_sub;
  // Workgroups are dealt round-robin to the 8 XCDs.  Which sub-pieces have something to sum is
  // periodic in the block index (with two segments per head every second group of state_sub
  // blocks is idle), and a period that divides 8 would leave whole XCDs without work: give each
  // XCD one contiguous run of the logical block order instead.
  int lb = blockIdx.x;
  {
    constexpr int kXcds = 8;
    const int total = gridDim.x, per = total / kXcds, rem = total % kXcds;
    const int xcd = lb % kXcds, slot = lb / kXcds;
    lb = xcd * per + min(xcd, rem) + slot;
  }
  int q, head, lc0, lc1;                     // workspace slot; chunks [lc0, lc1) of `head`
  if (a.causal) {
    q = lb + 1;
    const int e = q * ls;                    // the boundary, as a global chunk index
    if (e % a.vcph == 0) return;             // on a head boundary: nothing is carried
    head = e / a.vcph;
    const int next_main = (q + a.state_sub - 1) / a.state_sub * a.piece_chunks;
    if (next_main >= (head + 1) * a.vcph || next_main >= a.n_pieces * a.piece_chunks)
      return;                                // no piece starts later in this head: nobody reads it
    lc1 = e % a.vcph;
    lc0 = max(lc1 - ls, 0);
  } else {
    // bidirectional: every sub-piece is summed (pieces never straddle heads in this mode);
    // slot q holds the sum over sub-piece q itself
    q = lb;
    head = q * ls / a.vcph;
    lc0 = q * ls % a.vcph;
    lc1 = min(lc0 + ls, a.cph);
    if (lc0 >= lc1) return;                  // virtual padding only (the planner avoids it)
  }
  const HeadPtrs<D> hp = head_ptrs<D>(a, head);
  const int N = a.N;
  const int nchunks = lc1 - lc0;

  if (wave >= C::NWC) {
    // ---- producers ----
    const Staging<D> st(tid - C::NTC);
    const PieceOffsets<D> ko(st, a.k.sn), vo(st, a.v.sn);
    u32x4 ka[C::PIECES], va[C::PIECES], kb[C::PIECES], vb[C::PIECES];
    auto load = [&](u32x4 (&kr)[C::PIECES], u32x4 (&vr)[C::PIECES], int n) {
      const int t0 = (lc0 + n) * CH;
      // plain loads here: with two small workgroups per compute unit they measured 6 % faster
      // than the non-temporal ones the one-per-unit read-out kernel prefers (43 against 46 us)
      load_chunk<D, false>(kr, hp.k, t0, N, ko);
      load_chunk<D, false>(vr, hp.v, t0, N, vo);
    };
    auto stage = [&](const u32x4 (&kr)[C::PIECES], const u32x4 (&vr)[C::PIECES], int n) {
      const int t0 = (lc0 + n) * CH;
      StateTiles<D>& b = sm.buf[n & 1];
      const bool full = t0 + CH <= N;  // uniform; only a head's last chunk can be ragged
#pragma unroll
      for (int i = 0; i < C::PIECES; ++i) {
        const int row = st.r0 + i * C::RP;
        const bool valid = full || t0 + row < N;  // rows past the end contribute nothing
        const u32x4 fk = map_features<ELU1>(kr[i]);
        *reinterpret_cast<u32x4*>(&b.fk[row * C::KROW + st.col]) = valid ? fk : kZero4;
        *reinterpret_cast<u32x4*>(&b.v[row * C::VROW + st.col]) = valid ? vr[i] : kZero4;
      }
    };
    // chunk m travels in set m % 2; a set is reloaded (two chunks ahead) as soon as it is staged.
    // A sub-piece of more than four chunks runs a condition-free lead-in and condition-free
    // steady rounds, so that the compiler's wait counters know exactly which loads are in
    // flight; only its last rounds (and short sub-pieces) test before every load and stage.
    auto lead_in = [&](auto steady) {
      constexpr bool S = decltype(steady)::value;
      load(ka, va, 0);
      if (S || nchunks > 1) load(kb, vb, 1);
      stage(ka, va, 0);
      if (S || nchunks > 2) load(ka, va, 2);
      lds_barrier();
    };
    auto round2 = [&](int n, auto steady) {
      constexpr bool S = decltype(steady)::value;
      if (S || n + 1 < nchunks) stage(kb, vb, n + 1);
      if (S || n + 3 < nchunks) load(kb, vb, n + 3);
      lds_barrier();
      if (!S && n + 1 >= nchunks) return false;
      if (S || n + 2 < nchunks) stage(ka, va, n + 2);
      if (S || n + 4 < nchunks) load(ka, va, n + 4);
      lds_barrier();
      return true;
    };
    int n = 0;
    if (nchunks > 4) {
      lead_in(std::true_type{});
      for (; n + 4 < nchunks; n += 2) round2(n, std::true_type{});
    } else {
      lead_in(std::false_type{});
    }
    for (; n < nchunks; n += 2)
      if (!round2(n, std::false_type{})) break;
    return;
  }
  // ---- consumers ----
  f32x16 sacc[C::ET];
#pragma unroll
  for (int i = 0; i < C::ET; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[i][r] = 0.f;
  float zacc = 0.f;
  lds_barrier();
  for (int n = 0; n < nchunks; ++n) {
    zacc += update_state<D>(sacc, sm.buf[n & 1].fk, sm.buf[n & 1].v, wave, lane);
    lds_barrier();
  }
  float* dst = a.ws_states + (int64_t)q * C::STATE;
  state_store<D>(dst, sacc, wave, lane);
  zacc += __shfl_xor(zacc, 32, 64);
  if (lh == 0) dst[D * D + 32 * wave + ln] = zacc;
}

// (2) Slot j holds the sums over the part of its head that lies in sub-piece j-1.  Inside every
//     head, turn them into running sums: slot j = state of the head just before sub-piece j.
//     Stops after the head's last piece boundary (later slots were not written and are not read).
__global__ __launch_bounds__(256) void linear_prefix_kernel(float* ws, int n_heads, int vcph,
                                                             int sub_chunks, int n_sub, int state_sub,
                                                             int state_floats, int causal) {
  const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int head = blockIdx.y;
  if (x >= state_floats || head >= n_heads) return;
  const int64_t g_lo = (int64_t)head * vcph, g_hi = g_lo + vcph;
  if (!causal) {
    // bidirectional: the head's first slot receives the sum of all its slots
    const int64_t j0 = g_lo / sub_chunks, j1 = g_hi / sub_chunks;
    float tot = 0.f;
    for (int64_t j = j0; j < j1; ++j) tot += ws[j * state_floats + x];
    ws[j0 * state_floats + x] = tot;
    return;
  }
  const int64_t total = (int64_t)n_sub * sub_chunks;
  float run = 0.f;
  for (int64_t j = g_lo / sub_chunks + 1; j < n_sub && j * sub_chunks < g_hi; ++j) {
    const int64_t next_main = (j + state_sub - 1) / state_sub * state_sub * sub_chunks;
    if (next_main >= g_hi || next_main >= total) break;
    float* p = ws + j * state_floats + x;
    run += *p;
    *p = run;
  }
}

// -----------------------------------------------------------------------------------------
// (3) read-out.  Workgroup p walks the chunks of piece p carrying (A, Z); at a head's first
//     chunk the state restarts from zero, at a piece start inside a head from workspace slot p.
//     Waves [0, NWC): MFMA work, denominators, normalise.  Waves [NWC, 2 NWC): load chunk n+2
//     from global memory, apply phi to chunk n+1 and stage it in the other LDS buffer, write
//     chunk n-1's finished rows; the feature map's vector work thus overlaps the matrix work
//     of chunk n on every SIMD.  Two workgroup barriers per chunk: (a) masked products
//     visible, (b) buffers change hands.
// -----------------------------------------------------------------------------------------
//     CAUSAL = false is the bidirectional read-out: the state is the sum over the whole head and
//     never moves, K and V are not touched, and per chunk only the state read-out, phi(q).Z and
//     the normalisation remain (same barriers, same producer/consumer split).
//     EMIT (causal only): every head's (A, Z) after its last token is also written out, for a
//     decode step to continue from; a separate instantiation so that the plain layer pays nothing.
template <int D, bool ELU1, bool CAUSAL, bool EMIT>
__global__ __launch_bounds__(LinCfg<D>::NT, D == 64 ? 2 : 1) void linear_main_kernel(AttnArgs a) {
  using C = LinCfg<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  LinSmem<D>& sm = *reinterpret_cast<LinSmem<D>*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int n_heads = a.B * (a.H - a.H0);
  const int g0 = blockIdx.x * a.piece_chunks;
  const int nchunks = piece_chunk_count(a, g0, n_heads);
  if (nchunks <= 0) return;  // uniform
  const int N = a.N;

  if (wave >= C::NWC) {
    // ---- producers ----
    const Staging<D> st(tid - C::NTC);
    const PieceOffsets<D> qo(st, a.q.sn), ko(st, a.k.sn), vo(st, a.v.sn);
    ChunkCursor<D> cl(a, g0), cs(a, g0), co(a, g0);  // next chunk to load / stage / write out
    // NSETS register sets: chunk m travels in set m % NSETS; a set is reloaded with the chunk
    // NSETS further on as soon as it has been staged
    constexpr int NSETS = GF_MAIN_SETS;
    u32x4 qs[NSETS][C::PIECES], ks[NSETS][C::PIECES], vs[NSETS][C::PIECES];
    int nl = 0, no = 0;  // chunks loaded / written so far
    auto load_q = [&](u32x4 (&qr)[C::PIECES]) { load_chunk<D>(qr, cl.hp.q, cl.t0(), N, qo); };
    auto load_kv = [&](u32x4 (&kr)[C::PIECES], u32x4 (&vr)[C::PIECES]) {
      if constexpr (CAUSAL) {
        const int t0 = cl.t0();
        load_chunk<D>(kr, cl.hp.k, t0, N, ko);
        load_chunk<D>(vr, cl.hp.v, t0, N, vo);
      }
      ++nl;
      cl.next(a, nl < nchunks);
    };
    // phi(Q) of the chunk at `cs` -> buf[n % 2]
    auto stage_q = [&](const u32x4 (&qr)[C::PIECES], int n) {
      ChunkTiles<D>& b = sm.buf[n & 1];
#pragma unroll
      for (int i = 0; i < C::PIECES; ++i) {
        const u32x4 fqv = map_features<ELU1>(qr[i]);
        uint16_t* qd = &b.fq[(st.r0 + i * C::RP) * C::QROW + st.qcol];
        *reinterpret_cast<u32x2*>(qd) = u32x2{fqv[0], fqv[1]};
        *reinterpret_cast<u32x2*>(qd + 8) = u32x2{fqv[2], fqv[3]};
      }
    };
    // phi(K) and V of the chunk at `cs` -> buf[n % 2]; rows past the head's end become zeros
    auto stage_kv = [&](const u32x4 (&kr)[C::PIECES], const u32x4 (&vr)[C::PIECES], int n) {
      if constexpr (CAUSAL) {
        const int t0 = cs.t0();
        ChunkTiles<D>& b = sm.buf[n & 1];
        const bool full = t0 + CH <= N;  // uniform; only a head's last chunk can be ragged
#pragma unroll
        for (int i = 0; i < C::PIECES; ++i) {
          const int row = st.r0 + i * C::RP;
          const bool valid = full || t0 + row < N;
          const u32x4 fk = map_features<ELU1>(kr[i]);
          *reinterpret_cast<u32x4*>(&b.fk[row * C::KROW + st.col]) = valid ? fk : kZero4;
          *reinterpret_cast<u32x4*>(&b.v[row * C::VROW + st.col]) = valid ? vr[i] : kZero4;
        }
      }
      cs.next(a, n + 1 < nchunks);
    };
    // finished rows of the chunk at `co`: LDS -> global, 16 bytes per lane, whole rows per 16 lanes
    auto store_out = [&]() {
      const int t0 = co.t0();
#pragma unroll
      for (int i = 0; i < C::PIECES; ++i) {
        const int row = st.r0 + i * C::RP;
        const u32x4 o = *reinterpret_cast<const u32x4*>(&sm.ot[row * C::OROW + st.col]);
        if (t0 + row < N)
          __builtin_nontemporal_store(
              o, reinterpret_cast<u32x4*>(co.hp.o + (int64_t)(t0 + row) * a.osn + st.col));
      }
      ++no;
      co.next(a, no < nchunks);
    };
    // Per chunk n the consumers run [products, state read-out] (a) [denominators, in-chunk
    // part, state update] (b).  The producers' work for chunk n+1 is split the same way: phi(Q)
    // and its staging before (a); after (a) the write-out of chunk n-1, then phi(K), V and their
    // staging; each set's reload (chunk n+3) follows its staging.  The feature map is applied
    // where a tensor is staged: mapping parts of Q and K one phase early, in their registers, was
    // measured and is 2 % slower.  Two chunks per round (one per register set).
    //
    // The wait counters the compiler derives for a load that sits behind a condition assume it
    // may not have been issued, which makes the waits for older loads cover the newest ones as
    // well.  A piece of more than four chunks therefore runs a condition-free lead-in and
    // condition-free steady rounds; only its last rounds (and short pieces) take the general
    // code with a test in front of every load, stage and write-out.
    constexpr int kGeneral = 0, kFirst = 1, kSteady = 2;
    auto lead_in = [&](auto mode) {
      constexpr bool S = decltype(mode)::value != kGeneral;
#pragma unroll
      for (int i = 0; i < NSETS; ++i)
        if (S || nchunks > i) {
          load_q(qs[i]);
          load_kv(ks[i], vs[i]);
        }
      stage_q(qs[0], 0);
      stage_kv(ks[0], vs[0], 0);
      if (S || nchunks > NSETS) {
        load_q(qs[0]);
        load_kv(ks[0], vs[0]);
      }
      lds_barrier();  // chunk 0 staged
    };
    // while the consumers work on chunk n: stage chunk n + 1 out of its set, reload the set with
    // chunk n + 1 + NSETS, write out chunk n - 1.  False when chunk n was the piece's last.
    auto step = [&](auto set_tag, auto mode, int n) {
      constexpr int SET = decltype(set_tag)::value;
      constexpr int M = decltype(mode)::value;
      constexpr bool S = M != kGeneral;
      if (S || n + 1 < nchunks) stage_q(qs[SET], n + 1);
      if (S || n + 1 + NSETS < nchunks) load_q(qs[SET]);
      lds_barrier();  // (a)
      if (M == kSteady || n > 0) store_out();
      if (S || n + 1 < nchunks) stage_kv(ks[SET], vs[SET], n + 1);
      if (S || n + 1 + NSETS < nchunks) load_kv(ks[SET], vs[SET]);
      lds_barrier();  // (b)
      return S || n + 1 < nchunks;
    };
    // NSETS chunks per round, n a multiple of NSETS: chunk n + 1 + i sits in set (1 + i) % NSETS
    auto round = [&](int n, auto mode) {
      if (!step(std::integral_constant<int, 1 % NSETS>{}, mode, n)) return false;
      if (!step(std::integral_constant<int, 2 % NSETS>{}, mode, n + 1)) return false;
      if constexpr (NSETS == 3)
        if (!step(std::integral_constant<int, 0>{}, mode, n + 2)) return false;
      return true;
    };
    static_assert(NSETS == 2 || NSETS == 3, "rounds are written out for two or three sets");
    int n = 0;
    if (nchunks > 2 * NSETS) {
      lead_in(std::integral_constant<int, kFirst>{});
      round(0, std::integral_constant<int, kFirst>{});
      for (n = NSETS; n + 2 * NSETS < nchunks; n += NSETS) round(n, std::integral_constant<int, kSteady>{});
    } else {
      lead_in(std::integral_constant<int, kGeneral>{});
    }
    for (; n < nchunks; n += NSETS)
      if (!round(n, std::integral_constant<int, kGeneral>{})) break;
    lds_barrier();  // (c) last chunk's rows are in LDS
    store_out();
    return;
  }

  // ---- consumers ----
  // Z lives in LDS as fp32 plus a bf16 hi/lo split, in fq's permuted feature order
  auto put_z = [&](int buf, int zi, float zval) {
    sm.z[buf][zi] = zval;
    const uint16_t hi = (uint16_t)(pack_bf16(zval, 0.f) & 0xffffu);
    sm.zh[buf][zi] = hi;
    sm.zl[buf][zi] = (uint16_t)(pack_bf16(zval - __uint_as_float((uint32_t)hi << 16), 0.f) & 0xffffu);
  };
  f32x16 sacc[C::ET];
  int lc = g0 % a.vcph;  // chunk index inside the current head
#pragma unroll
  for (int ct = 0; ct < C::ET; ++ct)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[ct][r] = 0.f;
  float z0 = 0.f;
  if (CAUSAL ? (lc > 0 && a.ws_states) : a.ws_states != nullptr) {
    const int ls = a.piece_chunks / a.state_sub;
    int j_first, j_last;
    if (CAUSAL) {
      // state carried into this piece: the running sum of its head's sub-piece sums up to here
      j_last = g0 / ls;
      j_first = uses_prefix_kernel(a) ? j_last : (g0 - lc) / ls + 1;
    } else {
      // the state of the whole head: all of its sub-piece sums (or their total in its first slot)
      j_first = (g0 - lc) / ls;
      j_last = uses_prefix_kernel(a) ? j_first : j_first + a.vcph / ls - 1;
    }
    // two sums at a time: their loads are all in flight before the first is added, which halves
    // the number of trips to memory this prologue waits for (an odd one out is read twice and
    // counted once)
    for (int j = j_first; j <= j_last; j += 2) {
      const bool pair = j + 1 <= j_last;
      const float* s0 = a.ws_states + (int64_t)j * C::STATE;
      const float* s1 = a.ws_states + (int64_t)(pair ? j + 1 : j) * C::STATE;
      const float w1 = pair ? 1.f : 0.f;
      float4 t0[C::ET][4], t1[C::ET][4];
#pragma unroll
      for (int ct = 0; ct < C::ET; ++ct) {
        const int off = state_tile_offset<D>(ct, wave, lane);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          t0[ct][g] = reinterpret_cast<const float4*>(s0 + off)[g];
          t1[ct][g] = reinterpret_cast<const float4*>(s1 + off)[g];
        }
      }
      const float za = s0[D * D + 32 * wave + ln], zb = s1[D * D + 32 * wave + ln];
#pragma unroll
      for (int ct = 0; ct < C::ET; ++ct)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          sacc[ct][4 * g + 0] += t0[ct][g].x + w1 * t1[ct][g].x;
          sacc[ct][4 * g + 1] += t0[ct][g].y + w1 * t1[ct][g].y;
          sacc[ct][4 * g + 2] += t0[ct][g].z + w1 * t1[ct][g].z;
          sacc[ct][4 * g + 3] += t0[ct][g].w + w1 * t1[ct][g].w;
        }
      z0 += za + w1 * zb;
    }
  }
  if (lh == 0) {
    put_z(0, 32 * wave + kperm32(ln), z0);
    if (!CAUSAL) put_z(1, 32 * wave + kperm32(ln), z0);   // Z never moves: both buffers hold it
  }
  // the product tile above the diagonal (keys 32.., queries ..31) is never computed: it stays 0
  for (int x = tid; x < 32 * 32 / 8; x += C::NTC)
    *reinterpret_cast<u32x4*>(&sm.pt[(x / 4) * C::PROW + 32 + 8 * (x % 4)]) = kZero4;
  if (tid < CH) sm.den[tid] = 1.f;  // read by the first pass of the loop before any row exists
  __builtin_amdgcn_s_setprio(2);  // matrix waves first; the staging waves fill the gaps
  lds_barrier();  // chunk 0 staged, Z visible

  constexpr int PPT = C::NTC / CH;  // threads per query in the denominator
  // finished rows: divide by the denominators and hand them to the producers through LDS
  auto normalise = [&](const f32x16 (&num)[2]) {
#pragma unroll
    for (int tq = 0; tq < 2; ++tq) {
      const float inv = __builtin_amdgcn_rcpf(sm.den[32 * tq + ln]);
      uint16_t* orow = &sm.ot[(32 * tq + ln) * C::OROW + 32 * wave + 4 * lh];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(num[tq][4 * g + 0] * inv, num[tq][4 * g + 1] * inv);
        pk[1] = pack_bf16(num[tq][4 * g + 2] * inv, num[tq][4 * g + 3] * inv);
        *reinterpret_cast<u32x2*>(orow + 8 * g) = pk;
      }
    }
  };
  // Masked products P^T[key][query] = phi(k_key).phi(q_query), key <= query, are three 32x32
  // tiles (the fourth lies above the diagonal); tile t goes to wave t % NWC.  A wave left
  // without a tile repeats tile 0 and stores the same values to the same place, which keeps the
  // code free of branches: the products and the state read-out then interleave in one block and
  // neither chain of dependent matrix instructions has to wait for its own results.
  constexpr int NTILE = (3 + C::NWC - 1) / C::NWC;  // product tiles per wave
  constexpr int KS = D / 16;                        // contraction steps per product tile
  constexpr int G1N = NTILE * KS;                   // product steps per chunk
  static_assert(KS == 2 * C::ET, "a product tile and the read-out take the same contraction steps");
  f32x16 num[2];
#pragma unroll
  for (int tq = 0; tq < 2; ++tq)
#pragma unroll
    for (int r = 0; r < 16; ++r) num[tq][r] = 0.f;
  for (int n = 0; n < nchunks; ++n) {
    const int zc = n & 1;
    const ChunkTiles<D>& b = sm.buf[n & 1];
    const bool head_ends = (lc + 1 == a.vcph);  // the next chunk starts a new head from zero
    const bool head_done = (lc + 1 == a.cph);   // this chunk holds the head's last token
    lc = head_ends ? 0 : lc + 1;

    f32x16 p[NTILE];
    int tk[NTILE], tqa[NTILE];
#pragma unroll
    for (int rep = 0; rep < NTILE; ++rep) {
      const int tile = (wave + rep * C::NWC) % 3;
      tk[rep] = tile == 2 ? 1 : 0;
      tqa[rep] = tile == 0 ? 0 : 1;
    }
    // operands are fetched from LDS one step ahead of the matrix instructions that use them
    struct StepOps {
      bf16x8 kt, q0, q1;
    };
    auto fetch = [&](int i) {
      StepOps o;
      const int rep = i / KS, ks = i % KS;
      // k-slot 8*lh + 4*g + j of this step is feature 16*ks + 8*g + 4*lh + j
      if constexpr (CAUSAL) {
        const uint16_t* kr = &b.fk[(32 * tk[rep] + ln) * C::KROW + 16 * ks + 4 * lh];
        const u32x2 k0 = *reinterpret_cast<const u32x2*>(kr);
        const u32x2 k1 = *reinterpret_cast<const u32x2*>(kr + 8);
        o.kt = as_bf16x8(u32x4{k0[0], k0[1], k1[0], k1[1]});
      }
      // phi(Q) rows 0..31 and 32..63, features of contraction step ks: the read-out step
      // 2*ct + kb = ks uses both, the product tile the one of its query half
      o.q0 = lds_read16(&b.fq[ln * C::QROW + 16 * ks + 8 * lh]);
      o.q1 = lds_read16(&b.fq[(32 + ln) * C::QROW + 16 * ks + 8 * lh]);
      return o;
    };
    constexpr int PD = 2;  // steps between an operand fetch and its use (measured: 2 beats 1, 3 and 4)
    constexpr int NSTEP = CAUSAL ? G1N : KS;   // without product tiles only the read-out steps remain
    StepOps ops[NSTEP];
#pragma unroll
    for (int i = 0; i < PD && i < NSTEP; ++i) ops[i] = fetch(i);
    __builtin_amdgcn_sched_barrier(0);
    // rows of the previous chunk (at n = 0: zeros over den = 1, never written out), while the
    // first operands are on their way
    normalise(num);
#pragma unroll
    for (int tq = 0; tq < 2; ++tq)
#pragma unroll
      for (int r = 0; r < 16; ++r) num[tq][r] = 0.f;
#pragma unroll
    for (int rep = 0; rep < NTILE; ++rep)
#pragma unroll
      for (int r = 0; r < 16; ++r) p[rep][r] = 0.f;
#pragma unroll
    for (int i = 0; i < NSTEP; ++i) {
      if (i + PD < NSTEP) ops[i + PD] = fetch(i + PD);
      const StepOps& cur = ops[i];
      if constexpr (CAUSAL) p[i / KS] = mfma32(cur.kt, tqa[i / KS] ? cur.q1 : cur.q0, p[i / KS]);
      if (i / KS == 0) {
        // num^T = A^T phiQ^T with A straight from the state registers
        const int ct = i / 2, kb_ = i % 2;
        u32x4 sw;
#pragma unroll
        for (int x = 0; x < 4; ++x)
          sw[x] = pack_bf16(sacc[ct][8 * kb_ + 2 * x], sacc[ct][8 * kb_ + 2 * x + 1]);
        const bf16x8 sa = as_bf16x8(sw);
        num[0] = mfma32(sa, cur.q0, num[0]);
        num[1] = mfma32(sa, cur.q1, num[1]);
      }
      __builtin_amdgcn_sched_barrier(0);  // keep the fetches PD steps ahead of their use
    }
#pragma unroll
    for (int rep = 0; CAUSAL && rep < NTILE; ++rep) {
      // on the diagonal tile key row 8*(r/4) + 4*lh + r%4 must not exceed query column ln
      const int top = (tk[rep] == tqa[rep] ? ln : CH) - 4 * lh;
#pragma unroll
      for (int r = 0; r < 16; ++r) p[rep][r] = (8 * (r / 4) + (r % 4) > top) ? 0.f : p[rep][r];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(p[rep][4 * g + 0], p[rep][4 * g + 1]);
        pk[1] = pack_bf16(p[rep][4 * g + 2], p[rep][4 * g + 3]);
        *reinterpret_cast<u32x2*>(
            &sm.pt[(32 * tqa[rep] + ln) * C::PROW + 32 * tk[rep] + 8 * g + 4 * lh]) = pk;
      }
    }
    lds_barrier();  // (a) products visible

    // Over the chunk's tokens, 16 at a time, with one V^T operand serving both contractions:
    // num^T += V^T P^T (the first 32 queries see only the first 32 keys) and the state update
    // A += phiK^T V, Z += colsum(phiK); a new head starts from zero instead.  Operands are
    // fetched PDB steps ahead; the denominators are computed while the first ones arrive.
    {
      struct TokOps {
        bf16x8 vt, pb[2], fa[C::ET], fz;
      };
      auto fetch_tok = [&](int kk) {
        TokOps o;
        o.vt = lds_operand_tr(b.v, C::VROW, 16 * kk + 8 * lh, 16 * kk + 8 * lh + 4, 32 * wave, lane);
#pragma unroll
        for (int tq = 0; tq < 2; ++tq)
          if (16 * kk < 32 * (tq + 1))
            o.pb[tq] = lds_read16(&sm.pt[(32 * tq + ln) * C::PROW + 16 * kk + 8 * lh]);
#pragma unroll
        for (int ct = 0; ct < C::ET; ++ct)
          o.fa[ct] = lds_operand_tr(b.fk, C::KROW, 16 * kk + 8 * lh, 16 * kk + 8 * lh + 4, 32 * ct, lane);
        // the wave's own feature tile, for colsum(phiK): picked out of fa[] with wave-uniform
        // selects (a dozen vector moves; the LDS pipeline is the busier unit, a second read of the
        // tile costs it 9 cycles per wave)
        o.fz = o.fa[0];
#pragma unroll
        for (int ct = 1; ct < C::ET; ++ct) o.fz = wave == ct ? o.fa[ct] : o.fz;
        return o;
      };
      constexpr int NK = CAUSAL ? CH / 16 : 0, PDB = 2;   // no token work in the bidirectional read-out
      TokOps tok[NK > 0 ? NK : 1];
#pragma unroll
      for (int kk = 0; kk < PDB && kk < NK; ++kk) tok[kk] = fetch_tok(kk);
      __builtin_amdgcn_sched_barrier(0);
      // denominator: rowsum of the (rounded) products + phi(q).Z_prev, PPT threads per query,
      // all on packed bf16 pairs
      {
        const int qrow = tid / PPT, part = tid % PPT;
        constexpr int KW = CH / PPT;  // product slots per thread
        constexpr int CW = D / PPT;   // features per thread
        float s = 0.f;
#pragma unroll
        for (int x = 0; CAUSAL && x < KW; x += 8) {  // the never-visible tile holds zeros
          const u32x4 pv = *reinterpret_cast<const u32x4*>(&sm.pt[qrow * C::PROW + KW * part + x]);
#pragma unroll
          for (int w = 0; w < 4; ++w) s = dot2_bf16(pv[w], kOnesBf16x2, s);
        }
#pragma unroll
        for (int x = 0; x < CW; x += 8) {
          const u32x4 qv = *reinterpret_cast<const u32x4*>(&b.fq[qrow * C::QROW + CW * part + x]);
          const u32x4 zh = *reinterpret_cast<const u32x4*>(&sm.zh[zc][CW * part + x]);
          const u32x4 zl = *reinterpret_cast<const u32x4*>(&sm.zl[zc][CW * part + x]);
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            s = dot2_bf16(qv[w], zh[w], s);
            s = dot2_bf16(qv[w], zl[w], s);
          }
        }
#pragma unroll
        for (int o = 1; o < PPT; o <<= 1) s += __shfl_xor(s, o, 64);
        sm.den[qrow] = s + a.eps;  // every part holds the same sum
      }
      float zs = 0.f;
#pragma unroll
      for (int kk = 0; kk < NK; ++kk) {
        if (kk + PDB < NK) tok[kk + PDB] = fetch_tok(kk + PDB);
        const TokOps& cur = tok[kk];
#pragma unroll
        for (int tq = 0; tq < 2; ++tq)
          if (16 * kk < 32 * (tq + 1)) num[tq] = mfma32(cur.vt, cur.pb[tq], num[tq]);
        zs = sum8_bf16(cur.fz, zs);
#pragma unroll
        for (int ct = 0; ct < C::ET; ++ct) sacc[ct] = mfma32(cur.fa[ct], cur.vt, sacc[ct]);
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (CAUSAL) {
        zs += __shfl_xor(zs, 32, 64);
        const int zi = 32 * wave + kperm32(ln);
        const float znew = sm.z[zc][zi] + zs;
        if (EMIT && head_done) {
          // the state after the head's last token, for a decode step to continue from:
          // A row-major [feature][value] (lane = value column, register = feature row), then Z
          float* fs = a.final_state + (int64_t)((g0 + n) / a.vcph) * C::STATE;
          // four stores at a time: left to itself the scheduler forms all 64 addresses first and
          // spills half of the kernel's registers around this rarely taken block
#pragma unroll
          for (int ct = 0; ct < C::ET; ++ct)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              float* row = fs + (32 * ct + 8 * g + 4 * lh) * D + 32 * wave + ln;
#pragma unroll
              for (int x = 0; x < 4; ++x) row[x * D] = sacc[ct][4 * g + x];
              __builtin_amdgcn_sched_barrier(0);
            }
          if (lh == 0) fs[D * D + 32 * wave + ln] = znew;
        }
        if (lh == 0) put_z(zc ^ 1, zi, head_ends ? 0.f : znew);
        if (head_ends) {
#pragma unroll
          for (int ct = 0; ct < C::ET; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[ct][r] = 0.f;
        }
      }
    }
    lds_barrier();  // (b) denominators visible; this chunk's tiles are free again
  }
  normalise(num);  // the last chunk's rows
  lds_barrier();  // (c)
}

template <int D> hipError_t launch_state_t(const AttnArgs& a, hipStream_t s) {
  using C = LinCfg<D>;
  const int heads = a.B * (a.H - a.H0);
  const int smem = (int)sizeof(StateSmem<D>);
  const dim3 grid(a.n_pieces * a.state_sub - (a.causal ? 1 : 0)), block(C::NT);
  hipError_t e;
  if (a.phi == 0) {
    if ((e = allow_lds(linear_state_kernel<D, true>, smem)) != hipSuccess) return e;
    linear_state_kernel<D, true><<<grid, block, smem, s>>>(a);
  } else {
    if ((e = allow_lds(linear_state_kernel<D, false>, smem)) != hipSuccess) return e;
    linear_state_kernel<D, false><<<grid, block, smem, s>>>(a);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (uses_prefix_kernel(a)) {
    linear_prefix_kernel<<<dim3((C::STATE + 255) / 256, heads), dim3(256), 0, s>>>(
        a.ws_states, heads, a.vcph, a.piece_chunks / a.state_sub, a.n_pieces * a.state_sub,
        a.state_sub, C::STATE, a.causal);
    e = hipGetLastError();
  }
  return e;
}

template <int D> hipError_t launch_main_t(const AttnArgs& a, hipStream_t s) {
  using C = LinCfg<D>;
  const int smem = (int)sizeof(LinSmem<D>);
  const dim3 grid(a.n_pieces), block(C::NT);
  hipError_t e = hipSuccess;
  auto launch = [&](auto kern) {
    e = allow_lds(kern, smem);
    if (e == hipSuccess) kern<<<grid, block, smem, s>>>(a);
  };
  if (a.causal && a.final_state) {
    if (a.phi == 0) launch(linear_main_kernel<D, true, true, true>);
    else launch(linear_main_kernel<D, false, true, true>);
  } else if (a.causal) {
    if (a.phi == 0) launch(linear_main_kernel<D, true, true, false>);
    else launch(linear_main_kernel<D, false, true, false>);
  } else {
    if (a.phi == 0) launch(linear_main_kernel<D, true, false, false>);
    else launch(linear_main_kernel<D, false, false, false>);
  }
  return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace

hipError_t launch_linear_state_mfma(const AttnArgs& a, hipStream_t s) {
  if (a.H - a.H0 <= 0 || a.N <= 0 || a.B <= 0 || !a.ws_states) return hipSuccess;
  if (a.causal && a.n_pieces <= 1) return hipSuccess;
  return a.d == 64 ? launch_state_t<64>(a, s) : launch_state_t<128>(a, s);
}

hipError_t launch_linear_main_mfma(const AttnArgs& a, hipStream_t s) {
  if (a.H - a.H0 <= 0 || a.N <= 0 || a.B <= 0 || a.n_pieces <= 0) return hipSuccess;
  return a.d == 64 ? launch_main_t<64>(a, s) : launch_main_t<128>(a, s);
}

}  // namespace gformer
