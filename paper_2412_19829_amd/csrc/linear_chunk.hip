// Causal linear attention heads (section III-C, Algorithm 1) by chunks of C = 64, 128 or 256
// tokens on bf16 matrix cores: the read-out kernel for any of these chunk sizes.
//
// Algorithm 1 adds token i to (A, Z) and then reads row i.  By chunks of C tokens, with A_prev,
// Z_prev the sums over everything before the chunk:
//     num = tril(phiQ_c phiK_c^T) V_c + phiQ_c A_prev ,  den = rowsum(tril(phiQ_c phiK_c^T)) + phiQ_c.Z_prev
//     A += phiK_c^T V_c ,  Z += colsum(phiK_c)                      (once per chunk)
// The chunk size changes the work, not the result: the masked C x C product costs 2 C d FLOP per
// token next to the 4 d^2 of the two state products, while the state moves C / 64 times less often.
//
// One workgroup walks one piece (a run of whole chunks of one head) with the chunk's phi(Q),
// phi(K) and V resident in LDS.  The chunk's queries are taken in strips of 64: the strip's
// masked products with keys 0 .. 64 (s+1) - 1 of the chunk go through LDS as bf16, then every
// matrix wave contracts them with V for its 32 value columns and adds phiQ A_prev straight from
// its state registers (a lane's accumulator registers are the k-slots of an MFMA operand; phi(Q)
// is stored with its feature index permuted to match).  After the last strip the state takes the
// whole chunk in one contraction.
//
// Waves [0, NWC): matrix work, denominators, normalisation.  Waves [NWC, 2 NWC): they hold the
// next chunk in registers while the current one is computed (single-buffered tiles: C = 128 at
// d = 128 fills LDS), map and stage it when the tiles are free, and write finished rows.
// The kernel with C fixed at 64 in linear_mfma.hip double-buffers its tiles and overlaps the
// staging with the matrix work; this one is the general form, measured against it.
#include "linear_common.hpp"

namespace gformer {
namespace {

template <int D, int C> struct ChunkCfg {
  using L = LinCfg<D>;
  static constexpr int M = C / CH;           // strips of 64 queries per chunk
  // V rows: transpose reads only; the narrower stride keeps C = 256 at d = 64 inside 160 KB
  static constexpr int VROW = (D == 64 && C == 256) ? D + 8 : L::VROW;
  static constexpr int PROW = C + 8;         // masked products [query][key]: 4 dwords mod 64
};

template <int D, int C> struct ChunkSmem {
  using L = LinCfg<D>;
  using G = ChunkCfg<D, C>;
  uint16_t fq[C * L::QROW];     // phi(Q), feature index permuted by kperm32 inside 32-groups
  uint16_t fk[C * L::KROW];     // phi(K); rows past the head's end are zeros
  uint16_t v[C * G::VROW];      // V; rows past the head's end are zeros
  uint16_t pt[CH * G::PROW];    // one strip's masked products, [query][key]
  uint16_t ot[CH * L::OROW];    // one strip's finished rows, [query][value]
  float z[D];                   // Z in fq's permuted feature order
  uint16_t zh[D], zl[D];        // bf16(Z), bf16(Z - bf16(Z)) for the packed dot products
  float den[CH];
};

template <int D, int C, bool ELU1>
__global__ __launch_bounds__(LinCfg<D>::NT, 1) void linear_chunk_kernel(AttnArgs a) {
  using L = LinCfg<D>;
  using G = ChunkCfg<D, C>;
  constexpr int M = G::M;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  ChunkSmem<D, C>& sm = *reinterpret_cast<ChunkSmem<D, C>*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int n_heads = a.B * (a.H - a.H0);
  const int g0 = blockIdx.x * a.piece_chunks;             // in strips of 64 tokens
  const int nsub = piece_chunk_count(a, g0, n_heads);     // strips of this piece
  if (nsub <= 0) return;  // uniform
  // pieces of this kernel never straddle heads and start on a chunk boundary of their head
  const int head = g0 / a.vcph, lc0 = g0 % a.vcph;
  const HeadPtrs<D> hp = head_ptrs<D>(a, head);
  const int N = a.N;
  const int nmac = (nsub + M - 1) / M;                    // chunks of this piece

  if (wave >= L::NWC) {
    // ---- producers ----
    const Staging<D> st(tid - L::NTC);
    const PieceOffsets<D> qo(st, a.q.sn), ko(st, a.k.sn), vo(st, a.v.sn);
    u32x4 qr[M][L::PIECES], kr[M][L::PIECES], vr[M][L::PIECES];
    auto load = [&](int mc) {
#pragma unroll
      for (int s = 0; s < M; ++s) {
        // a strip past the piece's end repeats the last one (in bounds; staged as zeros)
        const int t0 = (lc0 + min(mc * M + s, nsub - 1)) * CH;
        load_chunk<D>(qr[s], hp.q, t0, N, qo);
        load_chunk<D>(kr[s], hp.k, t0, N, ko);
        load_chunk<D>(vr[s], hp.v, t0, N, vo);
      }
    };
    auto stage = [&](int mc) {
#pragma unroll
      for (int s = 0; s < M; ++s) {
        const int sub = mc * M + s;
        const int t0 = (lc0 + sub) * CH;
        const bool live = sub < nsub;   // uniform
#pragma unroll
        for (int i = 0; i < L::PIECES; ++i) {
          const int row = st.r0 + i * L::RP;
          const bool valid = live && t0 + row < N;   // rows past the end contribute nothing
          const u32x4 fqv = map_features<ELU1>(qr[s][i]);
          uint16_t* qd = &sm.fq[(CH * s + row) * L::QROW + st.qcol];
          *reinterpret_cast<u32x2*>(qd) = u32x2{fqv[0], fqv[1]};
          *reinterpret_cast<u32x2*>(qd + 8) = u32x2{fqv[2], fqv[3]};
          const u32x4 fkv = map_features<ELU1>(kr[s][i]);
          *reinterpret_cast<u32x4*>(&sm.fk[(CH * s + row) * L::KROW + st.col]) = valid ? fkv : kZero4;
          *reinterpret_cast<u32x4*>(&sm.v[(CH * s + row) * G::VROW + st.col]) = valid ? vr[s][i] : kZero4;
        }
      }
    };
    auto store_out = [&](int sub) {
      const int t0 = (lc0 + sub) * CH;
#pragma unroll
      for (int i = 0; i < L::PIECES; ++i) {
        const int row = st.r0 + i * L::RP;
        const u32x4 o = *reinterpret_cast<const u32x4*>(&sm.ot[row * L::OROW + st.col]);
        if (t0 + row < N)
          __builtin_nontemporal_store(
              o, reinterpret_cast<u32x4*>(hp.o + (int64_t)(t0 + row) * a.osn + st.col));
      }
    };
    load(0);
    stage(0);
    if (nmac > 1) load(1);
    lds_barrier();  // (e) chunk 0 staged
    for (int mc = 0; mc < nmac; ++mc) {
      const int ns = min(M, nsub - mc * M);
      for (int s = 0; s < ns; ++s) {
        lds_barrier();  // (a) products visible
        lds_barrier();  // (b) denominators visible
        lds_barrier();  // (c) the strip's rows are in LDS
        store_out(mc * M + s);
      }
      lds_barrier();    // (d) the state has taken the chunk: its tiles are free
      if (mc + 1 < nmac) {
        stage(mc + 1);
        if (mc + 2 < nmac) load(mc + 2);
      }
      lds_barrier();    // (e) next chunk staged
    }
    return;
  }

  // ---- consumers ----
  auto put_z = [&](int zi, float zval) {
    sm.z[zi] = zval;
    const uint16_t hi = (uint16_t)(pack_bf16(zval, 0.f) & 0xffffu);
    sm.zh[zi] = hi;
    sm.zl[zi] = (uint16_t)(pack_bf16(zval - __uint_as_float((uint32_t)hi << 16), 0.f) & 0xffffu);
  };
  f32x16 sacc[L::ET];
#pragma unroll
  for (int ct = 0; ct < L::ET; ++ct)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[ct][r] = 0.f;
  float z0 = 0.f;
  if (lc0 > 0 && a.ws_states) {
    // the state carried into this piece: the running sum of its head's sub-piece sums up to here
    // (one slot when the prefix kernel has run, else the sums in front of the piece, added here)
    const int ls = a.piece_chunks / a.state_sub;
    const int j_last = g0 / ls;
    const int j_first = uses_prefix_kernel(a) ? j_last : (g0 - lc0) / ls + 1;
    for (int j = j_first; j <= j_last; ++j) {
      const float* src = a.ws_states + (int64_t)j * L::STATE;
      state_add<D>(sacc, src, wave, lane);
      z0 += src[D * D + 32 * wave + ln];
    }
  }
  const int zi = 32 * wave + kperm32(ln);
  if (lh == 0) put_z(zi, z0);
  lds_barrier();  // (e) chunk 0 staged, Z visible

  constexpr int PPT = L::NTC / CH;   // threads per query in the denominator
  constexpr int KS = D / 16;         // contraction steps over the features
  for (int mc = 0; mc < nmac; ++mc) {
    const int ns = min(M, nsub - mc * M);
    for (int s = 0; s < ns; ++s) {
      // ---- (A) masked products of the strip's queries with keys 0 .. 64 (s+1) - 1 of the chunk:
      //      32 x 32 tiles P^T[key tile kt][query tile qt], dealt to the matrix waves in turn.  The
      //      two tiles of the chunk's diagonal block that the mask cuts are masked per element; the
      //      tile above the diagonal comes out as zeros.
      const int ntile = 4 * (s + 1);
      for (int t = wave; t < ntile; t += L::NWC) {
        const int kt = t >> 1, qt = t & 1;
        f32x16 p;
#pragma unroll
        for (int r = 0; r < 16; ++r) p[r] = 0.f;
        const uint16_t* krow = &sm.fk[(32 * kt + ln) * L::KROW + 4 * lh];
        const uint16_t* qrow = &sm.fq[(CH * s + 32 * qt + ln) * L::QROW + 8 * lh];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          // k-slot 8*lh + 4*g + j of this step is feature 16*ks + 8*g + 4*lh + j
          const u32x2 k0 = *reinterpret_cast<const u32x2*>(krow + 16 * ks);
          const u32x2 k1 = *reinterpret_cast<const u32x2*>(krow + 16 * ks + 8);
          const bf16x8 kop = as_bf16x8(u32x4{k0[0], k0[1], k1[0], k1[1]});
          p = mfma32(kop, lds_read16(qrow + 16 * ks), p);
        }
        // register r is key row 8*(r/4) + 4*lh + r%4 of the tile, the lane's column is query ln:
        // inside the diagonal block a key must not come after its query
        const int top = kt >= 2 * s ? 32 * qt + ln - 32 * (kt - 2 * s) - 4 * lh : CH;
#pragma unroll
        for (int r = 0; r < 16; ++r) p[r] = (8 * (r / 4) + (r % 4) > top) ? 0.f : p[r];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 pk;
          pk[0] = pack_bf16(p[4 * g + 0], p[4 * g + 1]);
          pk[1] = pack_bf16(p[4 * g + 2], p[4 * g + 3]);
          *reinterpret_cast<u32x2*>(&sm.pt[(32 * qt + ln) * G::PROW + 32 * kt + 8 * g + 4 * lh]) = pk;
        }
      }
      lds_barrier();  // (a)

      // ---- (B) denominators: rowsum of the rounded products + phi(q).Z_prev, PPT threads per
      //      query, all on packed bf16 pairs
      {
        const int qrow = tid / PPT, part = tid % PPT;
        constexpr int CW = D / PPT;   // features per thread
        float acc = 0.f;
        for (int x = 8 * part; x < CH * (s + 1); x += 8 * PPT) {
          const u32x4 pv = *reinterpret_cast<const u32x4*>(&sm.pt[qrow * G::PROW + x]);
#pragma unroll
          for (int w = 0; w < 4; ++w) acc = dot2_bf16(pv[w], kOnesBf16x2, acc);
        }
#pragma unroll
        for (int x = 0; x < CW; x += 8) {
          const u32x4 qv = *reinterpret_cast<const u32x4*>(&sm.fq[(CH * s + qrow) * L::QROW + CW * part + x]);
          const u32x4 zh = *reinterpret_cast<const u32x4*>(&sm.zh[CW * part + x]);
          const u32x4 zl = *reinterpret_cast<const u32x4*>(&sm.zl[CW * part + x]);
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            acc = dot2_bf16(qv[w], zh[w], acc);
            acc = dot2_bf16(qv[w], zl[w], acc);
          }
        }
#pragma unroll
        for (int o = 1; o < PPT; o <<= 1) acc += __shfl_xor(acc, o, 64);
        sm.den[qrow] = acc + a.eps;   // every part holds the same sum
      }
      // numerators for this wave's 32 value columns: num^T = V^T P^T over the strip's keys, 16 at
      // a time, plus A^T phiQ^T with A straight from the state registers
      f32x16 num[2];
#pragma unroll
      for (int tq = 0; tq < 2; ++tq)
#pragma unroll
        for (int r = 0; r < 16; ++r) num[tq][r] = 0.f;
      for (int kk = 0; kk < 4 * (s + 1); ++kk) {
        const bf16x8 vt =
            lds_operand_tr(sm.v, G::VROW, 16 * kk + 8 * lh, 16 * kk + 8 * lh + 4, 32 * wave, lane);
#pragma unroll
        for (int tq = 0; tq < 2; ++tq)
          num[tq] = mfma32(vt, lds_read16(&sm.pt[(32 * tq + ln) * G::PROW + 16 * kk + 8 * lh]), num[tq]);
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int ct = ks / 2, kb = ks % 2;
        u32x4 sw;
#pragma unroll
        for (int x = 0; x < 4; ++x)
          sw[x] = pack_bf16(sacc[ct][8 * kb + 2 * x], sacc[ct][8 * kb + 2 * x + 1]);
        const bf16x8 sa = as_bf16x8(sw);
#pragma unroll
        for (int tq = 0; tq < 2; ++tq)
          num[tq] = mfma32(sa, lds_read16(&sm.fq[(CH * s + 32 * tq + ln) * L::QROW + 16 * ks + 8 * lh]),
                           num[tq]);
      }
      lds_barrier();  // (b)

      // ---- (C) divide and hand the rows to the producers through LDS
#pragma unroll
      for (int tq = 0; tq < 2; ++tq) {
        const float inv = __builtin_amdgcn_rcpf(sm.den[32 * tq + ln]);
        uint16_t* orow = &sm.ot[(32 * tq + ln) * L::OROW + 32 * wave + 4 * lh];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 pk;
          pk[0] = pack_bf16(num[tq][4 * g + 0] * inv, num[tq][4 * g + 1] * inv);
          pk[1] = pack_bf16(num[tq][4 * g + 2] * inv, num[tq][4 * g + 3] * inv);
          *reinterpret_cast<u32x2*>(orow + 8 * g) = pk;
        }
      }
      lds_barrier();  // (c)
    }

    // ---- (D) the state takes the whole chunk: A += phiK^T V, Z += colsum(phiK)
    float zs = 0.f;
#pragma unroll 2
    for (int kk = 0; kk < C / 16; ++kk) {
      const bf16x8 vt =
          lds_operand_tr(sm.v, G::VROW, 16 * kk + 8 * lh, 16 * kk + 8 * lh + 4, 32 * wave, lane);
      bf16x8 fa[L::ET];
#pragma unroll
      for (int ct = 0; ct < L::ET; ++ct)
        fa[ct] = lds_operand_tr(sm.fk, L::KROW, 16 * kk + 8 * lh, 16 * kk + 8 * lh + 4, 32 * ct, lane);
      bf16x8 fz = fa[0];   // the wave's own feature tile, for colsum(phiK)
#pragma unroll
      for (int ct = 1; ct < L::ET; ++ct) fz = wave == ct ? fa[ct] : fz;
      zs = sum8_bf16(fz, zs);
#pragma unroll
      for (int ct = 0; ct < L::ET; ++ct) sacc[ct] = mfma32(fa[ct], vt, sacc[ct]);
    }
    zs += __shfl_xor(zs, 32, 64);
    if (lh == 0) put_z(zi, sm.z[zi] + zs);
    lds_barrier();  // (d)
    lds_barrier();  // (e)
  }
}

template <int D, int C> hipError_t launch_chunk_t(const AttnArgs& a, hipStream_t s) {
  const int smem = (int)sizeof(ChunkSmem<D, C>);
  static_assert(sizeof(ChunkSmem<D, C>) <= 160 * 1024, "one workgroup's tiles must fit the LDS of a compute unit");
  const dim3 grid(a.n_pieces), block(LinCfg<D>::NT);
  hipError_t e = hipSuccess;
  auto launch = [&](auto kern) {
    e = allow_lds(kern, smem);
    if (e == hipSuccess) kern<<<grid, block, smem, s>>>(a);
  };
  if (a.phi == 0) launch(linear_chunk_kernel<D, C, true>);
  else launch(linear_chunk_kernel<D, C, false>);
  return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace

bool linear_chunk_supported(int d, int chunk) {
  if (chunk != 64 && chunk != 128 && chunk != 256) return false;
  return d == 64 || (d == 128 && chunk <= 128);   // C = 256 at d = 128 would need 300 KB of LDS
}

// Read-out of the causal linear heads by chunks of a.chunk tokens.  The plan must hold uniform
// segments per head whose length is a multiple of the chunk (the planner's rule for this kernel).
hipError_t launch_linear_chunk(const AttnArgs& a, hipStream_t s) {
  if (a.H - a.H0 <= 0 || a.N <= 0 || a.B <= 0 || a.n_pieces <= 0) return hipSuccess;
  const int m = a.chunk / CH;
  if (!a.causal || !linear_chunk_supported(a.d, a.chunk) || a.piece_chunks % m != 0 ||
      a.vcph % a.piece_chunks != 0)
    return hipErrorInvalidValue;
  if (a.d == 64) {
    if (a.chunk == 64) return launch_chunk_t<64, 64>(a, s);
    if (a.chunk == 128) return launch_chunk_t<64, 128>(a, s);
    return launch_chunk_t<64, 256>(a, s);
  }
  if (a.chunk == 64) return launch_chunk_t<128, 64>(a, s);
  return launch_chunk_t<128, 128>(a, s);
}

}  // namespace gformer
