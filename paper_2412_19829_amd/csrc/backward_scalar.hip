// Backward pass of the causal layer, plain-FMA kernels (fp32 arithmetic on fp32 or bf16 storage).
//
// The paper trains its models (sections IV-B to IV-D) but prints no backward formulas; these are
// the derivatives of its two definitions.
//
// Nothing of the forward pass is taken as input: the forward result would arrive rounded to the
// storage type, and the differences below cancel too strongly for that.
//
// Windowed head (section III-B, Eq. 1), s_ij = scale q_i.k_j, p_ij = softmax over the window,
// o_i = sum_j p_ij v_j.  With D_i = dO_i.o_i = sum_j p_ij dO_i.v_j and ds_ij = p_ij (dO_i.v_j - D_i):
//   dq_i = scale sum_j ds_ij k_j,  dk_j = scale sum_i ds_ij q_i,  dv_j = sum_i p_ij dO_i.
// Two kernels: one wave per query row (recomputes the row's log-sum-exp, writes dq and leaves
// (lse_i, D_i) in the workspace), then one wave per key row over the queries that see it.
//
// Linear head (section II-B's ratio, Algorithm 1's running sums), fq = phi(q), fk = phi(k),
// den_i = fq_i.Z_i + eps, o_i = fq_i^T A_i / den_i.  With g_i = dO_i / den_i and
// c_i = (dO_i.o_i) / den_i = g_i.(fq_i^T A_i) / den_i:
//   dfq_i = A_i g_i - c_i Z_i                          (A_i, Z_i: sums over j <= i, forward scan)
//   dfk_j = B_j v_j - Y_j,  dv_j = B_j^T fk_j          (B_j = sum_{i>=j} fq_i g_i^T,
//                                                       Y_j = sum_{i>=j} c_i fq_i, reverse scan)
//   dq = dfq * phi'(q),  dk = dfk * phi'(k).
// Two kernels, one workgroup per head each, chunks of 32 tokens: inside a chunk the masked
// quadratic form, across chunks the carried d x d state in LDS, as in the forward kernel.
#include "common.hpp"
#include "scalar_util.hpp"

namespace gformer {

namespace {

constexpr int kBwdThreads = 256;
constexpr int kBwdRows = 16;   // rows per workgroup in the windowed kernels (4 per wave)

// ---------------------------------------------------------------------------------------
// windowed heads, per query row: dq_i, and (lse_i, D_i) for the key-row kernel
// grid = (ceil(N / kBwdRows), H0, B), block = 256
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kBwdThreads) void windowed_bwd_q_kernel(BwdArgs a) {
  constexpr int CPL = D / 64;  // columns per lane
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int h = blockIdx.y, b = blockIdx.z;
  const int64_t qoff = b * a.q.sb + h * a.q.sh;
  const int64_t koff = b * a.k.sb + h * a.k.sh;
  const int64_t voff = b * a.v.sb + h * a.v.sh;
  const int64_t ooff = b * a.dout.sb + h * a.dout.sh;
  float* ws = a.ws + ((int64_t)b * a.H + h) * a.N * 2;
  constexpr int rows_per_wave = kBwdRows / (kBwdThreads / 64);

  for (int r = 0; r < rows_per_wave; ++r) {
    const int i = blockIdx.x * kBwdRows + wave * rows_per_wave + r;
    if (i >= a.N) break;  // uniform per wave
    float qreg[CPL], doreg[CPL];
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc) {
      qreg[cc] = Storage<T>::load(a.q.base, qoff + i * a.q.sn + cc * 64 + lane);
      doreg[cc] = Storage<T>::load(a.dout.base, ooff + i * a.dout.sn + cc * 64 + lane);
    }
    const int lo = max(0, i - a.wleft), hi = min(a.N - 1, i + a.wright);
    // lane j's score against this query; lanes past the last visible key read that key again
    auto score = [&](int j) {
      return dot_row_with_spread<T, D>(a.k.base, koff + (int64_t)min(j, hi) * a.k.sn, qreg) * a.scale;
    };
    // lane j's dO_i.v_j
    auto dvalue = [&](int j) {
      return dot_row_with_spread<T, D>(a.v.base, voff + (int64_t)min(j, hi) * a.v.sn, doreg);
    };
    // dq_i += sum over one tile of ds_j k_j (lanes own columns)
    float acc[CPL];
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc) acc[cc] = 0.f;
    auto add_tile = [&](int j0, float ds) {
      const int cnt = min(64, hi - j0 + 1);
      for (int jj = 0; jj < cnt; ++jj) {
        const float dsj = lane_bcast(ds, jj);
        const int64_t kr = koff + (int64_t)(j0 + jj) * a.k.sn;
#pragma unroll
        for (int cc = 0; cc < CPL; ++cc)
          acc[cc] = fmaf(dsj, Storage<T>::load(a.k.base, kr + cc * 64 + lane), acc[cc]);
      }
    };
    float lse, Di;
    constexpr int KT = 4;   // windows of up to 64*KT keys keep their scores and dO.v in registers
    if (hi - lo < 64 * KT) {
      float sv[KT], dpv[KT];
      float m = -INFINITY;
#pragma unroll
      for (int t = 0; t < KT; ++t) {
        const int j = lo + 64 * t + lane;
        sv[t] = j <= hi ? score(j) : -INFINITY;
        dpv[t] = j <= hi ? dvalue(j) : 0.f;
        m = fmaxf(m, sv[t]);
      }
      m = wave_max(m);   // finite: key lo is always visible
      float l = 0.f;
#pragma unroll
      for (int t = 0; t < KT; ++t) {
        sv[t] = expf(sv[t] - m);   // 0 for lanes past the window
        l += sv[t];
      }
      l = wave_sum(l);
      lse = m + logf(l);
      const float inv = 1.f / l;
      float dsum = 0.f;
#pragma unroll
      for (int t = 0; t < KT; ++t) {
        sv[t] *= inv;              // p_ij
        dsum = fmaf(sv[t], dpv[t], dsum);
      }
      Di = wave_sum(dsum);
#pragma unroll
      for (int t = 0; t < KT; ++t)
        if (lo + 64 * t <= hi) add_tile(lo + 64 * t, sv[t] * (dpv[t] - Di));   // uniform condition
    } else {
      // wider windows: three walks over the window, recomputing the scores
      float m = -INFINITY, l = 0.f;
      for (int j0 = lo; j0 <= hi; j0 += 64) {
        const int j = j0 + lane;
        const float s = j <= hi ? score(j) : -INFINITY;
        const float m_new = fmaxf(m, wave_max(s));   // finite: key j0 is always visible
        l = l * expf(m - m_new) + wave_sum(j <= hi ? expf(s - m_new) : 0.f);
        m = m_new;
      }
      lse = m + logf(l);
      float dsum = 0.f;   // D_i = sum_j p_ij dO_i.v_j
      for (int j0 = lo; j0 <= hi; j0 += 64) {
        const int j = j0 + lane;
        if (j <= hi) dsum = fmaf(expf(score(j) - lse), dvalue(j), dsum);
      }
      Di = wave_sum(dsum);
      for (int j0 = lo; j0 <= hi; j0 += 64) {
        const int j = j0 + lane;
        const float p = j <= hi ? expf(score(j) - lse) : 0.f;
        add_tile(j0, p * (dvalue(j) - Di));
      }
    }
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc)
      Storage<T>::store(a.dq, qoff + i * a.q.sn + cc * 64 + lane, acc[cc] * a.scale);
    if (lane == 0) {
      ws[2 * (int64_t)i] = lse;
      ws[2 * (int64_t)i + 1] = Di;
    }
  }
}

// ---------------------------------------------------------------------------------------
// windowed heads, per key row: dk_j and dv_j over the queries that see key j (causal: j .. j + w - 1)
// grid = (ceil(N / kBwdRows), H0, B), block = 256; reads (lse_i, D_i) left by the kernel above
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kBwdThreads) void windowed_bwd_kv_kernel(BwdArgs a) {
  constexpr int CPL = D / 64;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int h = blockIdx.y, b = blockIdx.z;
  const int64_t qoff = b * a.q.sb + h * a.q.sh;
  const int64_t koff = b * a.k.sb + h * a.k.sh;
  const int64_t voff = b * a.v.sb + h * a.v.sh;
  const int64_t ooff = b * a.dout.sb + h * a.dout.sh;
  const float* ws = a.ws + ((int64_t)b * a.H + h) * a.N * 2;
  constexpr int rows_per_wave = kBwdRows / (kBwdThreads / 64);

  for (int r = 0; r < rows_per_wave; ++r) {
    const int j = blockIdx.x * kBwdRows + wave * rows_per_wave + r;
    if (j >= a.N) break;  // uniform per wave
    float kreg[CPL], vreg[CPL], acck[CPL], accv[CPL];
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc) {
      kreg[cc] = Storage<T>::load(a.k.base, koff + j * a.k.sn + cc * 64 + lane);
      vreg[cc] = Storage<T>::load(a.v.base, voff + j * a.v.sn + cc * 64 + lane);
      acck[cc] = 0.f;
      accv[cc] = 0.f;
    }
    // the queries that see key j: j - wright .. j + wleft, cut at the ends
    const int ilo = max(0, j - a.wright), ihi = min(a.N - 1, j + a.wleft);
    for (int i0 = ilo; i0 <= ihi; i0 += 64) {
      const int i = i0 + lane;
      const bool valid = i <= ihi;
      const int ii = min(i, ihi);   // lanes past the last query read that query again
      const float s = dot_row_with_spread<T, D>(a.q.base, qoff + (int64_t)ii * a.q.sn, kreg);
      const float dp = dot_row_with_spread<T, D>(a.dout.base, ooff + (int64_t)ii * a.dout.sn, vreg);
      const float lse = ws[2 * (int64_t)ii], Di = ws[2 * (int64_t)ii + 1];
      const float p = valid ? expf(s * a.scale - lse) : 0.f;
      const float ds = p * (dp - Di);
      const int cnt = min(64, ihi - i0 + 1);
      for (int t = 0; t < cnt; ++t) {
        const float pt = lane_bcast(p, t), dst = lane_bcast(ds, t);
        const int64_t qr = qoff + (int64_t)(i0 + t) * a.q.sn;
        const int64_t dr = ooff + (int64_t)(i0 + t) * a.dout.sn;
#pragma unroll
        for (int cc = 0; cc < CPL; ++cc) {
          acck[cc] = fmaf(dst, Storage<T>::load(a.q.base, qr + cc * 64 + lane), acck[cc]);
          accv[cc] = fmaf(pt, Storage<T>::load(a.dout.base, dr + cc * 64 + lane), accv[cc]);
        }
      }
    }
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc) {
      Storage<T>::store(a.dk, koff + j * a.k.sn + cc * 64 + lane, acck[cc] * a.scale);
      Storage<T>::store(a.dv, voff + j * a.v.sn + cc * 64 + lane, accv[cc]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// linear heads
// ---------------------------------------------------------------------------------------
constexpr int kBwdChunk = 32;
constexpr int kBwdLinThreads = 512;

// Token rows in LDS are D + 4 floats apart: 16-byte aligned, so that a row can be read four
// values at a time, and a column of 32 rows (the chunk's CH x CH products read those) spreads
// over 8 banks instead of falling into one.
template <int D> constexpr size_t linear_bwd_q_smem() {
  return sizeof(float) * (5 * kBwdChunk * (D + 4) + D * (D + 1) + D + 2 * kBwdChunk * (kBwdChunk + 1) + 2 * kBwdChunk);
}
template <int D> constexpr size_t linear_bwd_kv_smem() {
  return sizeof(float) * (4 * kBwdChunk * (D + 4) + D * (D + 1) + D + 2 * kBwdChunk * (kBwdChunk + 1) + kBwdChunk);
}

// Forward scan: dq, and (den_i, c_i) for the reverse scan.  grid = (H1, B), block = 512.
template <typename T, int D>
__global__ __launch_bounds__(kBwdLinThreads) void linear_bwd_q_kernel(BwdArgs a) {
  constexpr int CH = kBwdChunk;
  constexpr int G = kBwdLinThreads / D;   // thread groups along the token axis
  constexpr int NUM_T = CH / G;        // tokens per thread
  constexpr int UPD_C = D / G;         // state rows per thread in the update
  constexpr int SR = D + 1;            // state row stride: rows and columns both conflict-free
  constexpr int TR = D + 4;            // token row stride
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* fq = smem;                   // [CH][D] phi(q)
  float* fk = fq + CH * TR;            // [CH][D] phi(k)
  float* vv = fk + CH * TR;            // [CH][D]
  float* gg = vv + CH * TR;            // [CH][D] dO, then g = dO / den
  float* rr = gg + CH * TR;            // [CH][D] r_t = A g_t (state before the chunk)
  float* S = rr + CH * TR;             // [D][SR]  A: rows = feature c, columns = value e
  float* z = S + D * SR;              // [D]
  float* am = z + D;                  // [CH][CH+1] a[t][u] = phi(q_t).phi(k_u), u <= t
  float* gv = am + CH * (CH + 1);     // [CH][CH+1] g_t.v_u, then g_t.v_u - c_t, u <= t
  float* den = gv + CH * (CH + 1);    // [CH]
  float* cvec = den + CH;             // [CH]

  const int tid = threadIdx.x;
  const int h = a.H0 + blockIdx.x, b = blockIdx.y;
  const int64_t qoff = b * a.q.sb + h * a.q.sh;
  const int64_t koff = b * a.k.sb + h * a.k.sh;
  const int64_t voff = b * a.v.sb + h * a.v.sh;
  const int64_t ooff = b * a.dout.sb + h * a.dout.sh;   // layout of dO
  float* ws = a.ws + ((int64_t)b * a.H + h) * a.N * 2;

  for (int x = tid; x < D * SR; x += kBwdLinThreads) S[x] = 0.f;
  if (tid < D) z[tid] = 0.f;
  const int c = tid % D;   // the feature (or value) index this thread owns
  const int g = tid / D;

  for (int t0 = 0; t0 < a.N; t0 += CH) {
    __syncthreads();  // previous chunk fully consumed (and the zero fill above is visible)
    for (int x = tid; x < CH * D; x += kBwdLinThreads) {
      const int t = x / D, cc = x % D;
      const int n = t0 + t;
      float qv = 0.f, kv = 0.f, v_ = 0.f, d_ = 0.f;
      if (n < a.N) {
        qv = feature_map(Storage<T>::load(a.q.base, qoff + (int64_t)n * a.q.sn + cc), a.phi);
        kv = feature_map(Storage<T>::load(a.k.base, koff + (int64_t)n * a.k.sn + cc), a.phi);
        v_ = Storage<T>::load(a.v.base, voff + (int64_t)n * a.v.sn + cc);
        d_ = Storage<T>::load(a.dout.base, ooff + (int64_t)n * a.dout.sn + cc);
      }
      const int y = t * TR + cc;
      fq[y] = qv; fk[y] = kv; vv[y] = v_; gg[y] = d_;   // rows past N: zeros
    }
    __syncthreads();
    // a[t][u] = phi(q_t).phi(k_u), u <= t
    for (int x = tid; x < CH * CH; x += kBwdLinThreads) {
      const int t = x / CH, u = x % CH;
      float s = 0.f;
      if (u <= t)
        for (int cc = 0; cc < D; ++cc) s = fmaf(fq[t * TR + cc], fk[u * TR + cc], s);
      am[t * (CH + 1) + u] = s;
    }
    __syncthreads();
    if (tid < CH) {
      float s = 0.f;
      for (int u = 0; u <= tid; ++u) s += am[tid * (CH + 1) + u];
      float zz = 0.f;
      for (int cc = 0; cc < D; ++cc) zz = fmaf(fq[tid * TR + cc], z[cc], zz);
      // rows past N keep a harmless denominator of 1 (their dO is zero)
      den[tid] = (t0 + tid < a.N) ? s + zz + a.eps : 1.f;
    }
    __syncthreads();
    for (int x = tid; x < CH * D; x += kBwdLinThreads) gg[(x / D) * TR + x % D] /= den[x / D];   // g = dO / den
    __syncthreads();
    // gv[t][u] = g_t.v_u, u <= t
    for (int x = tid; x < CH * CH; x += kBwdLinThreads) {
      const int t = x / CH, u = x % CH;
      float s = 0.f;
      if (u <= t)
        for (int cc = 0; cc < D; ++cc) s = fmaf(gg[t * TR + cc], vv[u * TR + cc], s);
      gv[t * (CH + 1) + u] = s;
    }
    // r[t][c] = sum_e A[c][e] g_t[e]
    float acc[NUM_T];
#pragma unroll
    for (int i = 0; i < NUM_T; ++i) acc[i] = 0.f;
    for (int e = 0; e < D; e += 4) {
      const float s0 = S[c * SR + e], s1 = S[c * SR + e + 1], s2 = S[c * SR + e + 2], s3 = S[c * SR + e + 3];
#pragma unroll
      for (int i = 0; i < NUM_T; ++i) {
        const float4 g4 = *reinterpret_cast<const float4*>(&gg[(g + G * i) * TR + e]);   // same for all lanes
        acc[i] = fmaf(s0, g4.x, fmaf(s1, g4.y, fmaf(s2, g4.z, fmaf(s3, g4.w, acc[i]))));
      }
    }
#pragma unroll
    for (int i = 0; i < NUM_T; ++i) rr[(g + G * i) * TR + c] = acc[i];
    __syncthreads();
    // c_t = g_t.num_t / den_t with g_t.num_t = phi(q_t).r_t + sum_{u<=t} a[t][u] g_t.v_u
    if (tid < CH) {
      float s = 0.f;
      for (int cc = 0; cc < D; ++cc) s = fmaf(fq[tid * TR + cc], rr[tid * TR + cc], s);
      for (int u = 0; u <= tid; ++u) s = fmaf(am[tid * (CH + 1) + u], gv[tid * (CH + 1) + u], s);
      const float ct = s / den[tid];
      cvec[tid] = ct;
      if (t0 + tid < a.N) {
        ws[2 * (int64_t)(t0 + tid)] = den[tid];
        ws[2 * (int64_t)(t0 + tid) + 1] = ct;
      }
    }
    __syncthreads();
    // w[t][u] = g_t.v_u - c_t, u <= t
    for (int x = tid; x < CH * CH; x += kBwdLinThreads) {
      const int t = x / CH, u = x % CH;
      if (u <= t) gv[t * (CH + 1) + u] -= cvec[t];
    }
    __syncthreads();
    // dfq[t][c] = r_t[c] - c_t Z[c] + sum_{u<=t} w[t][u] phi(k_u)[c]
#pragma unroll
    for (int i = 0; i < NUM_T; ++i) acc[i] -= cvec[g + G * i] * z[c];
    for (int u = 0; u < CH; ++u) {
      const float fku = fk[u * TR + c];
#pragma unroll
      for (int i = 0; i < NUM_T; ++i) acc[i] = fmaf(gv[(g + G * i) * (CH + 1) + u], fku, acc[i]);
    }
#pragma unroll
    for (int i = 0; i < NUM_T; ++i) {
      const int t = g + G * i, n = t0 + t;
      if (n < a.N)
        Storage<T>::store(a.dq, qoff + (int64_t)n * a.q.sn + c,
                          acc[i] * feature_map_slope(fq[t * TR + c], a.phi));
    }
    __syncthreads();  // all reads of A and Z for this chunk are done
    // state update: A[cc][e] += sum_t phi(k_t)[cc] v_t[e];  Z[cc] += sum_t phi(k_t)[cc]
    {
      const int e = c;
      float vcol[CH];
#pragma unroll
      for (int t = 0; t < CH; ++t) vcol[t] = vv[t * TR + e];
      for (int i = 0; i < UPD_C / 4; ++i) {
        const int cc = 4 * (g + G * i);   // four state rows at a time: one 16-byte read per token
        float s0 = S[cc * SR + e], s1 = S[(cc + 1) * SR + e], s2 = S[(cc + 2) * SR + e], s3 = S[(cc + 3) * SR + e];
#pragma unroll
        for (int t = 0; t < CH; ++t) {
          const float4 f4 = *reinterpret_cast<const float4*>(&fk[t * TR + cc]);
          s0 = fmaf(f4.x, vcol[t], s0); s1 = fmaf(f4.y, vcol[t], s1);
          s2 = fmaf(f4.z, vcol[t], s2); s3 = fmaf(f4.w, vcol[t], s3);
        }
        S[cc * SR + e] = s0; S[(cc + 1) * SR + e] = s1; S[(cc + 2) * SR + e] = s2; S[(cc + 3) * SR + e] = s3;
      }
      if (tid < D) {
        float s = z[tid];
        for (int t = 0; t < CH; ++t) s += fk[t * TR + tid];
        z[tid] = s;
      }
    }
  }
}

// Reverse scan: dk and dv.  grid = (H1, B), block = 512; reads (den_i, c_i) left by the kernel above.
template <typename T, int D>
__global__ __launch_bounds__(kBwdLinThreads) void linear_bwd_kv_kernel(BwdArgs a) {
  constexpr int CH = kBwdChunk;
  constexpr int G = kBwdLinThreads / D;
  constexpr int NUM_T = CH / G;
  constexpr int UPD_C = D / G;
  constexpr int SR = D + 1;
  constexpr int TR = D + 4;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* fq = smem;                   // [CH][D]
  float* fk = fq + CH * TR;            // [CH][D]
  float* vv = fk + CH * TR;            // [CH][D]
  float* gg = vv + CH * TR;            // [CH][D] g = dO / den
  float* Bm = gg + CH * TR;            // [D][SR]  B: rows = feature c, columns = value e
  float* y = Bm + D * SR;             // [D]
  float* a1 = y + D;                  // [CH][CH+1] phi(q_t).phi(k_u), t >= u
  float* a2 = a1 + CH * (CH + 1);     // [CH][CH+1] g_t.v_u - c_t, t >= u
  float* cvec = a2 + CH * (CH + 1);   // [CH]

  const int tid = threadIdx.x;
  const int h = a.H0 + blockIdx.x, b = blockIdx.y;
  const int64_t qoff = b * a.q.sb + h * a.q.sh;
  const int64_t koff = b * a.k.sb + h * a.k.sh;
  const int64_t voff = b * a.v.sb + h * a.v.sh;
  const int64_t ooff = b * a.dout.sb + h * a.dout.sh;
  const float* ws = a.ws + ((int64_t)b * a.H + h) * a.N * 2;

  for (int x = tid; x < D * SR; x += kBwdLinThreads) Bm[x] = 0.f;
  if (tid < D) y[tid] = 0.f;
  const int c = tid % D;
  const int g = tid / D;

  const int nchunks = (a.N + CH - 1) / CH;
  for (int ch = nchunks - 1; ch >= 0; --ch) {
    const int t0 = ch * CH;
    __syncthreads();  // previous chunk fully consumed (and the zero fill above is visible)
    for (int x = tid; x < CH * D; x += kBwdLinThreads) {
      const int t = x / D, cc = x % D;
      const int n = t0 + t;
      float qv = 0.f, kv = 0.f, v_ = 0.f, g_ = 0.f;
      if (n < a.N) {
        qv = feature_map(Storage<T>::load(a.q.base, qoff + (int64_t)n * a.q.sn + cc), a.phi);
        kv = feature_map(Storage<T>::load(a.k.base, koff + (int64_t)n * a.k.sn + cc), a.phi);
        v_ = Storage<T>::load(a.v.base, voff + (int64_t)n * a.v.sn + cc);
        g_ = Storage<T>::load(a.dout.base, ooff + (int64_t)n * a.dout.sn + cc) / ws[2 * (int64_t)n];
      }
      const int y = t * TR + cc;
      fq[y] = qv; fk[y] = kv; vv[y] = v_; gg[y] = g_;   // rows past N: zeros, no contribution
    }
    if (tid < CH) cvec[tid] = (t0 + tid < a.N) ? ws[2 * (int64_t)(t0 + tid) + 1] : 0.f;
    __syncthreads();
    for (int x = tid; x < CH * CH; x += kBwdLinThreads) {
      const int t = x / CH, u = x % CH;
      float s1 = 0.f, s2 = 0.f;
      if (t >= u) {
        for (int cc = 0; cc < D; ++cc) {
          s1 = fmaf(fq[t * TR + cc], fk[u * TR + cc], s1);
          s2 = fmaf(gg[t * TR + cc], vv[u * TR + cc], s2);
        }
        s2 -= cvec[t];
        if (t0 + t >= a.N) { s1 = 0.f; s2 = 0.f; }   // a row past N weighs nothing
      }
      a1[t * (CH + 1) + u] = s1;
      a2[t * (CH + 1) + u] = s2;
    }
    __syncthreads();
    // thread (c, g) owns value column e = c of dv and feature c of dk for tokens u = g + G*i
    float accv[NUM_T], acck[NUM_T];
#pragma unroll
    for (int i = 0; i < NUM_T; ++i) { accv[i] = 0.f; acck[i] = -y[c]; }
    for (int cc = 0; cc < D; cc += 4) {
      float bce[4], bec[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        bce[r] = Bm[(cc + r) * SR + c];   // B[cc + r][e = c]
        bec[r] = Bm[c * SR + cc + r];     // B[c][e = cc + r]
      }
#pragma unroll
      for (int i = 0; i < NUM_T; ++i) {
        const float4 k4 = *reinterpret_cast<const float4*>(&fk[(g + G * i) * TR + cc]);
        const float4 v4 = *reinterpret_cast<const float4*>(&vv[(g + G * i) * TR + cc]);
        // dv_u[e] += B[cc][e] phi(k_u)[cc];  dfk_u[c] += B[c][cc] v_u[cc]
        accv[i] = fmaf(bce[0], k4.x, fmaf(bce[1], k4.y, fmaf(bce[2], k4.z, fmaf(bce[3], k4.w, accv[i]))));
        acck[i] = fmaf(bec[0], v4.x, fmaf(bec[1], v4.y, fmaf(bec[2], v4.z, fmaf(bec[3], v4.w, acck[i]))));
      }
    }
    for (int t = 0; t < CH; ++t) {
      const float gte = gg[t * TR + c], fqt = fq[t * TR + c];
#pragma unroll
      for (int i = 0; i < NUM_T; ++i) {
        accv[i] = fmaf(a1[t * (CH + 1) + g + G * i], gte, accv[i]);   // zero where t < u
        acck[i] = fmaf(a2[t * (CH + 1) + g + G * i], fqt, acck[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < NUM_T; ++i) {
      const int u = g + G * i, n = t0 + u;
      if (n < a.N) {
        Storage<T>::store(a.dv, voff + (int64_t)n * a.v.sn + c, accv[i]);
        Storage<T>::store(a.dk, koff + (int64_t)n * a.k.sn + c,
                          acck[i] * feature_map_slope(fk[u * TR + c], a.phi));
      }
    }
    __syncthreads();  // all reads of B and Y for this chunk are done
    // state update: B[cc][e] += sum_t phi(q_t)[cc] g_t[e];  Y[cc] += sum_t c_t phi(q_t)[cc]
    {
      const int e = c;
      float gcol[CH];
#pragma unroll
      for (int t = 0; t < CH; ++t) gcol[t] = gg[t * TR + e];
      for (int i = 0; i < UPD_C / 4; ++i) {
        const int cc = 4 * (g + G * i);   // four state rows at a time: one 16-byte read per token
        float s0 = Bm[cc * SR + e], s1 = Bm[(cc + 1) * SR + e], s2 = Bm[(cc + 2) * SR + e], s3 = Bm[(cc + 3) * SR + e];
#pragma unroll
        for (int t = 0; t < CH; ++t) {
          const float4 f4 = *reinterpret_cast<const float4*>(&fq[t * TR + cc]);
          s0 = fmaf(f4.x, gcol[t], s0); s1 = fmaf(f4.y, gcol[t], s1);
          s2 = fmaf(f4.z, gcol[t], s2); s3 = fmaf(f4.w, gcol[t], s3);
        }
        Bm[cc * SR + e] = s0; Bm[(cc + 1) * SR + e] = s1; Bm[(cc + 2) * SR + e] = s2; Bm[(cc + 3) * SR + e] = s3;
      }
      if (tid < D) {
        float s = y[tid];
        for (int t = 0; t < CH; ++t) s = fmaf(cvec[t], fq[t * TR + tid], s);
        y[tid] = s;
      }
    }
  }
}

template <typename T, int D>
hipError_t launch_bwd_t(const BwdArgs& a, bool windowed_heads, bool linear_heads, hipStream_t s) {
  if (windowed_heads && a.H0 > 0) {
    dim3 grid((a.N + kBwdRows - 1) / kBwdRows, a.H0, a.B);
    windowed_bwd_q_kernel<T, D><<<grid, dim3(kBwdThreads), 0, s>>>(a);
    windowed_bwd_kv_kernel<T, D><<<grid, dim3(kBwdThreads), 0, s>>>(a);
  }
  if (linear_heads && a.H0 < a.H) {
    dim3 grid(a.H - a.H0, a.B);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_bwd_q_kernel<T, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)linear_bwd_q_smem<D>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_bwd_kv_kernel<T, D>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)linear_bwd_kv_smem<D>());
    if (e != hipSuccess) return e;
    linear_bwd_q_kernel<T, D><<<grid, dim3(kBwdLinThreads), linear_bwd_q_smem<D>(), s>>>(a);
    linear_bwd_kv_kernel<T, D><<<grid, dim3(kBwdLinThreads), linear_bwd_kv_smem<D>(), s>>>(a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_backward_scalar(const BwdArgs& a, bool bf16, bool windowed_heads, bool linear_heads,
                                  hipStream_t s) {
  if (a.B <= 0 || a.H <= 0 || a.N <= 0) return hipSuccess;
  if (a.d == 64)
    return bf16 ? launch_bwd_t<uint16_t, 64>(a, windowed_heads, linear_heads, s)
                : launch_bwd_t<float, 64>(a, windowed_heads, linear_heads, s);
  return bf16 ? launch_bwd_t<uint16_t, 128>(a, windowed_heads, linear_heads, s)
              : launch_bwd_t<float, 128>(a, windowed_heads, linear_heads, s);
}

}  // namespace gformer
