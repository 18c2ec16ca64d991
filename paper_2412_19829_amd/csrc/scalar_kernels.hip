// Plain-FMA kernels: fp32 arithmetic on fp32 or bf16 storage.  They are the fp32 path of the
// library (reduced-precision operands never reach a matrix core here) and are written for
// clarity; the MFMA kernels carry the bf16 performance path.
#include "common.hpp"
#include "scalar_util.hpp"

namespace gformer {

namespace {

// ---------------------------------------------------------------------------------------
// Windowed softmax head (section III-B, Eq. 1), causal or centred.  One wave owns one query at a time;
// lanes own keys for the scores and value columns for the weighted sum.
// grid = (ceil(N / kScalarWindowRows), H0, B), block = 256.
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kScalarThreads) void windowed_scalar_kernel(AttnArgs a) {
  constexpr int CPL = D / 64;  // value columns per lane
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int h = blockIdx.y, b = blockIdx.z;
  const int64_t qoff = b * a.q.sb + h * a.q.sh;
  const int64_t koff = b * a.k.sb + h * a.k.sh;
  const int64_t voff = b * a.v.sb + h * a.v.sh;
  const int64_t ooff = b * a.osb + h * a.osh;
  constexpr int rows_per_wave = kScalarWindowRows / (kScalarThreads / 64);

  for (int r = 0; r < rows_per_wave; ++r) {
    const int i = blockIdx.x * kScalarWindowRows + wave * rows_per_wave + r;
    if (i >= a.N) break;  // uniform per wave
    float qreg[CPL];
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc) qreg[cc] = Storage<T>::load(a.q.base, qoff + i * a.q.sn + cc * 64 + lane);
    // visible keys lo..hi: the w tokens ending at i (causal) or centred on i (bidirectional)
    const int lo = max(0, i - a.wleft), hi = min(a.N - 1, i + a.wright);
    float m = -INFINITY, l = 0.f;
    float acc[CPL];
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc) acc[cc] = 0.f;

    for (int j0 = lo; j0 <= hi; j0 += 64) {
      const int j = j0 + lane;
      const bool valid = j <= hi;
      float s = 0.f;
      {
        // lanes past the last visible key read that key's row again (in bounds), masked below
        s = dot_row_with_spread<T, D>(a.k.base, koff + (int64_t)min(j, hi) * a.k.sn, qreg);
      }
      s = valid ? s * a.scale : -INFINITY;
      const float m_new = fmaxf(m, wave_max(s));  // finite: key j0 is always valid
      const float alpha = expf(m - m_new);        // exp(-inf) = 0 on the first tile
      const float p = valid ? expf(s - m_new) : 0.f;
      l = l * alpha + wave_sum(p);
#pragma unroll
      for (int cc = 0; cc < CPL; ++cc) acc[cc] *= alpha;
      const int cnt = min(64, hi - j0 + 1);
      for (int jj = 0; jj < cnt; ++jj) {
        const float pj = lane_bcast(p, jj);
        const int64_t vr = voff + (int64_t)(j0 + jj) * a.v.sn;
#pragma unroll
        for (int cc = 0; cc < CPL; ++cc)
          acc[cc] = fmaf(pj, Storage<T>::load(a.v.base, vr + cc * 64 + lane), acc[cc]);
      }
      m = m_new;
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int cc = 0; cc < CPL; ++cc)
      Storage<T>::store(a.out, ooff + i * a.osn + cc * 64 + lane, acc[cc] * inv);
  }
}

// ---------------------------------------------------------------------------------------
// Causal linear attention head (Algorithm 1), chunked: inside a chunk of CH tokens the masked
// quadratic form, across chunks the carried state A (D x D) and Z (D), all fp32 in LDS.
// One workgroup walks one head from token 0 to N-1.  grid = (H1, B), block = 256.
// ---------------------------------------------------------------------------------------
constexpr int kScalarChunk = 32;
template <int D> constexpr int kScalarTokenRow = D + 4;   // LDS stride of a token row (causal kernel)

template <typename T, int D>
__global__ __launch_bounds__(kScalarThreads) void linear_scalar_kernel(AttnArgs a) {
  constexpr int CH = kScalarChunk;
  constexpr int G = kScalarThreads / D;        // thread groups along the non-e axis
  constexpr int NUM_T = CH / G;                // tokens per thread in the read-out
  constexpr int UPD_C = D / G;                 // state rows per thread in the update
  // Token rows are D + 4 floats apart: 16-byte aligned, so that a row broadcast to a wave is read
  // four values at a time, and a column of 32 rows (the masked products read those) spreads over
  // 8 banks instead of falling into one.
  constexpr int TR = kScalarTokenRow<D>;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* fq = smem;                 // [CH][TR]
  float* fk = fq + CH * TR;         // [CH][TR]
  float* vv = fk + CH * TR;         // [CH][TR]
  float* S = vv + CH * TR;          // [D][D]   A of Algorithm 1, rows = feature c, cols = e
  float* z = S + D * D;             // [D]
  float* am = z + D;                // [CH][CH+1] masked feature products
  float* den = am + CH * (CH + 1);  // [CH]

  const int tid = threadIdx.x;
  const int h = a.H0 + blockIdx.x, b = blockIdx.y;
  const int64_t qoff = b * a.q.sb + h * a.q.sh;
  const int64_t koff = b * a.k.sb + h * a.k.sh;
  const int64_t voff = b * a.v.sb + h * a.v.sh;
  const int64_t ooff = b * a.osb + h * a.osh;

  for (int x = tid; x < D * D; x += kScalarThreads) S[x] = 0.f;
  if (tid < D) z[tid] = 0.f;

  const int e = tid % D;
  const int g = tid / D;

  for (int t0 = 0; t0 < a.N; t0 += CH) {
    __syncthreads();  // previous chunk fully consumed (and the zero fill above is visible)
    for (int x = tid; x < CH * D; x += kScalarThreads) {
      const int t = x / D, c = x % D;
      const int n = t0 + t;
      float qv = 0.f, kv = 0.f, v_ = 0.f;
      if (n < a.N) {
        qv = feature_map(Storage<T>::load(a.q.base, qoff + (int64_t)n * a.q.sn + c), a.phi);
        kv = feature_map(Storage<T>::load(a.k.base, koff + (int64_t)n * a.k.sn + c), a.phi);
        v_ = Storage<T>::load(a.v.base, voff + (int64_t)n * a.v.sn + c);
      }
      const int y = t * TR + c;
      fq[y] = qv; fk[y] = kv; vv[y] = v_;   // rows past N hold zeros and contribute nothing
    }
    __syncthreads();
    // masked products a[t][u] = phi(q_t).phi(k_u) for u <= t
    for (int x = tid; x < CH * CH; x += kScalarThreads) {
      const int t = x / CH, u = x % CH;
      float s = 0.f;
      if (u <= t) {
        for (int c = 0; c < D; ++c) s = fmaf(fq[t * TR + c], fk[u * TR + c], s);
      }
      am[t * (CH + 1) + u] = s;
    }
    __syncthreads();
    if (tid < CH) {
      float s = 0.f;
      for (int u = 0; u <= tid; ++u) s += am[tid * (CH + 1) + u];
      float zz = 0.f;
      for (int c = 0; c < D; ++c) zz = fmaf(fq[tid * TR + c], z[c], zz);
      den[tid] = s + zz + a.eps;
    }
    // read-out: num[t][e] = sum_u a[t][u] v[u][e] + sum_c phi(q_t)[c] A[c][e]
    float num[NUM_T];
#pragma unroll
    for (int i = 0; i < NUM_T; ++i) num[i] = 0.f;
    for (int c = 0; c < D; c += 4) {
      const float s0 = S[c * D + e], s1 = S[(c + 1) * D + e], s2 = S[(c + 2) * D + e], s3 = S[(c + 3) * D + e];
#pragma unroll
      for (int i = 0; i < NUM_T; ++i) {
        const float4 f4 = *reinterpret_cast<const float4*>(&fq[(g + G * i) * TR + c]);   // same for all lanes
        num[i] = fmaf(f4.x, s0, fmaf(f4.y, s1, fmaf(f4.z, s2, fmaf(f4.w, s3, num[i]))));
      }
    }
    for (int u = 0; u < CH; ++u) {
      const float vue = vv[u * TR + e];
#pragma unroll
      for (int i = 0; i < NUM_T; ++i) num[i] = fmaf(am[(g + G * i) * (CH + 1) + u], vue, num[i]);
    }
    __syncthreads();  // den ready; all reads of S for this chunk done
#pragma unroll
    for (int i = 0; i < NUM_T; ++i) {
      const int n = t0 + g + G * i;
      if (n < a.N) Storage<T>::store(a.out, ooff + (int64_t)n * a.osn + e, num[i] / den[g + G * i]);
    }
    // state update: A[c][e] += sum_t phi(k_t)[c] v_t[e];  Z[c] += sum_t phi(k_t)[c]
    float vcol[CH];
#pragma unroll
    for (int t = 0; t < CH; ++t) vcol[t] = vv[t * TR + e];
    for (int i = 0; i < UPD_C / 4; ++i) {
      const int c = 4 * (g + G * i);   // four state rows at a time: one 16-byte read per token
      float s0 = S[c * D + e], s1 = S[(c + 1) * D + e], s2 = S[(c + 2) * D + e], s3 = S[(c + 3) * D + e];
#pragma unroll
      for (int t = 0; t < CH; ++t) {
        const float4 f4 = *reinterpret_cast<const float4*>(&fk[t * TR + c]);
        s0 = fmaf(f4.x, vcol[t], s0); s1 = fmaf(f4.y, vcol[t], s1);
        s2 = fmaf(f4.z, vcol[t], s2); s3 = fmaf(f4.w, vcol[t], s3);
      }
      S[c * D + e] = s0; S[(c + 1) * D + e] = s1; S[(c + 2) * D + e] = s2; S[(c + 3) * D + e] = s3;
    }
    if (tid < D) {
      float s = z[tid];
      for (int t = 0; t < CH; ++t) s += fk[t * TR + tid];
      z[tid] = s;
    }
  }
  if (a.final_state) {   // (A, Z) after the last token, for a decode step to continue from
    __syncthreads();
    float* fs = a.final_state + ((int64_t)b * (a.H - a.H0) + blockIdx.x) * (D * D + D);
    for (int x = tid; x < D * D; x += kScalarThreads) fs[x] = S[x];
    if (tid < D) fs[D * D + tid] = z[tid];
  }
}

// The last `window` keys and values of every windowed head, token t in ring slot t % window
// (what the decode step attends to).  grid = (min(window, N) rows, H0, B), block = 64.
template <typename T>
__global__ void fill_rings_kernel(AttnArgs a) {
  const int h = blockIdx.y, b = blockIdx.z;
  const int first = max(0, a.N - a.window);
  const int t = first + blockIdx.x;
  if (t >= a.N) return;
  const int slot = t % a.window;
  const int64_t ring = (((int64_t)b * a.H0 + h) * a.window + slot) * a.d;
  for (int c = threadIdx.x; c < a.d; c += blockDim.x) {
    Storage<T>::store(a.kring, ring + c, Storage<T>::load(a.k.base, b * a.k.sb + h * a.k.sh + (int64_t)t * a.k.sn + c));
    Storage<T>::store(a.vring, ring + c, Storage<T>::load(a.v.base, b * a.v.sb + h * a.v.sh + (int64_t)t * a.v.sn + c));
  }
}

// ---------------------------------------------------------------------------------------
// Non-causal linear attention head (section II-B): S = phi(K)^T V and z = phi(K)^T 1 over the
// whole sequence first, then out_i = phi(q_i)^T S / (phi(q_i).z + eps).  Same LDS layout and
// launch geometry as the causal kernel; two passes over the head.
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kScalarThreads) void linear_scalar_bidir_kernel(AttnArgs a) {
  constexpr int CH = kScalarChunk;
  constexpr int G = kScalarThreads / D;
  constexpr int NUM_T = CH / G;
  constexpr int UPD_C = D / G;
  extern __shared__ float smem[];
  float* fq = smem;                 // [CH][D]
  float* fk = fq + CH * D;          // [CH][D]
  float* vv = fk + CH * D;          // [CH][D]
  float* S = vv + CH * D;           // [D][D]
  float* z = S + D * D;             // [D]
  float* den = z + D;               // [CH]

  const int tid = threadIdx.x;
  const int h = a.H0 + blockIdx.x, b = blockIdx.y;
  const int64_t qoff = b * a.q.sb + h * a.q.sh;
  const int64_t koff = b * a.k.sb + h * a.k.sh;
  const int64_t voff = b * a.v.sb + h * a.v.sh;
  const int64_t ooff = b * a.osb + h * a.osh;
  const int e = tid % D, g = tid / D;

  for (int x = tid; x < D * D; x += kScalarThreads) S[x] = 0.f;
  if (tid < D) z[tid] = 0.f;
  // pass 1: the state of the whole head
  for (int t0 = 0; t0 < a.N; t0 += CH) {
    __syncthreads();
    for (int x = tid; x < CH * D; x += kScalarThreads) {
      const int n = t0 + x / D, c = x % D;
      float kv = 0.f, v_ = 0.f;
      if (n < a.N) {
        kv = feature_map(Storage<T>::load(a.k.base, koff + (int64_t)n * a.k.sn + c), a.phi);
        v_ = Storage<T>::load(a.v.base, voff + (int64_t)n * a.v.sn + c);
      }
      fk[x] = kv; vv[x] = v_;   // rows past N hold zeros and contribute nothing
    }
    __syncthreads();
    float vcol[CH];
#pragma unroll
    for (int t = 0; t < CH; ++t) vcol[t] = vv[t * D + e];
    for (int i = 0; i < UPD_C; ++i) {
      const int c = g + G * i;
      float s = S[c * D + e];
#pragma unroll
      for (int t = 0; t < CH; ++t) s = fmaf(fk[t * D + c], vcol[t], s);
      S[c * D + e] = s;
    }
    if (tid < D) {
      float s = z[tid];
      for (int t = 0; t < CH; ++t) s += fk[t * D + tid];
      z[tid] = s;
    }
  }
  // pass 2: read-out of every token against the same state
  for (int t0 = 0; t0 < a.N; t0 += CH) {
    __syncthreads();  // state complete (first round) / previous chunk consumed
    for (int x = tid; x < CH * D; x += kScalarThreads) {
      const int n = t0 + x / D, c = x % D;
      fq[x] = n < a.N ? feature_map(Storage<T>::load(a.q.base, qoff + (int64_t)n * a.q.sn + c), a.phi) : 0.f;
    }
    __syncthreads();
    if (tid < CH) {
      float zz = 0.f;
      for (int c = 0; c < D; ++c) zz = fmaf(fq[tid * D + c], z[c], zz);
      den[tid] = zz + a.eps;
    }
    float num[NUM_T];
#pragma unroll
    for (int i = 0; i < NUM_T; ++i) num[i] = 0.f;
    for (int c = 0; c < D; ++c) {
      const float sce = S[c * D + e];
#pragma unroll
      for (int i = 0; i < NUM_T; ++i) num[i] = fmaf(fq[(g + G * i) * D + c], sce, num[i]);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NUM_T; ++i) {
      const int n = t0 + g + G * i;
      if (n < a.N) Storage<T>::store(a.out, ooff + (int64_t)n * a.osn + e, num[i] / den[g + G * i]);
    }
  }
}

template <int D> size_t linear_scalar_smem() {
  constexpr int CH = kScalarChunk;
  return sizeof(float) * (size_t)(3 * CH * kScalarTokenRow<D> + D * D + D + CH * (CH + 1) + CH);
}

}  // namespace

hipError_t launch_windowed_scalar(const AttnArgs& a, bool bf16, hipStream_t s) {
  if (a.H0 <= 0 || a.N <= 0 || a.B <= 0) return hipSuccess;
  dim3 grid((a.N + kScalarWindowRows - 1) / kScalarWindowRows, a.H0, a.B);
  dim3 block(kScalarThreads);
  if (a.d == 64) {
    if (bf16) windowed_scalar_kernel<uint16_t, 64><<<grid, block, 0, s>>>(a);
    else windowed_scalar_kernel<float, 64><<<grid, block, 0, s>>>(a);
  } else {
    if (bf16) windowed_scalar_kernel<uint16_t, 128><<<grid, block, 0, s>>>(a);
    else windowed_scalar_kernel<float, 128><<<grid, block, 0, s>>>(a);
  }
  return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_linear_scalar_t(const AttnArgs& a, hipStream_t s) {
  const size_t smem = linear_scalar_smem<D>();
  auto kern = a.causal ? linear_scalar_kernel<T, D> : linear_scalar_bidir_kernel<T, D>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  dim3 grid(a.H - a.H0, a.B);
  kern<<<grid, dim3(kScalarThreads), smem, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_fill_rings(const AttnArgs& a, bool bf16, hipStream_t s) {
  if (a.H0 <= 0 || a.N <= 0 || a.B <= 0 || !a.kring || !a.vring) return hipSuccess;
  const int rows = a.N < a.window ? a.N : a.window;
  const dim3 grid(rows, a.H0, a.B), block(64);
  if (bf16) fill_rings_kernel<uint16_t><<<grid, block, 0, s>>>(a);
  else fill_rings_kernel<float><<<grid, block, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_linear_scalar(const AttnArgs& a, bool bf16, hipStream_t s) {
  if (a.H - a.H0 <= 0 || a.N <= 0 || a.B <= 0) return hipSuccess;
  if (a.d == 64)
    return bf16 ? launch_linear_scalar_t<uint16_t, 64>(a, s) : launch_linear_scalar_t<float, 64>(a, s);
  return bf16 ? launch_linear_scalar_t<uint16_t, 128>(a, s) : launch_linear_scalar_t<float, 128>(a, s);
}

}  // namespace gformer
