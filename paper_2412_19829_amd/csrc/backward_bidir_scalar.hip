// Backward pass of the bidirectional linear heads, plain-FMA kernels (fp32 arithmetic on fp32 or
// bf16 storage).
//
// Section II-B's ratio over all keys: with fq = phi(q), fk = phi(k),
//     S = sum_j fk_j v_j^T,  z = sum_j fk_j,  den_i = fq_i.z + eps,  o_i = fq_i^T S / den_i.
// Its derivatives, with g_i = dO_i / den_i, r_i = S g_i and c_i = fq_i.r_i / den_i (= g_i.o_i):
//     dfq_i = r_i - c_i z
//     B = sum_i fq_i g_i^T,  Y = sum_i c_i fq_i
//     dfk_j = B v_j - Y,  dv_j = B^T fk_j
//     dq = dfq * phi'(q),  dk = dfk * phi'(k).
// Nothing depends on the position, so the pass is three sweeps over the head, one workgroup per
// (batch, head) each, chunks of 32 tokens: (1) S and z, (2) dq while B and Y are summed,
// (3) dk and dv.  The d x d sums travel between the kernels through the workspace; inside a
// kernel the sum being built lives in registers (a thread owns one row and a run of columns) and
// the sum being read lives in LDS with rows d + 1 floats apart (rows and columns both
// conflict-free).  Token rows in LDS are d + 4 floats apart.
#include "common.hpp"
#include "scalar_util.hpp"

namespace gformer {
namespace {

constexpr int kThreads = 512;
constexpr int kChunk = 32;

template <int D> struct BidirCfg {
  static constexpr int G = kThreads / D;        // thread groups: group g owns a run of columns / tokens
  static constexpr int EPT = D / G;             // columns of the d x d sum per thread
  static constexpr int TPT = kChunk / G;        // tokens per thread in the per-token products
  static constexpr int SR = D + 1, TR = D + 4;  // row strides of the d x d sum and of token tiles
  static constexpr int STATE = D * D + D;
};

struct HeadOffsets {
  int64_t q, k, v, o;
  float* state;   // this head's first sum; the second starts kBidirStateSlots blocks further on
};
template <int D> __device__ __forceinline__ HeadOffsets head_offsets(const BwdArgs& a) {
  const int h = a.H0 + blockIdx.x, b = blockIdx.y;
  HeadOffsets o;
  o.q = b * a.q.sb + h * a.q.sh;
  o.k = b * a.k.sb + h * a.k.sh;
  o.v = b * a.v.sb + h * a.v.sh;
  o.o = b * a.dout.sb + h * a.dout.sh;
  o.state = a.ws_state + ((int64_t)b * (a.H - a.H0) + blockIdx.x) * 2 * kBidirStateSlots * BidirCfg<D>::STATE;
  return o;
}

// (1) S = sum_j phi(k_j) v_j^T, z = sum_j phi(k_j)  ->  state block 0 (S row-major [feature][value], then z)
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void linear_bidir_state_kernel(BwdArgs a) {
  using C = BidirCfg<D>;
  __shared__ float fk[kChunk * C::TR], vv[kChunk * C::TR];
  const int tid = threadIdx.x, c = tid % D, g = tid / D, e0 = g * C::EPT;
  const HeadOffsets ho = head_offsets<D>(a);
  float acc[C::EPT], zc = 0.f;
#pragma unroll
  for (int x = 0; x < C::EPT; ++x) acc[x] = 0.f;
  for (int t0 = 0; t0 < a.N; t0 += kChunk) {
    __syncthreads();
    for (int x = tid; x < kChunk * D; x += kThreads) {
      const int t = x / D, cc = x % D, n = t0 + t;
      float kv = 0.f, v_ = 0.f;   // rows past N: zeros, they add nothing
      if (n < a.N) {
        kv = feature_map(Storage<T>::load(a.k.base, ho.k + (int64_t)n * a.k.sn + cc), a.phi);
        v_ = Storage<T>::load(a.v.base, ho.v + (int64_t)n * a.v.sn + cc);
      }
      fk[t * C::TR + cc] = kv;
      vv[t * C::TR + cc] = v_;
    }
    __syncthreads();
    for (int t = 0; t < kChunk; ++t) {
      const float f = fk[t * C::TR + c];
#pragma unroll
      for (int x = 0; x < C::EPT; ++x) acc[x] = fmaf(f, vv[t * C::TR + e0 + x], acc[x]);
      if (g == 0) zc += f;
    }
  }
#pragma unroll
  for (int x = 0; x < C::EPT; ++x) ho.state[c * D + e0 + x] = acc[x];
  if (g == 0) ho.state[D * D + c] = zc;
}

template <int D> constexpr size_t bidir_dq_smem() {
  using C = BidirCfg<D>;
  return sizeof(float) * (D * C::SR + D + 3 * kChunk * C::TR + 2 * kChunk);
}

// (2) dq, and B = sum_i phi(q_i) g_i^T, Y = sum_i c_i phi(q_i)  ->  state block 1
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void linear_bidir_dq_kernel(BwdArgs a) {
  using C = BidirCfg<D>;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* S = smem;                      // [D][SR]
  float* z = S + D * C::SR;             // [D]
  float* fq = z + D;                    // [CH][TR] phi(q)
  float* gg = fq + kChunk * C::TR;      // [CH][TR] dO, then g = dO / den
  float* rr = gg + kChunk * C::TR;      // [CH][TR] r_t = S g_t
  float* den = rr + kChunk * C::TR;     // [CH]
  float* cvec = den + kChunk;           // [CH]
  const int tid = threadIdx.x, c = tid % D, g = tid / D, e0 = g * C::EPT;
  const HeadOffsets ho = head_offsets<D>(a);
  for (int x = tid; x < D * D; x += kThreads) S[(x / D) * C::SR + x % D] = ho.state[x];
  if (tid < D) z[tid] = ho.state[D * D + tid];
  float bacc[C::EPT], yc = 0.f;
#pragma unroll
  for (int x = 0; x < C::EPT; ++x) bacc[x] = 0.f;

  for (int t0 = 0; t0 < a.N; t0 += kChunk) {
    __syncthreads();   // previous chunk consumed (first pass: S and z visible)
    for (int x = tid; x < kChunk * D; x += kThreads) {
      const int t = x / D, cc = x % D, n = t0 + t;
      float qv = 0.f, d_ = 0.f;   // rows past N: zeros
      if (n < a.N) {
        qv = feature_map(Storage<T>::load(a.q.base, ho.q + (int64_t)n * a.q.sn + cc), a.phi);
        d_ = Storage<T>::load(a.dout.base, ho.o + (int64_t)n * a.dout.sn + cc);
      }
      fq[t * C::TR + cc] = qv;
      gg[t * C::TR + cc] = d_;
    }
    __syncthreads();
    if (tid < kChunk) {
      float s = 0.f;
      for (int cc = 0; cc < D; ++cc) s = fmaf(fq[tid * C::TR + cc], z[cc], s);
      den[tid] = (t0 + tid < a.N) ? s + a.eps : 1.f;   // rows past N: a harmless 1 under a zero dO
    }
    __syncthreads();
    for (int x = tid; x < kChunk * D; x += kThreads) gg[(x / D) * C::TR + x % D] /= den[x / D];
    __syncthreads();
    // r[t][c] = sum_e S[c][e] g_t[e], tokens t = g, g + G, ...
    {
      float acc[C::TPT];
#pragma unroll
      for (int i = 0; i < C::TPT; ++i) acc[i] = 0.f;
      for (int e = 0; e < D; e += 4) {
        const float s0 = S[c * C::SR + e], s1 = S[c * C::SR + e + 1], s2 = S[c * C::SR + e + 2],
                    s3 = S[c * C::SR + e + 3];
#pragma unroll
        for (int i = 0; i < C::TPT; ++i) {
          const float4 g4 = *reinterpret_cast<const float4*>(&gg[(g + C::G * i) * C::TR + e]);
          acc[i] = fmaf(s0, g4.x, fmaf(s1, g4.y, fmaf(s2, g4.z, fmaf(s3, g4.w, acc[i]))));
        }
      }
#pragma unroll
      for (int i = 0; i < C::TPT; ++i) rr[(g + C::G * i) * C::TR + c] = acc[i];
    }
    __syncthreads();
    if (tid < kChunk) {
      float s = 0.f;
      for (int cc = 0; cc < D; ++cc) s = fmaf(fq[tid * C::TR + cc], rr[tid * C::TR + cc], s);
      cvec[tid] = s / den[tid];
    }
    __syncthreads();
    // dq_t = (r_t - c_t z) * phi'(q_t)
    for (int x = tid; x < kChunk * D; x += kThreads) {
      const int t = x / D, cc = x % D, n = t0 + t;
      if (n < a.N) {
        const float f = fq[t * C::TR + cc];
        Storage<T>::store(a.dq, ho.q + (int64_t)n * a.q.sn + cc,
                          (rr[t * C::TR + cc] - cvec[t] * z[cc]) * feature_map_slope(f, a.phi));
      }
    }
    // B[c][e0..] += sum_t phi(q_t)[c] g_t[e],  Y[c] += sum_t c_t phi(q_t)[c]
    for (int t = 0; t < kChunk; ++t) {
      const float f = fq[t * C::TR + c];
#pragma unroll
      for (int x = 0; x < C::EPT; ++x) bacc[x] = fmaf(f, gg[t * C::TR + e0 + x], bacc[x]);
      if (g == 0) yc = fmaf(cvec[t], f, yc);
    }
  }
  float* out = ho.state + kBidirStateSlots * C::STATE;
#pragma unroll
  for (int x = 0; x < C::EPT; ++x) out[c * D + e0 + x] = bacc[x];
  if (g == 0) out[D * D + c] = yc;
}

template <int D> constexpr size_t bidir_dkv_smem() {
  using C = BidirCfg<D>;
  return sizeof(float) * (D * C::SR + D + 2 * kChunk * C::TR);
}

// (3) dk_j = (B v_j - Y) * phi'(k_j),  dv_j = B^T phi(k_j)
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void linear_bidir_dkv_kernel(BwdArgs a) {
  using C = BidirCfg<D>;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* Bm = smem;                     // [D][SR] rows = feature, columns = value
  float* y = Bm + D * C::SR;            // [D]
  float* fk = y + D;                    // [CH][TR]
  float* vv = fk + kChunk * C::TR;      // [CH][TR]
  const int tid = threadIdx.x, c = tid % D, g = tid / D;
  const HeadOffsets ho = head_offsets<D>(a);
  const float* in = ho.state + kBidirStateSlots * C::STATE;
  for (int x = tid; x < D * D; x += kThreads) Bm[(x / D) * C::SR + x % D] = in[x];
  if (tid < D) y[tid] = in[D * D + tid];

  for (int t0 = 0; t0 < a.N; t0 += kChunk) {
    __syncthreads();
    for (int x = tid; x < kChunk * D; x += kThreads) {
      const int t = x / D, cc = x % D, n = min(t0 + t, a.N - 1);   // rows past N repeat the last one
      fk[t * C::TR + cc] = feature_map(Storage<T>::load(a.k.base, ho.k + (int64_t)n * a.k.sn + cc), a.phi);
      vv[t * C::TR + cc] = Storage<T>::load(a.v.base, ho.v + (int64_t)n * a.v.sn + cc);
    }
    __syncthreads();
    float ak[C::TPT], av[C::TPT];
#pragma unroll
    for (int i = 0; i < C::TPT; ++i) { ak[i] = 0.f; av[i] = 0.f; }
    // feature c: sum_e B[c][e] v_t[e];  value column c: sum_f B[f][c] phi(k_t)[f]
    for (int e = 0; e < D; e += 4) {
      const float b0 = Bm[c * C::SR + e], b1 = Bm[c * C::SR + e + 1], b2 = Bm[c * C::SR + e + 2],
                  b3 = Bm[c * C::SR + e + 3];
      const float t0_ = Bm[e * C::SR + c], t1_ = Bm[(e + 1) * C::SR + c], t2_ = Bm[(e + 2) * C::SR + c],
                  t3_ = Bm[(e + 3) * C::SR + c];
#pragma unroll
      for (int i = 0; i < C::TPT; ++i) {
        const float4 v4 = *reinterpret_cast<const float4*>(&vv[(g + C::G * i) * C::TR + e]);
        const float4 f4 = *reinterpret_cast<const float4*>(&fk[(g + C::G * i) * C::TR + e]);
        ak[i] = fmaf(b0, v4.x, fmaf(b1, v4.y, fmaf(b2, v4.z, fmaf(b3, v4.w, ak[i]))));
        av[i] = fmaf(t0_, f4.x, fmaf(t1_, f4.y, fmaf(t2_, f4.z, fmaf(t3_, f4.w, av[i]))));
      }
    }
#pragma unroll
    for (int i = 0; i < C::TPT; ++i) {
      const int t = g + C::G * i, n = t0 + t;
      if (n < a.N) {
        const float f = fk[t * C::TR + c];
        Storage<T>::store(a.dk, ho.k + (int64_t)n * a.k.sn + c, (ak[i] - y[c]) * feature_map_slope(f, a.phi));
        Storage<T>::store(a.dv, ho.v + (int64_t)n * a.v.sn + c, av[i]);
      }
    }
  }
}

template <typename T, int D> hipError_t launch_bidir_t(const BwdArgs& a, hipStream_t s) {
  const dim3 grid(a.H - a.H0, a.B), block(kThreads);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_bidir_dq_kernel<T, D>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)bidir_dq_smem<D>());
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_bidir_dkv_kernel<T, D>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)bidir_dkv_smem<D>());
  if (e != hipSuccess) return e;
  linear_bidir_state_kernel<T, D><<<grid, block, 0, s>>>(a);
  linear_bidir_dq_kernel<T, D><<<grid, block, bidir_dq_smem<D>(), s>>>(a);
  linear_bidir_dkv_kernel<T, D><<<grid, block, bidir_dkv_smem<D>(), s>>>(a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_linear_backward_bidir(const BwdArgs& a, bool bf16, hipStream_t s) {
  if (a.H - a.H0 <= 0 || a.N <= 0 || a.B <= 0 || !a.ws_state) return hipSuccess;
  if (a.d == 64) return bf16 ? launch_bidir_t<uint16_t, 64>(a, s) : launch_bidir_t<float, 64>(a, s);
  return bf16 ? launch_bidir_t<uint16_t, 128>(a, s) : launch_bidir_t<float, 128>(a, s);
}

}  // namespace gformer
