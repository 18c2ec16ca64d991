// Positive random features as a pre-map of Q or K for the linear heads (section III-A names
// them, Algorithm 1 calls them "random feature maps"; the formula is the construction of the
// work they cite):
//     out[t][i] = exp(w_i . x_t - |x_t|^2 / 2) / sqrt(m),   i = 0..m-1,  m = d here.
// The mapped tensor is then given to the attention call with the identity feature map.
//
// bf16 kernel: one GEMM tile per wave on the matrix cores, computed transposed,
//     C^T[feature][token] = W X^T,
// so that a lane owns one token: its half of the squared norm comes from the very registers it
// feeds the matrix cores with, and exponent, scaling and rounding are lane-local.  X operands are
// loaded from global memory directly in operand layout (16 bytes per lane and k-step); W sits in
// LDS for the lifetime of the workgroup; finished rows leave through LDS as whole rows.
// HBM-bound: 2*d*2 bytes per token-head against 2*d*m FLOP.
#include "common.hpp"
#include "mfma.hpp"

namespace gformer {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kFeatThreads = 256;
constexpr int kFeatRows = 128;   // tokens per workgroup step (32 per wave)

template <int D> struct FeatSmem {
  static constexpr int WROW = D + 8;    // row stride = 4 dwords mod 64: conflict-free b128 reads
  static constexpr int OROW = D + 8;
  uint16_t w[D * WROW];                 // W, row-major [feature][input]
  uint16_t ot[kFeatRows * OROW];        // finished rows on their way to memory
};

template <int D>
__global__ __launch_bounds__(kFeatThreads, 2) void random_features_mfma_kernel(FeatureArgs a) {
  constexpr int KS = D / 16, NT = D / 32;
  using Smem = FeatSmem<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int N = a.N;

  // W -> LDS, once
  const uint16_t* wp = reinterpret_cast<const uint16_t*>(a.w);
  for (int c = tid; c < D * (D / 8); c += kFeatThreads) {
    const int row = c / (D / 8), col = 8 * (c % (D / 8));
    *reinterpret_cast<u32x4*>(&sm.w[row * Smem::WROW + col]) =
        *reinterpret_cast<const u32x4*>(wp + (int64_t)row * D + col);
  }
  lds_barrier();

  const int tiles_per_head = (N + kFeatRows - 1) / kFeatRows;
  const int heads = a.head_end - a.head_begin;
  const int total = a.B * heads * tiles_per_head;
  // exp(acc - |x|^2/2) / sqrt(m) = 2^((acc - |x|^2/2) * log2(e) - log2(m)/2)
  const float shift = 0.5f * __log2f((float)D);
  for (int tile = blockIdx.x; tile < total; tile += gridDim.x) {   // uniform trip count
    const int tt = tile % tiles_per_head, hh = (tile / tiles_per_head) % heads;
    const int b = tile / (tiles_per_head * heads), h = a.head_begin + hh;
    const uint16_t* xp = reinterpret_cast<const uint16_t*>(a.x.base) + b * a.x.sb + h * a.x.sh;
    uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + b * a.osb + h * a.osh;
    const int t0 = tt * kFeatRows;
    // this lane's token; rows past N-1 re-read row N-1 (in bounds) and are not written
    const int tok = min(t0 + 32 * wave + ln, N - 1);
    const uint16_t* xr = xp + (int64_t)tok * a.x.sn + 8 * lh;
    bf16x8 xb[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      xb[ks] = as_bf16x8(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xr + 16 * ks)));
    // half of |x|^2 from this lane's share of the row, the other half from lane ^ 32
    float sq = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const u32x4 u = as_u32x4(xb[ks]);
#pragma unroll
      for (int i = 0; i < 4; ++i) sq = dot2_bf16(u[i], u[i], sq);
    }
    sq += __shfl_xor(sq, 32, 64);
    const float bias = -(0.5f * sq) * kLog2e - shift;

    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nt][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 wa = lds_read16(&sm.w[(32 * nt + ln) * Smem::WROW + 16 * ks + 8 * lh]);
        acc[nt] = mfma32(wa, xb[ks], acc[nt]);
      }
    }
    // register r of tile nt is feature 32*nt + 8*(r/4) + 4*lh + r%4 of this lane's token
    uint16_t* orow = &sm.ot[(32 * wave + ln) * Smem::OROW + 4 * lh];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) e[j] = __builtin_amdgcn_exp2f(fmaf(acc[nt][4 * g + j], kLog2e, bias));
        u32x2 pk;
        pk[0] = pack_bf16(e[0], e[1]);
        pk[1] = pack_bf16(e[2], e[3]);
        *reinterpret_cast<u32x2*>(orow + 32 * nt + 8 * g) = pk;
      }
    }
    lds_barrier();  // rows visible
    constexpr int OPIECES = kFeatRows * (D / 8) / kFeatThreads;
#pragma unroll
    for (int i = 0; i < OPIECES; ++i) {
      const int c = tid + i * kFeatThreads;
      const int row = c / (D / 8), col = 8 * (c % (D / 8));
      if (t0 + row < N) {
        const u32x4 o = *reinterpret_cast<const u32x4*>(&sm.ot[row * Smem::OROW + col]);
        __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(op + (int64_t)(t0 + row) * a.osn + col));
      }
    }
    lds_barrier();  // staging free again
  }
}

// fp32 arithmetic, fp32 or bf16 storage: one workgroup per token, one thread per feature.  The
// row is copied to LDS first, so the map may run in place.
template <typename T>
__global__ __launch_bounds__(128) void random_features_scalar_kernel(FeatureArgs a) {
  __shared__ float xs[128];
  __shared__ float red[128];
  const int d = a.d, N = a.N, heads = a.head_end - a.head_begin;
  const int64_t row = blockIdx.x;                       // over B * heads * N
  const int n = (int)(row % N), hh = (int)((row / N) % heads), b = (int)(row / ((int64_t)N * heads));
  const int h = a.head_begin + hh, i = threadIdx.x;
  const int64_t xo = b * a.x.sb + h * a.x.sh + (int64_t)n * a.x.sn;
  const int64_t oo = b * a.osb + h * a.osh + (int64_t)n * a.osn;
  float v = 0.f;
  if (i < d) v = Storage<T>::load(a.x.base, xo + i);
  xs[i] = v;
  red[i] = v * v;
  __syncthreads();
  for (int s = 64; s > 0; s >>= 1) {
    if (i < s) red[i] += red[i + s];
    __syncthreads();
  }
  if (i >= d) return;
  const float half_sq = 0.5f * red[0];
  float dot = 0.f;
  for (int c = 0; c < d; ++c) dot = fmaf(Storage<T>::load(a.w, (int64_t)i * d + c), xs[c], dot);
  Storage<T>::store(a.out, oo + i, expf(dot - half_sq) * rsqrtf((float)d));
}

template <int D> hipError_t launch_mfma_t(const FeatureArgs& a, hipStream_t s) {
  const int heads = a.head_end - a.head_begin;
  const long total = (long)a.B * heads * ((a.N + kFeatRows - 1) / kFeatRows);
  const int grid = (int)(total < 512 ? total : 512);   // two resident workgroups per compute unit
  const int smem = (int)sizeof(FeatSmem<D>);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(random_features_mfma_kernel<D>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (e != hipSuccess) return e;
  random_features_mfma_kernel<D><<<dim3(grid), dim3(kFeatThreads), smem, s>>>(a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_random_features(const FeatureArgs& a, bool bf16, bool mfma, hipStream_t s) {
  const int heads = a.head_end - a.head_begin;
  if (a.B <= 0 || heads <= 0 || a.N <= 0) return hipSuccess;
  if (mfma) return a.d == 64 ? launch_mfma_t<64>(a, s) : launch_mfma_t<128>(a, s);
  const int64_t rows = (int64_t)a.B * heads * a.N;
  if (bf16) random_features_scalar_kernel<uint16_t><<<dim3((unsigned)rows), dim3(128), 0, s>>>(a);
  else random_features_scalar_kernel<float><<<dim3((unsigned)rows), dim3(128), 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace gformer
