// Decode step of the causal layer: token t of every (batch, head) from what the layer keeps
// between steps.  Windowed heads (section III-B) keep the last `window` keys and values in a ring
// (slot t % window) and compute row t of Eq. 1 over the filled slots; linear heads run the loop
// body of Algorithm 1 once on their carried A (d x d) and Z (d).  GEMV-shaped and bound by
// reading the ring (2*w*d elements) or the state (d*d floats) once: plain fp32 FMAs, one
// workgroup per (batch, head), no matrix cores.
#include "common.hpp"

namespace gformer {
namespace {

constexpr int kDecodeThreads = 256;

__device__ __forceinline__ float phi_of(float x, int phi) {
  if (phi != 0) return x;
  return x > 0.f ? x + 1.f : expf(x);   // section II-B: elu(x) + 1
}

// 8 consecutive elements (16-byte aligned for bf16, 32-byte for fp32) widened to fp32
template <typename T> __device__ __forceinline__ void load8(const void* p, int64_t i, float (&x)[8]) {
  if constexpr (sizeof(T) == 2) {
    const uint4 u = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(p) + i);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      x[2 * j] = __uint_as_float(w[j] << 16);
      x[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
    }
  } else {
    const float4 a = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p) + i);
    const float4 b = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p) + i + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
}

__device__ __forceinline__ float block_reduce(float x, float* red, bool is_max) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float y = __shfl_xor(x, o, 64);
    x = is_max ? fmaxf(x, y) : x + y;
  }
  __syncthreads();            // red free again
  if (lane == 0) red[wave] = x;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < kDecodeThreads / 64; ++w) r = is_max ? fmaxf(r, red[w]) : r + red[w];
  return r;
}

template <typename T, int D>
__global__ __launch_bounds__(kDecodeThreads) void decode_kernel(DecodeArgs a) {
  extern __shared__ float smem[];
  __shared__ float red[kDecodeThreads / 64];
  const int tid = threadIdx.x;
  const int h = blockIdx.x, b = blockIdx.y;
  const int64_t tok = ((int64_t)b * a.H + h) * D;   // q, k, v, out are dense [B, H, d]

  if (h < a.H0) {
    // ---- windowed head ----
    float* s = smem;                 // [cnt] scores, then weights
    float* qs = smem + a.window;     // [D]
    const int w = a.window;
    const int cnt = (int)(a.t + 1 < (int64_t)w ? a.t + 1 : (int64_t)w);
    const int slot = (int)(a.t % w);
    const int64_t ring = ((int64_t)b * a.H0 + h) * w * D;
    if constexpr (sizeof(T) == 2) {
      if (w <= kDecodeThreads) {
        // Rings of at most one row per thread in 16-bit storage: every load of the step -- this
        // thread's key row and its pieces of the value rows -- is issued before anything waits, so
        // the step costs one trip to memory instead of three in a row.  The row of slot t % w is
        // taken from the new token itself (its copy into the ring is under way in the same step).
        constexpr int C8 = D / 8, RG = kDecodeThreads / C8, VR = kDecodeThreads / RG;
        const int c0 = 8 * (tid % C8), g = tid / C8;
        const uint16_t* kin = reinterpret_cast<const uint16_t*>(a.k) + tok;
        const uint16_t* vin = reinterpret_cast<const uint16_t*>(a.v) + tok;
        const uint16_t* kring = reinterpret_cast<const uint16_t*>(a.kcache) + ring;
        const uint16_t* vring = reinterpret_cast<const uint16_t*>(a.vcache) + ring;
        uint4 kr[C8], vr[VR];
        if (tid < cnt) {
          const uint16_t* src = tid == slot ? kin : kring + (int64_t)tid * D;
#pragma unroll
          for (int c = 0; c < C8; ++c) kr[c] = *reinterpret_cast<const uint4*>(src + 8 * c);
        }
#pragma unroll
        for (int i = 0; i < VR; ++i) {
          const int r = g + RG * i;
          if (r < cnt) {
            const uint16_t* src = r == slot ? vin : vring + (int64_t)r * D;
            vr[i] = *reinterpret_cast<const uint4*>(src + c0);
          }
        }
        if (tid < D) {
          Storage<T>::store(a.kcache, ring + (int64_t)slot * D + tid, Storage<T>::load(a.k, tok + tid));
          Storage<T>::store(a.vcache, ring + (int64_t)slot * D + tid, Storage<T>::load(a.v, tok + tid));
          qs[tid] = Storage<T>::load(a.q, tok + tid);
        }
        __syncthreads();
        auto widen = [](const uint4& u, float (&x)[8]) {
          const uint32_t wd[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            x[2 * j] = __uint_as_float(wd[j] << 16);
            x[2 * j + 1] = __uint_as_float(wd[j] & 0xffff0000u);
          }
        };
        float mloc = -INFINITY;
        if (tid < cnt) {
          float acc = 0.f;
#pragma unroll
          for (int c = 0; c < C8; ++c) {
            float kx[8];
            widen(kr[c], kx);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc = fmaf(qs[8 * c + j], kx[j], acc);
          }
          acc *= a.scale;
          s[tid] = acc;
          mloc = acc;
        }
        const float m = block_reduce(mloc, red, true);   // also makes s[] visible
        float lloc = 0.f;
        if (tid < cnt) {
          const float p = expf(s[tid] - m);
          s[tid] = p;
          lloc = p;
        }
        const float l = block_reduce(lloc, red, false);
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;
#pragma unroll
        for (int i = 0; i < VR; ++i) {
          const int r = g + RG * i;
          if (r < cnt) {
            float vx[8];
            widen(vr[i], vx);
            const float p = s[r];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = fmaf(p, vx[j], acc[j]);
          }
        }
        float* part = qs + D;            // [RG][D]
#pragma unroll
        for (int j = 0; j < 8; ++j) part[g * D + c0 + j] = acc[j];
        __syncthreads();
        if (tid < D) {
          float o = 0.f;
#pragma unroll
          for (int gg = 0; gg < RG; ++gg) o += part[gg * D + tid];
          Storage<T>::store(a.out, tok + tid, o / l);
        }
        return;
      }
    }
    if (tid < D) {
      Storage<T>::store(a.kcache, ring + (int64_t)slot * D + tid, Storage<T>::load(a.k, tok + tid));
      Storage<T>::store(a.vcache, ring + (int64_t)slot * D + tid, Storage<T>::load(a.v, tok + tid));
      qs[tid] = Storage<T>::load(a.q, tok + tid);
    }
    __syncthreads();   // the new row is visible to the whole workgroup
    // while t < window the ring is filled from slot 0 up: rows 0..cnt-1 are the visible keys
    // one thread per ring row: the whole dot product from 16-byte loads, no cross-lane traffic
    float mloc = -INFINITY;
    for (int r = tid; r < cnt; r += kDecodeThreads) {
      float acc = 0.f;
#pragma unroll
      for (int c = 0; c < D; c += 8) {
        float kx[8];
        load8<T>(a.kcache, ring + (int64_t)r * D + c, kx);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc = fmaf(qs[c + j], kx[j], acc);
      }
      acc *= a.scale;
      s[r] = acc;
      mloc = fmaxf(mloc, acc);
    }
    const float m = block_reduce(mloc, red, true);   // also makes s[] visible
    float lloc = 0.f;
    for (int r = tid; r < cnt; r += kDecodeThreads) {
      const float p = expf(s[r] - m);
      s[r] = p;
      lloc += p;
    }
    const float l = block_reduce(lloc, red, false);
    // out[c] = sum_r p[r] V[r][c] / l: thread = (row group, 8 columns), 16-byte loads, all of a
    // thread's rows in flight together; the row groups meet in LDS
    constexpr int C8 = D / 8, RG = kDecodeThreads / C8;
    const int c0 = 8 * (tid % C8), g = tid / C8;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    for (int r = g; r < cnt; r += RG) {
      float vx[8];
      load8<T>(a.vcache, ring + (int64_t)r * D + c0, vx);
      const float p = s[r];
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = fmaf(p, vx[j], acc[j]);
    }
    float* part = qs + D;            // [RG][D]
#pragma unroll
    for (int j = 0; j < 8; ++j) part[g * D + c0 + j] = acc[j];
    __syncthreads();
    if (tid < D) {
      float o = 0.f;
#pragma unroll
      for (int gg = 0; gg < RG; ++gg) o += part[gg * D + tid];
      Storage<T>::store(a.out, tok + tid, o / l);
    }
    return;
  }

  // ---- linear head: A += phi(k) (x) v, Z += phi(k), H = phi(q)^T A / (phi(q).Z + eps) ----
  float* fq = smem;          // [D]
  float* fk = fq + D;        // [D]
  float* vv = fk + D;        // [D]
  float* part = vv + D;      // [G][D]
  constexpr int G = kDecodeThreads / D;
  float* st = a.state + ((int64_t)b * (a.H - a.H0) + (h - a.H0)) * (D * D + D);
  float zq = 0.f;
  if (tid < D) {
    fq[tid] = phi_of(Storage<T>::load(a.q, tok + tid), a.phi);
    const float f = phi_of(Storage<T>::load(a.k, tok + tid), a.phi);
    fk[tid] = f;
    vv[tid] = Storage<T>::load(a.v, tok + tid);
    const float z = st[D * D + tid] + f;
    st[D * D + tid] = z;
    zq = fq[tid] * z;
  }
  const float den = block_reduce(zq, red, false) + a.eps;   // also makes fq, fk, vv visible
  const int e = tid % D, g = tid / D;
  // this thread's D/G state elements: all loads first (independent, in flight together), then
  // the update and the read-out from registers, then the stores
  constexpr int PER = D / G;
  float x[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) x[i] = st[(g + G * i) * D + e];
  float num = 0.f;
  const float ve = vv[e];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    x[i] = fmaf(fk[g + G * i], ve, x[i]);
    num = fmaf(fq[g + G * i], x[i], num);
  }
#pragma unroll
  for (int i = 0; i < PER; ++i) st[(g + G * i) * D + e] = x[i];
  part[g * D + e] = num;
  __syncthreads();
  if (tid < D) {
    float o = 0.f;
#pragma unroll
    for (int gg = 0; gg < G; ++gg) o += part[gg * D + tid];
    Storage<T>::store(a.out, tok + tid, o / den);
  }
}

}  // namespace

size_t decode_smem_bytes(int d, int window, int H0) {
  const size_t g = kDecodeThreads / d;
  const size_t win = H0 > 0 ? (size_t)window + d + (size_t)(kDecodeThreads / (d / 8)) * d : 0;
  const size_t lin = 3 * (size_t)d + g * d;
  return sizeof(float) * (win > lin ? win : lin);
}

hipError_t launch_decode(const DecodeArgs& a, bool bf16, hipStream_t s) {
  if (a.B <= 0 || a.H <= 0) return hipSuccess;
  const dim3 grid(a.H, a.B), block(kDecodeThreads);
  const int smem = (int)decode_smem_bytes(a.d, a.window, a.H0);
  hipError_t e = hipSuccess;
  auto launch = [&](auto kern) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e == hipSuccess) kern<<<grid, block, smem, s>>>(a);
  };
  if (a.d == 64) {
    if (bf16) launch(decode_kernel<uint16_t, 64>); else launch(decode_kernel<float, 64>);
  } else {
    if (bf16) launch(decode_kernel<uint16_t, 128>); else launch(decode_kernel<float, 128>);
  }
  return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace gformer
