// Shared host/device declarations of the GFormer attention library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gformer {

// One [B,H,N,d] tensor: element (b,h,n,c) at base + b*sb + h*sh + n*sn + c (elements).
struct TensorView {
  const void* base;
  int64_t sb, sh, sn;
};

// Everything a kernel needs to know about one attention call.
struct AttnArgs {
  TensorView q, k, v;
  void* out;
  int64_t osb, osh, osn;
  int B, H, N, d;
  int window;
  int causal;        // 1: causal (window ends at the token, linear prefix); 0: bidirectional
  int wleft, wright; // windowed heads: token i sees keys i - wleft .. i + wright (cut at the ends)
  int H0;            // heads [0,H0) windowed, [H0,H) linear
  int phi;           // gf_phi
  float scale;       // softmax scale (windowed heads)
  float eps;         // linear denominator epsilon
  // Linear-attention work split.  The chunks (64 tokens) of all linear heads form one list in
  // which head i owns virtual chunks [i*vcph, (i+1)*vcph), the first `cph` of them real.  The
  // list is cut into `n_pieces` pieces of `piece_chunks` chunks; one workgroup walks one piece.
  // vcph == cph: pieces are cut with no regard to head boundaries (balanced);
  // vcph  > cph: every head is padded to a whole number of pieces (uniform segments per head).
  int chunk;         // tokens per chunk of the causal read-out (64, 128, 256)
  // the four counts below are in strips of 64 tokens whatever the chunk ("chunks" of the fixed-64 kernels)
  int cph;           // real strips per head = ceil(N / 64)
  int vcph;          // virtual chunks per head
  int piece_chunks;  // chunks per piece
  int n_pieces;      // pieces = workgroups of the read-out kernel
  int state_sub;     // the state pass cuts every piece into this many equal sub-pieces (1, 2 or 4)
  float* final_state; // optional [B*(H-H0), d*d + d] fp32: every linear head's (A, Z) after its last
                     // token, A row-major [feature][value] (what the decode step carries on from)
  void *kring, *vring; // optional [B, H0, window, d] rings: the last `window` keys / values of every
                     // windowed head, token t in slot t % window
  // Streaming windowed kernel: every (batch, windowed head) is cut into `win_pieces_per_head`
  // pieces of `win_pairs_per_piece` pairs of 32-query groups (set by its launcher).
  int win_pairs_per_piece, win_pieces_per_head;
  float* ws_states;  // [n_pieces*state_sub, d*d + d] fp32: slot j = (A, Z) of its head just
                     // before global chunk j*piece_chunks/state_sub (piece p reads slot p*state_sub)
};

// With few carried boundaries per head the read-out kernel adds up the per-sub-piece sums
// itself (independent loads, no extra launch); with many, a prefix kernel runs first and the
// read-out kernel reads a single slot.
__host__ __device__ inline bool uses_prefix_kernel(const AttnArgs& a) {
  const int ls = a.piece_chunks / a.state_sub;
  if (!a.causal) return a.vcph / ls > 6;   // every piece adds up its whole head
  // a causal piece adds up the sub-pieces in front of it inside its head; the latest start is
  // the head's last piece when pieces never straddle heads, else the head's last chunk
  const int last_start = a.vcph % a.piece_chunks == 0 ? a.vcph - a.piece_chunks : a.vcph - 1;
  return last_start / ls > 6;
}

// bf16 storage helpers (round to nearest even on store).
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T> struct Storage;
template <> struct Storage<float> {
  static __device__ __forceinline__ float load(const void* p, int64_t i) {
    return reinterpret_cast<const float*>(p)[i];
  }
  static __device__ __forceinline__ void store(void* p, int64_t i, float v) {
    reinterpret_cast<float*>(p)[i] = v;
  }
};
template <> struct Storage<uint16_t> {  // bf16 bit patterns
  static __device__ __forceinline__ float load(const void* p, int64_t i) {
    return bf16_bits_to_float(reinterpret_cast<const uint16_t*>(p)[i]);
  }
  static __device__ __forceinline__ void store(void* p, int64_t i, float v) {
    reinterpret_cast<uint16_t*>(p)[i] = float_to_bf16_bits(v);
  }
};

// One call of the backward pass: q, k, v and the gradient dout of the output in; dq, dk, dv out
// (dq is laid out like q, dk like k, dv like v).
struct BwdArgs {
  TensorView q, k, v, dout;
  void *dq, *dk, *dv;
  int B, H, N, d;
  int window;         // causal calls: tokens in the window, cut at N
  int wleft, wright;  // windowed heads: token i sees keys i - wleft .. i + wright (cut at the ends)
  int causal;         // 1: causal layer; 0: bidirectional (centred window, linear heads over all keys)
  int H0;
  int phi;
  float scale, eps;
  float* ws_state;    // bidirectional linear heads: [B * (H - H0)][2][4][d*d + d] fp32: the sums
                      // (S, z) and (B, Y) of every head, each in up to four per-segment partials
                      // (matrix row-major [feature][value], then the vector)
  int lin_segments;   // workgroups per linear head in the matrix-core scans (set by their launcher)
  int lin_bounds[5];  // segment s covers chunks [lin_bounds[s], lin_bounds[s+1]) (reverse scan: mirrored)
  float* ws;   // [B, H, N, 2] fp32: windowed heads (log-sum-exp, dO.o), linear heads (den, dO.o / den),
               // written by the per-query kernels, read by the per-key kernels
};
// plain-FMA kernels: the windowed heads, the linear heads, or both
hipError_t launch_backward_scalar(const BwdArgs& a, bool bf16, bool windowed_heads, bool linear_heads,
                                  hipStream_t s);
// bf16 matrix-core kernels for the windowed heads and for the linear heads
hipError_t launch_windowed_backward_mfma(const BwdArgs& a, hipStream_t s);
hipError_t launch_linear_backward_mfma(const BwdArgs& a, hipStream_t s);
// bidirectional linear heads: plain-FMA kernels on either storage type, matrix-core kernels (bf16)
hipError_t launch_linear_backward_bidir(const BwdArgs& a, bool bf16, hipStream_t s);
hipError_t launch_linear_backward_bidir_mfma(const BwdArgs& a, hipStream_t s);
constexpr int kBidirStateSlots = 4;   // per-segment partials kept per sum

// One call of the random-feature pre-map: heads [head_begin, head_end) of x -> the same heads of out.
struct FeatureArgs {
  TensorView x;
  const void* w;     // [d, d] row-major, same element type as x
  void* out;
  int64_t osb, osh, osn;
  int B, H, N, d;
  int head_begin, head_end;
};

// One decode step: the new token of every (batch, head), the windowed heads' key/value rings
// and the linear heads' carried states.
struct DecodeArgs {
  const void *q, *k, *v;   // [B, H, d] dense
  void* out;               // [B, H, d] dense
  void *kcache, *vcache;   // [B, H0, window, d] dense rings
  float* state;            // [B, H - H0, d*d + d] fp32: A row-major [feature][value], then Z
  int B, H, d, window, H0, phi;
  int64_t t;               // position of the token, 0-based
  float scale, eps;
};

// Host-side launchers, one per kernel family.  Each returns the hipError_t of its launch.
hipError_t launch_windowed_scalar(const AttnArgs& a, bool bf16, hipStream_t s);
hipError_t launch_linear_scalar(const AttnArgs& a, bool bf16, hipStream_t s);
hipError_t launch_windowed_mfma(const AttnArgs& a, hipStream_t s);
// The streaming form of the same heads, for windows that span at most kStreamSlots key tiles.
constexpr int kStreamSlots = 5;
struct StreamPlan {
  bool applies;          // the window fits the kernel
  bool preferred;        // ... and the problem is large enough for it to beat the query-block kernel
  int pairs_per_piece;   // 64-query pairs one workgroup walks
  int pieces_per_head;
  int64_t blocks;        // workgroups = heads * pieces_per_head
  int threads;
};
StreamPlan windowed_stream_plan(int64_t heads, int N, int wleft, int wright);
hipError_t launch_windowed_stream(const AttnArgs& a, hipStream_t s);
hipError_t launch_linear_state_mfma(const AttnArgs& a, hipStream_t s);
hipError_t launch_linear_main_mfma(const AttnArgs& a, hipStream_t s);
// The causal read-out for chunks of 64, 128 or 256 tokens (the general form of the kernel above).
bool linear_chunk_supported(int d, int chunk);
hipError_t launch_linear_chunk(const AttnArgs& a, hipStream_t s);
hipError_t launch_fill_rings(const AttnArgs& a, bool bf16, hipStream_t s);
hipError_t launch_random_features(const FeatureArgs& a, bool bf16, bool mfma, hipStream_t s);
hipError_t launch_decode(const DecodeArgs& a, bool bf16, hipStream_t s);
size_t decode_smem_bytes(int d, int window, int H0);

// Launch geometry shared by the planner and the launchers.
constexpr int kScalarWindowRows = 16;   // query rows per workgroup, scalar windowed kernel
constexpr int kScalarThreads = 256;
constexpr int kMfmaWindowRows = 128;    // query rows per workgroup, MFMA windowed kernel
constexpr int kMfmaWindowThreads = 256;
int mfma_linear_threads(int d);
int device_compute_units();   // of the current device; 256 (MI355X) in a process without one

}  // namespace gformer
