// C ABI of the GFormer attention library: argument validation, launch planning, dispatch.
// Everything up to the first launch is plain host code and can be exercised without a GPU.
#include "../../include/gformer.h"

#include <string.h>

#include <mutex>

#include "common.hpp"

#include <atomic>

namespace gformer {

int mfma_linear_threads(int d) { return d == 128 ? 512 : 256; }

// Compute units of the current device, asked once per device; a process without a device (the
// planner is host arithmetic and is also called there) plans for an MI355X.
int device_compute_units() {
  constexpr int kDefault = 256, kSlots = 64;
  static std::atomic<int> cached[kSlots];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kSlots) {
    (void)hipGetLastError();
    return kDefault;
  }
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n > 0) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
    (void)hipGetLastError();
    return kDefault;
  }
  cached[dev].store(n, std::memory_order_relaxed);
  return n;
}

namespace {

struct Resolved {
  gformer_plan plan;
  int64_t qs[3], ks[3], vs[3], os[3];
  int cph, vcph, piece_chunks, state_sub;
  bool stream;   // MFMA path: the windowed heads go to the streaming kernel
  bool general_chunk;  // MFMA path, causal: the linear read-out goes to the general-chunk kernel
};

// One side stream and a fork/join event pair per device, created on first use and kept for the
// life of the process.  Default priority on purpose.
constexpr int kMaxDevices = 64;
struct SideStream {
  bool ready = false;
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
};
SideStream g_side[kMaxDevices];
std::mutex g_enqueue_mutex;

// The device a call works on: the current one, which must also be the device of the caller's
// stream when that is not the null stream (kernels launched on a stream run on the stream's
// device, while per-device state below is looked up by the current one).
hipError_t call_device(hipStream_t s, int* dev) {
  hipError_t e = hipGetDevice(dev);
  if (e != hipSuccess) return e;
  if (s != nullptr) {
    int sdev = -1;
    // a stream under capture may refuse the query; the device check is then skipped
    if (hipStreamGetDevice(s, &sdev) == hipSuccess) {
      if (sdev != *dev) return hipErrorInvalidDevice;
    } else {
      (void)hipGetLastError();
    }
  }
  if (*dev < 0 || *dev >= kMaxDevices) return hipErrorInvalidDevice;
  return hipSuccess;
}

hipError_t side_stream_for_current_device(hipStream_t caller, SideStream** out) {
  int dev = 0;
  hipError_t e = call_device(caller, &dev);
  if (e != hipSuccess) return e;
  SideStream& s = g_side[dev];
  if (!s.ready) {
    if ((e = hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking)) != hipSuccess) return e;
    if ((e = hipEventCreateWithFlags(&s.fork, hipEventDisableTiming)) != hipSuccess) return e;
    if ((e = hipEventCreateWithFlags(&s.join, hipEventDisableTiming)) != hipSuccess) return e;
    s.ready = true;
  }
  *out = &s;
  return hipSuccess;
}

// Scratch of the entry point that allocates nothing: the carried linear-attention states live in
// this file-scope device array instead of a caller's workspace.  Every device the library runs
// on holds its own copy, at its own address, from the moment the code object is loaded until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// address that kernels receive is looked up once per device, with that device current.
constexpr size_t kScratchBytes = GFORMER_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
std::atomic<void*> g_scratch_ptr[kMaxDevices];

hipError_t scratch_for_current_device(hipStream_t caller, void** out) {
  int dev = 0;
  hipError_t e = call_device(caller, &dev);
  if (e != hipSuccess) return e;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return hipSuccess;
}

constexpr int64_t kMaxRowStride = 1 << 20;  // elements

bool strides_all_zero(const int64_t* s) { return s[0] == 0 && s[1] == 0 && s[2] == 0; }

void dense_strides(int64_t* s, int H, int N, int d) {
  s[0] = (int64_t)H * N * d;
  s[1] = (int64_t)N * d;
  s[2] = d;
}

gf_status check_strides(const int64_t* in, int64_t* out, int H, int N, int d) {
  if (strides_all_zero(in)) {
    dense_strides(out, H, N, d);
    return GF_OK;
  }
  for (int i = 0; i < 3; ++i) {
    if (in[i] < 0 || (in[i] % 8) != 0) return GF_ERR_INVALID_ARG;
    out[i] = in[i];
  }
  if (N > 1 && in[2] < d) return GF_ERR_INVALID_ARG;  // rows would overlap
  if (in[2] > kMaxRowStride) return GF_ERR_UNSUPPORTED;  // kernels keep in-chunk offsets in 32 bits
  return GF_OK;
}


// Chunks per piece when every linear head is cut into the same whole number of pieces (one
// workgroup per piece, at most one per compute unit, pieces of 8 chunks or more), or 0 when that
// would leave more than a fifth of the compute units without a piece.
long aligned_piece(long heads_lin, long cph, long kComputeUnits) {
  if (heads_lin <= 0 || cph <= 0) return 0;
  long k = kComputeUnits / heads_lin;
  if (k > cph / 8) k = cph / 8;
  if (k < 1) return 0;
  const long piece = (cph + k - 1) / k;
  const long per_head = (cph + piece - 1) / piece;
  if (heads_lin * per_head * 5 < (long)kComputeUnits * 4) return 0;
  return piece;
}

// Shared by gformer_attn_plan, gformer_attn_workspace_bytes and gformer_attn_fwd.
// Token i of a windowed head sees keys i - left .. i + right (cut at the sequence ends): the w
// tokens ending at i, or (bidirectional) the w tokens centred on it.
// Both reaches are cut at N - 1 here, once: a token cannot see further than the sequence, and
// the tile arithmetic of the kernels and planners (reach + tile size, row + reach) then stays far
// from the end of the int range for any window up to INT_MAX (the natural way to ask for full
// attention).
int window_left(int window, int bidirectional, int N) {
  const int reach = bidirectional ? window / 2 : window - 1;
  return reach < N - 1 ? reach : (N > 1 ? N - 1 : 0);
}
int window_right(int window, int bidirectional, int N) {
  const int reach = bidirectional ? window - 1 - window / 2 : 0;
  return reach < N - 1 ? reach : (N > 1 ? N - 1 : 0);
}

gf_status resolve(int B, int H, int N, int d, int window, const gformer_params* p, Resolved* r) {
  memset(r, 0, sizeof(*r));
  if (!p) return GF_ERR_INVALID_ARG;
  if (p->struct_size != sizeof(gformer_params)) return GF_ERR_INVALID_ARG;
  if (B < 0 || H < 0 || N < 0 || d < 1 || window < 1) return GF_ERR_INVALID_ARG;
  if (p->dtype != GF_F32 && p->dtype != GF_BF16) return GF_ERR_INVALID_ARG;
  if (p->phi != GF_PHI_ELU1 && p->phi != GF_PHI_IDENTITY) return GF_ERR_INVALID_ARG;
  if (p->impl != GF_IMPL_AUTO && p->impl != GF_IMPL_SCALAR && p->impl != GF_IMPL_MFMA &&
      p->impl != GF_IMPL_MFMA_BLOCKED && p->impl != GF_IMPL_MFMA_STREAM &&
      p->impl != GF_IMPL_MFMA_CHUNK)
    return GF_ERR_INVALID_ARG;
  if (p->n_sparse_heads < 0 || p->n_sparse_heads > H) return GF_ERR_INVALID_ARG;
  if (p->chunk < 0 || p->segment_len < 0) return GF_ERR_INVALID_ARG;
  if (p->launch_mask < 0 || p->launch_mask > 7) return GF_ERR_INVALID_ARG;
  if (p->overlap != 0 && p->overlap != 1) return GF_ERR_INVALID_ARG;
  if (p->bidirectional != 0 && p->bidirectional != 1) return GF_ERR_INVALID_ARG;
  if (!(p->softmax_scale == p->softmax_scale) || !(p->eps >= 0.f)) return GF_ERR_INVALID_ARG;
  if (B > 65535 || H > 65535) return GF_ERR_UNSUPPORTED;  // grid y/z limits
  gf_status st;
  if ((st = check_strides(p->q_stride, r->qs, H, N, d)) != GF_OK) return st;
  if ((st = check_strides(p->k_stride, r->ks, H, N, d)) != GF_OK) return st;
  if ((st = check_strides(p->v_stride, r->vs, H, N, d)) != GF_OK) return st;
  if ((st = check_strides(p->o_stride, r->os, H, N, d)) != GF_OK) return st;
  if (d != 64 && d != 128) return GF_ERR_UNSUPPORTED;

  int impl = p->impl;
  if (impl == GF_IMPL_AUTO) impl = (p->dtype == GF_BF16) ? GF_IMPL_MFMA : GF_IMPL_SCALAR;
  // the others differ from GF_IMPL_MFMA only in which kernel runs the windowed heads or the
  // linear read-out
  if (impl == GF_IMPL_MFMA_BLOCKED || impl == GF_IMPL_MFMA_STREAM || impl == GF_IMPL_MFMA_CHUNK)
    impl = GF_IMPL_MFMA;
  if (impl == GF_IMPL_MFMA && p->dtype != GF_BF16) return GF_ERR_UNSUPPORTED;
  if (p->chunk != 0 && p->chunk != 64 && p->chunk != 128 && p->chunk != 256) return GF_ERR_UNSUPPORTED;

  gformer_plan& pl = r->plan;
  pl.impl = impl;
  const long kComputeUnits = device_compute_units();
  const int H0 = p->n_sparse_heads, H1 = H - H0;
  const long heads_lin = (long)B * H1;
  if (impl == GF_IMPL_SCALAR) {
    pl.chunk = 32;  // fixed by the fp32 kernel
    pl.segment_len = N;
    pl.n_segments = (H1 > 0 && N > 0) ? (int)heads_lin : 0;  // one workgroup walks a whole head
    if (p->segment_len != 0 && p->segment_len < N) return GF_ERR_UNSUPPORTED;
    pl.windowed_threads = kScalarThreads;
    pl.windowed_blocks = (H0 > 0 && N > 0) ? B * H0 * ((N + kScalarWindowRows - 1) / kScalarWindowRows) : 0;
    pl.linear_threads = kScalarThreads;
    pl.linear_blocks = (H1 > 0 && N > 0) ? (int)heads_lin : 0;
    pl.state_blocks = 0;
    pl.workspace_bytes = 0;
    return GF_OK;
  }
  pl.chunk = p->chunk ? p->chunk : 64;
  // Everything below counts in strips of 64 tokens (the tile every kernel works in); a chunk is
  // one, two or four of them.  Chunks of more than one strip (and GF_IMPL_MFMA_CHUNK at any
  // size) take the causal read-out to the general-chunk kernel, whose pieces are whole chunks of
  // one head.  The bidirectional read-out has no in-chunk part: there the chunk only sets the
  // granularity of segment_len.
  constexpr long kStrip = 64;
  const long cm = pl.chunk / kStrip;
  r->general_chunk = !p->bidirectional && (cm > 1 || p->impl == GF_IMPL_MFMA_CHUNK);
  if (r->general_chunk && H1 > 0 && !linear_chunk_supported(d, pl.chunk)) return GF_ERR_UNSUPPORTED;
  const long cph = N > 0 ? (N + kStrip - 1) / kStrip : 0;  // real strips per head
  long piece = 0, vcph = cph, pieces = 0, mid = 0, sub = 1;
  if (p->segment_len != 0 && p->segment_len % pl.chunk != 0) return GF_ERR_INVALID_ARG;
  if (p->bidirectional && heads_lin > 0 && cph > 0) {
    // Bidirectional linear heads: every piece needs the state of its whole head, so pieces never
    // straddle heads (uniform segments per head) and every one of them is summed by the state
    // pass.  Without a request: as many pieces per head as keep every compute unit at one piece.
    if (p->segment_len != 0) {
      piece = p->segment_len / kStrip;
    } else {
      long per = kComputeUnits / heads_lin;
      if (per < 1) per = 1;
      if (per > cph) per = cph;
      piece = (cph + per - 1) / per;
    }
    const long per_head = (cph + piece - 1) / piece;
    vcph = per_head * piece;
    pieces = heads_lin * per_head;
    mid = pieces;
  } else if (p->segment_len != 0 ||
             (heads_lin > 0 && cph > 0 &&
              (r->general_chunk || aligned_piece(heads_lin, cph, kComputeUnits) > 0))) {
    // Uniform segments per head: asked for, needed by the general-chunk kernel, or chosen
    // because a whole number of them per head keeps at least 4 of 5 compute units busy.  Pieces
    // that never straddle heads leave the state pass the least to re-read (a head's last segment
    // is never summed).
    piece = p->segment_len != 0 ? p->segment_len / kStrip : aligned_piece(heads_lin, cph, kComputeUnits);
    if (piece == 0) {
      // general-chunk kernel with too few or too many heads for a good whole-number cut: as many
      // pieces per head as there are compute units for, none shorter than 8 strips
      long k = kComputeUnits / heads_lin;
      if (k > cph / 8) k = cph / 8;
      if (k < 1) k = 1;
      piece = (cph + k - 1) / k;
    }
    if (r->general_chunk) piece = (piece + cm - 1) / cm * cm;   // whole chunks
    const long per_head = cph > 0 ? (cph + piece - 1) / piece : 0;
    vcph = per_head * piece;
    pieces = heads_lin * per_head;
    // The state pass walks a head's segments but the last one.  A workgroup of it is bound by
    // its own chunk-by-chunk walk, so segments are cut into up to four sub-pieces as long as the
    // sub-pieces stay 4 chunks or longer and fit two workgroups per compute unit.
    const long carried = heads_lin * (per_head > 0 ? per_head - 1 : 0);
    for (sub = 4; sub > 1; sub /= 2)
      if (piece % sub == 0 && piece / sub >= 4 && carried * sub <= 2 * kComputeUnits) break;
    mid = carried * sub;
  } else if (heads_lin > 0 && cph > 0) {
    // One workgroup per compute unit (its LDS holds one), each with the same number of chunks;
    // pieces no shorter than 8 chunks so the carried state (d*d fp32 in, d*d out) stays a small
    // share of the traffic.
    const long total = heads_lin * cph;
    piece = (total + kComputeUnits - 1) / kComputeUnits;
    if (piece < 8) piece = 8;
    if (piece > total) piece = total;
    if (piece % 2 != 0 && piece < total) ++piece;  // even, so the state pass can halve it
    pieces = (total + piece - 1) / piece;
    // Here the state pass works on half pieces (two workgroups per compute unit fit there), which
    // evens out its load: a sub-piece is summed iff a piece boundary follows it inside its head.
    sub = piece % 2 == 0 ? 2 : 1;
    const long ls = piece / sub;
    for (long j = 1; j < pieces * sub; ++j) {
      const long e = j * ls, next_main = (j + sub - 1) / sub * piece;
      mid += (e % cph) != 0 && next_main < (e / cph + 1) * cph && next_main < total;
    }
  }
  if (pieces > 0x7fffffffL / 64) return GF_ERR_UNSUPPORTED;
  r->cph = (int)cph;
  r->vcph = (int)vcph;
  r->piece_chunks = (int)piece;
  r->state_sub = (int)sub;
  pl.segment_len = (int)(piece * kStrip);
  pl.n_segments = (int)pieces;
  pl.windowed_threads = kMfmaWindowThreads;
  pl.windowed_blocks = (H0 > 0 && N > 0) ? B * H0 * ((N + kMfmaWindowRows - 1) / kMfmaWindowRows) : 0;
  {
    const StreamPlan sp = windowed_stream_plan((int64_t)B * H0, N, window_left(window, p->bidirectional, N),
                                               window_right(window, p->bidirectional, N));
    if (p->impl == GF_IMPL_MFMA_STREAM && H0 > 0 && !sp.applies) return GF_ERR_UNSUPPORTED;
    r->stream = p->impl == GF_IMPL_MFMA_STREAM || (p->impl != GF_IMPL_MFMA_BLOCKED && sp.preferred);
    if (r->stream && H0 > 0 && N > 0) {
      pl.windowed_threads = sp.threads;
      pl.windowed_blocks = (int)sp.blocks;
    }
  }
  pl.linear_threads = mfma_linear_threads(d);
  pl.linear_blocks = (int)pieces;
  pl.state_blocks = (int)mid;
  pl.workspace_bytes = mid > 0 ? (uint64_t)pieces * sub * ((uint64_t)d * d + d) * sizeof(float) : 0;
  return GF_OK;
}

}  // namespace
}  // namespace gformer

using namespace gformer;

extern "C" {

void gformer_params_init(gformer_params* p) {
  if (!p) return;
  memset(p, 0, sizeof(*p));
  p->struct_size = sizeof(gformer_params);
  p->dtype = GF_BF16;
  p->phi = GF_PHI_ELU1;
  p->impl = GF_IMPL_AUTO;
  p->softmax_scale = 1.0f;
  p->eps = 0.0f;
}

size_t gformer_attn_workspace_bytes(int B, int H, int N, int d, int window,
                                    const gformer_params* p) {
  Resolved r;
  if (resolve(B, H, N, d, window, p, &r) != GF_OK) return 0;
  return (size_t)r.plan.workspace_bytes;
}

gf_status gformer_attn_plan(int B, int H, int N, int d, int window, const gformer_params* p,
                            gformer_plan* plan) {
  if (!plan) return GF_ERR_INVALID_ARG;
  Resolved r;
  gf_status st = resolve(B, H, N, d, window, p, &r);
  *plan = r.plan;
  return st;
}

}  // extern "C"

namespace {

// The whole layer; with rings / final states it also leaves what a decode step continues from.
gf_status attn_forward(const void* q, const void* k, const void* v, void* out, void* kring,
                       void* vring, float* final_state, int B, int H, int N, int d, int window,
                       const gformer_params* p, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
  Resolved r;
  gf_status st = resolve(B, H, N, d, window, p, &r);
  if (st != GF_OK) return st;
  if (B == 0 || H == 0 || N == 0) return GF_OK;
  if (!q || !k || !v || !out) return GF_ERR_INVALID_ARG;
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15u) return GF_ERR_INVALID_ARG;
  if (out == q || out == k || out == v) return GF_ERR_INVALID_ARG;
  if (r.plan.workspace_bytes > 0) {
    if (!workspace || workspace_bytes < r.plan.workspace_bytes) return GF_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 255u) return GF_ERR_INVALID_ARG;
  }
  // only the kernel specialised for chunks of 64 writes the states a decode step continues from
  if (final_state && r.general_chunk && p->n_sparse_heads < H) return GF_ERR_UNSUPPORTED;

  AttnArgs a;
  memset(&a, 0, sizeof(a));
  a.q = TensorView{q, r.qs[0], r.qs[1], r.qs[2]};
  a.k = TensorView{k, r.ks[0], r.ks[1], r.ks[2]};
  a.v = TensorView{v, r.vs[0], r.vs[1], r.vs[2]};
  a.out = out;
  a.osb = r.os[0]; a.osh = r.os[1]; a.osn = r.os[2];
  a.B = B; a.H = H; a.N = N; a.d = d;
  a.window = window;
  a.causal = p->bidirectional ? 0 : 1;
  a.wleft = window_left(window, p->bidirectional, N);
  a.wright = window_right(window, p->bidirectional, N);
  a.H0 = p->n_sparse_heads;
  a.phi = p->phi;
  a.scale = p->softmax_scale;
  a.eps = p->eps;
  a.chunk = r.plan.chunk;
  a.cph = r.cph;
  a.vcph = r.vcph;
  a.piece_chunks = r.piece_chunks;
  a.n_pieces = r.plan.n_segments;
  a.state_sub = r.state_sub;
  a.ws_states = r.plan.workspace_bytes > 0 ? reinterpret_cast<float*>(workspace) : nullptr;
  a.final_state = final_state;
  a.kring = kring;
  a.vring = vring;

  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  const int mask = p->launch_mask ? p->launch_mask : 7;
  const bool bf16 = p->dtype == GF_BF16;
  hipError_t e = hipSuccess;
  if (r.plan.impl == GF_IMPL_SCALAR) {
    if ((mask & GF_LAUNCH_WINDOWED) && e == hipSuccess) e = launch_windowed_scalar(a, bf16, s);
    if ((mask & GF_LAUNCH_LINEAR_MAIN) && e == hipSuccess) e = launch_linear_scalar(a, bf16, s);
  } else {
    const bool win = (mask & GF_LAUNCH_WINDOWED) && a.H0 > 0;
    // large problems with windows of at most five key tiles stream; the rest goes query block
    // by query block
    const bool stream = r.stream;
    auto launch_windowed = [&](hipStream_t on) {
      return stream ? launch_windowed_stream(a, on) : launch_windowed_mfma(a, on);
    };
    const bool lin = (mask & (GF_LAUNCH_LINEAR_STATE | GF_LAUNCH_LINEAR_MAIN)) && a.H0 < a.H;
    std::lock_guard<std::mutex> lock(g_enqueue_mutex);
    SideStream* side = nullptr;
    if (win && lin && p->overlap) e = side_stream_for_current_device(s, &side);
    bool forked = false;
    if (side && e == hipSuccess) {
      // fork: the windowed heads wait for what is already in `s`, then run beside the linear ones
      e = hipEventRecord(side->fork, s);
      if (e == hipSuccess) e = hipStreamWaitEvent(side->stream, side->fork, 0);
      forked = e == hipSuccess;
      if (e == hipSuccess) e = launch_windowed(side->stream);
    }
    // The read-out kernel wants every compute unit at once (one piece each), so only the state
    // pass, whose small workgroups pack two to a unit, shares the chip with the windowed heads.
    if ((mask & GF_LAUNCH_LINEAR_STATE) && e == hipSuccess) e = launch_linear_state_mfma(a, s);
    if (forked) {
      // join, also after a failed launch: a side stream left waiting on the fork would break a
      // capture in progress and leave `s` unordered against what did get enqueued
      const hipError_t j1 = hipEventRecord(side->join, side->stream);
      const hipError_t j2 = j1 == hipSuccess ? hipStreamWaitEvent(s, side->join, 0) : j1;
      if (e == hipSuccess) e = j2;
    } else if (win && !side && e == hipSuccess) {
      e = launch_windowed(s);
    }
    if ((mask & GF_LAUNCH_LINEAR_MAIN) && e == hipSuccess)
      e = r.general_chunk ? launch_linear_chunk(a, s) : launch_linear_main_mfma(a, s);
  }
  if (e == hipSuccess) e = launch_fill_rings(a, bf16, s);
  return e == hipSuccess ? GF_OK : GF_ERR_DEVICE;
}

}  // namespace

extern "C" {

gf_status gformer_attn_fwd(const void* q, const void* k, const void* v, void* out, int B, int H,
                           int N, int d, int window, const gformer_params* p, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  return attn_forward(q, k, v, out, nullptr, nullptr, nullptr, B, H, N, d, window, p, workspace,
                      workspace_bytes, hip_stream);
}

gf_status gformer_attn_fwd_noalloc(const void* q, const void* k, const void* v, void* out, int B,
                                   int H, int N, int d, int window, const gformer_params* p,
                                   void* hip_stream) {
  Resolved r;
  const gf_status st = resolve(B, H, N, d, window, p, &r);
  if (st != GF_OK) return st;
  if (p->overlap != 0) return GF_ERR_UNSUPPORTED;   // the side stream is created on first use
  if (r.plan.workspace_bytes > kScratchBytes) return GF_ERR_WORKSPACE;
  if (B == 0 || H == 0 || N == 0) return GF_OK;
  void* ws = nullptr;
  if (r.plan.workspace_bytes > 0) {
    std::lock_guard<std::mutex> lock(g_enqueue_mutex);
    if (scratch_for_current_device(reinterpret_cast<hipStream_t>(hip_stream), &ws) != hipSuccess) {
      (void)hipGetLastError();
      return GF_ERR_DEVICE;
    }
  }
  return attn_forward(q, k, v, out, nullptr, nullptr, nullptr, B, H, N, d, window, p, ws,
                      ws ? kScratchBytes : 0, hip_stream);
}

gf_status gformer_attn_prefill(const void* q, const void* k, const void* v, void* out, void* kcache,
                               void* vcache, float* state, int B, int H, int N, int d, int window,
                               const gformer_params* p, void* workspace, size_t workspace_bytes,
                               void* hip_stream) {
  if (!p || p->struct_size != sizeof(gformer_params)) return GF_ERR_INVALID_ARG;
  if (p->bidirectional != 0 || p->launch_mask != 0) return GF_ERR_INVALID_ARG;
  if (B > 0 && H > 0 && N > 0) {
    const int H0 = p->n_sparse_heads;
    if (H0 > 0 && H0 <= H && (!kcache || !vcache)) return GF_ERR_INVALID_ARG;
    if (H0 >= 0 && H0 < H && !state) return GF_ERR_INVALID_ARG;
    if (((uintptr_t)kcache | (uintptr_t)vcache | (uintptr_t)state) & 15u) return GF_ERR_INVALID_ARG;
  }
  return attn_forward(q, k, v, out, kcache, vcache, state, B, H, N, d, window, p, workspace,
                      workspace_bytes, hip_stream);
}

gf_status gformer_attn_decode(const void* q, const void* k, const void* v, void* out, void* kcache,
                              void* vcache, float* state, int B, int H, int d, int window,
                              int64_t t, const gformer_params* p, void* hip_stream) {
  if (!p || p->struct_size != sizeof(gformer_params)) return GF_ERR_INVALID_ARG;
  if (B < 0 || H < 0 || d < 1 || window < 1 || t < 0) return GF_ERR_INVALID_ARG;
  if (p->dtype != GF_F32 && p->dtype != GF_BF16) return GF_ERR_INVALID_ARG;
  if (p->phi != GF_PHI_ELU1 && p->phi != GF_PHI_IDENTITY) return GF_ERR_INVALID_ARG;
  if (p->n_sparse_heads < 0 || p->n_sparse_heads > H) return GF_ERR_INVALID_ARG;
  if (!(p->softmax_scale == p->softmax_scale) || !(p->eps >= 0.f)) return GF_ERR_INVALID_ARG;
  if (p->bidirectional != 0) return GF_ERR_INVALID_ARG;   // a token cannot see what is not there yet
  if (B > 65535) return GF_ERR_UNSUPPORTED;
  if (d != 64 && d != 128) return GF_ERR_UNSUPPORTED;
  const int H0 = p->n_sparse_heads;
  if (decode_smem_bytes(d, window, H0) > 64 * 1024) return GF_ERR_UNSUPPORTED;  // ring scores in LDS
  if (B == 0 || H == 0) return GF_OK;
  if (!q || !k || !v || !out) return GF_ERR_INVALID_ARG;
  if (H0 > 0 && (!kcache || !vcache)) return GF_ERR_INVALID_ARG;
  if (H0 < H && !state) return GF_ERR_INVALID_ARG;
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out | (uintptr_t)kcache |
       (uintptr_t)vcache | (uintptr_t)state) & 15u)
    return GF_ERR_INVALID_ARG;
  if (out == q || out == k || out == v) return GF_ERR_INVALID_ARG;

  DecodeArgs a;
  memset(&a, 0, sizeof(a));
  a.q = q; a.k = k; a.v = v; a.out = out;
  a.kcache = kcache; a.vcache = vcache; a.state = state;
  a.B = B; a.H = H; a.d = d; a.window = window; a.H0 = H0; a.phi = p->phi;
  a.t = t;
  a.scale = p->softmax_scale;
  a.eps = p->eps;
  const hipError_t e = launch_decode(a, p->dtype == GF_BF16, reinterpret_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? GF_OK : GF_ERR_DEVICE;
}

void gformer_feature_params_init(gformer_feature_params* p) {
  if (!p) return;
  memset(p, 0, sizeof(*p));
  p->struct_size = sizeof(gformer_feature_params);
  p->dtype = GF_BF16;
  p->impl = GF_IMPL_AUTO;
}

gf_status gformer_random_features(const void* x, const void* w, void* out, int B, int H, int N,
                                  int d, int m, const gformer_feature_params* p, void* hip_stream) {
  if (!p || p->struct_size != sizeof(gformer_feature_params)) return GF_ERR_INVALID_ARG;
  if (B < 0 || H < 0 || N < 0 || d < 1 || m < 1) return GF_ERR_INVALID_ARG;
  if (p->dtype != GF_F32 && p->dtype != GF_BF16) return GF_ERR_INVALID_ARG;
  if (p->impl != GF_IMPL_AUTO && p->impl != GF_IMPL_SCALAR && p->impl != GF_IMPL_MFMA)
    return GF_ERR_INVALID_ARG;
  if (p->head_begin < 0 || p->head_end < p->head_begin || p->head_end > H) return GF_ERR_INVALID_ARG;
  if (B > 65535 || H > 65535) return GF_ERR_UNSUPPORTED;
  int64_t xs[3], os[3];
  gf_status st;
  if ((st = check_strides(p->x_stride, xs, H, N, d)) != GF_OK) return st;
  if ((st = check_strides(p->o_stride, os, H, N, m)) != GF_OK) return st;
  if (m != d || (d != 64 && d != 128)) return GF_ERR_UNSUPPORTED;
  int impl = p->impl;
  if (impl == GF_IMPL_AUTO) impl = (p->dtype == GF_BF16) ? GF_IMPL_MFMA : GF_IMPL_SCALAR;
  if (impl == GF_IMPL_MFMA && p->dtype != GF_BF16) return GF_ERR_UNSUPPORTED;
  if (B == 0 || N == 0 || p->head_end == p->head_begin) return GF_OK;
  if (!x || !w || !out) return GF_ERR_INVALID_ARG;
  if (((uintptr_t)x | (uintptr_t)w | (uintptr_t)out) & 15u) return GF_ERR_INVALID_ARG;
  if (out == w) return GF_ERR_INVALID_ARG;
  // in place is fine only when every element keeps its address
  if (out == x && (xs[0] != os[0] || xs[1] != os[1] || xs[2] != os[2])) return GF_ERR_INVALID_ARG;
  if ((int64_t)B * (p->head_end - p->head_begin) * N > 0x7fffffffLL) return GF_ERR_UNSUPPORTED;

  FeatureArgs a;
  memset(&a, 0, sizeof(a));
  a.x = TensorView{x, xs[0], xs[1], xs[2]};
  a.w = w;
  a.out = out;
  a.osb = os[0]; a.osh = os[1]; a.osn = os[2];
  a.B = B; a.H = H; a.N = N; a.d = d;
  a.head_begin = p->head_begin;
  a.head_end = p->head_end;
  const hipError_t e = launch_random_features(a, p->dtype == GF_BF16, impl == GF_IMPL_MFMA,
                                              reinterpret_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? GF_OK : GF_ERR_DEVICE;
}

namespace {
// per-token statistics [B, H, N, 2] fp32, rounded up to 256 bytes
size_t bwd_stats_bytes(int B, int H, int N) {
  return ((size_t)B * H * N * 2 * sizeof(float) + 255) / 256 * 256;
}
}  // namespace

size_t gformer_attn_bwd_workspace_bytes(int B, int H, int N, int d, int window,
                                        const gformer_params* p) {
  (void)window;
  if (B <= 0 || H <= 0 || N <= 0) return 0;
  size_t need = bwd_stats_bytes(B, H, N);
  // bidirectional linear heads: the two d x d sums (and their vectors) of every head, each in up
  // to kBidirStateSlots per-segment partials
  if (p && p->bidirectional == 1 && p->n_sparse_heads >= 0 && p->n_sparse_heads < H && d > 0)
    need += (size_t)B * (H - p->n_sparse_heads) * 2 * kBidirStateSlots * ((size_t)d * d + d) * sizeof(float);
  return need;
}

gf_status gformer_attn_bwd(const void* q, const void* k, const void* v, const void* dout, void* dq,
                           void* dk, void* dv, int B, int H, int N, int d, int window,
                           const gformer_params* p, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
  if (!p) return GF_ERR_INVALID_ARG;
  if (p->struct_size != sizeof(gformer_params)) return GF_ERR_INVALID_ARG;
  // a bf16 call runs on the matrix-core kernels (AUTO, MFMA) unless SCALAR asks for the plain-FMA
  // kernels, which are also the fp32 path and, on either storage type, the linear heads of the
  // bidirectional layer.
  if (p->impl == GF_IMPL_MFMA_BLOCKED || p->impl == GF_IMPL_MFMA_STREAM ||
      p->impl == GF_IMPL_MFMA_CHUNK)
    return GF_ERR_UNSUPPORTED;
  if (p->impl == GF_IMPL_MFMA && p->dtype != GF_BF16) return GF_ERR_UNSUPPORTED;
  gformer_params pp = *p;
  pp.impl = GF_IMPL_SCALAR;
  pp.segment_len = 0;
  Resolved r;
  const gf_status st = resolve(B, H, N, d, window, &pp, &r);
  if (st != GF_OK) return st;
  if (p->launch_mask != 0) return GF_ERR_INVALID_ARG;
  if (B == 0 || H == 0 || N == 0) return GF_OK;
  if (!q || !k || !v || !dout || !dq || !dk || !dv) return GF_ERR_INVALID_ARG;
  const void* ins[4] = {q, k, v, dout};
  void* outs[3] = {dq, dk, dv};
  for (const void* x : ins)
    if ((uintptr_t)x & 15u) return GF_ERR_INVALID_ARG;
  for (void* y : outs) {
    if ((uintptr_t)y & 15u) return GF_ERR_INVALID_ARG;
    for (const void* x : ins)
      if (x == y) return GF_ERR_INVALID_ARG;
  }
  if (dq == dk || dq == dv || dk == dv) return GF_ERR_INVALID_ARG;
  const size_t need = gformer_attn_bwd_workspace_bytes(B, H, N, d, window, p);
  if (!workspace || workspace_bytes < need) return GF_ERR_WORKSPACE;
  if ((uintptr_t)workspace & 255u) return GF_ERR_INVALID_ARG;

  BwdArgs a;
  memset(&a, 0, sizeof(a));
  a.q = TensorView{q, r.qs[0], r.qs[1], r.qs[2]};
  a.k = TensorView{k, r.ks[0], r.ks[1], r.ks[2]};
  a.v = TensorView{v, r.vs[0], r.vs[1], r.vs[2]};
  a.dout = TensorView{dout, r.os[0], r.os[1], r.os[2]};
  a.dq = dq; a.dk = dk; a.dv = dv;
  a.B = B; a.H = H; a.N = N; a.d = d;
  a.window = window < N ? window : N;   // a wider window sees no more keys; keeps row + window in range
  a.causal = p->bidirectional ? 0 : 1;
  a.wleft = window_left(window, p->bidirectional, N);
  a.wright = window_right(window, p->bidirectional, N);
  a.H0 = p->n_sparse_heads;
  a.phi = p->phi;
  a.scale = p->softmax_scale;
  a.eps = p->eps;
  a.ws = reinterpret_cast<float*>(workspace);
  a.ws_state = a.causal ? nullptr
                        : reinterpret_cast<float*>(static_cast<char*>(workspace) + bwd_stats_bytes(B, H, N));
  auto launch_linear = [&](hipStream_t on) {
    return a.causal ? launch_linear_backward_mfma(a, on) : launch_linear_backward_bidir_mfma(a, on);
  };
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const bool bf16 = p->dtype == GF_BF16;
  const bool mfma = bf16 && p->impl != GF_IMPL_SCALAR;
  hipError_t e = hipSuccess;
  if (mfma) {
    // The linear scans are one workgroup per head and segment: with fewer of those than compute
    // units the rest of the chip is idle for their whole duration.  With overlap = 1 the windowed
    // heads' passes therefore run beside them on the library's side stream (forked from and
    // joined to the caller's stream by events), and the scans are enqueued first so that their
    // workgroups get their compute units.
    const bool both = a.H0 > 0 && a.H0 < a.H;
    std::lock_guard<std::mutex> lock(g_enqueue_mutex);
    SideStream* side = nullptr;
    if (both && p->overlap) e = side_stream_for_current_device(stream, &side);
    if (side && e == hipSuccess) {
      e = hipEventRecord(side->fork, stream);
      if (e == hipSuccess) {
        e = launch_linear(stream);
        hipError_t f = hipStreamWaitEvent(side->stream, side->fork, 0);
        if (f == hipSuccess) {
          if (e == hipSuccess) e = launch_windowed_backward_mfma(a, side->stream);
          // join whatever happened after the fork
          f = hipEventRecord(side->join, side->stream);
          if (f == hipSuccess) f = hipStreamWaitEvent(stream, side->join, 0);
        }
        if (e == hipSuccess) e = f;
      }
    } else if (e == hipSuccess) {
      e = launch_windowed_backward_mfma(a, stream);
      if (e == hipSuccess) e = launch_linear(stream);
    }
  } else if (a.causal) {
    e = launch_backward_scalar(a, bf16, true, true, stream);
  } else {
    e = launch_backward_scalar(a, bf16, true, false, stream);   // the windowed heads
    if (e == hipSuccess) e = launch_linear_backward_bidir(a, bf16, stream);
  }
  return e == hipSuccess ? GF_OK : GF_ERR_DEVICE;
}

const char* gformer_status_string(gf_status s) {
  switch (s) {
    case GF_OK: return "ok";
    case GF_ERR_INVALID_ARG: return "invalid argument";
    case GF_ERR_UNSUPPORTED: return "unsupported configuration";
    case GF_ERR_WORKSPACE: return "workspace missing or too small";
    case GF_ERR_DEVICE: return "HIP launch or runtime failure";
  }
  return "unknown status";
}

int gformer_version(void) { return 100; }

}  // extern "C"
