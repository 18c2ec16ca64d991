/*
 * gformer.h - C ABI of the GFormer attention forward library for AMD MI355X (gfx950).
 *
 * One call computes one attention layer forward over all heads, as defined in
 * "GFormer: Accelerating Large Language Models with Optimized Transformers on
 * Gaudi Processors" (arXiv 2412.19829):
 *
 *   - Section III-A (overview, Fig. 4): Q, K, V are split along the head dimension.
 *     Heads [0, n_sparse_heads) run windowed causal softmax attention, heads
 *     [n_sparse_heads, H) run causal linear attention.  Head h's result is written to
 *     head h's slot of `out`; the two groups are never summed.
 *   - Section III-B + Eq. 1: windowed head.  Token i attends to the `window` tokens
 *     ending at itself, j in [max(0, i-window+1), i]:
 *         out_i = sum_j softmax_j(softmax_scale * q_i.k_j) v_j
 *   - Section III-C, Algorithm 1: linear head.  With A_i = sum_{j<=i} phi(k_j) (x) v_j and
 *     Z_i = sum_{j<=i} phi(k_j) (token i included before row i is read out):
 *         out_i = phi(q_i)^T A_i / (phi(q_i).Z_i + eps)
 *   - Section II-B: phi(x) = elu(x) + 1 (GF_PHI_ELU1).  GF_PHI_IDENTITY lets the caller
 *     pass already-mapped, strictly positive features (e.g. random features).
 *
 * Conventions
 *   - q, k, v, out are DEVICE pointers, 16-byte aligned, owned by the caller.  The library
 *     never allocates, frees or keeps a pointer.  `out` must not alias an input.
 *   - Element (b, h, n, c) of a tensor lives at base + b*stride[0] + h*stride[1] +
 *     n*stride[2] + c (strides in elements, last dimension contiguous).  All-zero strides
 *     mean dense [B, H, N, d].  The paper's [B, N, H, E] layout is stride = {N*H*d, d, H*d}.
 *     Strides must be multiples of 8 elements (16-byte rows for bf16); the row stride
 *     stride[2] may not exceed 2^20 elements (GF_ERR_UNSUPPORTED beyond).
 *   - `workspace` is a DEVICE pointer of at least gformer_attn_workspace_bytes(...) bytes,
 *     256-byte aligned; may be NULL when that size is 0.  It holds the linear-attention
 *     states carried into each piece and is rewritten by every call that uses it.
 *   - `hip_stream` is a hipStream_t (NULL = default stream).  The call enqueues kernels and
 *     returns; it never synchronises.  With params.overlap = 1 and both head groups present
 *     the windowed heads are enqueued on one library-owned, default-priority side stream per
 *     device that waits for the work already in `hip_stream` and that `hip_stream` waits for
 *     before going on
 *     (an event fork/join, also valid under stream capture); the stream and its two events are
 *     created on first use and kept until the process ends.  Calls are serialised by a mutex
 *     while they enqueue.  Per-device state (that side stream, the scratch of
 *     gformer_attn_fwd_noalloc) is looked up by the CURRENT device: call with the device of
 *     `hip_stream` current; a non-NULL stream of another device is refused with GF_ERR_DEVICE
 *     before anything is launched.
 *   - No exception crosses this boundary.  Argument errors are detected on the host before
 *     anything is launched and reported through gf_status.
 *   - Supported: d in {64, 128}; any N >= 0 (N == 0 or B*H == 0 is a no-op); any window >= 1
 *     (window >= N is full causal attention); 0 <= n_sparse_heads <= H;
 *     chunk in {0, 64, 128, 256} (256 only with d = 64).  Everything else returns
 *     GF_ERR_UNSUPPORTED; nothing falls back silently.
 */
#ifndef GFORMER_H
#define GFORMER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GF_OK = 0,
  GF_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad enum, misaligned pointer/stride */
  GF_ERR_UNSUPPORTED = 2, /* valid request outside what the kernels cover (d, chunk, ...)   */
  GF_ERR_WORKSPACE = 3,   /* workspace missing or smaller than gformer_attn_workspace_bytes */
  GF_ERR_DEVICE = 4       /* a HIP launch or runtime call failed                             */
} gf_status;

typedef enum { GF_F32 = 0, GF_BF16 = 1 } gf_dtype; /* q, k, v, out share one dtype */
typedef enum { GF_PHI_ELU1 = 0, GF_PHI_IDENTITY = 1 } gf_phi;

/* Which implementation runs.  GF_IMPL_AUTO picks the MFMA kernels for bf16 and the scalar
 * fp32 kernels for fp32.  GF_IMPL_SCALAR forces the plain-FMA kernels (fp32 arithmetic on
 * either storage type); GF_IMPL_MFMA with GF_F32 is GF_ERR_UNSUPPORTED.
 * GF_IMPL_MFMA runs the windowed heads by one of two kernels with the same results: a streaming
 * kernel (windows of at most 257 tokens; chosen when the call has at least 1024 blocks of 128
 * queries over all windowed heads) or a kernel that gives each workgroup one block of 128
 * queries (everything else).  GF_IMPL_MFMA_BLOCKED / GF_IMPL_MFMA_STREAM force one of them, for
 * comparison and tests; GF_IMPL_MFMA_STREAM with a wider window is GF_ERR_UNSUPPORTED. */
typedef enum {
  GF_IMPL_AUTO = 0,
  GF_IMPL_SCALAR = 1,
  GF_IMPL_MFMA = 2,
  GF_IMPL_MFMA_BLOCKED = 3,
  GF_IMPL_MFMA_STREAM = 4,
  GF_IMPL_MFMA_CHUNK = 5 /* as GF_IMPL_MFMA, with the causal linear heads read out by the kernel */
                         /* that takes any chunk size, also at chunk 64 (for comparison)        */
} gf_impl;

typedef struct gformer_params {
  uint32_t struct_size;   /* = sizeof(gformer_params); anything else is GF_ERR_INVALID_ARG   */
  int32_t dtype;          /* gf_dtype                                                        */
  int32_t phi;            /* gf_phi, linear heads only                                       */
  int32_t n_sparse_heads; /* H0: heads [0,H0) windowed softmax, heads [H0,H) causal linear   */
  int32_t chunk;          /* linear-attention chunk C of Algorithm 1's chunked form: 64, 128  */
                          /* or 256 tokens, 0 = library picks (64).  The result does not      */
                          /* depend on it.  64 runs a kernel specialised for it; 128 and 256  */
                          /* (256: d = 64 only, a larger tile set does not fit the LDS of a   */
                          /* compute unit) run the general-chunk kernel, causal layers only   */
                          /* in the sense that the bidirectional read-out has no in-chunk     */
                          /* part (there the chunk only sets the granularity of segment_len). */
                          /* The fp32 kernels work in chunks of 32 whatever is asked.         */
  int32_t segment_len;    /* 0 = library picks: every linear head is cut into the same whole */
                          /* number of pieces when that fills most of the chip, else the     */
                          /* chunks of all linear heads are cut into equal pieces with no    */
                          /* regard to head boundaries; one workgroup per piece.  > 0        */
                          /* (multiple of chunk): every head is cut into segments of this    */
                          /* many tokens.  Either way pieces run in parallel and are         */
                          /* stitched with a prefix over their (A, Z) states.                */
  int32_t impl;           /* gf_impl                                                         */
  int32_t launch_mask;    /* 0 = everything.  Otherwise a bit set of GF_LAUNCH_*: only those */
                          /* kernels are enqueued (profiling aid; the skipped stages' data   */
                          /* is taken as already present in the workspace).                  */
  int32_t overlap;        /* 0: everything is enqueued on `hip_stream` one after another.    */
                          /* 1: the windowed heads run on a library-owned side stream that   */
                          /* forks from and joins `hip_stream`, next to the state pass (in   */
                          /* gformer_attn_bwd: next to the linear heads' scans).             */
  int32_t bidirectional;  /* 0: causal (sections III-B, III-C).  1: the encoder / image form of  */
                          /* section IV: windowed heads see the w tokens centred on the token */
                          /* (w/2 to the left, w-1-w/2 to the right, cut at the ends; the     */
                          /* paper does not say how w splits), linear heads see every key:    */
                          /* out_i = phi(q_i)^T (sum_j phi(k_j) v_j^T) / (phi(q_i).sum_j      */
                          /* phi(k_j) + eps), section II-B.                                   */
  float softmax_scale;    /* multiplies q.k on windowed heads; 1.0 when Q is pre-scaled      */
  float eps;              /* added to the linear denominator; 0 follows Algorithm 1          */
  int64_t q_stride[3], k_stride[3], v_stride[3], o_stride[3]; /* (b, h, n) element strides   */
} gformer_params;

enum {
  GF_LAUNCH_WINDOWED = 1,     /* windowed softmax heads                                */
  GF_LAUNCH_LINEAR_STATE = 2, /* per-piece (A, Z) sums + their prefix inside each head */
  GF_LAUNCH_LINEAR_MAIN = 4   /* linear heads read-out                                 */
};

/* What a call with these arguments would launch (host-only; touches no device). */
typedef struct gformer_plan {
  int32_t impl;             /* resolved gf_impl (SCALAR or MFMA)                        */
  int32_t chunk;            /* resolved linear chunk C                                  */
  int32_t segment_len;      /* resolved tokens per piece of linear-attention work       */
  int32_t n_segments;       /* pieces in total (= linear_blocks)                        */
  int32_t windowed_blocks;  /* workgroups of the windowed kernel (0 if H0 == 0)         */
  int32_t windowed_threads;
  int32_t linear_blocks;    /* workgroups of the linear read-out kernel (0 if H0 == H)  */
  int32_t linear_threads;
  int32_t state_blocks;     /* pieces that start inside a head and need a carried state */
  int32_t reserved;
  uint64_t workspace_bytes;
} gformer_plan;

/* Fills `p` with defaults: struct_size, dtype = GF_BF16, phi = GF_PHI_ELU1, H0 = 0, chunk,
 * segment_len, impl, launch_mask = 0, overlap = 0, bidirectional = 0, softmax_scale = 1, eps = 0, dense
 * strides. */
void gformer_params_init(gformer_params* p);

/* Bytes of device workspace gformer_attn_fwd needs for these arguments (0 if none).
 * Returns 0 as well when the arguments are invalid; gformer_attn_fwd reports why. */
size_t gformer_attn_workspace_bytes(int B, int H, int N, int d, int window,
                                    const gformer_params* p);

/* Validates like gformer_attn_fwd (pointers excepted) and describes the launch. */
gf_status gformer_attn_plan(int B, int H, int N, int d, int window, const gformer_params* p,
                            gformer_plan* plan);

/* GFormer attention forward (section III; see the top of this file).
 *   q, k, v : device, read-only, [B,H,N,d] through the strides in `p`
 *   out     : device, written,   [B,H,N,d] through o_stride
 * Enqueues on `hip_stream` and returns without synchronising.
 * Errors: GF_ERR_INVALID_ARG / GF_ERR_UNSUPPORTED / GF_ERR_WORKSPACE before any launch;
 * GF_ERR_DEVICE if HIP reports a launch failure. */
gf_status gformer_attn_fwd(const void* q, const void* k, const void* v, void* out, int B, int H,
                           int N, int d, int window, const gformer_params* p, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

/* gformer_attn_fwd for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results (bit for bit), conventions and errors as gformer_attn_fwd, without
 * `workspace`: the carried linear-attention states go to a device array of
 * GFORMER_NOALLOC_SCRATCH_BYTES that is part of the library's code object (every device that
 * loads the library holds its own copy until the process ends).  The call allocates and frees
 * nothing, on the host or on the device, and creates no stream or event.
 *   - gformer_attn_workspace_bytes(...) > GFORMER_NOALLOC_SCRATCH_BYTES: GF_ERR_WORKSPACE, before
 *     anything is launched (the headline layer B=4 H=32 N=8192 d=128 needs 52.4 MiB, 64.5 MiB with all heads linear).
 *   - params.overlap = 1 (library-owned side stream, created on first use): GF_ERR_UNSUPPORTED.
 *   - Call it with the device of `hip_stream` current.  The first call on a device looks up that
 *     device's address of the array (hipGetSymbolAddress, no allocation); make that first call
 *     outside stream capture.
 *   - All calls on one device share the one array, which keeps the last call's contents: nothing
 *     in it has to start at zero (every slot a call reads was written by that same call), but two
 *     calls that overlap in time on one device (different streams, or graph branches) race.
 *     Calls on one stream, one after another, are safe. */
#define GFORMER_NOALLOC_SCRATCH_BYTES ((size_t)72 << 20)
gf_status gformer_attn_fwd_noalloc(const void* q, const void* k, const void* v, void* out, int B,
                                   int H, int N, int d, int window, const gformer_params* p,
                                   void* hip_stream);

/* One decode step of the causal layer: token `t` of every (batch, head) from what the layer keeps
 * between steps (autoregressive generation; the paper targets LLM inference, its evaluation runs
 * whole sequences).  Windowed heads (section III-B, Eq. 1): the last `window` keys and values live
 * in rings, slot t % window is overwritten with the new row and the min(t+1, window) filled slots
 * are attended to.  Linear heads (Algorithm 1, one pass of its loop): A += phi(k) (x) v,
 * Z += phi(k), out = phi(q)^T A / (phi(q).Z + eps).  Decoding t = 0, 1, ... from zeroed states
 * reproduces gformer_attn_fwd row by row (fp32 arithmetic throughout; bf16 only as storage).
 *   q, k, v : device, dense [B,H,d], the new token, read
 *   out     : device, dense [B,H,d], written; must not alias q, k, v
 *   kcache, vcache : device, dense [B,H0,window,d] rings of the same element type, read and
 *             written; caller-owned, kept between steps; may be NULL when H0 == 0
 *   state   : device, fp32 [B,H-H0,d*d+d]: A row-major [feature][value], then Z; read and
 *             written; zero it before t = 0; may be NULL when H0 == H
 * Of `p` only dtype, phi, n_sparse_heads, softmax_scale and eps are used; bidirectional must be
 * 0.  d in {64,128}; window up to what fits 64 KB of LDS as fp32 scores (about 16,000), else
 * GF_ERR_UNSUPPORTED.  No workspace; asynchronous on `hip_stream`; one step per call, steps of
 * one sequence must be enqueued in order. */
gf_status gformer_attn_decode(const void* q, const void* k, const void* v, void* out, void* kcache,
                              void* vcache, float* state, int B, int H, int d, int window,
                              int64_t t, const gformer_params* p, void* hip_stream);

/* gformer_attn_fwd (causal) that also leaves what gformer_attn_decode continues from: the last
 * `window` keys and values of every windowed head in ring order (token t in slot t % window;
 * slots of tokens that do not exist are left alone) and every linear head's (A, Z) after its last
 * token.  Same arguments, conventions and errors as gformer_attn_fwd, plus
 *   kcache, vcache : device, dense [B,H0,window,d], element type of q; may be NULL when H0 == 0
 *   state          : device, fp32 dense [B,H-H0,d*d+d]; may be NULL when H0 == H
 * params.bidirectional and params.launch_mask must be 0.  The next token to decode is t = N. */
gf_status gformer_attn_prefill(const void* q, const void* k, const void* v, void* out, void* kcache,
                               void* vcache, float* state, int B, int H, int N, int d, int window,
                               const gformer_params* p, void* workspace, size_t workspace_bytes,
                               void* hip_stream);

/* Backward pass of the layer, causal or bidirectional (params.bidirectional): the gradients of a
 * scalar loss with respect to Q, K and V from its gradient with respect to the layer's output.
 * The paper trains its models (sections IV-B to IV-D) but prints no backward formulas: these are
 * the derivatives of section III-B, Eq. 1 (softmax over the window) and of section II-B's ratio
 * with Algorithm 1's running sums (bidirectional: with the sums over all keys), the feature map's
 * slope included.
 *   q, k, v : device, as for gformer_attn_fwd, read
 *   dout    : device, gradient with respect to the layer's output, layout of o_stride, read
 *             (the forward result itself is not an input: what the derivatives need of it is
 *             recomputed in fp32, since the stored result is rounded to the element type)
 *   dq, dk, dv : device, written; laid out like q, k, v (their strides); must not overlap any
 *             input or each other
 *   workspace : device, gformer_attn_bwd_workspace_bytes bytes, 256-byte aligned: 8 bytes per
 *             token and head (per-row softmax statistics / denominators), rounded up to 256,
 *             plus, for a bidirectional call, two (d*d + d) fp32 sums per linear head
 * Kernels: a bf16 call runs on the matrix cores (params.impl GF_IMPL_AUTO or GF_IMPL_MFMA: bf16
 * products, fp32 accumulation, softmax statistics, denominators and carried sums in fp32; the
 * two operands of the linear heads whose rounding would cost more than the bf16 mode's 2e-2 per
 * row, T' and the in-chunk weights of the numerator, travel as bf16 pairs);
 * GF_IMPL_SCALAR and every fp32 call run on plain-FMA kernels (fp32 arithmetic on either
 * storage type).  The linear heads of a bidirectional call take three sweeps over each head (the
 * sums over all keys, dq with the sums over all queries, dk and dv), on the matrix cores for a
 * bf16 call, with the d x d sums and dO / den as bf16 pairs where a difference of nearly equal
 * terms depends on them.  GF_IMPL_MFMA with fp32 storage, GF_IMPL_MFMA_BLOCKED, GF_IMPL_MFMA_STREAM and
 * GF_IMPL_MFMA_CHUNK are GF_ERR_UNSUPPORTED.  params.launch_mask must be 0; segment_len and chunk
 * are ignored.  params.overlap = 1 (matrix-core kernels, both head groups present): the windowed
 * heads' passes run on the library's side stream beside the linear heads' scans, which leave
 * compute units idle when there are fewer heads than units; same fork/join as in
 * gformer_attn_fwd, same results.
 * Asynchronous on `hip_stream`; errors as for gformer_attn_fwd. */
size_t gformer_attn_bwd_workspace_bytes(int B, int H, int N, int d, int window,
                                        const gformer_params* p);
gf_status gformer_attn_bwd(const void* q, const void* k, const void* v, const void* dout, void* dq,
                           void* dk, void* dv, int B, int H, int N, int d, int window,
                           const gformer_params* p, void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/* Positive random features as a pre-map of Q or K for the linear heads.  Section III-A names
 * "positive orthogonal random features" for the linear part and Algorithm 1 "random feature
 * maps"; neither prints them, so the formula is the construction of the work they cite:
 *     out[b,h,n,i] = exp( sum_c w[i][c] * x[b,h,n,c]  -  |x[b,h,n,:]|^2 / 2 ) / sqrt(m)
 * for heads head_begin <= h < head_end (the linear heads); other heads of `out` are not touched.
 * The mapped tensors are then passed to gformer_attn_fwd with phi = GF_PHI_IDENTITY (the windowed
 * heads of that call still read the unmapped heads, so map in place or into a copy).
 *   x   : device, [B,H,N,d] through x_stride, read
 *   w   : device, [m,d] dense row-major, same element type as x; drawing (and orthogonalising)
 *         its rows is the caller's business
 *   out : device, [B,H,N,m] through o_stride, written; may be the same buffer and strides as x
 *         (in place), must not overlap it otherwise
 * Supported: m == d in {64,128} (the carried state of the linear heads is d x d); anything else
 * GF_ERR_UNSUPPORTED.  No workspace.  Asynchronous on `hip_stream`.  Values outside the range of
 * the element type overflow like any other float expression: keep |x| moderate (the cited
 * construction subtracts a stabiliser, which cancels in the attention ratio). */
typedef struct gformer_feature_params {
  uint32_t struct_size;   /* = sizeof(gformer_feature_params)                                */
  int32_t dtype;          /* gf_dtype of x, w and out                                        */
  int32_t head_begin;     /* first head to map                                               */
  int32_t head_end;       /* one past the last head to map                                   */
  int32_t impl;           /* gf_impl; AUTO = MFMA for bf16, scalar for fp32                  */
  int32_t reserved0;
  int64_t x_stride[3], o_stride[3]; /* (b, h, n) element strides; all-zero = dense [B,H,N,d] */
} gformer_feature_params;

/* struct_size set, dtype = GF_BF16, head_begin = head_end = 0, impl = AUTO, dense strides */
void gformer_feature_params_init(gformer_feature_params* p);

gf_status gformer_random_features(const void* x, const void* w, void* out, int B, int H, int N,
                                  int d, int m, const gformer_feature_params* p, void* hip_stream);

/* ---- Head partition model (Section III-D, Algorithm 2 and the two latency estimates) -------
 * Host arithmetic only: no device is touched and no stream is taken.
 *
 * gformer_partition_balance is Algorithm 2 as printed: a share p of `size` units goes to
 * partition 0 and 1-p to partition 1; each partition's latency is its FLOPs (share x size x
 * FLOPs per unit) over its average performance; the result p' is the share at which the two
 * latencies are equal,  p' = (flops_per1/perf1) / (flops_per0/perf0 + flops_per1/perf1).
 *   in       : host, read.  size, perf0, perf1 > 0; flops_per0, flops_per1 >= 0 and not both 0;
 *              p in [0,1] (the initial share; it only selects what latency[0..1] report)
 *   p_prime  : host, written
 *   latency  : host, 4 doubles written, or NULL: latency0(p), latency1(p), latency0(p'),
 *              latency1(p') in seconds when perf is in FLOP/s
 * GF_ERR_INVALID_ARG for a null pointer, a wrong struct_size, a non-finite or out-of-range field. */
typedef struct gformer_partition_inputs {
  uint32_t struct_size;   /* = sizeof(gformer_partition_inputs)                              */
  int32_t reserved0;      /* 0                                                               */
  double p;               /* initial share of partition 0                                    */
  double size;            /* problem size, in the units the FLOP counts are per              */
  double flops_per0, flops_per1; /* FLOPs per unit of partition 0 / 1                        */
  double perf0, perf1;    /* average performance of partition 0 / 1, FLOP/s                  */
} gformer_partition_inputs;

gf_status gformer_partition_balance(const gformer_partition_inputs* in, double* p_prime,
                                    double* latency);

/* The same balance over whole heads, with the FLOP counts of Section III-D: H0 windowed heads
 * cost 2*B*H0*E*N*W (scores) + 3*B*H0*N*W (softmax) FLOPs (the two terms as printed; the total
 * printed under them drops the factor E of the first and is not used), H1 = H-H0 linear heads
 * cost 8*B*N*(H1*E)^2 with GF_FLOPS_PAPER (the printed count, which treats the linear heads as
 * one contraction of width H1*E) or 8*B*N*H1*E^2 with GF_FLOPS_PER_HEAD (heads independent, as
 * the kernels of this library run them).  Returns in *H0 the head count in [0,H] whose two
 * latencies are closest (the smaller count on a tie), and in latency[0..1] (may be NULL) the
 * windowed and the linear latency at that count.
 *   perf_sparse, perf_linear : measured average FLOP/s of the two head kinds under the same
 *                              FLOP count, > 0
 * GF_ERR_INVALID_ARG for null H0, sizes < 1, a bad flop_model or a non-positive performance. */
typedef enum gf_flop_model { GF_FLOPS_PAPER = 0, GF_FLOPS_PER_HEAD = 1 } gf_flop_model;

gf_status gformer_partition_heads(int B, int H, int N, int E, int W, double perf_sparse,
                                  double perf_linear, int flop_model, int* H0, double* latency);

const char* gformer_status_string(gf_status s);

/* major*10000 + minor*100 + patch */
int gformer_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GFORMER_H */
