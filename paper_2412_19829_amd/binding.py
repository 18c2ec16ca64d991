"""Thin ctypes binding of libgformer_attn.so (see include/gformer.h).

Argument marshalling only: every step of the attention forward runs in the HIP
kernels behind the C ABI.  torch is used by callers for device memory and
streams; this module only reads `data_ptr()` / shapes / strides from tensors.
There is no CPU fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libgformer_attn.so")

GF_OK, GF_ERR_INVALID_ARG, GF_ERR_UNSUPPORTED, GF_ERR_WORKSPACE, GF_ERR_DEVICE = range(5)
GF_F32, GF_BF16 = 0, 1
GF_PHI_ELU1, GF_PHI_IDENTITY = 0, 1
GF_FLOPS_PAPER, GF_FLOPS_PER_HEAD = 0, 1
GF_IMPL_AUTO, GF_IMPL_SCALAR, GF_IMPL_MFMA, GF_IMPL_MFMA_BLOCKED, GF_IMPL_MFMA_STREAM = 0, 1, 2, 3, 4
GF_IMPL_MFMA_CHUNK = 5
GF_LAUNCH_WINDOWED, GF_LAUNCH_LINEAR_STATE, GF_LAUNCH_LINEAR_MAIN = 1, 2, 4

EXPORTS = ("gformer_params_init", "gformer_attn_workspace_bytes", "gformer_attn_plan",
           "gformer_attn_fwd", "gformer_attn_fwd_noalloc", "gformer_attn_prefill", "gformer_attn_decode",
           "gformer_attn_bwd_workspace_bytes", "gformer_attn_bwd",
           "gformer_feature_params_init",
           "gformer_random_features",
           "gformer_partition_balance", "gformer_partition_heads",
           "gformer_status_string", "gformer_version")


class GformerParams(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("phi", ctypes.c_int32), ("n_sparse_heads", ctypes.c_int32),
                ("chunk", ctypes.c_int32), ("segment_len", ctypes.c_int32),
                ("impl", ctypes.c_int32), ("launch_mask", ctypes.c_int32),
                ("overlap", ctypes.c_int32), ("bidirectional", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float), ("eps", ctypes.c_float),
                ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3),
                ("v_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3)]


class GformerPlan(ctypes.Structure):
    _fields_ = [("impl", ctypes.c_int32), ("chunk", ctypes.c_int32),
                ("segment_len", ctypes.c_int32), ("n_segments", ctypes.c_int32),
                ("windowed_blocks", ctypes.c_int32), ("windowed_threads", ctypes.c_int32),
                ("linear_blocks", ctypes.c_int32), ("linear_threads", ctypes.c_int32),
                ("state_blocks", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("workspace_bytes", ctypes.c_uint64)]

    def as_dict(self) -> dict:
        return {n: int(getattr(self, n)) for n, _ in self._fields_ if n != "reserved"}


class GformerFeatureParams(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("head_begin", ctypes.c_int32), ("head_end", ctypes.c_int32),
                ("impl", ctypes.c_int32), ("reserved0", ctypes.c_int32),
                ("x_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3)]


class GformerPartitionInputs(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("reserved0", ctypes.c_int32),
                ("p", ctypes.c_double), ("size", ctypes.c_double),
                ("flops_per0", ctypes.c_double), ("flops_per1", ctypes.c_double),
                ("perf0", ctypes.c_double), ("perf1", ctypes.c_double)]


class GformerError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"gformer status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """Load the shared library (built by paper_2412_19829_amd/build.py).  Fails loudly."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: run `python -m paper_2412_19829_amd.build` "
                "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        P = ctypes.POINTER(GformerParams)
        L.gformer_params_init.restype = None
        L.gformer_params_init.argtypes = [P]
        L.gformer_attn_workspace_bytes.restype = ctypes.c_size_t
        L.gformer_attn_workspace_bytes.argtypes = [ctypes.c_int] * 5 + [P]
        L.gformer_attn_plan.restype = ctypes.c_int
        L.gformer_attn_plan.argtypes = [ctypes.c_int] * 5 + [P, ctypes.POINTER(GformerPlan)]
        L.gformer_attn_fwd.restype = ctypes.c_int
        L.gformer_attn_fwd.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 5 + \
            [P, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.gformer_attn_fwd_noalloc.restype = ctypes.c_int
        L.gformer_attn_fwd_noalloc.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 5 + \
            [P, ctypes.c_void_p]
        L.gformer_attn_prefill.restype = ctypes.c_int
        L.gformer_attn_prefill.argtypes = [ctypes.c_void_p] * 7 + [ctypes.c_int] * 5 + \
            [P, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.gformer_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.gformer_attn_bwd_workspace_bytes.argtypes = [ctypes.c_int] * 5 + [P]
        L.gformer_attn_bwd.restype = ctypes.c_int
        L.gformer_attn_bwd.argtypes = [ctypes.c_void_p] * 7 + [ctypes.c_int] * 5 + \
            [P, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.gformer_attn_decode.restype = ctypes.c_int
        L.gformer_attn_decode.argtypes = [ctypes.c_void_p] * 7 + [ctypes.c_int] * 4 + \
            [ctypes.c_int64, P, ctypes.c_void_p]
        FP = ctypes.POINTER(GformerFeatureParams)
        L.gformer_feature_params_init.restype = None
        L.gformer_feature_params_init.argtypes = [FP]
        L.gformer_random_features.restype = ctypes.c_int
        L.gformer_random_features.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int] * 5 + \
            [FP, ctypes.c_void_p]
        L.gformer_partition_balance.restype = ctypes.c_int
        L.gformer_partition_balance.argtypes = [ctypes.POINTER(GformerPartitionInputs),
                                                ctypes.POINTER(ctypes.c_double),
                                                ctypes.POINTER(ctypes.c_double)]
        L.gformer_partition_heads.restype = ctypes.c_int
        L.gformer_partition_heads.argtypes = [ctypes.c_int] * 5 + [ctypes.c_double] * 2 + \
            [ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_double)]
        L.gformer_status_string.restype = ctypes.c_char_p
        L.gformer_status_string.argtypes = [ctypes.c_int]
        L.gformer_version.restype = ctypes.c_int
        L.gformer_version.argtypes = []
        _lib = L
    return _lib


def gformer_params_init() -> GformerParams:
    p = GformerParams()
    lib().gformer_params_init(ctypes.byref(p))
    return p


def make_params(dtype=GF_BF16, n_sparse_heads=0, phi=GF_PHI_ELU1, chunk=0, segment_len=0,
                impl=GF_IMPL_AUTO, launch_mask=0, overlap=0, bidirectional=0, softmax_scale=1.0,
                eps=0.0, q_stride=None, k_stride=None, v_stride=None, o_stride=None) -> GformerParams:
    p = gformer_params_init()
    p.dtype, p.n_sparse_heads, p.phi = int(dtype), int(n_sparse_heads), int(phi)
    p.chunk, p.segment_len, p.impl, p.launch_mask = int(chunk), int(segment_len), int(impl), int(launch_mask)
    p.overlap = int(overlap)
    p.bidirectional = int(bidirectional)
    p.softmax_scale, p.eps = float(softmax_scale), float(eps)
    for name, val in (("q_stride", q_stride), ("k_stride", k_stride),
                      ("v_stride", v_stride), ("o_stride", o_stride)):
        if val is not None:
            setattr(p, name, (ctypes.c_int64 * 3)(*[int(x) for x in val]))
    return p


def gformer_status_string(status: int) -> str:
    return lib().gformer_status_string(int(status)).decode()


def gformer_version() -> int:
    return int(lib().gformer_version())


def gformer_attn_workspace_bytes(B, H, N, d, window, params: GformerParams) -> int:
    return int(lib().gformer_attn_workspace_bytes(B, H, N, d, window, ctypes.byref(params)))


def gformer_attn_plan(B, H, N, d, window, params: GformerParams):
    """Returns (status, GformerPlan)."""
    plan = GformerPlan()
    st = lib().gformer_attn_plan(B, H, N, d, window, ctypes.byref(params), ctypes.byref(plan))
    return int(st), plan


def gformer_attn_fwd_raw(q_ptr, k_ptr, v_ptr, out_ptr, B, H, N, d, window, params: GformerParams,
                         workspace_ptr=0, workspace_bytes=0, stream=0) -> int:
    """Direct call with integer device addresses; returns the gf_status."""
    return int(lib().gformer_attn_fwd(
        ctypes.c_void_p(q_ptr or None), ctypes.c_void_p(k_ptr or None),
        ctypes.c_void_p(v_ptr or None), ctypes.c_void_p(out_ptr or None),
        int(B), int(H), int(N), int(d), int(window), ctypes.byref(params),
        ctypes.c_void_p(workspace_ptr or None), ctypes.c_size_t(int(workspace_bytes)),
        ctypes.c_void_p(stream or None)))


GFORMER_NOALLOC_SCRATCH_BYTES = 72 << 20


def gformer_attn_fwd_noalloc_raw(q_ptr, k_ptr, v_ptr, out_ptr, B, H, N, d, window,
                                 params: GformerParams, stream=0) -> int:
    """Direct call with integer device addresses; returns the gf_status."""
    return int(lib().gformer_attn_fwd_noalloc(
        ctypes.c_void_p(q_ptr or None), ctypes.c_void_p(k_ptr or None),
        ctypes.c_void_p(v_ptr or None), ctypes.c_void_p(out_ptr or None),
        int(B), int(H), int(N), int(d), int(window), ctypes.byref(params),
        ctypes.c_void_p(stream or None)))


def _strides3(t):
    s = t.stride()
    if s[3] != 1 and t.shape[3] > 1:
        raise ValueError("last dimension must be contiguous")
    return (s[0], s[1], s[2])


def gformer_attn_fwd(q, k, v, out, window: int, n_sparse_heads: int, *, phi=GF_PHI_ELU1,
                     chunk=0, segment_len=0, impl=GF_IMPL_AUTO, launch_mask=0, overlap=0,
                     bidirectional=0, softmax_scale=1.0, eps=0.0, workspace=None,
                     stream: Optional[int] = None):
    """GFormer attention forward on torch device tensors shaped [B, H, N, d] (any strides with
    a contiguous last dimension, e.g. a permuted [B, N, H, d] buffer).

    `out` is written in place and returned.  `workspace` is an optional uint8 device tensor
    of at least gformer_attn_workspace_bytes(...) bytes; when omitted and one is needed it is
    allocated with torch.empty (plumbing: the library itself never allocates).  The call is
    asynchronous on `stream` (a raw hipStream_t; default: torch's current stream)."""
    import torch

    if not (q.is_cuda and k.is_cuda and v.is_cuda and out.is_cuda):
        raise ValueError("q, k, v, out must be device tensors: there is no CPU path")
    if not (q.dtype == k.dtype == v.dtype == out.dtype):
        raise ValueError("q, k, v, out must share one dtype")
    if q.dtype == torch.bfloat16:
        dtype = GF_BF16
    elif q.dtype == torch.float32:
        dtype = GF_F32
    else:
        raise ValueError(f"unsupported dtype {q.dtype}")
    if not (q.shape == k.shape == v.shape == out.shape) or q.dim() != 4:
        raise ValueError("q, k, v, out must all be [B, H, N, d]")
    B, H, N, d = (int(x) for x in q.shape)
    params = make_params(dtype=dtype, n_sparse_heads=n_sparse_heads, phi=phi, chunk=chunk,
                         segment_len=segment_len, impl=impl, launch_mask=launch_mask,
                         overlap=overlap, bidirectional=bidirectional,
                         softmax_scale=softmax_scale, eps=eps,
                         q_stride=_strides3(q), k_stride=_strides3(k),
                         v_stride=_strides3(v), o_stride=_strides3(out))
    need = gformer_attn_workspace_bytes(B, H, N, d, window, params)
    ws_ptr, ws_bytes = 0, 0
    if need > 0:
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    st = gformer_attn_fwd_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                              B, H, N, d, window, params, ws_ptr, ws_bytes, stream)
    if st != GF_OK:
        raise GformerError(st, gformer_status_string(st))
    return out


def gformer_feature_params_init() -> GformerFeatureParams:
    p = GformerFeatureParams()
    lib().gformer_feature_params_init(ctypes.byref(p))
    return p


def make_feature_params(dtype=GF_BF16, head_begin=0, head_end=0, impl=GF_IMPL_AUTO,
                        x_stride=None, o_stride=None) -> GformerFeatureParams:
    p = gformer_feature_params_init()
    p.dtype, p.head_begin, p.head_end, p.impl = int(dtype), int(head_begin), int(head_end), int(impl)
    for name, val in (("x_stride", x_stride), ("o_stride", o_stride)):
        if val is not None:
            setattr(p, name, (ctypes.c_int64 * 3)(*[int(v) for v in val]))
    return p


def gformer_random_features_raw(x_ptr, w_ptr, out_ptr, B, H, N, d, m, params: GformerFeatureParams,
                                stream=0) -> int:
    """Direct call with integer device addresses; returns the gf_status."""
    return int(lib().gformer_random_features(
        ctypes.c_void_p(x_ptr or None), ctypes.c_void_p(w_ptr or None),
        ctypes.c_void_p(out_ptr or None), int(B), int(H), int(N), int(d), int(m),
        ctypes.byref(params), ctypes.c_void_p(stream or None)))


def gformer_random_features(x, w, out, head_begin: int, head_end: int, *, impl=GF_IMPL_AUTO,
                            stream: Optional[int] = None):
    """Positive random features of heads [head_begin, head_end) of x ([B,H,N,d] device tensor)
    under the projection w ([d,d], dense), written to the same heads of `out` (may be x itself)."""
    import torch

    if not (x.is_cuda and w.is_cuda and out.is_cuda):
        raise ValueError("x, w, out must be device tensors: there is no CPU path")
    if not (x.dtype == w.dtype == out.dtype):
        raise ValueError("x, w, out must share one dtype")
    if x.dtype == torch.bfloat16:
        dtype = GF_BF16
    elif x.dtype == torch.float32:
        dtype = GF_F32
    else:
        raise ValueError(f"unsupported dtype {x.dtype}")
    if x.dim() != 4 or out.shape != x.shape or w.dim() != 2 or not w.is_contiguous():
        raise ValueError("x, out must be [B, H, N, d] and w a dense [m, d] matrix")
    B, H, N, d = (int(v) for v in x.shape)
    params = make_feature_params(dtype=dtype, head_begin=head_begin, head_end=head_end, impl=impl,
                                 x_stride=_strides3(x), o_stride=_strides3(out))
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    st = gformer_random_features_raw(x.data_ptr(), w.data_ptr(), out.data_ptr(), B, H, N, d,
                                     int(w.shape[0]), params, stream)
    if st != GF_OK:
        raise GformerError(st, gformer_status_string(st))
    return out


def gformer_attn_decode_raw(q_ptr, k_ptr, v_ptr, out_ptr, kcache_ptr, vcache_ptr, state_ptr, B, H, d,
                            window, t, params: GformerParams, stream=0) -> int:
    """Direct call with integer device addresses; returns the gf_status."""
    vp = lambda x: ctypes.c_void_p(x or None)
    return int(lib().gformer_attn_decode(vp(q_ptr), vp(k_ptr), vp(v_ptr), vp(out_ptr), vp(kcache_ptr),
                                         vp(vcache_ptr), vp(state_ptr), int(B), int(H), int(d),
                                         int(window), ctypes.c_int64(int(t)), ctypes.byref(params),
                                         vp(stream)))


def gformer_attn_decode(q, k, v, out, kcache, vcache, state, window: int, n_sparse_heads: int, t: int,
                        *, phi=GF_PHI_ELU1, softmax_scale=1.0, eps=0.0, stream: Optional[int] = None):
    """One decode step on dense device tensors: q, k, v, out [B, H, d]; kcache, vcache
    [B, H0, window, d] (or None when H0 == 0); state fp32 [B, H - H0, d*d + d] (or None)."""
    import torch

    ts = [x for x in (q, k, v, out, kcache, vcache, state) if x is not None]
    if not all(x.is_cuda and x.is_contiguous() for x in ts):
        raise ValueError("decode tensors must be dense device tensors: there is no CPU path")
    if q.dtype == torch.bfloat16:
        dtype = GF_BF16
    elif q.dtype == torch.float32:
        dtype = GF_F32
    else:
        raise ValueError(f"unsupported dtype {q.dtype}")
    B, H, d = (int(x) for x in q.shape)
    if any(x.shape != q.shape or x.dtype != q.dtype for x in (k, v, out)):
        raise ValueError("q, k, v, out must all be [B, H, d] of one dtype")
    H0 = int(n_sparse_heads)
    if H0 > 0 and (kcache is None or vcache is None or kcache.dtype != q.dtype
                   or tuple(kcache.shape) != (B, H0, window, d) or vcache.shape != kcache.shape):
        raise ValueError("kcache, vcache must be [B, H0, window, d] of the same dtype")
    if H0 < H and (state is None or state.dtype != torch.float32
                   or tuple(state.shape) != (B, H - H0, d * d + d)):
        raise ValueError("state must be fp32 [B, H - H0, d*d + d]")
    params = make_params(dtype=dtype, n_sparse_heads=H0, phi=phi, softmax_scale=softmax_scale, eps=eps)
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    ptr = lambda x: 0 if x is None else x.data_ptr()
    st = gformer_attn_decode_raw(ptr(q), ptr(k), ptr(v), ptr(out), ptr(kcache), ptr(vcache), ptr(state),
                                 B, H, d, window, t, params, stream)
    if st != GF_OK:
        raise GformerError(st, gformer_status_string(st))
    return out


def gformer_attn_prefill_raw(q_ptr, k_ptr, v_ptr, out_ptr, kcache_ptr, vcache_ptr, state_ptr, B, H, N, d,
                             window, params: GformerParams, workspace_ptr=0, workspace_bytes=0,
                             stream=0) -> int:
    """Direct call with integer device addresses; returns the gf_status."""
    vp = lambda x: ctypes.c_void_p(x or None)
    return int(lib().gformer_attn_prefill(vp(q_ptr), vp(k_ptr), vp(v_ptr), vp(out_ptr), vp(kcache_ptr),
                                          vp(vcache_ptr), vp(state_ptr), int(B), int(H), int(N), int(d),
                                          int(window), ctypes.byref(params), vp(workspace_ptr),
                                          ctypes.c_size_t(int(workspace_bytes)), vp(stream)))


def gformer_attn_prefill(q, k, v, out, kcache, vcache, state, window: int, n_sparse_heads: int, *,
                         phi=GF_PHI_ELU1, impl=GF_IMPL_AUTO, softmax_scale=1.0, eps=0.0,
                         workspace=None, stream: Optional[int] = None):
    """The causal layer on [B, H, N, d] device tensors that also fills the decode step's rings
    (kcache, vcache: dense [B, H0, window, d]) and carried states (fp32 [B, H - H0, d*d + d])."""
    import torch

    if not all(x.is_cuda for x in (q, k, v, out)):
        raise ValueError("q, k, v, out must be device tensors: there is no CPU path")
    dtype = GF_BF16 if q.dtype == torch.bfloat16 else GF_F32
    B, H, N, d = (int(x) for x in q.shape)
    for x in (kcache, vcache, state):
        if x is not None and not (x.is_cuda and x.is_contiguous()):
            raise ValueError("rings and states must be dense device tensors")
    params = make_params(dtype=dtype, n_sparse_heads=n_sparse_heads, phi=phi, impl=impl,
                         softmax_scale=softmax_scale, eps=eps, q_stride=_strides3(q),
                         k_stride=_strides3(k), v_stride=_strides3(v), o_stride=_strides3(out))
    need = gformer_attn_workspace_bytes(B, H, N, d, window, params)
    ws_ptr, ws_bytes = 0, 0
    if need > 0:
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    ptr = lambda x: 0 if x is None else x.data_ptr()
    st = gformer_attn_prefill_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), ptr(kcache),
                                  ptr(vcache), ptr(state), B, H, N, d, window, params, ws_ptr, ws_bytes,
                                  stream)
    if st != GF_OK:
        raise GformerError(st, gformer_status_string(st))
    return out


def gformer_attn_bwd_workspace_bytes(B, H, N, d, window, params: GformerParams) -> int:
    return int(lib().gformer_attn_bwd_workspace_bytes(B, H, N, d, window, ctypes.byref(params)))


def gformer_attn_bwd_raw(q_ptr, k_ptr, v_ptr, dout_ptr, dq_ptr, dk_ptr, dv_ptr, B, H, N, d, window,
                         params: GformerParams, workspace_ptr=0, workspace_bytes=0, stream=0) -> int:
    """Direct call with integer device addresses; returns the gf_status."""
    vp = lambda x: ctypes.c_void_p(x or None)
    return int(lib().gformer_attn_bwd(vp(q_ptr), vp(k_ptr), vp(v_ptr), vp(dout_ptr), vp(dq_ptr),
                                      vp(dk_ptr), vp(dv_ptr), int(B), int(H), int(N), int(d), int(window),
                                      ctypes.byref(params), vp(workspace_ptr),
                                      ctypes.c_size_t(int(workspace_bytes)), vp(stream)))


def gformer_attn_bwd(q, k, v, dout, dq, dk, dv, window: int, n_sparse_heads: int, *,
                     phi=GF_PHI_ELU1, impl=GF_IMPL_AUTO, softmax_scale=1.0, eps=0.0, overlap=0,
                     bidirectional=0, workspace=None, stream: Optional[int] = None):
    """Backward of the layer (causal or bidirectional) on [B, H, N, d] device tensors: fills dq,
    dk, dv (laid out like q, k, v) from `dout`, the gradient with respect to the layer's output."""
    import torch

    if not all(x.is_cuda for x in (q, k, v, dout, dq, dk, dv)):
        raise ValueError("all tensors must be device tensors: there is no CPU path")
    if _strides3(dq) != _strides3(q) or _strides3(dk) != _strides3(k) or _strides3(dv) != _strides3(v):
        raise ValueError("dq, dk, dv must be laid out like q, k, v")
    dtype = GF_BF16 if q.dtype == torch.bfloat16 else GF_F32
    B, H, N, d = (int(x) for x in q.shape)
    params = make_params(dtype=dtype, n_sparse_heads=n_sparse_heads, phi=phi, impl=impl,
                         softmax_scale=softmax_scale, eps=eps, overlap=overlap,
                         bidirectional=bidirectional, q_stride=_strides3(q),
                         k_stride=_strides3(k), v_stride=_strides3(v), o_stride=_strides3(dout))
    need = gformer_attn_bwd_workspace_bytes(B, H, N, d, window, params)
    ws_ptr, ws_bytes = 0, 0
    if need > 0:
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    st = gformer_attn_bwd_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(),
                              dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), B, H, N, d, window, params,
                              ws_ptr, ws_bytes, stream)
    if st != GF_OK:
        raise GformerError(st, gformer_status_string(st))
    return dq, dk, dv


def gformer_partition_balance(p, size, flops_per0, flops_per1, perf0, perf1):
    """Algorithm 2 through the C ABI (host arithmetic).  Returns (p', [latency0(p), latency1(p),
    latency0(p'), latency1(p')])."""
    inp = GformerPartitionInputs(ctypes.sizeof(GformerPartitionInputs), 0, p, size, flops_per0,
                                 flops_per1, perf0, perf1)
    pp = ctypes.c_double()
    lat = (ctypes.c_double * 4)()
    st = int(lib().gformer_partition_balance(ctypes.byref(inp), ctypes.byref(pp), lat))
    if st != GF_OK:
        raise GformerError(st, gformer_status_string(st))
    return pp.value, list(lat)


def gformer_partition_heads(B, H, N, E, W, perf_sparse, perf_linear, flop_model=GF_FLOPS_PAPER):
    """The balance of Section III-D over whole heads.  Returns (H0, [windowed latency, linear
    latency])."""
    h0 = ctypes.c_int()
    lat = (ctypes.c_double * 2)()
    st = int(lib().gformer_partition_heads(int(B), int(H), int(N), int(E), int(W), float(perf_sparse),
                                           float(perf_linear), int(flop_model), ctypes.byref(h0), lat))
    if st != GF_OK:
        raise GformerError(st, gformer_status_string(st))
    return h0.value, list(lat)
