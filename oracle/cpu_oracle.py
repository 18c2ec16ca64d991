"""ctypes front end of the C fp64 oracle (oracle/gformer_oracle.c).  TEST INFRASTRUCTURE ONLY.

All functions take and return float64 numpy arrays; layout [B, H, N, d] for the
layer call and [N, d] for the per-head calls.  See the C file for the passages of
the paper each routine follows.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

PHI_ELU1 = 0
PHI_IDENTITY = 1
LINEAR_QUADRATIC = 0
LINEAR_RECURRENT = 1

_lib = None
_dp = ctypes.POINTER(ctypes.c_double)


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        L.gformer_oracle_windowed_head_f64.restype = ctypes.c_int
        L.gformer_oracle_windowed_head_f64.argtypes = [_dp, _dp, _dp, _dp, ctypes.c_int,
                                                       ctypes.c_int, ctypes.c_int, ctypes.c_double]
        for name in ("gformer_oracle_linear_head_quadratic_f64",
                     "gformer_oracle_linear_head_recurrent_f64"):
            f = getattr(L, name)
            f.restype = ctypes.c_int
            f.argtypes = [_dp, _dp, _dp, _dp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                          ctypes.c_double]
        L.gformer_oracle_fwd_f64.restype = ctypes.c_int
        L.gformer_oracle_fwd_f64.argtypes = [_dp, _dp, _dp, _dp] + [ctypes.c_int] * 7 + \
            [ctypes.c_double, ctypes.c_double, ctypes.c_int, ctypes.c_int]
        L.gformer_oracle_windowed_head_bidir_f64.restype = ctypes.c_int
        L.gformer_oracle_windowed_head_bidir_f64.argtypes = L.gformer_oracle_windowed_head_f64.argtypes
        for name in ("gformer_oracle_linear_head_bidir_f64", "gformer_oracle_linear_head_bidir_state_f64"):
            f = getattr(L, name)
            f.restype = ctypes.c_int
            f.argtypes = L.gformer_oracle_linear_head_quadratic_f64.argtypes
        L.gformer_oracle_fwd_bidir_f64.restype = ctypes.c_int
        L.gformer_oracle_fwd_bidir_f64.argtypes = L.gformer_oracle_fwd_f64.argtypes
        L.gformer_oracle_decode_windowed_f64.restype = ctypes.c_int
        L.gformer_oracle_decode_windowed_f64.argtypes = [_dp] * 6 + [ctypes.c_int, ctypes.c_int,
                                                                  ctypes.c_long, ctypes.c_double]
        L.gformer_oracle_decode_linear_f64.restype = ctypes.c_int
        L.gformer_oracle_decode_linear_f64.argtypes = [_dp] * 6 + [ctypes.c_int, ctypes.c_int,
                                                                ctypes.c_double]
        L.gformer_oracle_windowed_head_bwd_f64.restype = ctypes.c_int
        L.gformer_oracle_windowed_head_bwd_f64.argtypes = [_dp] * 7 + [ctypes.c_int] * 3 + [ctypes.c_double]
        L.gformer_oracle_linear_head_bwd_f64.restype = ctypes.c_int
        L.gformer_oracle_linear_head_bwd_f64.argtypes = [_dp] * 7 + [ctypes.c_int] * 3 + [ctypes.c_double]
        L.gformer_oracle_bwd_f64.restype = ctypes.c_int
        L.gformer_oracle_bwd_f64.argtypes = [_dp] * 7 + [ctypes.c_int] * 7 + [ctypes.c_double] * 2
        for name, like in (("gformer_oracle_windowed_head_bidir_bwd_f64", L.gformer_oracle_windowed_head_bwd_f64),
                           ("gformer_oracle_linear_head_bidir_bwd_f64", L.gformer_oracle_linear_head_bwd_f64),
                           ("gformer_oracle_bwd_bidir_f64", L.gformer_oracle_bwd_f64)):
            f = getattr(L, name)
            f.restype = ctypes.c_int
            f.argtypes = like.argtypes
        L.gformer_oracle_max_threads.restype = ctypes.c_int
        L.gformer_oracle_random_features_f64.restype = ctypes.c_int
        L.gformer_oracle_random_features_f64.argtypes = [_dp, _dp, _dp, ctypes.c_long,
                                                         ctypes.c_int, ctypes.c_int]
        _lib = L
    return _lib


def _c(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_dp)


def windowed_head(q, k, v, window, scale=1.0, bidirectional=False):
    """Causal: the w tokens ending at i.  Bidirectional: the w tokens centred on i."""
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v)
    N, d = q.shape
    out = np.empty((N, d), np.float64)
    fn = (lib().gformer_oracle_windowed_head_bidir_f64 if bidirectional
          else lib().gformer_oracle_windowed_head_f64)
    rc = fn(qp, kp, vp, out.ctypes.data_as(_dp), N, d, int(window), float(scale))
    if rc:
        raise RuntimeError(f"oracle windowed head failed: {rc}")
    return out


def linear_head(q, k, v, phi=PHI_ELU1, eps=0.0, form=LINEAR_QUADRATIC, bidirectional=False):
    """form: explicit sum over keys (LINEAR_QUADRATIC) or running / total state (LINEAR_RECURRENT)."""
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v)
    N, d = q.shape
    out = np.empty((N, d), np.float64)
    if bidirectional:
        fn = (lib().gformer_oracle_linear_head_bidir_state_f64 if form == LINEAR_RECURRENT
              else lib().gformer_oracle_linear_head_bidir_f64)
    else:
        fn = (lib().gformer_oracle_linear_head_recurrent_f64 if form == LINEAR_RECURRENT
              else lib().gformer_oracle_linear_head_quadratic_f64)
    rc = fn(qp, kp, vp, out.ctypes.data_as(_dp), N, d, int(phi), float(eps))
    if rc:
        raise RuntimeError(f"oracle linear head failed: {rc}")
    return out


def attn_fwd(q, k, v, window, n_sparse_heads, phi=PHI_ELU1, softmax_scale=1.0, eps=0.0,
             linear_form=LINEAR_QUADRATIC, threads=0, bidirectional=False):
    """Whole layer over dense [B, H, N, d]; heads [0, n_sparse_heads) windowed, rest linear."""
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v)
    B, H, N, d = q.shape
    out = np.empty((B, H, N, d), np.float64)
    fwd = lib().gformer_oracle_fwd_bidir_f64 if bidirectional else lib().gformer_oracle_fwd_f64
    rc = fwd(qp, kp, vp, out.ctypes.data_as(_dp), B, H, N, d,
                                      int(window), int(n_sparse_heads), int(phi),
                                      float(softmax_scale), float(eps), int(linear_form),
                                      int(threads))
    if rc:
        raise RuntimeError(f"oracle layer call failed: {rc}")
    return out


def windowed_head_bwd(q, k, v, dout, window, scale=1.0, bidirectional=False):
    """Gradients (dq, dk, dv) of a windowed head (causal window, or the window centred on the
    token), [N, d] each, for output gradient dout."""
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v); dout, dop = _c(dout)
    N, d = q.shape
    dq, dk, dv = (np.empty((N, d), np.float64) for _ in range(3))
    fn = lib().gformer_oracle_windowed_head_bidir_bwd_f64 if bidirectional else \
        lib().gformer_oracle_windowed_head_bwd_f64
    rc = fn(qp, kp, vp, dop, dq.ctypes.data_as(_dp),
                                                    dk.ctypes.data_as(_dp), dv.ctypes.data_as(_dp),
                                                    N, d, int(window), float(scale))
    if rc:
        raise RuntimeError(f"oracle windowed backward failed: {rc}")
    return dq, dk, dv


def linear_head_bwd(q, k, v, dout, phi=PHI_ELU1, eps=0.0, bidirectional=False):
    """Gradients (dq, dk, dv) of a linear head (causal, or over all keys), [N, d] each, for output
    gradient dout."""
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v); dout, dop = _c(dout)
    N, d = q.shape
    dq, dk, dv = (np.empty((N, d), np.float64) for _ in range(3))
    fn = lib().gformer_oracle_linear_head_bidir_bwd_f64 if bidirectional else \
        lib().gformer_oracle_linear_head_bwd_f64
    rc = fn(qp, kp, vp, dop, dq.ctypes.data_as(_dp),
                                                  dk.ctypes.data_as(_dp), dv.ctypes.data_as(_dp),
                                                  N, d, int(phi), float(eps))
    if rc:
        raise RuntimeError(f"oracle linear backward failed: {rc}")
    return dq, dk, dv


def attn_bwd(q, k, v, dout, window, n_sparse_heads, phi=PHI_ELU1, softmax_scale=1.0, eps=0.0,
             bidirectional=False):
    """Backward of the layer (causal or bidirectional) over dense [B, H, N, d]: (dq, dk, dv)."""
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v); dout, dop = _c(dout)
    B, H, N, d = q.shape
    dq, dk, dv = (np.empty((B, H, N, d), np.float64) for _ in range(3))
    fn = lib().gformer_oracle_bwd_bidir_f64 if bidirectional else lib().gformer_oracle_bwd_f64
    rc = fn(qp, kp, vp, dop, dq.ctypes.data_as(_dp), dk.ctypes.data_as(_dp),
                                      dv.ctypes.data_as(_dp), B, H, N, d, int(window),
                                      int(n_sparse_heads), int(phi), float(softmax_scale), float(eps))
    if rc:
        raise RuntimeError(f"oracle layer backward failed: {rc}")
    return dq, dk, dv


def _inplace(a):
    if not (isinstance(a, np.ndarray) and a.dtype == np.float64 and a.flags.c_contiguous):
        raise ValueError("state arrays must be C-contiguous float64 (they are updated in place)")
    return a.ctypes.data_as(_dp)


def decode_windowed(q, k, v, kring, vring, t, scale=1.0):
    """One decode step of a windowed head: q, k, v are [d]; kring, vring [window, d] are updated
    in place (slot t % window); returns row t of the causal windowed head."""
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v)
    window, d = kring.shape
    out = np.empty(d, np.float64)
    rc = lib().gformer_oracle_decode_windowed_f64(qp, kp, vp, out.ctypes.data_as(_dp), _inplace(kring),
                                                  _inplace(vring), d, window, int(t), float(scale))
    if rc:
        raise RuntimeError(f"oracle windowed decode failed: {rc}")
    return out


def decode_linear(q, k, v, A, Z, phi=PHI_ELU1, eps=0.0):
    """One decode step of a linear head (Algorithm 1's loop body): A [d, d] and Z [d] are updated
    in place; returns H_t."""
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v)
    d = q.shape[0]
    out = np.empty(d, np.float64)
    rc = lib().gformer_oracle_decode_linear_f64(qp, kp, vp, out.ctypes.data_as(_dp), _inplace(A),
                                                _inplace(Z), d, int(phi), float(eps))
    if rc:
        raise RuntimeError(f"oracle linear decode failed: {rc}")
    return out


def random_features(x, w):
    """Positive random features of the rows of x ([..., d]) under projection w ([m, d]):
    exp(w_i . x - |x|^2 / 2) / sqrt(m), shape [..., m] (section III-A's alternative phi)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    w, wp = _c(w)
    m, d = w.shape
    if x.shape[-1] != d:
        raise ValueError("x and w disagree on d")
    rows = int(np.prod(x.shape[:-1], dtype=np.int64))
    out = np.empty(x.shape[:-1] + (m,), np.float64)
    rc = lib().gformer_oracle_random_features_f64(x.ctypes.data_as(_dp), wp, out.ctypes.data_as(_dp),
                                                  rows, d, m)
    if rc:
        raise RuntimeError(f"oracle random features failed: {rc}")
    return out


def max_threads() -> int:
    return int(lib().gformer_oracle_max_threads())


# ---- Head partition model (Section III-D) -------------------------------------------------
# Plain Python floats (fp64).  The "find p'" step of Algorithm 2 is done here by bisection on
# the share: latency0 grows and latency1 shrinks with it, so their difference crosses zero once.

FLOPS_PAPER = 0      # linear heads counted as one contraction of width H1*E (the printed count)
FLOPS_PER_HEAD = 1   # linear heads counted one by one


def partition_latencies(p, size, flops_per0, flops_per1, perf0, perf1):
    """The first four steps of Algorithm 2 at share p: FLOPs of each partition, then latency =
    FLOPs / average performance."""
    flops_p0 = p * size * flops_per0
    flops_p1 = (1.0 - p) * size * flops_per1
    latency0 = flops_p0 / perf0
    latency1 = flops_p1 / perf1
    return latency0, latency1


def partition_balance(p, size, flops_per0, flops_per1, perf0, perf1, iters=200):
    """Algorithm 2: the share p' of partition 0 at which latency0 == latency1.  `p` is the
    initial share of the printed algorithm; the search does not depend on it."""
    lo, hi = 0.0, 1.0
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        l0, l1 = partition_latencies(mid, size, flops_per0, flops_per1, perf0, perf1)
        if l0 < l1:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def sparse_flops(B, H0, N, E, W):
    """Section III-D: scores 2*B*H0*E*N*W plus softmax 3*B*H0*N*W (the two printed terms)."""
    return 2.0 * B * H0 * E * N * W + 3.0 * B * H0 * N * W


def linear_flops(B, H1, N, E, flop_model=FLOPS_PAPER):
    """Section III-D: feature maps 4BN(H1 E)^2, phi(K)^T V 2BN(H1 E)^2, phi(Q) C 2BN(H1 E)^2."""
    if flop_model == FLOPS_PAPER:
        width2 = float(H1 * E) ** 2
    else:
        width2 = float(H1) * float(E) ** 2
    return 4.0 * B * N * width2 + 2.0 * B * N * width2 + 2.0 * B * N * width2


def partition_heads(B, H, N, E, W, perf_sparse, perf_linear, flop_model=FLOPS_PAPER):
    """The head count H0 in [0,H] whose windowed latency (sparse FLOPs / perf_sparse) is closest
    to the linear latency of the other H-H0 heads; the smaller count on a tie.  Returns
    (H0, latency_sparse, latency_linear)."""
    best = None
    for h0 in range(H + 1):
        ls = sparse_flops(B, h0, N, E, W) / perf_sparse
        ll = linear_flops(B, H - h0, N, E, flop_model) / perf_linear
        gap = abs(ls - ll)
        if best is None or gap < best[0]:
            best = (gap, h0, ls, ll)
    return best[1], best[2], best[3]
