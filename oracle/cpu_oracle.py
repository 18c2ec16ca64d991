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
