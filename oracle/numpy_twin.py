"""Second, independently written fp64 statement of GFormer attention forward, in
numpy with plain Python loops over tokens.  TEST INFRASTRUCTURE ONLY; for small N.

It exists so that the C oracle is not its own only witness: the two were written
separately from the paper's definitions (section III-A head split, section III-B
window, Eq. 1 softmax, Algorithm 1 recurrence, section II-B feature map) and are
compared on small shapes by the CPU tests.
"""
from __future__ import annotations

import numpy as np


def phi_elu1(x: np.ndarray) -> np.ndarray:
    """Section II-B: phi(x) = elu(x) + 1."""
    x = np.asarray(x, np.float64)
    return np.where(x > 0, x + 1.0, np.exp(np.minimum(x, 0.0)))


def windowed_head(q, k, v, window: int, scale: float = 1.0) -> np.ndarray:
    """Section III-B: token i sees keys i-w+1 .. i (clipped at 0); Eq. 1 softmax over them."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    N, d = q.shape
    out = np.zeros((N, d))
    for i in range(N):
        lo = max(0, i - window + 1)
        s = scale * (k[lo:i + 1] @ q[i])
        e = np.exp(s - s.max())
        out[i] = (e / e.sum()) @ v[lo:i + 1]
    return out


def linear_head_recurrent(q, k, v, phi=phi_elu1, eps: float = 0.0) -> np.ndarray:
    """Algorithm 1: A += phi(K_i) (x) V_i ; Z += phi(K_i) ; H_i = phi(Q_i)^T A / (phi(Q_i).Z)."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    N, d = q.shape
    A = np.zeros((d, v.shape[1]))
    Z = np.zeros(d)
    out = np.zeros((N, v.shape[1]))
    for i in range(N):
        qp, kp = phi(q[i]), phi(k[i])
        A += np.outer(kp, v[i])
        Z += kp
        out[i] = (qp @ A) / (qp @ Z + eps)
    return out


def linear_head_quadratic(q, k, v, phi=phi_elu1, eps: float = 0.0) -> np.ndarray:
    """Section II-B form restricted to j <= i: weights a_ij = phi(q_i).phi(k_j)."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    a = np.tril(phi(q) @ phi(k).T)
    return (a @ v) / (a.sum(axis=1, keepdims=True) + eps)


def attn_fwd(q, k, v, window: int, n_sparse_heads: int, phi=phi_elu1, softmax_scale: float = 1.0,
             eps: float = 0.0) -> np.ndarray:
    """Section III-A: heads [0, H0) windowed, heads [H0, H) linear; [B, H, N, d]."""
    q = np.asarray(q, np.float64)
    B, H, N, d = q.shape
    out = np.zeros((B, H, N, d))
    for b in range(B):
        for h in range(H):
            if h < n_sparse_heads:
                out[b, h] = windowed_head(q[b, h], k[b, h], v[b, h], window, softmax_scale)
            else:
                out[b, h] = linear_head_recurrent(q[b, h], k[b, h], v[b, h], phi, eps)
    return out
