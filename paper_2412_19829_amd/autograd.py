"""The layer as a differentiable PyTorch operation: gformer_attn_fwd in forward,
gformer_attn_bwd in backward.

Plumbing only: tensors are allocated here (PyTorch is used for device memory and streams) and
every arithmetic step runs in the HIP kernels behind the C ABI.  There is no CPU path.
"""
from __future__ import annotations

import torch

from . import binding as gb


class _GformerAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, window, n_sparse_heads, phi, softmax_scale, eps, bidirectional):
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
        gb.gformer_attn_fwd(q, k, v, out, window, n_sparse_heads, phi=phi, softmax_scale=softmax_scale,
                            eps=eps, bidirectional=bidirectional)
        ctx.save_for_backward(q, k, v)
        ctx.cfg = (int(window), int(n_sparse_heads), int(phi), float(softmax_scale), float(eps),
                   int(bidirectional))
        return out

    @staticmethod
    def backward(ctx, dout):
        q, k, v = ctx.saved_tensors
        window, n_sparse_heads, phi, softmax_scale, eps, bidirectional = ctx.cfg
        if dout.stride(-1) != 1:
            dout = dout.contiguous()
        # gradients are laid out like the tensors they belong to
        dq, dk, dv = (torch.empty_strided(t.shape, t.stride(), dtype=t.dtype, device=t.device)
                      for t in (q, k, v))
        gb.gformer_attn_bwd(q, k, v, dout, dq, dk, dv, window, n_sparse_heads, phi=phi,
                            softmax_scale=softmax_scale, eps=eps, bidirectional=bidirectional)
        return dq, dk, dv, None, None, None, None, None, None


def gformer_attention(q, k, v, window: int, n_sparse_heads: int, *, phi=gb.GF_PHI_ELU1,
                      softmax_scale: float = 1.0, eps: float = 0.0, bidirectional: int = 0):
    """GFormer attention on [B, H, N, d] device tensors (bf16 or fp32, any strides with a
    contiguous last dimension): heads [0, n_sparse_heads) windowed softmax, the rest linear.
    Differentiable with respect to q, k and v."""
    return _GformerAttention.apply(q, k, v, window, n_sparse_heads, phi, softmax_scale, eps,
                                   bidirectional)
