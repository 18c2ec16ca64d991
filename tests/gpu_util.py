"""Plumbing for the GPU tests: numpy -> device tensors -> C ABI -> numpy.  No arithmetic."""
from __future__ import annotations

import numpy as np

from paper_2412_19829_amd import binding as gb
from paper_2412_19829_amd import inputs as gi

F32_MAX_ABS = 1e-5      # fp32 mode: max-abs error vs the fp64 oracle
BF16_ROW_REL_L2 = 2e-2  # bf16 mode: per-row ||gpu - oracle||_2 / ||oracle||_2


def to_device(x: np.ndarray, dtype: str):
    import torch
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda()
    bits = gi.f32_to_bf16_bits(x)
    assert np.array_equal(gi.bf16_bits_to_f32(bits), x.astype(np.float32)), "inputs must be bf16-exact"
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_host(t) -> np.ndarray:
    import torch
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return gi.bf16_bits_to_f32(bits).astype(np.float64)
    return t.float().cpu().numpy().astype(np.float64)


def run_gpu(q, k, v, dtype: str, window: int, n_sparse_heads: int, layout: str = "bhnd", **kw):
    """q, k, v: float32 numpy [B,H,N,d] (bf16-exact when dtype == 'bf16').  Returns float64."""
    import torch
    tq, tk, tv = (to_device(x, dtype) for x in (q, k, v))
    if layout == "bnhd":   # the paper's [B, N, H, E] storage, viewed as [B, H, N, d]
        tq, tk, tv = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (tq, tk, tv))
        out = torch.full_like(tq.permute(0, 2, 1, 3).contiguous(), float("nan")).permute(0, 2, 1, 3)
    else:
        out = torch.full_like(tq, float("nan"))
    gb.gformer_attn_fwd(tq, tk, tv, out, window, n_sparse_heads, **kw)
    torch.cuda.synchronize()
    return to_host(out)
