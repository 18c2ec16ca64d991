"""The differentiable wrapper: loss.backward() through gformer_attention gives the oracle's
gradients (fp32: 1e-5 relative to the gradient's size; bf16: 2e-2 per row)."""
from __future__ import annotations

import numpy as np
import pytest

from oracle import cpu_oracle as co
from paper_2412_19829_amd import inputs as gi
from tests.gpu_util import to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bidirectional", [0, 1], ids=["causal", "bidirectional"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_through_the_wrapper(dtype, bidirectional):
    import torch
    from paper_2412_19829_amd.autograd import gformer_attention
    from tests.test_gpu_parity import check, check_grad
    B, H, N, d, w, H0 = 2, 3, 300, 64, 50, 1
    wl = gi.Workload("ag", B, H, N, d, w, dtype, 4711)
    q, k, v = gi.make_qkv(wl)
    dout = gi.make_qkv(gi.Workload("ag", B, H, N, d, w, dtype, 4712))[2]
    # the paper's [B, N, H, E] storage, handed over as strided [B, H, N, d] views
    tq, tk, tv = (to_device(x, dtype).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3).requires_grad_(True)
                  for x in (q, k, v))
    out = gformer_attention(tq, tk, tv, w, H0, eps=0.25, bidirectional=bidirectional)
    check(to_host(out.detach()), co.attn_fwd(q, k, v, w, H0, eps=0.25, bidirectional=bool(bidirectional)),
          dtype, "forward through the wrapper")
    (out * to_device(dout, dtype)).sum().backward()
    ref = co.attn_bwd(q, k, v, dout, w, H0, eps=0.25, bidirectional=bool(bidirectional))
    for t, r, name in zip((tq, tk, tv), ref, ("dq", "dk", "dv")):
        assert t.grad is not None and t.grad.stride() == t.stride()
        check_grad(to_host(t.grad), r, dtype, name, dout, 0)
