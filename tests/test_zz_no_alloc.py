"""The entry point that allocates nothing (gformer_attn_fwd_noalloc: carried states in a device
array inside the library) against gformer_attn_fwd with a caller's workspace, through the C ABI:
same bits, on two calls in a row, the second with a smaller input (the shared array keeps the
first call's contents).  Collected last: it shares one device array with nothing else."""
from __future__ import annotations

import numpy as np
import pytest

from oracle import cpu_oracle as co
from paper_2412_19829_amd import binding as gb
from paper_2412_19829_amd import inputs as gi
from tests.gpu_util import BF16_ROW_REL_L2, to_device, to_host
from tests.helpers import row_rel_l2


def _params(B, H, N, d, H0, t):
    def strides(x):
        s = x.stride()
        return (s[0], s[1], s[2])
    return gb.make_params(dtype=gb.GF_BF16, n_sparse_heads=H0, q_stride=strides(t), k_stride=strides(t),
                          v_stride=strides(t), o_stride=strides(t))


def test_noalloc_argument_checks_on_the_host():
    # a plan whose carried states do not fit the library's array is refused before any launch
    p = gb.make_params(n_sparse_heads=0, segment_len=512)   # 16 pieces per head
    shape = (4, 32, 8192, 128, 256)
    assert gb.gformer_attn_workspace_bytes(*shape, p) > gb.GFORMER_NOALLOC_SCRATCH_BYTES
    assert gb.gformer_attn_fwd_noalloc_raw(256, 512, 768, 1024, *shape, p) == gb.GF_ERR_WORKSPACE
    # the side stream is created on first use: not in a call that must not allocate
    p1 = gb.make_params(n_sparse_heads=1, overlap=1)
    assert gb.gformer_attn_fwd_noalloc_raw(256, 512, 768, 1024, 1, 2, 128, 64, 16, p1) == gb.GF_ERR_UNSUPPORTED
    # argument errors and empty problems as in gformer_attn_fwd
    assert gb.gformer_attn_fwd_noalloc_raw(0, 0, 0, 0, 1, 2, 128, 64, 16, gb.make_params()) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_attn_fwd_noalloc_raw(0, 0, 0, 0, 0, 2, 128, 64, 16, gb.make_params()) == gb.GF_OK
    assert gb.gformer_attn_fwd_noalloc_raw(256, 512, 768, 1024, 1, 2, 128, 96, 16, gb.make_params()) == gb.GF_ERR_UNSUPPORTED


@pytest.mark.gpu
def test_noalloc_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    # (B, H, N, d, window, H0): both need carried states; the second is smaller in every respect
    for case, seed in (((2, 5, 4096, 128, 200, 1), 31), ((1, 3, 1000, 64, 64, 1), 32)):
        B, H, N, d, w, H0 = case
        wl = gi.Workload("noalloc", B, H, N, d, w, "bf16", seed)
        q, k, v = gi.make_qkv(wl)
        tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
        p = _params(B, H, N, d, H0, tq)
        need = gb.gformer_attn_workspace_bytes(B, H, N, d, w, p)
        assert 0 < need <= gb.GFORMER_NOALLOC_SCRATCH_BYTES, "the case must use the scratch array"
        want = torch.full_like(tq, float("nan"))
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        st = gb.gformer_attn_fwd_raw(tq.data_ptr(), tk.data_ptr(), tv.data_ptr(), want.data_ptr(),
                                     B, H, N, d, w, p, ws.data_ptr(), need, stream)
        assert st == gb.GF_OK
        got = torch.full_like(tq, float("nan"))
        st = gb.gformer_attn_fwd_noalloc_raw(tq.data_ptr(), tk.data_ptr(), tv.data_ptr(), got.data_ptr(),
                                             B, H, N, d, w, p, stream)
        assert st == gb.GF_OK, gb.gformer_status_string(st)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), f"{case}: bits differ"
        # and both are the layer: per-row relative L2 against the fp64 oracle
        ref = co.attn_fwd(q, k, v, w, H0, linear_form=co.LINEAR_RECURRENT)
        assert float(row_rel_l2(to_host(got), ref).max()) <= BF16_ROW_REL_L2
