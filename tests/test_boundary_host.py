"""Host-side behaviour of the C ABI (no GPU needed): the library loads, exports every symbol
the header declares, validates arguments before any launch, and plans launches sensibly."""
from __future__ import annotations

import ctypes
import os
import re

import numpy as np
import pytest

from paper_2412_19829_amd import binding as gb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_functions():
    text = open(os.path.join(ROOT, "include", "gformer.h"), encoding="utf-8").read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gformer_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = gb.lib()
    names = _header_functions()
    assert set(names) == set(gb.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_status_strings():
    assert gb.gformer_version() >= 100
    seen = {gb.gformer_status_string(s) for s in range(5)}
    assert len(seen) == 5 and "ok" in seen
    assert "unknown" in gb.gformer_status_string(99)


def test_params_init_defaults_and_struct_size():
    p = gb.gformer_params_init()
    assert p.struct_size == ctypes.sizeof(gb.GformerParams)
    assert p.dtype == gb.GF_BF16 and p.phi == gb.GF_PHI_ELU1 and p.n_sparse_heads == 0
    assert p.softmax_scale == 1.0 and p.eps == 0.0 and p.launch_mask == 0
    assert list(p.q_stride) == [0, 0, 0] and list(p.o_stride) == [0, 0, 0]


def _plan(B, H, N, d, w, **kw):
    st, plan = gb.gformer_attn_plan(B, H, N, d, w, gb.make_params(**kw))
    return st, plan.as_dict()


def test_plan_headline_config():
    st, pl = _plan(4, 32, 8192, 128, 256, n_sparse_heads=6)
    assert st == gb.GF_OK and pl["impl"] == gb.GF_IMPL_MFMA
    # 104 linear heads x 128 chunks: two pieces per head (208 of 256 compute units busy, no piece
    # straddles a head)
    assert pl["chunk"] == 64 and pl["segment_len"] == 64 * 64
    assert pl["n_segments"] == 208 and pl["linear_blocks"] == 208
    # window 256 spans five key tiles: the streaming kernel, 24 (batch, head) pairs cut into
    # 256 // 24 = 10 pieces of ceil(128 / 10) = 13 pairs of 32-query groups each
    assert pl["windowed_blocks"] == 24 * 10 and pl["windowed_threads"] == 768
    st, blocked = _plan(4, 32, 8192, 128, 256, n_sparse_heads=6, impl=gb.GF_IMPL_MFMA_BLOCKED)
    assert st == gb.GF_OK and blocked["impl"] == gb.GF_IMPL_MFMA
    assert blocked["windowed_blocks"] == 4 * 6 * (8192 // 128) and blocked["windowed_threads"] == 256
    st, wide = _plan(4, 32, 8192, 128, 258, n_sparse_heads=6)     # six tiles: query blocks
    assert st == gb.GF_OK and wide["windowed_blocks"] == 4 * 6 * (8192 // 128)
    st, centred = _plan(4, 32, 8192, 128, 257, n_sparse_heads=6, bidirectional=1)
    assert st == gb.GF_OK and centred["windowed_threads"] == 768
    # a small call (192 blocks of 128 queries) goes query block by query block unless told otherwise
    st, small = _plan(1, 12, 2048, 64, 128, n_sparse_heads=12)
    assert st == gb.GF_OK and small["windowed_threads"] == 256 and small["windowed_blocks"] == 12 * 16
    st, forced = _plan(1, 12, 2048, 64, 128, n_sparse_heads=12, impl=gb.GF_IMPL_MFMA_STREAM)
    assert st == gb.GF_OK and forced["windowed_threads"] == 768 and forced["impl"] == gb.GF_IMPL_MFMA
    # with no windowed head the forced streaming choice has nothing to refuse
    st, _none = _plan(1, 2, 600, 64, 300, n_sparse_heads=0, impl=gb.GF_IMPL_MFMA_STREAM)
    assert st == gb.GF_OK
    # The state pass sums the first piece of every head, in four sub-pieces of 16 chunks.
    assert pl["state_blocks"] == 104 * 4
    want_ws = 208 * 4 * (128 * 128 + 128) * 4
    assert pl["workspace_bytes"] == want_ws
    assert gb.gformer_attn_workspace_bytes(4, 32, 8192, 128, 256, gb.make_params(n_sparse_heads=6)) == want_ws
    # 7 heads x 128 chunks: no whole number of pieces per head fills the chip (16 per head would be
    # the limit of 8 chunks a piece: 112 pieces), so the chunk list is cut into 256 equal pieces of
    # ceil(896 / 256) = 4 -> 8 chunks (the minimum), half pieces of 4 in the state pass
    st, eq = _plan(1, 7, 8192, 128, 256, n_sparse_heads=0)
    assert st == gb.GF_OK and eq["segment_len"] == 8 * 64 and eq["n_segments"] == 112


def test_plan_modes_and_overrides():
    st, pl = _plan(1, 1, 256, 64, 32, dtype=gb.GF_F32, n_sparse_heads=1)
    assert st == gb.GF_OK and pl["impl"] == gb.GF_IMPL_SCALAR and pl["workspace_bytes"] == 0
    assert pl["linear_blocks"] == 0 and pl["windowed_blocks"] == 16
    # uniform segments per head on request
    st, pl = _plan(1, 32, 32768, 128, 512, n_sparse_heads=0, chunk=64, segment_len=1024)
    assert st == gb.GF_OK and pl["chunk"] == 64 and pl["segment_len"] == 1024 and pl["n_segments"] == 32 * 32
    assert pl["state_blocks"] == 32 * 31 and pl["windowed_blocks"] == 0
    assert pl["workspace_bytes"] == 32 * 32 * (128 * 128 + 128) * 4
    st, pl = _plan(1, 2, 100, 64, 8, n_sparse_heads=0, segment_len=64)
    assert st == gb.GF_OK and pl["n_segments"] == 4 and pl["state_blocks"] == 2
    # short problems: one piece, nothing carried, no workspace
    st, pl = _plan(1, 2, 100, 64, 8, n_sparse_heads=0)
    assert st == gb.GF_OK and pl["n_segments"] == 1 and pl["segment_len"] == 4 * 64 and pl["workspace_bytes"] == 0
    st, pl = _plan(1, 2, 100, 64, 8, n_sparse_heads=2)
    assert st == gb.GF_OK and pl["linear_blocks"] == 0 and pl["workspace_bytes"] == 0
    st, pl = _plan(2, 4, 0, 64, 8)
    assert st == gb.GF_OK and pl["linear_blocks"] == 0 and pl["windowed_blocks"] == 0
    # pieces that divide the head length carry nothing across their aligned boundaries
    st, pl = _plan(1, 64, 8192, 128, 256, n_sparse_heads=0)   # 64 heads x 128 chunks / 256 = 32
    assert st == gb.GF_OK and pl["segment_len"] == 32 * 64 and pl["n_segments"] == 256
    assert pl["state_blocks"] == 64 * 6    # half pieces of 16 chunks: 6 summed boundaries per head


@pytest.mark.parametrize("args,kw,want", [
    ((1, 1, 16, 64, 0), {}, gb.GF_ERR_INVALID_ARG),               # window < 1
    ((-1, 1, 16, 64, 4), {}, gb.GF_ERR_INVALID_ARG),
    ((1, 1, -5, 64, 4), {}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"n_sparse_heads": 3}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"n_sparse_heads": -1}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"dtype": 7}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"phi": 2}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"impl": 9}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"eps": -1.0}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"eps": float("nan")}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"launch_mask": 8}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"overlap": 2}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"bidirectional": 2}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"q_stride": (1024, 512, 60)}, gb.GF_ERR_INVALID_ARG),   # not 16-byte rows
    ((1, 2, 16, 64, 4), {"o_stride": (2048, 1024, 32)}, gb.GF_ERR_INVALID_ARG),  # rows overlap
    ((1, 2, 16, 64, 4), {"k_stride": (1 << 26, 1 << 25, (1 << 20) + 8)}, gb.GF_ERR_UNSUPPORTED),  # row stride limit
    ((1, 2, 256, 64, 4), {"chunk": 64, "segment_len": 96}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 96, 4), {}, gb.GF_ERR_UNSUPPORTED),               # head size
    ((1, 2, 16, 64, 4), {"chunk": 48}, gb.GF_ERR_UNSUPPORTED),
    ((1, 2, 16, 64, 4), {"chunk": 512}, gb.GF_ERR_UNSUPPORTED),
    ((1, 2, 16, 128, 4), {"chunk": 256}, gb.GF_ERR_UNSUPPORTED),   # its tiles do not fit the LDS
    ((1, 2, 256, 64, 4), {"chunk": 128, "segment_len": 192}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"dtype": gb.GF_F32, "impl": gb.GF_IMPL_MFMA}, gb.GF_ERR_UNSUPPORTED),
    ((1, 2, 16, 64, 4), {"dtype": gb.GF_F32, "impl": gb.GF_IMPL_MFMA_BLOCKED}, gb.GF_ERR_UNSUPPORTED),
    ((1, 2, 16, 64, 4), {"impl": 6}, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 16, 64, 4), {"dtype": gb.GF_F32, "impl": gb.GF_IMPL_MFMA_CHUNK}, gb.GF_ERR_UNSUPPORTED),
    ((1, 2, 600, 64, 258), {"impl": gb.GF_IMPL_MFMA_STREAM, "n_sparse_heads": 1}, gb.GF_ERR_UNSUPPORTED),
    ((1, 2, 256, 64, 4), {"dtype": gb.GF_F32, "segment_len": 64}, gb.GF_ERR_UNSUPPORTED),
    ((70000, 2, 16, 64, 4), {}, gb.GF_ERR_UNSUPPORTED),
])
def test_argument_errors_are_reported_by_plan_and_fwd(args, kw, want):
    p = gb.make_params(**kw)
    st, _ = gb.gformer_attn_plan(*args, p)
    assert st == want
    assert gb.gformer_attn_workspace_bytes(*args, p) == 0
    # the forward call rejects the same arguments on the host, before touching any device
    assert gb.gformer_attn_fwd_raw(0x1000, 0x2000, 0x3000, 0x4000, *args, p) == want


def test_fwd_pointer_checks_happen_on_the_host():
    p = gb.make_params(dtype=gb.GF_F32, n_sparse_heads=1)
    a = (1, 1, 16, 64, 4)
    assert gb.gformer_attn_fwd_raw(0, 0x2000, 0x3000, 0x4000, *a, p) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_attn_fwd_raw(0x1000, 0x2000, 0x3000, 0, *a, p) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_attn_fwd_raw(0x1008, 0x2000, 0x3000, 0x4000, *a, p) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_attn_fwd_raw(0x1000, 0x2000, 0x3000, 0x2000, *a, p) == gb.GF_ERR_INVALID_ARG  # alias
    # empty problems are a no-op even with null pointers
    assert gb.gformer_attn_fwd_raw(0, 0, 0, 0, 1, 1, 0, 64, 4, p) == gb.GF_OK
    assert gb.gformer_attn_fwd_raw(0, 0, 0, 0, 0, 1, 16, 64, 4, p) == gb.GF_OK
    bad = gb.make_params()
    bad.struct_size = 12
    assert gb.gformer_attn_fwd_raw(0x1000, 0x2000, 0x3000, 0x4000, *a, bad) == gb.GF_ERR_INVALID_ARG
    assert gb.lib().gformer_attn_plan(1, 1, 16, 64, 4, None, ctypes.byref(gb.GformerPlan())) == gb.GF_ERR_INVALID_ARG


def test_workspace_is_required_when_segments_are_used():
    p = gb.make_params(n_sparse_heads=0, chunk=64, segment_len=64)
    a = (1, 2, 256, 64, 8)
    need = gb.gformer_attn_workspace_bytes(*a, p)
    assert need == 1 * 2 * 4 * (64 * 64 + 64) * 4   # one slot per piece
    assert gb.gformer_attn_fwd_raw(0x1000, 0x2000, 0x3000, 0x4000, *a, p, 0, 0) == gb.GF_ERR_WORKSPACE
    assert gb.gformer_attn_fwd_raw(0x1000, 0x2000, 0x3000, 0x4000, *a, p, 0x10000, need - 1) == gb.GF_ERR_WORKSPACE
    assert gb.gformer_attn_fwd_raw(0x1000, 0x2000, 0x3000, 0x4000, *a, p, 0x10010, need) == gb.GF_ERR_INVALID_ARG


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 1, 8, 64)
    with pytest.raises(ValueError):
        gb.gformer_attn_fwd(x, x, x, torch.empty_like(x), 4, 1)


# ---------------------------------------------------------------------------------------
# gformer_random_features: host-side checks
# ---------------------------------------------------------------------------------------

def test_feature_params_defaults():
    p = gb.gformer_feature_params_init()
    assert p.struct_size == ctypes.sizeof(gb.GformerFeatureParams)
    assert p.dtype == gb.GF_BF16 and p.head_begin == 0 and p.head_end == 0 and p.impl == gb.GF_IMPL_AUTO
    assert list(p.x_stride) == [0, 0, 0] and list(p.o_stride) == [0, 0, 0]


@pytest.mark.parametrize("args,kw,want", [
    ((1, 4, 16, 64, 64), {"head_begin": 1, "head_end": 5}, gb.GF_ERR_INVALID_ARG),
    ((1, 4, 16, 64, 64), {"head_begin": 3, "head_end": 2}, gb.GF_ERR_INVALID_ARG),
    ((1, 4, 16, 64, 64), {"head_begin": -1, "head_end": 2}, gb.GF_ERR_INVALID_ARG),
    ((1, 4, 16, 64, 64), {"head_end": 4, "dtype": 5}, gb.GF_ERR_INVALID_ARG),
    ((1, 4, 16, 64, 64), {"head_end": 4, "impl": 7}, gb.GF_ERR_INVALID_ARG),
    ((1, 4, -1, 64, 64), {"head_end": 4}, gb.GF_ERR_INVALID_ARG),
    ((1, 4, 16, 64, 64), {"head_end": 4, "x_stride": (4096, 1024, 60)}, gb.GF_ERR_INVALID_ARG),
    ((1, 4, 16, 64, 128), {"head_end": 4}, gb.GF_ERR_UNSUPPORTED),    # m != d
    ((1, 4, 16, 96, 96), {"head_end": 4}, gb.GF_ERR_UNSUPPORTED),     # head size
    ((1, 4, 16, 64, 64), {"head_end": 4, "dtype": gb.GF_F32, "impl": gb.GF_IMPL_MFMA}, gb.GF_ERR_UNSUPPORTED),
])
def test_feature_argument_errors_are_reported_on_the_host(args, kw, want):
    p = gb.make_feature_params(**kw)
    assert gb.gformer_random_features_raw(0x1000, 0x2000, 0x3000, *args, p) == want


def test_feature_pointer_checks_and_empty_problems():
    p = gb.make_feature_params(dtype=gb.GF_F32, head_end=2)
    a = (1, 2, 16, 64, 64)
    assert gb.gformer_random_features_raw(0, 0x2000, 0x3000, *a, p) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_random_features_raw(0x1000, 0x2008, 0x3000, *a, p) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_random_features_raw(0x1000, 0x2000, 0x2000, *a, p) == gb.GF_ERR_INVALID_ARG  # out is w
    # in place needs identical strides
    q = gb.make_feature_params(dtype=gb.GF_F32, head_end=2, x_stride=(4096, 1024, 64), o_stride=(8192, 2048, 128))
    assert gb.gformer_random_features_raw(0x1000, 0x2000, 0x1000, *a, q) == gb.GF_ERR_INVALID_ARG
    # nothing to do: fine even with null pointers
    assert gb.gformer_random_features_raw(0, 0, 0, 0, 2, 16, 64, 64, p) == gb.GF_OK
    assert gb.gformer_random_features_raw(0, 0, 0, 1, 2, 0, 64, 64, p) == gb.GF_OK
    e = gb.make_feature_params(dtype=gb.GF_F32, head_begin=1, head_end=1)
    assert gb.gformer_random_features_raw(0, 0, 0, *a, e) == gb.GF_OK
    with pytest.raises(ValueError):
        import torch
        t = torch.zeros(1, 2, 16, 64)
        gb.gformer_random_features(t, torch.zeros(64, 64), t, 0, 2)   # host tensors: no CPU path


def test_plan_bidirectional_pieces_never_straddle_heads():
    """Every piece needs the state of its whole head: uniform segments per head, every piece
    summed by the state pass, one piece per compute unit at most."""
    st, pl = _plan(4, 32, 8192, 128, 256, n_sparse_heads=6, bidirectional=1)
    assert st == gb.GF_OK
    # 104 linear heads, 128 chunks each: two pieces of 64 chunks per head
    assert pl["segment_len"] == 64 * 64 and pl["n_segments"] == 208 and pl["state_blocks"] == 208
    assert pl["workspace_bytes"] == 208 * (128 * 128 + 128) * 4
    st, pl = _plan(1, 3, 1100, 64, 40, n_sparse_heads=1, bidirectional=1, segment_len=64)
    assert st == gb.GF_OK and pl["n_segments"] == 2 * 18 and pl["state_blocks"] == 36
    # one short head: a single piece, still summed first
    st, pl = _plan(1, 1, 100, 64, 8, n_sparse_heads=0, bidirectional=1)
    assert st == gb.GF_OK and pl["n_segments"] == 2 and pl["state_blocks"] == 2 and pl["workspace_bytes"] > 0


# ---------------------------------------------------------------------------------------
# gformer_attn_decode: host-side checks
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("shape,kw,t,want", [
    ((1, 2, 64, 4), {"n_sparse_heads": 3}, 0, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 64, 4), {"n_sparse_heads": 1, "bidirectional": 1}, 0, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 64, 4), {"n_sparse_heads": 1}, -1, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 64, 0), {"n_sparse_heads": 1}, 0, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 64, 4), {"n_sparse_heads": 1, "eps": -1.0}, 0, gb.GF_ERR_INVALID_ARG),
    ((1, 2, 96, 4), {"n_sparse_heads": 1}, 0, gb.GF_ERR_UNSUPPORTED),
    ((1, 2, 64, 1 << 20), {"n_sparse_heads": 1}, 0, gb.GF_ERR_UNSUPPORTED),   # ring scores do not fit LDS
    ((70000, 2, 64, 4), {"n_sparse_heads": 1}, 0, gb.GF_ERR_UNSUPPORTED),
])
def test_decode_argument_errors_are_reported_on_the_host(shape, kw, t, want):
    B, H, d, w = shape
    p = gb.make_params(**kw)
    got = gb.gformer_attn_decode_raw(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000, B, H, d, w, t, p)
    assert got == want


def test_decode_pointer_checks_and_empty_problems():
    p = gb.make_params(dtype=gb.GF_F32, n_sparse_heads=1)
    a = (1, 2, 64, 8, 5)
    ok = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000]
    for i in range(7):                      # every pointer is needed when both head kinds exist
        bad = list(ok); bad[i] = 0
        assert gb.gformer_attn_decode_raw(*bad, *a, p) == gb.GF_ERR_INVALID_ARG
    mis = list(ok); mis[4] = 0x5008
    assert gb.gformer_attn_decode_raw(*mis, *a, p) == gb.GF_ERR_INVALID_ARG
    alias = list(ok); alias[3] = alias[1]
    assert gb.gformer_attn_decode_raw(*alias, *a, p) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_attn_decode_raw(0, 0, 0, 0, 0, 0, 0, 0, 2, 64, 8, 5, p) == gb.GF_OK


def test_prefill_argument_checks_on_the_host():
    p = gb.make_params(dtype=gb.GF_F32, n_sparse_heads=1)
    a = (1, 2, 16, 64, 4)
    ok = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000]
    for i in (4, 5, 6):                     # rings and states are needed when both head kinds exist
        bad = list(ok); bad[i] = 0
        assert gb.gformer_attn_prefill_raw(*bad, *a, p) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_attn_prefill_raw(*ok, *a, gb.make_params(dtype=gb.GF_F32, n_sparse_heads=1, bidirectional=1)) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_attn_prefill_raw(*ok, *a, gb.make_params(dtype=gb.GF_F32, n_sparse_heads=1, launch_mask=1)) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_attn_prefill_raw(*ok, 1, 2, 16, 96, 4, p) == gb.GF_ERR_UNSUPPORTED
    assert gb.gformer_attn_prefill_raw(0, 0, 0, 0, 0, 0, 0, 1, 2, 0, 64, 4, p) == gb.GF_OK


def test_prefill_with_the_general_chunk_kernel_is_refused_on_the_host():
    """Only the kernel specialised for chunks of 64 writes the states a decode step continues
    from: a prefill call that would run the general-chunk kernel says so before any launch."""
    ptrs = (0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000)
    a = (1, 2, 256, 64, 4)
    ws = (0x10000, 1 << 24)
    for kw in (dict(chunk=128), dict(chunk=256), dict(impl=gb.GF_IMPL_MFMA_CHUNK)):
        p = gb.make_params(n_sparse_heads=1, **kw)
        assert gb.gformer_attn_prefill_raw(*ptrs, *a, p, *ws) == gb.GF_ERR_UNSUPPORTED
    # all heads windowed: no linear state to write, nothing to refuse on that account ... but the
    # call would launch, so it is only planned here
    p = gb.make_params(n_sparse_heads=2, chunk=128)
    assert gb.gformer_attn_plan(*a, p)[0] == gb.GF_OK


def test_backward_argument_checks_on_the_host():
    p = gb.make_params(dtype=gb.GF_F32, n_sparse_heads=1)
    a = (1, 2, 16, 64, 4)
    ptrs = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000]
    ws = (0x10000, 1 << 20)
    assert gb.gformer_attn_bwd_workspace_bytes(*a, p) == 1 * 2 * 16 * 2 * 4    # 8 bytes per token and head
    assert gb.gformer_attn_bwd_workspace_bytes(1, 2, 17, 64, 4, p) == 512      # ... rounded up to 256
    # the bidirectional layer also parks two (d*d + d) sums per linear head there, each in up to
    # four per-segment partials
    pb = gb.make_params(dtype=gb.GF_F32, n_sparse_heads=1, bidirectional=1)
    assert gb.gformer_attn_bwd_workspace_bytes(*a, pb) == 256 + 1 * 1 * 2 * 4 * (64 * 64 + 64) * 4
    assert gb.gformer_attn_bwd_raw(*ptrs, *a, pb, ws[0], 256) == gb.GF_ERR_WORKSPACE
    assert gb.gformer_attn_bwd_workspace_bytes(0, 2, 16, 64, 4, p) == 0
    for i in range(7):                      # any null pointer
        bad = list(ptrs)
        bad[i] = 0
        assert gb.gformer_attn_bwd_raw(*bad, *a, p, *ws) == gb.GF_ERR_INVALID_ARG
    mis = list(ptrs)
    mis[3] += 8                             # misaligned dout
    assert gb.gformer_attn_bwd_raw(*mis, *a, p, *ws) == gb.GF_ERR_INVALID_ARG
    for i, j in ((4, 0), (5, 1), (6, 3), (4, 5), (5, 6)):   # an output on an input or on another output
        al = list(ptrs)
        al[i] = al[j]
        assert gb.gformer_attn_bwd_raw(*al, *a, p, *ws) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_attn_bwd_raw(*ptrs, *a, p, 0, 0) == gb.GF_ERR_WORKSPACE
    assert gb.gformer_attn_bwd_raw(*ptrs, *a, p, ws[0], 255) == gb.GF_ERR_WORKSPACE
    assert gb.gformer_attn_bwd_raw(*ptrs, *a, p, ws[0] + 16, ws[1]) == gb.GF_ERR_INVALID_ARG
    # what the backward pass does not cover
    for impl in (gb.GF_IMPL_MFMA_BLOCKED, gb.GF_IMPL_MFMA_STREAM):     # forward-only kernel choices
        q = gb.make_params(n_sparse_heads=1, impl=impl)
        assert gb.gformer_attn_bwd_raw(*ptrs, *a, q, *ws) == gb.GF_ERR_UNSUPPORTED
    q = gb.make_params(dtype=gb.GF_F32, n_sparse_heads=1, impl=gb.GF_IMPL_MFMA)   # matrix cores: bf16 only
    assert gb.gformer_attn_bwd_raw(*ptrs, *a, q, *ws) == gb.GF_ERR_UNSUPPORTED
    assert gb.gformer_attn_bwd_raw(*ptrs, *a, gb.make_params(n_sparse_heads=1, launch_mask=1), *ws) == gb.GF_ERR_INVALID_ARG
    assert gb.gformer_attn_bwd_raw(*ptrs, 1, 2, 16, 96, 4, p, *ws) == gb.GF_ERR_UNSUPPORTED     # head size
    assert gb.gformer_attn_bwd_raw(*ptrs, 1, 2, 16, 64, 0, p, *ws) == gb.GF_ERR_INVALID_ARG     # window
    assert gb.gformer_attn_bwd_raw(*ptrs, 1, 2, 16, 64, 4, gb.make_params(n_sparse_heads=3), *ws) == gb.GF_ERR_INVALID_ARG
    # empty problems are a no-op even with null pointers
    assert gb.gformer_attn_bwd_raw(0, 0, 0, 0, 0, 0, 0, 1, 2, 0, 64, 4, p) == gb.GF_OK


def test_plan_invariants_over_random_shapes():
    """Whatever way the planner cuts the linear heads, the pieces must cover every chunk of every
    head, the workspace must hold one (A, Z) per state-pass slot, and the launch must stay at one
    workgroup per compute unit unless the pieces are already at their minimum length."""
    rng = np.random.default_rng(77)
    for _ in range(400):
        d = int(rng.choice([64, 128]))
        B = int(rng.integers(1, 9))
        H = int(rng.integers(1, 65))
        H0 = int(rng.integers(0, H + 1))
        N = int(rng.choice([int(rng.integers(1, 300)), int(rng.integers(300, 5000)), int(rng.integers(5000, 40000))]))
        bidir = int(rng.integers(0, 4) == 0)
        st, pl = _plan(B, H, N, d, 64, n_sparse_heads=H0, bidirectional=bidir)
        assert st == gb.GF_OK, (B, H, N, d, H0, bidir)
        heads, cph = B * (H - H0), -(-N // 64)
        if heads == 0:
            assert pl["linear_blocks"] == 0 and pl["workspace_bytes"] == 0
            continue
        assert pl["chunk"] == 64 and pl["segment_len"] % 64 == 0 and pl["segment_len"] > 0
        piece = pl["segment_len"] // 64
        assert pl["linear_blocks"] == pl["n_segments"] >= 1
        assert pl["n_segments"] * piece >= heads * cph                      # every chunk is in a piece
        assert (pl["n_segments"] - 1) * piece < heads * -(-cph // piece) * piece   # and no piece is idle
        assert pl["n_segments"] <= 256 or piece <= 8 or heads > 256, (B, H, N, H0, pl)
        state = (d * d + d) * 4
        if pl["state_blocks"] == 0:
            assert pl["workspace_bytes"] == 0
        else:
            assert pl["workspace_bytes"] % (pl["n_segments"] * state) == 0
            sub = pl["workspace_bytes"] // (pl["n_segments"] * state)
            assert sub in (1, 2, 4) and piece % sub == 0
            assert pl["state_blocks"] <= pl["n_segments"] * sub
            # causal: nothing is carried into the very first piece
            assert bidir or pl["state_blocks"] <= pl["n_segments"] * sub - 1
        assert gb.gformer_attn_workspace_bytes(B, H, N, d, 64, gb.make_params(n_sparse_heads=H0, bidirectional=bidir)) \
            == pl["workspace_bytes"]


@pytest.mark.parametrize("bidirectional", [0, 1])
@pytest.mark.parametrize("shape", [(4, 32, 8192, 128, 6), (1, 12, 2048, 64, 12), (2, 3, 100, 64, 2)])
def test_plan_of_a_window_at_the_end_of_the_int_range(shape, bidirectional):
    """A window no sequence can fill (INT_MAX is the natural way to ask for full attention) is
    planned exactly like a window of the whole sequence: the reach is cut at N - 1 on the host,
    before any tile arithmetic could leave the int range."""
    B, H, N, d, H0 = shape
    full = 2 * N if bidirectional else N
    st, want = _plan(B, H, N, d, full, n_sparse_heads=H0, bidirectional=bidirectional)
    assert st == gb.GF_OK
    for w in (2 ** 31 - 1, 2 ** 31 - 40, 2 ** 30, full + 1):
        st, got = _plan(B, H, N, d, w, n_sparse_heads=H0, bidirectional=bidirectional)
        assert st == gb.GF_OK and got == want, (w, got, want)
    # such a window never fits the streaming kernel (five key tiles) once N is larger than that
    if N > 400:
        st, _pl = _plan(B, H, N, d, 2 ** 31 - 1, n_sparse_heads=H0, bidirectional=bidirectional,
                        impl=gb.GF_IMPL_MFMA_STREAM)
        assert st == gb.GF_ERR_UNSUPPORTED


@pytest.mark.parametrize("d,chunk", [(64, 64), (64, 128), (64, 256), (128, 64), (128, 128)])
def test_plan_of_the_general_chunk_kernel(d, chunk):
    """Chunks of 128 and 256 tokens (and GF_IMPL_MFMA_CHUNK at 64) go to the general-chunk kernel,
    whose pieces are whole chunks of one head: uniform segments per head, a multiple of the chunk
    long, whatever the head count."""
    impl = gb.GF_IMPL_MFMA_CHUNK if chunk == 64 else gb.GF_IMPL_MFMA
    for (B, H, N, H0) in [(4, 32, 8192, 6), (1, 3, 5000, 0), (2, 7, 333, 2), (40, 9, 700, 1), (1, 1, 64, 0)]:
        st, pl = _plan(B, H, N, d, 256, n_sparse_heads=H0, chunk=chunk, impl=impl)
        assert st == gb.GF_OK and pl["chunk"] == chunk
        seg = pl["segment_len"]
        assert seg % chunk == 0 and seg > 0
        per_head = -(-N // seg)
        assert pl["n_segments"] == B * (H - H0) * per_head == pl["linear_blocks"]
        # asked-for segments keep their length when it is a multiple of the chunk
        st, pl2 = _plan(B, H, N, d, 256, n_sparse_heads=H0, chunk=chunk, impl=impl, segment_len=2 * chunk)
        assert st == gb.GF_OK and pl2["segment_len"] == 2 * chunk
    # the headline layer: two segments of 64 strips per head, as with the specialised kernel
    st, pl = _plan(4, 32, 8192, d, 256, n_sparse_heads=6, chunk=chunk, impl=impl)
    assert pl["segment_len"] == 4096 and pl["n_segments"] == 208
    # the bidirectional read-out has no in-chunk part: any chunk plans like 64
    st, bi = _plan(4, 32, 8192, d, 256, n_sparse_heads=6, chunk=chunk, bidirectional=1)
    st, bi64 = _plan(4, 32, 8192, d, 256, n_sparse_heads=6, chunk=64, bidirectional=1)
    assert {k: v for k, v in bi.items() if k != "chunk"} == {k: v for k, v in bi64.items() if k != "chunk"}
