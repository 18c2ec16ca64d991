"""Head partition model (Section III-D, Algorithm 2): the library's host functions against the
oracle.  Host arithmetic only, so these run without a GPU."""
from __future__ import annotations

import ctypes
import random

import pytest

from oracle import cpu_oracle as co
from paper_2412_19829_amd import binding as gb


@pytest.mark.parametrize("seed", range(20))
def test_balance_matches_oracle(seed):
    rng = random.Random(seed)
    p = rng.random()
    size = 10.0 ** rng.uniform(0, 9)
    f0, f1 = 10.0 ** rng.uniform(-2, 6), 10.0 ** rng.uniform(-2, 6)
    g0, g1 = 10.0 ** rng.uniform(9, 15), 10.0 ** rng.uniform(9, 15)
    pp, lat = gb.gformer_partition_balance(p, size, f0, f1, g0, g1)
    want = co.partition_balance(p, size, f0, f1, g0, g1)
    assert abs(pp - want) <= 1e-13
    l0, l1 = co.partition_latencies(p, size, f0, f1, g0, g1)
    assert abs(lat[0] - l0) <= 1e-12 * max(l0, 1e-300) and abs(lat[1] - l1) <= 1e-12 * max(l1, 1e-300)
    b0, b1 = co.partition_latencies(want, size, f0, f1, g0, g1)
    full = size * max(f0 / g0, f1 / g1)        # the latency of giving everything to the slower side
    assert abs(lat[2] - b0) <= 1e-12 * full and abs(lat[3] - b1) <= 1e-12 * full
    assert abs(lat[2] - lat[3]) <= 1e-12 * full


def test_balance_edge_shares():
    # one side free of cost: everything goes to it
    assert gb.gformer_partition_balance(0.5, 4.0, 0.0, 1.0, 1.0, 1.0)[0] == 1.0
    assert gb.gformer_partition_balance(0.5, 4.0, 1.0, 0.0, 1.0, 1.0)[0] == 0.0
    assert co.partition_balance(0.5, 4.0, 0.0, 1.0, 1.0, 1.0) == pytest.approx(1.0, abs=1e-15)
    assert co.partition_balance(0.5, 4.0, 1.0, 0.0, 1.0, 1.0) == pytest.approx(0.0, abs=1e-15)


@pytest.mark.parametrize("seed", range(20))
@pytest.mark.parametrize("model", [gb.GF_FLOPS_PAPER, gb.GF_FLOPS_PER_HEAD])
def test_heads_match_oracle(seed, model):
    rng = random.Random(1000 + seed)
    B, H, N = rng.randint(1, 8), rng.randint(1, 96), rng.randint(1, 65536)
    E, W = rng.choice([32, 64, 128, 256]), rng.randint(1, 2048)
    ps, pl = 10.0 ** rng.uniform(11, 15), 10.0 ** rng.uniform(11, 15)
    h0, lat = gb.gformer_partition_heads(B, H, N, E, W, ps, pl, model)
    want, ls, ll = co.partition_heads(B, H, N, E, W, ps, pl, model)
    assert h0 == want                                  # an integer decision: exact
    assert abs(lat[0] - ls) <= 1e-12 * max(ls, 1e-300) and abs(lat[1] - ll) <= 1e-12 * max(ll, 1e-300)


def test_heads_headline_shape_and_extremes():
    B, H, N, E, W = 4, 32, 8192, 128, 256
    for model in (gb.GF_FLOPS_PAPER, gb.GF_FLOPS_PER_HEAD):
        assert gb.gformer_partition_heads(B, H, N, E, W, 1e14, 1e14, model)[0] == \
            co.partition_heads(B, H, N, E, W, 1e14, 1e14, model)[0]
    # a windowed side that is far faster takes (nearly) every head, and the other way round
    assert gb.gformer_partition_heads(B, H, N, E, W, 1e20, 1e12, gb.GF_FLOPS_PER_HEAD)[0] == H
    assert gb.gformer_partition_heads(B, H, N, E, W, 1e8, 1e16, gb.GF_FLOPS_PER_HEAD)[0] == 0


def test_argument_errors():
    L = gb.lib()
    pp = ctypes.c_double()
    ok = gb.GformerPartitionInputs(ctypes.sizeof(gb.GformerPartitionInputs), 0, 0.5, 1.0, 1.0, 1.0, 1.0, 1.0)
    assert L.gformer_partition_balance(ctypes.byref(ok), ctypes.byref(pp), None) == gb.GF_OK
    assert L.gformer_partition_balance(None, ctypes.byref(pp), None) == gb.GF_ERR_INVALID_ARG
    assert L.gformer_partition_balance(ctypes.byref(ok), None, None) == gb.GF_ERR_INVALID_ARG
    for field, bad in (("struct_size", 8), ("reserved0", 1), ("p", -0.1), ("p", 1.5), ("p", float("nan")),
                       ("size", 0.0), ("perf0", 0.0), ("perf1", -1.0), ("flops_per0", -1.0),
                       ("flops_per1", float("inf"))):
        inp = gb.GformerPartitionInputs(ctypes.sizeof(gb.GformerPartitionInputs), 0, 0.5, 1.0, 1.0, 1.0, 1.0, 1.0)
        setattr(inp, field, bad)
        assert L.gformer_partition_balance(ctypes.byref(inp), ctypes.byref(pp), None) == gb.GF_ERR_INVALID_ARG, field
    both_free = gb.GformerPartitionInputs(ctypes.sizeof(gb.GformerPartitionInputs), 0, 0.5, 1.0, 0.0, 0.0, 1.0, 1.0)
    assert L.gformer_partition_balance(ctypes.byref(both_free), ctypes.byref(pp), None) == gb.GF_ERR_INVALID_ARG
    h0 = ctypes.c_int()
    assert L.gformer_partition_heads(1, 4, 8, 64, 8, 1.0, 1.0, 0, None, None) == gb.GF_ERR_INVALID_ARG
    for args in ((0, 4, 8, 64, 8, 1.0, 1.0, 0), (1, 0, 8, 64, 8, 1.0, 1.0, 0), (1, 4, 8, 64, 0, 1.0, 1.0, 0),
                 (1, 4, 8, 64, 8, 0.0, 1.0, 0), (1, 4, 8, 64, 8, 1.0, float("nan"), 0), (1, 4, 8, 64, 8, 1.0, 1.0, 2)):
        assert L.gformer_partition_heads(*args, ctypes.byref(h0), None) == gb.GF_ERR_INVALID_ARG, args
    with pytest.raises(gb.GformerError):
        gb.gformer_partition_heads(1, 4, 8, 64, 8, -1.0, 1.0)
