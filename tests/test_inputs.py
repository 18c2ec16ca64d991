"""Seeded input generators: determinism, per-head streams, bf16 rounding (CPU only)."""
import numpy as np
import torch

from paper_2412_19829_amd import inputs as gi


def test_bf16_rounding_matches_library_conversion():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65504.0, 1e-30, -1e30,
                                  np.float32(1 + 2 ** -8), np.float32(1 + 3 * 2 ** -8)], np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16)
    bits = gi.f32_to_bf16_bits(x)
    assert np.array_equal(bits, want.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(gi.bf16_bits_to_f32(bits), want.float().numpy())
    assert np.array_equal(gi.round_to_bf16(gi.round_to_bf16(x)), gi.round_to_bf16(x))


def test_heads_are_independent_streams_and_deterministic():
    wl = gi.WORKLOADS["gpt2_small"].with_(N=64)
    q, k, v = gi.make_qkv(wl)
    assert q.shape == (1, 12, 64, 64) and q.dtype == np.float32
    q5, k5, v5 = gi.make_head(wl, 0, 5)
    assert np.array_equal(q[0, 5], q5) and np.array_equal(k[0, 5], k5) and np.array_equal(v[0, 5], v5)
    qs, ks, vs = gi.make_qkv(wl, heads=[(0, 5), (0, 0)])
    assert np.array_equal(qs[0], q5) and np.array_equal(vs[1], v[0, 0])
    assert not np.array_equal(q[0, 0], q[0, 1])
    assert np.array_equal(gi.round_to_bf16(q), q)          # already bf16-representable
    assert abs(float(q.std()) - 1 / 8) < 0.01 and abs(float(k.std()) - 1.0) < 0.03


def test_outlier_recipe_and_unscaled_queries():
    wl = gi.WORKLOADS["long32k"].with_(N=256)
    q, k, v = gi.make_head(wl, 0, 3)
    assert abs(float(q.std()) - 0.5) < 0.02                  # Q not pre-scaled in this workload
    ratio = np.abs(k[::64]).mean() / np.abs(np.delete(k, np.s_[::64], axis=0)).mean()
    assert 6.0 < ratio < 10.0


def test_f32_workload_is_not_rounded():
    wl = gi.WORKLOADS["tiny_f32"]
    q, k, v = gi.make_head(wl, 0, 0)
    assert q.shape == (256, 64)
    assert not np.array_equal(gi.round_to_bf16(k), k)


def test_sample_heads_covers_both_groups():
    wl = gi.WORKLOADS["llm7b"]
    s = gi.sample_heads(wl, 6)
    assert (0, 0) in s and (wl.B - 1, 5) in s and (0, 6) in s and (wl.B - 1, 31) in s
    assert all(0 <= b < wl.B and 0 <= h < wl.H for b, h in s)
    assert gi.sample_heads(wl, 0)[0] == (0, 0) and all(h >= 0 for _, h in gi.sample_heads(wl, 0))
