"""Pins for the fp64 oracle (CPU only).

The oracle is checked against things it did not produce: hand-derived exact
examples (tests/golden), a library softmax-attention routine, exact rational
brute force, closed forms and invariants of the definitions.  A set of planted
wrong readings (written here, on the CPU) must each be rejected by the goldens.
"""
from __future__ import annotations

import json
import math
import os
import random
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import cpu_oracle as co
from oracle import numpy_twin as tw
from tests.helpers import load_golden, max_abs, parse_matrix, parse_scalar

TIGHT = 1e-12


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


# ---------------------------------------------------------------------------
# hand examples (exact rationals)
# ---------------------------------------------------------------------------

WINDOW_IMPLS = {
    "c": lambda q, k, v, w: co.windowed_head(q, k, v, w, 1.0),
    "numpy": lambda q, k, v, w: tw.windowed_head(q, k, v, w, 1.0),
}
LINEAR_IMPLS = {
    "c_quadratic": lambda q, k, v: co.linear_head(q, k, v, form=co.LINEAR_QUADRATIC),
    "c_recurrent": lambda q, k, v: co.linear_head(q, k, v, form=co.LINEAR_RECURRENT),
    "numpy_recurrent": lambda q, k, v: tw.linear_head_recurrent(q, k, v),
    "numpy_quadratic": lambda q, k, v: tw.linear_head_quadratic(q, k, v),
}


@pytest.mark.parametrize("impl", sorted(WINDOW_IMPLS))
def test_window_example_exact(impl):
    g = load_golden("window_4token.json")
    q, k, v = parse_matrix(g["q"]), parse_matrix(g["k"]), parse_matrix(g["v"])
    for w, rows in g["expected"].items():
        got = WINDOW_IMPLS[impl](q, k, v, int(w))
        assert max_abs(got, parse_matrix(rows)) < 1e-14, (impl, w)


@pytest.mark.parametrize("impl", sorted(LINEAR_IMPLS))
def test_linear_example_exact(impl):
    g = load_golden("linear_4token.json")
    q, k, v = parse_matrix(g["q"]), parse_matrix(g["k"]), parse_matrix(g["v"])
    got = LINEAR_IMPLS[impl](q, k, v)
    assert max_abs(got, parse_matrix(g["expected"])) < 1e-14
    # the order of operations printed in the paper's PyTorch listing is not Algorithm 1
    assert max_abs(got, parse_matrix(g["must_reject"])) > 0.05


def test_linear_example_intermediates():
    """The fixture's own phi, num and den columns are consistent with its inputs."""
    g = load_golden("linear_4token.json")
    q, k, v = parse_matrix(g["q"]), parse_matrix(g["k"]), parse_matrix(g["v"])
    assert max_abs(tw.phi_elu1(q), parse_matrix(g["phi_q"])) < 1e-15
    assert max_abs(tw.phi_elu1(k), parse_matrix(g["phi_k"])) < 1e-15
    fq = [[Fraction(t) for t in r] for r in g["phi_q"]]
    fk = [[Fraction(t) for t in r] for r in g["phi_k"]]
    fv = [[Fraction(t) for t in r] for r in g["v"]]
    for i in range(4):
        a = [sum(fq[i][c] * fk[j][c] for c in range(2)) for j in range(i + 1)]
        assert sum(a) == Fraction(g["den"][i])
        for e in range(2):
            assert sum(a[j] * fv[j][e] for j in range(i + 1)) == Fraction(g["num"][i][e])
            assert sum(a[j] * fv[j][e] for j in range(i + 1)) / sum(a) == Fraction(g["expected"][i][e])


@pytest.mark.parametrize("impl", sorted(LINEAR_IMPLS))
def test_linear_head_size_one(impl):
    g = load_golden("linear_d1.json")
    q, k, v = parse_matrix(g["q"]), parse_matrix(g["k"]), parse_matrix(g["v"])
    assert max_abs(LINEAR_IMPLS[impl](q, k, v), parse_matrix(g["expected"])) < 1e-14


# ---------------------------------------------------------------------------
# planted wrong readings must fail the goldens (mistakes are planted here, on the CPU)
# ---------------------------------------------------------------------------

def _wrong_window(q, k, v, w, kind):
    N, d = q.shape
    out = np.zeros((N, d))
    for i in range(N):
        if kind == "w_plus_one":
            lo, hi = max(0, i - w), i
        elif kind == "exclude_self":
            lo, hi = max(0, i - w), max(0, i - 1)
        elif kind == "not_causal":
            lo, hi = max(0, i - w + 1), min(N - 1, i + w - 1)
        else:
            lo, hi = max(0, i - w + 1), i
        s = k[lo:hi + 1] @ q[i]
        if kind == "transposed_qk":
            s = q[lo:hi + 1] @ k[i]
        if kind == "half_scale":
            s = 0.5 * s
        e = np.exp(s - s.max())
        if kind == "no_normalise":
            out[i] = e @ v[lo:hi + 1]
        else:
            out[i] = (e / e.sum()) @ v[lo:hi + 1]
    return out


@pytest.mark.parametrize("kind", ["w_plus_one", "exclude_self", "not_causal", "transposed_qk",
                                  "half_scale", "no_normalise"])
def test_window_golden_rejects_wrong_readings(kind):
    g = load_golden("window_4token.json")
    q, k, v = parse_matrix(g["q"]), parse_matrix(g["k"]), parse_matrix(g["v"])
    worst = max(max_abs(_wrong_window(q, k, v, int(w), kind), parse_matrix(rows))
                for w, rows in g["expected"].items())
    assert worst > 1e-3, kind


def _wrong_linear(q, k, v, kind):
    N, d = q.shape
    fq, fk = tw.phi_elu1(q), tw.phi_elu1(k)
    if kind == "elu_without_plus_one":
        fq, fk = fq - 1.0, fk - 1.0
    if kind == "phi_on_q_only":
        fk = k
    A = np.zeros((d, d)); Z = np.zeros(d); out = np.zeros((N, d))
    for i in range(N):
        if kind == "exclusive_prefix":
            num, den = fq[i] @ A, fq[i] @ Z
            A += np.outer(fk[i], v[i]); Z += fk[i]
            out[i] = num / den if den != 0 else 0.0
            continue
        if kind == "transposed_state":
            A += np.outer(v[i], fk[i])
        else:
            A += np.outer(fk[i], v[i])
        Z += fk[i]
        if kind == "k_reads_state":      # the garbled last line of Algorithm 1 taken literally
            out[i] = (fk[i] @ A) / (fq[i] @ Z)
        elif kind == "no_normaliser":
            out[i] = fq[i] @ A
        else:
            out[i] = (fq[i] @ A) / (fq[i] @ Z)
    return out


@pytest.mark.parametrize("kind", ["exclusive_prefix", "transposed_state", "k_reads_state",
                                  "no_normaliser", "elu_without_plus_one", "phi_on_q_only"])
def test_linear_golden_rejects_wrong_readings(kind):
    g = load_golden("linear_4token.json")
    q, k, v = parse_matrix(g["q"]), parse_matrix(g["k"]), parse_matrix(g["v"])
    with np.errstate(all="ignore"):
        got = _wrong_linear(q, k, v, kind)
    assert not np.allclose(got, parse_matrix(g["expected"]), atol=1e-3, equal_nan=False), kind


# ---------------------------------------------------------------------------
# feature map (section II-B)
# ---------------------------------------------------------------------------

def test_feature_map_values_through_the_oracle():
    """With d = 1, N = 1 .. the first output is v_0; use a 2-token probe to read phi(k) back:
    out_1 = (phi(k0) v0 + phi(k1) v1) / (phi(k0) + phi(k1)) with v = (0, 1), k0 = 0 (phi = 1)."""
    for x, want in [(0.0, 1.0), (-math.log(2.0), 0.5), (2.5, 3.5), (-30.0, math.exp(-30.0)),
                    (1e-9, 1.0 + 1e-9), (-1e-9, math.exp(-1e-9))]:
        q = np.array([[0.3], [0.7]]); k = np.array([[0.0], [x]]); v = np.array([[0.0], [1.0]])
        for form in (co.LINEAR_QUADRATIC, co.LINEAR_RECURRENT):
            got = co.linear_head(q, k, v, form=form)[1, 0]
            assert abs(got - want / (1.0 + want)) < 1e-15 * max(1.0, want), (x, form)


def test_feature_map_positive_and_continuous():
    x = np.linspace(-40, 40, 4001)
    y = tw.phi_elu1(x)
    assert (y > 0).all()
    assert np.all(np.diff(y) > 0)
    assert abs(tw.phi_elu1(np.array([0.0]))[0] - 1.0) == 0.0


# ---------------------------------------------------------------------------
# library second opinion: Eq. 1 with the causal mask == torch SDPA (fp64, CPU)
# ---------------------------------------------------------------------------

def _sdpa(q, k, v, mask=None, causal=False):
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))[None, None]
    o = torch.nn.functional.scaled_dot_product_attention(
        t(q), t(k), t(v), attn_mask=mask, is_causal=causal, scale=1.0)
    return o[0, 0].numpy()


@pytest.mark.parametrize("N,d,w", [(37, 8, 37), (64, 16, 100), (5, 3, 5)])
def test_window_covering_sequence_is_full_causal_attention(N, d, w):
    q, k, v = _rand((N, d), 1), _rand((N, d), 2), _rand((N, d), 3)
    want = _sdpa(q, k, v, causal=True)
    assert max_abs(co.windowed_head(q, k, v, w), want) < TIGHT
    assert max_abs(tw.windowed_head(q, k, v, w), want) < TIGHT


@pytest.mark.parametrize("N,d,w", [(50, 8, 1), (50, 8, 2), (67, 16, 13), (130, 4, 64), (96, 32, 33)])
def test_window_matches_library_attention_with_band_mask(N, d, w):
    q, k, v = _rand((N, d), 4), _rand((N, d), 5), _rand((N, d), 6)
    i = torch.arange(N)[:, None]; j = torch.arange(N)[None, :]
    mask = (j <= i) & (j > i - w)
    want = _sdpa(q, k, v, mask=mask)
    assert max_abs(co.windowed_head(q, k, v, w), want) < TIGHT
    assert max_abs(tw.windowed_head(q, k, v, w), want) < TIGHT


def test_softmax_scale_is_applied_to_scores():
    N, d, w = 40, 8, 9
    q, k, v = _rand((N, d), 7), _rand((N, d), 8), _rand((N, d), 9)
    s = 1.0 / math.sqrt(d)
    assert max_abs(co.windowed_head(q, k, v, w, s), co.windowed_head(q * s, k, v, w, 1.0)) < TIGHT
    i = torch.arange(N)[:, None]; j = torch.arange(N)[None, :]
    mask = (j <= i) & (j > i - w)
    assert max_abs(co.windowed_head(q, k, v, w, s), _sdpa(q * s, k, v, mask=mask)) < TIGHT


# ---------------------------------------------------------------------------
# exact rational brute force (independent arithmetic)
# ---------------------------------------------------------------------------

def _frac_matrix(rng, n, d, lo=1, hi=9, signed=False):
    m = [[Fraction(int(rng.integers(lo, hi)), int(rng.integers(1, 7))) for _ in range(d)]
         for _ in range(n)]
    if signed:
        m = [[x * (1 if rng.integers(0, 2) else -1) for x in r] for r in m]
    return m


def _to_np(m):
    return np.array([[float(x) for x in r] for r in m])


@pytest.mark.parametrize("seed", range(4))
def test_linear_identity_phi_against_exact_rationals(seed):
    rng = np.random.default_rng(100 + seed)
    N, d = 8, 2 + seed % 2
    fq, fk = _frac_matrix(rng, N, d), _frac_matrix(rng, N, d)   # positive features
    fv = _frac_matrix(rng, N, d, signed=True)
    want = []
    for i in range(N):
        a = [sum(fq[i][c] * fk[j][c] for c in range(d)) for j in range(i + 1)]
        want.append([sum(a[j] * fv[j][e] for j in range(i + 1)) / sum(a) for e in range(d)])
    want = _to_np(want)
    for form in (co.LINEAR_QUADRATIC, co.LINEAR_RECURRENT):
        got = co.linear_head(_to_np(fq), _to_np(fk), _to_np(fv), phi=co.PHI_IDENTITY, form=form)
        assert max_abs(got, want) < 1e-13
    got = tw.linear_head_recurrent(_to_np(fq), _to_np(fk), _to_np(fv), phi=lambda x: x)
    assert max_abs(got, want) < 1e-13


@pytest.mark.parametrize("seed,w", [(0, 1), (1, 3), (2, 5), (3, 8)])
def test_window_against_exact_rationals(seed, w):
    """Keys are logs of rationals along q's only non-zero axis, so softmax weights are rational."""
    rng = np.random.default_rng(200 + seed)
    N, d = 8, 2
    r = [Fraction(int(rng.integers(1, 12)), int(rng.integers(1, 5))) for _ in range(N)]
    fv = _frac_matrix(rng, N, d, signed=True)
    q = np.tile(np.array([[0.0, 1.0]]), (N, 1))
    k = np.array([[float(rng.standard_normal()), math.log(float(x))] for x in r])
    want = []
    for i in range(N):
        lo = max(0, i - w + 1)
        tot = sum(r[lo:i + 1])
        want.append([sum(r[j] * fv[j][e] for j in range(lo, i + 1)) / tot for e in range(d)])
    assert max_abs(co.windowed_head(q, k, _to_np(fv), w), _to_np(want)) < 1e-13
    assert max_abs(tw.windowed_head(q, k, _to_np(fv), w), _to_np(want)) < 1e-13


# ---------------------------------------------------------------------------
# equivalence of forms and of the two implementations
# ---------------------------------------------------------------------------

def chunked_linear(q, k, v, C, phi=tw.phi_elu1, eps=0.0):
    """Chunk-parallel rearrangement of Algorithm 1 (host-side statement of what the GPU kernel
    does): inside a chunk the masked quadratic form, across chunks the carried state."""
    N, d = q.shape
    S = np.zeros((d, d)); z = np.zeros(d); out = np.zeros((N, d))
    for s0 in range(0, N, C):
        fq, fk, vc = phi(q[s0:s0 + C]), phi(k[s0:s0 + C]), v[s0:s0 + C]
        a = np.tril(fq @ fk.T)
        num = a @ vc + fq @ S
        den = a.sum(1) + fq @ z + eps
        out[s0:s0 + C] = num / den[:, None]
        S += fk.T @ vc
        z += fk.sum(0)
    return out


@pytest.mark.parametrize("N,d", [(1, 4), (2, 1), (33, 8), (100, 16), (257, 64)])
def test_linear_forms_agree(N, d):
    q, k, v = _rand((N, d), 11), _rand((N, d), 12), _rand((N, d), 13)
    a = co.linear_head(q, k, v, form=co.LINEAR_QUADRATIC)
    b = co.linear_head(q, k, v, form=co.LINEAR_RECURRENT)
    c = tw.linear_head_recurrent(q, k, v)
    e = tw.linear_head_quadratic(q, k, v)
    assert max_abs(a, b) < 1e-11 and max_abs(a, c) < 1e-11 and max_abs(a, e) < 1e-11
    for C in (1, 3, 7, 64, N, N + 5):
        assert max_abs(a, chunked_linear(q, k, v, C)) < 1e-11, C


def test_c_oracle_matches_numpy_twin_on_a_layer():
    B, H, N, d, w, H0 = 2, 5, 70, 8, 17, 2
    q, k, v = _rand((B, H, N, d), 21, 0.7), _rand((B, H, N, d), 22), _rand((B, H, N, d), 23)
    a = co.attn_fwd(q, k, v, w, H0, softmax_scale=0.8, eps=0.0)
    b = tw.attn_fwd(q, k, v, w, H0, softmax_scale=0.8)
    assert max_abs(a, b) < 1e-11
    r = co.attn_fwd(q, k, v, w, H0, softmax_scale=0.8, linear_form=co.LINEAR_RECURRENT, threads=3)
    assert max_abs(a, r) < 1e-11
    # head split (section III-A): slot h holds head h; the scale touches windowed heads only
    for b_ in range(B):
        for h in range(H):
            if h < H0:
                one = co.windowed_head(q[b_, h], k[b_, h], v[b_, h], w, 0.8)
            else:
                one = co.linear_head(q[b_, h], k[b_, h], v[b_, h])
            assert max_abs(a[b_, h], one) == 0.0


def test_head_result_depends_only_on_its_side_of_the_split():
    B, H, N, d, w = 1, 4, 40, 8, 6
    q, k, v = _rand((B, H, N, d), 31), _rand((B, H, N, d), 32), _rand((B, H, N, d), 33)
    o1, o2, o3 = (co.attn_fwd(q, k, v, w, h0) for h0 in (1, 2, 3))
    assert max_abs(o1[:, 0], o2[:, 0]) == 0.0 and max_abs(o2[:, 0], o3[:, 0]) == 0.0  # windowed
    assert max_abs(o1[:, 3], o2[:, 3]) == 0.0 and max_abs(o2[:, 3], o3[:, 3]) == 0.0  # linear
    assert max_abs(o2[:, 1], o3[:, 1]) == 0.0 and max_abs(o1[:, 1], o2[:, 1]) > 1e-3
    perm = [2, 3, 0, 1]   # permuting heads inside one mode group permutes outputs
    op = co.attn_fwd(q[:, perm], k[:, perm], v[:, perm], w, 0)
    assert max_abs(op, co.attn_fwd(q, k, v, w, 0)[:, perm]) == 0.0


# ---------------------------------------------------------------------------
# invariants and closed forms
# ---------------------------------------------------------------------------

def _both_paths(q, k, v, w):
    return [("window", co.windowed_head(q, k, v, w)),
            ("linear_q", co.linear_head(q, k, v, form=co.LINEAR_QUADRATIC)),
            ("linear_r", co.linear_head(q, k, v, form=co.LINEAR_RECURRENT))]


def test_weights_sum_to_one():
    N, d, w = 60, 8, 11
    q, k = _rand((N, d), 41), _rand((N, d), 42)
    for name, o in _both_paths(q, k, np.ones((N, d)), w):
        assert max_abs(o, np.ones((N, d))) < 1e-13, name
    const = np.tile(np.arange(d, dtype=np.float64)[None] - 3.0, (N, 1))
    for name, o in _both_paths(q, k, const, w):
        assert max_abs(o, const) < 1e-12, name


def test_outputs_lie_in_convex_hull_of_visible_values():
    N, d, w = 80, 6, 9
    q, k, v = _rand((N, d), 43), _rand((N, d), 44), _rand((N, d), 45)
    ow = co.windowed_head(q, k, v, w)
    ol = co.linear_head(q, k, v)
    for i in range(N):
        lo = max(0, i - w + 1)
        assert (ow[i] <= v[lo:i + 1].max(0) + 1e-12).all() and (ow[i] >= v[lo:i + 1].min(0) - 1e-12).all()
        assert (ol[i] <= v[:i + 1].max(0) + 1e-12).all() and (ol[i] >= v[:i + 1].min(0) - 1e-12).all()


def test_zero_queries_or_keys_give_plain_means():
    N, d, w = 50, 5, 7
    k, v = _rand((N, d), 46), _rand((N, d), 47)
    zero = np.zeros((N, d))
    win_mean = np.stack([v[max(0, i - w + 1):i + 1].mean(0) for i in range(N)])
    pre_mean = np.cumsum(v, 0) / np.arange(1, N + 1)[:, None]
    assert max_abs(co.windowed_head(zero, k, v, w), win_mean) < 1e-13
    assert max_abs(co.windowed_head(k, zero, v, w), win_mean) < 1e-13
    # phi(0) = 1 on every feature: all keys weigh the same whatever q is
    assert max_abs(co.linear_head(k, zero, v), pre_mean) < 1e-12
    assert max_abs(co.linear_head(k, zero, v, form=co.LINEAR_RECURRENT), pre_mean) < 1e-12


def test_first_token_returns_its_own_value():
    N, d = 9, 4
    q, k, v = _rand((N, d), 48), _rand((N, d), 49), _rand((N, d), 50)
    for name, o in _both_paths(q, k, v, 3):
        assert max_abs(o[0], v[0]) < 1e-14, name


def test_causality_and_window_locality():
    N, d, w, t = 70, 6, 8, 31
    q, k, v = _rand((N, d), 51), _rand((N, d), 52), _rand((N, d), 53)
    k2, v2 = k.copy(), v.copy()
    k2[t] += 1.0; v2[t] -= 2.0
    base, pert = _both_paths(q, k, v, w), _both_paths(q, k2, v2, w)
    for (name, a), (_, b) in zip(base, pert):
        assert max_abs(a[:t], b[:t]) == 0.0, name          # nothing before t moves
        assert max_abs(a[t], b[t]) > 1e-6, name
        if name == "window":
            assert max_abs(a[t + w:], b[t + w:]) == 0.0      # and nothing past the window
            assert max_abs(a[t + w - 1], b[t + w - 1]) > 1e-9
        else:
            assert max_abs(a[-1], b[-1]) > 1e-9              # the linear state remembers
    q2 = q.copy(); q2[t] *= -0.5
    for (name, a), (_, b) in zip(base, _both_paths(q2, k, v, w)):
        rows = np.abs(a - b).max(1)
        assert rows[t] > 1e-9 and rows[:t].max() == 0.0 and rows[t + 1:].max() == 0.0, name


def test_softmax_shift_invariance_with_large_shift():
    N, d, w = 40, 8, 10
    q, k, v = _rand((N, d), 54), _rand((N, d), 55), _rand((N, d), 56)
    shift = 300.0 * _rand((1, d), 57)     # adds q_i.shift (hundreds) to every score of row i
    assert max_abs(co.windowed_head(q, k, v, w), co.windowed_head(q, k + shift, v, w)) < 1e-9
    big = co.windowed_head(50.0 * q, 50.0 * k, v, w)   # scores in the thousands: no overflow
    assert np.isfinite(big).all()


def test_linearity_in_values():
    N, d, w = 45, 7, 6
    q, k = _rand((N, d), 58), _rand((N, d), 59)
    v1, v2 = _rand((N, d), 60), _rand((N, d), 61)
    for (name, a), (_, b), (_, c) in zip(_both_paths(q, k, 2.0 * v1 - 3.0 * v2, w),
                                         _both_paths(q, k, v1, w), _both_paths(q, k, v2, w)):
        assert max_abs(a, 2.0 * b - 3.0 * c) < 1e-12, name


def test_linear_scale_invariance_identity_phi():
    N, d = 30, 5
    rng = np.random.default_rng(62)
    fq, fk = rng.uniform(0.1, 2.0, (N, d)), rng.uniform(0.1, 2.0, (N, d))
    v = _rand((N, d), 63)
    base = co.linear_head(fq, fk, v, phi=co.PHI_IDENTITY)
    rowscale = rng.uniform(0.5, 4.0, (N, 1))
    assert max_abs(base, co.linear_head(fq * rowscale, fk, v, phi=co.PHI_IDENTITY)) < 1e-13
    assert max_abs(base, co.linear_head(fq, 7.5 * fk, v, phi=co.PHI_IDENTITY)) < 1e-13


def test_eps_enters_the_linear_denominator_only():
    N, d = 12, 3
    q, k, v = _rand((N, d), 64), _rand((N, d), 65), _rand((N, d), 66)
    a = tw.phi_elu1(q) @ tw.phi_elu1(k).T
    a = np.tril(a)
    want = (a @ v) / (a.sum(1, keepdims=True) + 0.25)
    for form in (co.LINEAR_QUADRATIC, co.LINEAR_RECURRENT):
        assert max_abs(co.linear_head(q, k, v, eps=0.25, form=form), want) < 1e-13


def test_degenerate_shapes_and_errors():
    z = np.zeros((0, 4))
    assert co.windowed_head(z, z, z, 3).shape == (0, 4)
    assert co.linear_head(z, z, z).shape == (0, 4)
    one = np.ones((1, 1))
    assert co.windowed_head(one, one, 2 * one, 1)[0, 0] == 2.0
    assert co.linear_head(one, one, 2 * one)[0, 0] == 2.0
    with pytest.raises(RuntimeError):
        co.windowed_head(one, one, one, 0)
    with pytest.raises(RuntimeError):
        co.attn_fwd(np.ones((1, 2, 3, 4)), np.ones((1, 2, 3, 4)), np.ones((1, 2, 3, 4)), 2, 3)


# ---------------------------------------------------------------------------------------
# positive random features (section III-A's alternative feature map)
# ---------------------------------------------------------------------------------------

def _rf_expected(g):
    const = {"sqrt_e": g["sqrt_e"], "inv_sqrt_e": g["inv_sqrt_e"], "e_m3_2": g["e_m3_2"], "one": 1.0}
    return np.array([[const[t] * g["inv_sqrt_3"] for t in row] for row in g["expected_terms"]])


def test_random_features_worked_example():
    g = load_golden("random_features_3.json")
    got = co.random_features(np.array(g["x"], float), np.array(g["w"], float))
    assert got.shape == (2, 3)
    assert max_abs(got, _rf_expected(g)) < 1e-15


@pytest.mark.parametrize("kind", ["no_norm_term", "plus_norm_term", "no_sqrt_m"])
def test_random_features_golden_rejects_wrong_readings(kind):
    """Dropping the -|x|^2/2 term, flipping its sign or forgetting 1/sqrt(m) all miss the fixture."""
    g = load_golden("random_features_3.json")
    wrong = np.array(g["must_reject"][kind]) * (1.0 if kind == "no_sqrt_m" else g["inv_sqrt_3"])
    assert max_abs(wrong, _rf_expected(g)[0]) > 0.1


def test_random_features_estimate_the_exponential_kernel():
    """E over Gaussian rows of phi(q).phi(k) is exp(q.k): the defining property of the
    construction, checked by Monte Carlo with 400k rows (standard error well below the bound)."""
    rng = np.random.default_rng(77)
    d, m = 4, 400_000
    w = rng.standard_normal((m, d))
    for _ in range(3):
        q = rng.standard_normal(d) * 0.4
        k = rng.standard_normal(d) * 0.4
        est = float(co.random_features(q[None], w)[0] @ co.random_features(k[None], w)[0])
        assert abs(est / math.exp(float(q @ k)) - 1.0) < 0.02


def test_random_features_log_is_linear_minus_half_square():
    """log phi(x+y) = log phi(x) + log phi(y) - x.y + log(m)/2 for every feature, and
    log phi(2x) = 4 log phi(x) - 2 w.x + 3 log(m)/2: both fix the -1/2 of the squared norm and
    the 1/sqrt(m) without evaluating an exponential in the test."""
    rng = np.random.default_rng(78)
    d, m = 5, 7
    w = rng.standard_normal((m, d))
    x, y = rng.standard_normal(d), rng.standard_normal(d)
    lx, ly, lxy, l2x = (np.log(co.random_features(v[None], w)[0]) for v in (x, y, x + y, 2 * x))
    assert max_abs(lxy, lx + ly - float(x @ y) + 0.5 * math.log(m)) < 1e-12
    assert max_abs(l2x, 4 * lx - 2 * (w @ x) + 1.5 * math.log(m)) < 1e-12
    # rows of W enter one feature each, in order
    w2 = w.copy(); w2[3] += 1.0
    delta = np.log(co.random_features(x[None], w2)[0]) - lx
    assert max_abs(delta, np.eye(m)[3] * float(x.sum())) < 1e-12


def test_random_features_feed_algorithm_1_as_kernel_weights():
    """Linear head with pre-mapped features and the identity map == causal kernel regression
    with weights phi(q_i).phi(k_j), written out here with a dense matrix."""
    rng = np.random.default_rng(79)
    N, d = 9, 4
    q, k, v = (rng.standard_normal((N, d)) * 0.5 for _ in range(3))
    w = rng.standard_normal((d, d))
    fq, fk = co.random_features(q, w), co.random_features(k, w)
    got = co.linear_head(fq, fk, v, phi=co.PHI_IDENTITY)
    a = np.tril(fq @ fk.T)
    assert max_abs(got, (a @ v) / a.sum(1, keepdims=True)) < 1e-12
    assert (fq > 0).all() and (fk > 0).all()


# ---------------------------------------------------------------------------------------
# bidirectional variant: window centred on the token, linear head over all keys
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("w", [1, 2, 3, 4, 5, 9])
def test_bidirectional_window_example_exact(w):
    g, b = load_golden("window_4token.json"), load_golden("bidirectional_examples.json")
    q, k, v = (parse_matrix(g[n]) for n in "qkv")
    got = co.windowed_head(q, k, v, w, bidirectional=True)
    assert max_abs(got, parse_matrix(b["window_expected"][str(w)])) < 1e-14
    if w <= 2:   # nothing to the right of the token: the causal head gives the same rows
        assert max_abs(got, co.windowed_head(q, k, v, w)) < 1e-15


def test_bidirectional_window_golden_rejects_wrong_splits():
    b = load_golden("bidirectional_examples.json")
    exp4 = parse_matrix(b["window_expected"]["4"])[0]
    exp3 = parse_matrix(b["window_expected"]["3"])[0]
    assert max_abs(parse_matrix([b["window_must_reject"]["right_heavy_w4_row0"]])[0], exp4) > 0.1
    assert max_abs(parse_matrix([b["window_must_reject"]["causal_w3_row0"]])[0], exp3) > 0.1


@pytest.mark.parametrize("form", [co.LINEAR_QUADRATIC, co.LINEAR_RECURRENT])
def test_bidirectional_linear_example_exact(form):
    b = load_golden("bidirectional_examples.json")["linear"]
    q, k, v = (parse_matrix(b[n]) for n in "qkv")
    got = co.linear_head(q, k, v, phi=co.PHI_IDENTITY, form=form, bidirectional=True)
    assert max_abs(got, parse_matrix(b["expected"])) < 1e-15
    # the causal head differs already in row 0
    assert max_abs(co.linear_head(q, k, v, phi=co.PHI_IDENTITY)[0], parse_matrix([b["causal_expected_row0"]])[0]) < 1e-15
    d1 = load_golden("linear_d1.json")
    q1, k1, v1 = (parse_matrix(d1[n]) for n in "qkv")
    want = parse_matrix(load_golden("bidirectional_examples.json")["linear_d1_expected"])
    assert max_abs(co.linear_head(q1, k1, v1, form=form, bidirectional=True), want) < 1e-14


@pytest.mark.parametrize("N,d,w", [(37, 8, 5), (50, 16, 12), (23, 4, 1), (40, 8, 200)])
def test_bidirectional_window_matches_library_attention_with_band_mask(N, d, w):
    rng = np.random.default_rng(500 + N + w)
    q, k, v = (rng.standard_normal((N, d)) for _ in range(3))
    i, j = np.arange(N)[:, None], np.arange(N)[None, :]
    left = w // 2
    band = (j >= i - left) & (j <= i + (w - 1 - left))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None],
        attn_mask=torch.from_numpy(band)[None], scale=0.7)[0].numpy()
    assert max_abs(co.windowed_head(q, k, v, w, scale=0.7, bidirectional=True), ref) < 1e-12
    if w >= 2 * N:   # the window covers everything: plain softmax attention, no mask at all
        full = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None], scale=0.7)[0].numpy()
        assert max_abs(ref, full) < 1e-12


def test_bidirectional_symmetries_and_links_to_the_causal_heads():
    rng = np.random.default_rng(601)
    N, d = 29, 6
    q, k, v = (rng.standard_normal((N, d)) for _ in range(3))
    lin = co.linear_head(q, k, v, bidirectional=True)
    # the order of the (key, value) pairs does not matter to a head that sees them all
    perm = rng.permutation(N)
    assert max_abs(co.linear_head(q, k[perm], v[perm], bidirectional=True), lin) < 1e-12
    # the last token of the causal head already sees every key
    assert max_abs(lin[-1], co.linear_head(q, k, v)[-1]) < 1e-12
    assert max_abs(co.linear_head(q, k, v, form=co.LINEAR_RECURRENT, bidirectional=True), lin) < 1e-12
    # odd window: reversing the sequence reverses the output
    for w in (1, 5, 11):
        a = co.windowed_head(q, k, v, w, bidirectional=True)
        b = co.windowed_head(q[::-1], k[::-1], v[::-1], w, bidirectional=True)[::-1]
        assert max_abs(a, b) < 1e-12
    # even window: one more key on the left than on the right
    v_ones = np.zeros((N, d)); v_ones[:, 0] = np.arange(N)
    k0 = np.zeros((N, d))       # uniform weights: output = mean index over the window
    mid = co.windowed_head(q, k0, v_ones, 4, bidirectional=True)[10, 0]
    assert abs(mid - (8 + 9 + 10 + 11) / 4) < 1e-12
    # layer driver: head split and both linear forms
    Q, K, V = (rng.standard_normal((2, 3, 17, 4)) for _ in range(3))
    out = co.attn_fwd(Q, K, V, 6, 1, bidirectional=True)
    assert max_abs(out[1, 0], co.windowed_head(Q[1, 0], K[1, 0], V[1, 0], 6, bidirectional=True)) < 1e-15
    assert max_abs(out[0, 2], co.linear_head(Q[0, 2], K[0, 2], V[0, 2], bidirectional=True)) < 1e-15
    out2 = co.attn_fwd(Q, K, V, 6, 1, bidirectional=True, linear_form=co.LINEAR_RECURRENT)
    assert max_abs(out, out2) < 1e-12


@pytest.mark.parametrize("seed", [1, 2])
def test_bidirectional_linear_against_exact_rationals(seed):
    rng = np.random.default_rng(700 + seed)
    N, d = 6, 2
    qi, ki, vi = (rng.integers(1, 6, (N, d)) for _ in range(3))
    want = []
    for i in range(N):
        a = [sum(Fraction(int(qi[i, c])) * int(ki[j, c]) for c in range(d)) for j in range(N)]
        den = sum(a)
        want.append([float(sum(a[j] * int(vi[j, e]) for j in range(N)) / den) for e in range(d)])
    got = co.linear_head(qi.astype(float), ki.astype(float), vi.astype(float), phi=co.PHI_IDENTITY,
                         bidirectional=True)
    assert max_abs(got, np.array(want)) < 1e-14


# ---------------------------------------------------------------------------------------
# decode step: one token at a time reproduces the full causal forward
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("N,d,w", [(40, 6, 7), (25, 4, 1), (30, 8, 64), (33, 5, 32)])
def test_decode_steps_reproduce_the_full_forward(N, d, w):
    rng = np.random.default_rng(800 + N + w)
    q, k, v = (rng.standard_normal((N, d)) for _ in range(3))
    full_w = co.windowed_head(q, k, v, w, scale=0.6)
    full_l = co.linear_head(q, k, v, eps=0.125)
    kring, vring = np.full((w, d), np.nan), np.full((w, d), np.nan)   # unused slots are never read
    A, Z = np.zeros((d, d)), np.zeros(d)
    for t in range(N):
        ow = co.decode_windowed(q[t], k[t], v[t], kring, vring, t, scale=0.6)
        ol = co.decode_linear(q[t], k[t], v[t], A, Z, eps=0.125)
        assert max_abs(ow, full_w[t]) < 1e-12, t
        assert max_abs(ol, full_l[t]) < 1e-12, t
    # what is kept between steps: the last w keys in ring order, and Algorithm 1's running sums
    for t in range(max(0, N - w), N):
        assert np.array_equal(kring[t % w], k[t]) and np.array_equal(vring[t % w], v[t])
    fk = np.where(k > 0, k + 1, np.exp(k))
    assert max_abs(A, fk.T @ v) < 1e-12 and max_abs(Z, fk.sum(0)) < 1e-12


def test_decode_linear_worked_example_and_identity_map():
    g = load_golden("linear_4token.json")
    q, k, v = (parse_matrix(g[n]) for n in "qkv")
    d = q.shape[1]
    A, Z = np.zeros((d, d)), np.zeros(d)
    rows = [co.decode_linear(q[t], k[t], v[t], A, Z, phi=co.PHI_ELU1 if g.get("phi", "elu1") == "elu1" else co.PHI_IDENTITY)
            for t in range(q.shape[0])]
    assert max_abs(np.array(rows), co.linear_head(q, k, v)) < 1e-13
    with pytest.raises(ValueError):
        co.decode_linear(q[0], k[0], v[0], A.astype(np.float32), Z)


# ---- Head partition model (Section III-D, Algorithm 2) ---------------------------------------

def _partition_golden():
    with open(os.path.join(os.path.dirname(__file__), "golden", "partition_examples.json")) as f:
        return json.load(f)


def _fr(x):
    return Fraction(x)


@pytest.mark.parametrize("case", range(3))
def test_partition_balance_worked_examples(case):
    ex = _partition_golden()["balance"][case]
    args = [float(_fr(ex[k])) for k in ("p", "size", "flops_per0", "flops_per1", "perf0", "perf1")]
    pp = co.partition_balance(*args)
    assert abs(pp - float(_fr(ex["p_prime"]))) <= 1e-14, ex["why"]
    l0, l1 = co.partition_latencies(pp, *args[1:])
    want = float(_fr(ex["latency_at_p_prime"]))
    assert abs(l0 - want) <= 1e-12 * want and abs(l1 - want) <= 1e-12 * want


@pytest.mark.parametrize("seed", range(6))
def test_partition_balance_against_exact_rationals(seed):
    """Equal latencies p' c0 = (1-p') c1 with c = FLOPs per unit / performance, solved in exact
    rationals: p' = c1 / (c0 + c1).  Also: independent of size and of the initial share, and
    swapping the two partitions gives 1 - p'."""
    rng = random.Random(seed)
    f0, f1 = Fraction(rng.randint(1, 999), rng.randint(1, 99)), Fraction(rng.randint(1, 999), rng.randint(1, 99))
    g0, g1 = Fraction(rng.randint(1, 999), rng.randint(1, 99)), Fraction(rng.randint(1, 999), rng.randint(1, 99))
    size = Fraction(rng.randint(1, 10 ** 6))
    c0, c1 = f0 / g0, f1 / g1
    want = c1 / (c0 + c1)
    got = co.partition_balance(0.25, float(size), float(f0), float(f1), float(g0), float(g1))
    assert abs(got - float(want)) <= 1e-13
    assert abs(co.partition_balance(0.9, 3.0 * float(size), float(f0), float(f1), float(g0), float(g1)) - got) <= 1e-13
    swapped = co.partition_balance(0.25, float(size), float(f1), float(f0), float(g1), float(g0))
    assert abs(swapped - (1.0 - got)) <= 1e-13
    # a dropped (1-p), a latency written as perf/FLOPs or a swapped performance would each move p'
    wrong = [c0 / (c0 + c1), (f1 * g1) / (f0 * g0 + f1 * g1), (f1 / g0) / (f0 / g1 + f1 / g0)]
    assert all(abs(float(wv) - got) > 1e-6 for wv in wrong if wv != want)


def test_partition_latencies_follow_the_printed_steps():
    # share 1/4 of 8 units at 6 FLOPs per unit and 4 FLOP/s: 12 FLOPs, 3 s; the rest: 6 units at 1 FLOP, 2 FLOP/s: 3 s
    assert co.partition_latencies(0.25, 8.0, 6.0, 1.0, 4.0, 2.0) == (3.0, 3.0)
    assert co.partition_latencies(1.0, 8.0, 6.0, 1.0, 4.0, 2.0) == (12.0, 0.0)
    assert co.partition_latencies(0.0, 8.0, 6.0, 1.0, 4.0, 2.0) == (0.0, 4.0)


def test_partition_flop_counts_are_the_printed_ones():
    B, N, E, W = 3, 7, 5, 11
    # windowed: 2 B H0 E N W + 3 B H0 N W
    assert co.sparse_flops(B, 2, N, E, W) == 2 * B * 2 * E * N * W + 3 * B * 2 * N * W
    # linear: (4 + 2 + 2) B N (H1 E)^2
    assert co.linear_flops(B, 4, N, E, co.FLOPS_PAPER) == 8 * B * N * (4 * E) ** 2
    assert co.linear_flops(B, 4, N, E, co.FLOPS_PER_HEAD) == 8 * B * N * 4 * E ** 2
    assert co.linear_flops(B, 1, N, E, co.FLOPS_PAPER) == co.linear_flops(B, 1, N, E, co.FLOPS_PER_HEAD)
    assert co.sparse_flops(B, 0, N, E, W) == 0 and co.linear_flops(B, 0, N, E) == 0


@pytest.mark.parametrize("case", range(4))
def test_partition_heads_worked_examples(case):
    ex = _partition_golden()["heads"][case]
    model = co.FLOPS_PAPER if ex["flop_model"] == "paper" else co.FLOPS_PER_HEAD
    h0, ls, ll = co.partition_heads(ex["B"], ex["H"], ex["N"], ex["E"], ex["W"], float(_fr(ex["perf_sparse"])),
                                    float(_fr(ex["perf_linear"])), model)
    assert h0 == ex["H0"], ex["why"]
    assert ls == float(_fr(ex["latency_sparse"])) and ll == float(_fr(ex["latency_linear"]))


@pytest.mark.parametrize("seed", range(8))
def test_partition_heads_against_exact_rational_search(seed):
    rng = random.Random(100 + seed)
    B, H, N, E, W = rng.randint(1, 4), rng.randint(1, 40), rng.randint(1, 4096), rng.choice([16, 64, 128]), rng.randint(1, 512)
    ps, pl = Fraction(rng.randint(1, 10 ** 6)), Fraction(rng.randint(1, 10 ** 6))
    for model in (co.FLOPS_PAPER, co.FLOPS_PER_HEAD):
        gaps = []
        for h0 in range(H + 1):
            fs = Fraction(2 * B * h0 * E * N * W + 3 * B * h0 * N * W)
            h1 = H - h0
            fl = Fraction(8 * B * N * ((h1 * E) ** 2 if model == co.FLOPS_PAPER else h1 * E * E))
            gaps.append(abs(fs / ps - fl / pl))
        want = min(range(H + 1), key=lambda h: (gaps[h], h))
        got, ls, ll = co.partition_heads(B, H, N, E, W, float(ps), float(pl), model)
        # the float search may only differ from the exact one on a near-tie
        assert got == want or abs(float(gaps[got] - gaps[want])) <= 1e-9 * float(max(gaps))
        assert abs(abs(ls - ll) - float(gaps[got])) <= 1e-9 * float(max(gaps))


def test_partition_heads_follows_the_continuous_balance():
    """With heads counted one by one both latencies are linear in the head count, so the head
    search must land within one head of H times the share Algorithm 2 returns."""
    B, H, N, E, W = 4, 32, 8192, 128, 256
    ps, pl = 3.0e14, 2.0e14
    pp = co.partition_balance(0.5, float(H), co.sparse_flops(B, 1, N, E, W), co.linear_flops(B, 1, N, E, co.FLOPS_PER_HEAD), ps, pl)
    h0, _, _ = co.partition_heads(B, H, N, E, W, ps, pl, co.FLOPS_PER_HEAD)
    assert abs(h0 - pp * H) <= 0.5 + 1e-9


# ---- Backward pass ---------------------------------------------------------------------------

def _bwd_golden():
    with open(os.path.join(os.path.dirname(__file__), "golden", "backward_2token.json")) as f:
        return json.load(f)


def _gval(x):
    """'3/4', '-ln2', '3/4*ln3' -> float."""
    x = x.replace("ln3", repr(math.log(3.0))).replace("ln2", repr(math.log(2.0)))
    if "*" in x:
        a, b = x.split("*")
        return float(Fraction(a)) * float(b)
    if x.startswith("-") and not x[1:].replace("/", "").replace(".", "").isdigit():
        return -float(x[1:])
    try:
        return float(Fraction(x))
    except ValueError:
        return float(x)


def _gcol(ex, key):
    return np.array([[_gval(x)] for x in ex[key]], dtype=np.float64)


def test_backward_worked_examples():
    g = _bwd_golden()
    ex = g["window"]
    dq, dk, dv = co.windowed_head_bwd(_gcol(ex, "q"), _gcol(ex, "k"), _gcol(ex, "v"), _gcol(ex, "dout"), 2)
    for got, key in ((dq, "dq"), (dk, "dk"), (dv, "dv")):
        assert max_abs(got, _gcol(ex, key)) <= 1e-14, (key, ex["why"])
    for name, phi in (("linear_identity", co.PHI_IDENTITY), ("linear_elu", co.PHI_ELU1)):
        ex = g[name]
        dq, dk, dv = co.linear_head_bwd(_gcol(ex, "q"), _gcol(ex, "k"), _gcol(ex, "v"), _gcol(ex, "dout"), phi=phi)
        for got, key in ((dq, "dq"), (dk, "dk"), (dv, "dv")):
            assert max_abs(got, _gcol(ex, key)) <= 1e-14, (name, key, ex["why"])


def _central_differences(f, x, dout, h=1e-6):
    """d/dx of sum(f(x) * dout) by central differences, every element of x."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    while not it.finished:
        idx = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        g[idx] = ((f(xp) - f(xm)) * dout).sum() / (2 * h)
        it.iternext()
    return g


@pytest.mark.parametrize("N,d,w", [(9, 3, 4), (7, 4, 1), (6, 2, 50)])
def test_windowed_backward_is_the_derivative_of_the_forward(N, d, w):
    """Central differences of the (separately pinned) forward oracle, every input element."""
    q, k, v, do = (_rand((N, d), 300 + s) for s in range(4))
    dq, dk, dv = co.windowed_head_bwd(q, k, v, do, w, 0.7)
    assert max_abs(dq, _central_differences(lambda x: co.windowed_head(x, k, v, w, 0.7), q, do)) <= 1e-7
    assert max_abs(dk, _central_differences(lambda x: co.windowed_head(q, x, v, w, 0.7), k, do)) <= 1e-7
    assert max_abs(dv, _central_differences(lambda x: co.windowed_head(q, k, x, w, 0.7), v, do)) <= 1e-7


@pytest.mark.parametrize("phi", [co.PHI_ELU1, co.PHI_IDENTITY])
@pytest.mark.parametrize("N,d", [(8, 3), (5, 4)])
def test_linear_backward_is_the_derivative_of_the_forward(N, d, phi):
    q, k, v, do = (_rand((N, d), 310 + s) for s in range(4))
    if phi == co.PHI_IDENTITY:      # keep the denominators away from zero
        q, k = np.abs(q) + 0.5, np.abs(k) + 0.5
    eps = 0.25
    f = lambda a, b, c: co.linear_head(a, b, c, phi=phi, eps=eps, form=co.LINEAR_QUADRATIC)
    dq, dk, dv = co.linear_head_bwd(q, k, v, do, phi=phi, eps=eps)
    assert max_abs(dq, _central_differences(lambda x: f(x, k, v), q, do)) <= 1e-7
    assert max_abs(dk, _central_differences(lambda x: f(q, x, v), k, do)) <= 1e-7
    assert max_abs(dv, _central_differences(lambda x: f(q, k, x), v, do)) <= 1e-7


def test_backward_against_library_autograd():
    """The two definitions written with library tensor routines (band-masked softmax; cumulative
    sums for Algorithm 1) and differentiated by the library's reverse mode."""
    N, d, w = 150, 8, 37
    q, k, v, do = (torch.tensor(_rand((N, d), 320 + s)) for s in range(4))
    idx = torch.arange(N)
    band = (idx[None, :] <= idx[:, None]) & (idx[None, :] > idx[:, None] - w)
    tq, tk, tv = (t.clone().requires_grad_(True) for t in (q, k, v))
    s = (tq @ tk.T) * 0.3
    o = torch.softmax(s.masked_fill(~band, float("-inf")), dim=-1) @ tv
    (o * do).sum().backward()
    dq, dk, dv = co.windowed_head_bwd(q.numpy(), k.numpy(), v.numpy(), do.numpy(), w, 0.3)
    assert max_abs(dq, tq.grad.numpy()) <= 1e-12 and max_abs(dk, tk.grad.numpy()) <= 1e-12
    assert max_abs(dv, tv.grad.numpy()) <= 1e-12
    tq, tk, tv = (t.clone().requires_grad_(True) for t in (q, k, v))
    fq, fk = torch.nn.functional.elu(tq) + 1, torch.nn.functional.elu(tk) + 1
    A = torch.cumsum(fk[:, :, None] * tv[:, None, :], dim=0)        # Algorithm 1's running sums
    Z = torch.cumsum(fk, dim=0)
    o = torch.einsum("nc,nce->ne", fq, A) / ((fq * Z).sum(-1, keepdim=True) + 0.125)
    (o * do).sum().backward()
    dq, dk, dv = co.linear_head_bwd(q.numpy(), k.numpy(), v.numpy(), do.numpy(), eps=0.125)
    assert max_abs(dq, tq.grad.numpy()) <= 1e-11 and max_abs(dk, tk.grad.numpy()) <= 1e-11
    assert max_abs(dv, tv.grad.numpy()) <= 1e-11


def test_backward_closed_forms():
    N, d = 40, 6
    q, k, v, do = (_rand((N, d), 330 + s) for s in range(4))
    # window 1: every token returns its own value, so dv = dO and nothing depends on q or k
    dq, dk, dv = co.windowed_head_bwd(q, k, v, do, 1)
    assert max_abs(dq, 0 * q) == 0 and max_abs(dk, 0 * k) == 0 and max_abs(dv, do) <= 1e-15
    # the softmax Jacobian annihilates constants: sum_j ds_ij = 0 for every query.  With one common
    # query vector qc, dk_j = scale * qc * sum_i ds_ij, so the dk rows add up to zero
    qc = np.tile(_rand((1, d), 340), (N, 1))
    dq, dk, dv = co.windowed_head_bwd(qc, k, v, do, N)       # full causal attention
    assert max_abs(dk.sum(axis=0), np.zeros(d)) <= 1e-12
    # linear head: the ratio is unchanged when every phi(k_j) is scaled by one factor (identity
    # map, eps = 0), so sum_j k_j . dk_j = 0; and likewise q_i . dq_i = 0 for every token
    qp, kp = np.abs(q) + 0.5, np.abs(k) + 0.5
    dq, dk, dv = co.linear_head_bwd(qp, kp, v, do, phi=co.PHI_IDENTITY)
    assert abs((kp * dk).sum()) <= 1e-11
    assert max_abs((qp * dq).sum(axis=1), np.zeros(N)) <= 1e-11
    # first token of a linear head: out_0 = v_0 (eps = 0)
    dq1, dk1, dv1 = co.linear_head_bwd(q[:1], k[:1], v[:1], do[:1])
    assert max_abs(dv1, do[:1]) <= 1e-15 and max_abs(dq1, 0 * dq1) <= 1e-15 and max_abs(dk1, 0 * dk1) <= 1e-15


def test_backward_is_linear_in_the_output_gradient_and_splits_by_head():
    B, H, N, d, w, H0 = 2, 3, 30, 4, 7, 1
    q, k, v, d1, d2 = (_rand((B, H, N, d), 350 + s) for s in range(5))
    a = co.attn_bwd(q, k, v, d1, w, H0, softmax_scale=0.5, eps=0.1)
    b = co.attn_bwd(q, k, v, d2, w, H0, softmax_scale=0.5, eps=0.1)
    c = co.attn_bwd(q, k, v, 2 * d1 - 3 * d2, w, H0, softmax_scale=0.5, eps=0.1)
    for x, y, z in zip(a, b, c):
        assert max_abs(z, 2 * x - 3 * y) <= 1e-12
    for bb in range(B):
        ref = co.windowed_head_bwd(q[bb, 0], k[bb, 0], v[bb, 0], d1[bb, 0], w, 0.5)
        for x, y in zip(a, ref):
            assert max_abs(x[bb, 0], y) == 0
        ref = co.linear_head_bwd(q[bb, 2], k[bb, 2], v[bb, 2], d1[bb, 2], eps=0.1)
        for x, y in zip(a, ref):
            assert max_abs(x[bb, 2], y) == 0


# ---------------------------------------------------------------------------------------
# backward pass of the bidirectional variant
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("N,d,w", [(9, 3, 4), (7, 4, 1), (8, 2, 5), (6, 2, 50)])
def test_bidirectional_windowed_backward_is_the_derivative_of_the_forward(N, d, w):
    """Central differences of the (separately pinned) bidirectional forward oracle."""
    q, k, v, do = (_rand((N, d), 400 + s) for s in range(4))
    f = lambda a, b, c: co.windowed_head(a, b, c, w, 0.7, bidirectional=True)
    dq, dk, dv = co.windowed_head_bwd(q, k, v, do, w, 0.7, bidirectional=True)
    assert max_abs(dq, _central_differences(lambda x: f(x, k, v), q, do)) <= 1e-7
    assert max_abs(dk, _central_differences(lambda x: f(q, x, v), k, do)) <= 1e-7
    assert max_abs(dv, _central_differences(lambda x: f(q, k, x), v, do)) <= 1e-7


@pytest.mark.parametrize("phi", [co.PHI_ELU1, co.PHI_IDENTITY])
@pytest.mark.parametrize("N,d", [(8, 3), (5, 4)])
def test_bidirectional_linear_backward_is_the_derivative_of_the_forward(N, d, phi):
    q, k, v, do = (_rand((N, d), 410 + s) for s in range(4))
    if phi == co.PHI_IDENTITY:
        q, k = np.abs(q) + 0.5, np.abs(k) + 0.5
    eps = 0.25
    f = lambda a, b, c: co.linear_head(a, b, c, phi=phi, eps=eps, bidirectional=True)
    dq, dk, dv = co.linear_head_bwd(q, k, v, do, phi=phi, eps=eps, bidirectional=True)
    assert max_abs(dq, _central_differences(lambda x: f(x, k, v), q, do)) <= 1e-7
    assert max_abs(dk, _central_differences(lambda x: f(q, x, v), k, do)) <= 1e-7
    assert max_abs(dv, _central_differences(lambda x: f(q, k, x), v, do)) <= 1e-7


def test_bidirectional_backward_against_library_autograd():
    """The two definitions written with library tensor routines (softmax under a centred band
    mask; state first for the linear head) and differentiated by the library's reverse mode."""
    N, d = 150, 8
    q, k, v, do = (torch.tensor(_rand((N, d), 420 + s)) for s in range(4))
    idx = torch.arange(N)
    for w in (37, 38, 1, 400):       # odd, even (one more on the left), self only, everything
        left, right = w // 2, w - 1 - w // 2
        band = (idx[None, :] >= idx[:, None] - left) & (idx[None, :] <= idx[:, None] + right)
        tq, tk, tv = (t.clone().requires_grad_(True) for t in (q, k, v))
        o = torch.softmax(((tq @ tk.T) * 0.3).masked_fill(~band, float("-inf")), dim=-1) @ tv
        (o * do).sum().backward()
        dq, dk, dv = co.windowed_head_bwd(q.numpy(), k.numpy(), v.numpy(), do.numpy(), w, 0.3, bidirectional=True)
        assert max_abs(dq, tq.grad.numpy()) <= 1e-12 and max_abs(dk, tk.grad.numpy()) <= 1e-12, w
        assert max_abs(dv, tv.grad.numpy()) <= 1e-12, w
    tq, tk, tv = (t.clone().requires_grad_(True) for t in (q, k, v))
    fq, fk = torch.nn.functional.elu(tq) + 1, torch.nn.functional.elu(tk) + 1
    o = (fq @ (fk.T @ tv)) / ((fq @ fk.sum(0))[:, None] + 0.125)      # section II-B, state first
    (o * do).sum().backward()
    dq, dk, dv = co.linear_head_bwd(q.numpy(), k.numpy(), v.numpy(), do.numpy(), eps=0.125, bidirectional=True)
    assert max_abs(dq, tq.grad.numpy()) <= 1e-11 and max_abs(dk, tk.grad.numpy()) <= 1e-11
    assert max_abs(dv, tv.grad.numpy()) <= 1e-11
    # a window that covers everything is full softmax attention: the library's fused routine
    tq, tk, tv = (t.clone().requires_grad_(True) for t in (q, k, v))
    o = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None], tv[None], scale=0.3)[0]
    (o * do).sum().backward()
    dq, dk, dv = co.windowed_head_bwd(q.numpy(), k.numpy(), v.numpy(), do.numpy(), 2 * N, 0.3, bidirectional=True)
    assert max_abs(dq, tq.grad.numpy()) <= 1e-12 and max_abs(dk, tk.grad.numpy()) <= 1e-12
    assert max_abs(dv, tv.grad.numpy()) <= 1e-12


def test_bidirectional_backward_closed_forms_and_relations():
    N, d = 40, 6
    q, k, v, do = (_rand((N, d), 430 + s) for s in range(4))
    # windows of one and two tokens coincide with the causal window (nothing to the right)
    for w in (1, 2):
        for a, b in zip(co.windowed_head_bwd(q, k, v, do, w, 0.5, bidirectional=True),
                        co.windowed_head_bwd(q, k, v, do, w, 0.5)):
            assert max_abs(a, b) == 0
    # the linear head does not know the order of the (key, value) pairs: permuting them permutes
    # dk and dv and leaves dq alone
    perm = np.random.default_rng(7).permutation(N)
    a = co.linear_head_bwd(q, k, v, do, eps=0.1, bidirectional=True)
    b = co.linear_head_bwd(q, k[perm], v[perm], do, eps=0.1, bidirectional=True)
    assert max_abs(a[0], b[0]) <= 1e-12 and max_abs(a[1][perm], b[1]) <= 1e-12 and max_abs(a[2][perm], b[2]) <= 1e-12
    # only the last token's output gets a gradient: the last causal row sees every key too
    last = np.zeros_like(do)
    last[-1] = do[-1]
    for x, y in zip(co.linear_head_bwd(q, k, v, last, eps=0.1, bidirectional=True),
                    co.linear_head_bwd(q, k, v, last, eps=0.1)):
        assert max_abs(x, y) <= 1e-13
    # scale invariance of the ratio (identity map, eps = 0): sum_j k_j.dk_j = 0, q_i.dq_i = 0
    qp, kp = np.abs(q) + 0.5, np.abs(k) + 0.5
    dq, dk, dv = co.linear_head_bwd(qp, kp, v, do, phi=co.PHI_IDENTITY, bidirectional=True)
    assert abs((kp * dk).sum()) <= 1e-11 and max_abs((qp * dq).sum(axis=1), np.zeros(N)) <= 1e-11
    # weights sum to one: with a constant added to every value nothing but dv could change, and
    # sum_j dv_j = sum_i dO_i (eps = 0)
    dq2, dk2, dv2 = co.linear_head_bwd(q, k, v + 3.0, do, bidirectional=True)
    dq1, dk1, dv1 = co.linear_head_bwd(q, k, v, do, bidirectional=True)
    assert max_abs(dq1, dq2) <= 1e-11 and max_abs(dk1, dk2) <= 1e-11 and max_abs(dv1, dv2) <= 1e-13
    assert max_abs(dv1.sum(axis=0), do.sum(axis=0)) <= 1e-12
    # the layer driver places heads like the forward one
    B, H, w, H0 = 2, 3, 7, 1
    q4, k4, v4, d4 = (_rand((B, H, 30, 4), 440 + s) for s in range(4))
    full = co.attn_bwd(q4, k4, v4, d4, w, H0, softmax_scale=0.5, eps=0.1, bidirectional=True)
    for bb in range(B):
        for x, y in zip(full, co.windowed_head_bwd(q4[bb, 0], k4[bb, 0], v4[bb, 0], d4[bb, 0], w, 0.5, bidirectional=True)):
            assert max_abs(x[bb, 0], y) == 0
        for x, y in zip(full, co.linear_head_bwd(q4[bb, 2], k4[bb, 2], v4[bb, 2], d4[bb, 2], eps=0.1, bidirectional=True)):
            assert max_abs(x[bb, 2], y) == 0
