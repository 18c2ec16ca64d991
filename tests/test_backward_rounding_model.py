"""Which operands of the matrix-core backward pass may be one bf16 and which may not (CPU only).

The matrix-core kernels of the linear heads work in chunks of 64 tokens with bf16 operands
(phi(q), phi(k), the in-chunk weights S and T', g = dO/den and the copy of the carried sum) and
fp32 accumulation.  This file writes those chunked formulas out in numpy, exactly and with the
operands rounded where a kernel could round them, and compares with the oracle:
  * without rounding the chunked form IS the oracle's derivative (to fp64 rounding), so the
    rearrangement the kernels use is right;
  * with every operand rounded to one bf16, rows of dk that are small because their terms cancel
    come out 2-4 % off in relative L2 although the average row is within 1 %: not within the
    2e-2 per row that the bf16 mode is held to;
  * with T' = tril(g v^T - c 1^T) carried as a bf16 pair (high half + rounded remainder) wherever
    it is an operand, and S = tril(phiQ phiK^T) as a pair in the numerator and the denominator of
    the forward scan (c = dO.num / den^2 enters every T' of its row), the worst row is back under
    1.5e-2 - which is what the kernels do.  The other operands stay one bf16.
"""
import numpy as np

from oracle import cpu_oracle as co
from paper_2412_19829_amd import inputs as gi

CH = 64


def _rb(x):
    return gi.round_to_bf16(x.astype(np.float32)).astype(np.float64)


def _phi(x):
    return np.where(x > 0, x + 1, np.exp(x))


def _pair(x):
    hi = _rb(x)
    return hi + _rb(x - hi)


def chunked_linear_bwd(q, k, v, dout, rounded, pairs=False):
    """dq, dk, dv of one causal linear head by the chunked forward and reverse scans.
    rounded: every matrix operand is rounded to bf16; pairs: T' (both scans) and the S of the
    forward scan's numerator and denominator are bf16 pairs instead."""
    R = _rb if rounded else (lambda x: x)
    RT = _pair if pairs else R
    N, d = q.shape
    fq, fk = R(_phi(q)), R(_phi(k))
    nch = (N + CH - 1) // CH
    A, Z = np.zeros((d, d)), np.zeros(d)
    den, c, dfq = np.zeros(N), np.zeros(N), np.zeros((N, d))
    for n in range(nch):                      # forward scan
        sl = slice(n * CH, min(N, (n + 1) * CH))
        Sm = RT(np.tril(fq[sl] @ fk[sl].T))
        num = Sm @ v[sl] + fq[sl] @ R(A)
        den[sl] = Sm.sum(1) + fq[sl] @ Z
        c[sl] = (dout[sl] * num).sum(1) / den[sl] ** 2
        g = R(dout[sl] / den[sl][:, None])
        Tp = RT(np.tril((dout[sl] @ v[sl].T) / den[sl][:, None] - c[sl][:, None]))
        dfq[sl] = Tp @ fk[sl] + g @ R(A).T - c[sl][:, None] * Z[None, :]
        A += fk[sl].T @ v[sl]
        Z += fk[sl].sum(0)
    Bn, Y = np.zeros((d, d)), np.zeros(d)
    dfk, dv = np.zeros((N, d)), np.zeros((N, d))
    for n in reversed(range(nch)):            # reverse scan
        sl = slice(n * CH, min(N, (n + 1) * CH))
        Sm = R(np.tril(fq[sl] @ fk[sl].T))
        g = R(dout[sl] / den[sl][:, None])
        Tp = RT(np.tril((dout[sl] @ v[sl].T) / den[sl][:, None] - c[sl][:, None]))
        dfk[sl] = Tp.T @ fq[sl] + v[sl] @ R(Bn).T - Y[None, :]
        dv[sl] = Sm.T @ g + fk[sl] @ R(Bn)
        Bn += fq[sl].T @ g
        Y += fq[sl].T @ c[sl]
    slope = lambda f: np.where(f > 1, 1.0, f)
    return dfq * slope(fq), dfk * slope(fk), dv


def _case(N=281, d=64, seed=1182):
    wl = gi.Workload("case", 1, 1, N, d, 1, "bf16", seed)
    q, k, v = gi.make_qkv(wl)
    dout = gi.make_qkv(gi.Workload("case", 1, 1, N, d, 1, "bf16", seed + 1))[2]
    ref = co.attn_bwd(q, k, v, dout, 1, 0)
    return tuple(x[0, 0].astype(np.float64) for x in (q, k, v, dout)), tuple(r[0, 0] for r in ref)


def _row_rel(got, ref):
    """Per-row relative L2 error; rows that are exactly zero (dq of the first token, which sees
    only itself) are left out."""
    norm = np.sqrt((ref ** 2).sum(-1))
    keep = norm > 0
    return np.sqrt(((got - ref) ** 2).sum(-1))[keep] / norm[keep]


def test_chunked_scans_are_the_oracles_derivative():
    (q, k, v, dout), ref = _case()
    got = chunked_linear_bwd(q, k, v, dout, rounded=False)
    for g, r in zip(got, ref):
        assert np.abs(g - r).max() <= 1e-10 * max(1.0, np.abs(r).max())


def test_bf16_operands_alone_cost_a_few_percent_on_cancelling_rows():
    (q, k, v, dout), ref = _case()
    got = chunked_linear_bwd(q, k, v, dout, rounded=True)
    rel = [_row_rel(g, r) for g, r in zip(got, ref)]
    worst = max(float(x.max()) for x in rel)
    mean = max(float(x.mean()) for x in rel)
    assert mean < 1e-2            # the average row is fine
    assert 2e-2 < worst < 4e-2    # single rows are not within 2e-2 with one bf16 per operand


def _gpu_measure(got, ref, dout):
    """The GPU tests' measure: per-row L2 error over the row's norm, rows that vanish by
    cancellation measured against 1 % of a typical dO row."""
    err = np.sqrt(((got - ref) ** 2).sum(-1))
    floor = 1e-2 * float(np.median(np.sqrt((dout ** 2).sum(-1))))
    return err / np.maximum(np.sqrt((ref ** 2).sum(-1)), floor)


def test_bf16_pairs_for_the_two_cancelling_operands_bring_every_row_under_the_bar():
    rng = np.random.default_rng(1)
    worst_single, worst_pairs = 0.0, 0.0
    for _ in range(12):
        N, d, seed = int(rng.integers(100, 500)), int(rng.choice([64, 128])), int(rng.integers(0, 10 ** 6))
        (q, k, v, dout), ref = _case(N, d, seed)
        single = chunked_linear_bwd(q, k, v, dout, rounded=True)
        pairs = chunked_linear_bwd(q, k, v, dout, rounded=True, pairs=True)
        worst_single = max(worst_single, max(float(_gpu_measure(g, r, dout).max()) for g, r in zip(single, ref)))
        worst_pairs = max(worst_pairs, max(float(_gpu_measure(g, r, dout).max()) for g, r in zip(pairs, ref)))
    assert worst_single > 2e-2     # one bf16 per operand misses the bar on some input
    assert worst_pairs < 1.5e-2    # the kernels' choice meets it with room to spare
