"""Where the bf16 tolerance of the matrix-core backward pass comes from (CPU only).

The matrix-core kernels of the linear heads work in chunks of 64 tokens with bf16 operands
(phi(q), phi(k), the in-chunk weights S and T', g = dO/den and the copy of the carried sum) and
fp32 accumulation.  This file writes those chunked formulas out in numpy, once exactly and once
with every operand rounded to bf16 where the kernels round, and compares with the oracle:
  * without rounding the chunked form IS the oracle's derivative (to fp64 rounding), so the
    rearrangement the kernels use is right;
  * with rounding, rows of dk that are small because their terms cancel come out 2-4 % off in
    relative L2 although the average row is within 1 %: that is the arithmetic, not the kernel,
    and it is why the GPU test allows 4e-2 per row for the matrix-core kernels where it allows
    2e-2 for the fp32-arithmetic kernels.
"""
import numpy as np

from oracle import cpu_oracle as co
from paper_2412_19829_amd import inputs as gi

CH = 64


def _rb(x):
    return gi.round_to_bf16(x.astype(np.float32)).astype(np.float64)


def _phi(x):
    return np.where(x > 0, x + 1, np.exp(x))


def chunked_linear_bwd(q, k, v, dout, rounded):
    """dq, dk, dv of one causal linear head by the chunked forward and reverse scans."""
    R = _rb if rounded else (lambda x: x)
    N, d = q.shape
    fq, fk = R(_phi(q)), R(_phi(k))
    nch = (N + CH - 1) // CH
    A, Z = np.zeros((d, d)), np.zeros(d)
    den, c, dfq = np.zeros(N), np.zeros(N), np.zeros((N, d))
    for n in range(nch):                      # forward scan
        sl = slice(n * CH, min(N, (n + 1) * CH))
        Sm = R(np.tril(fq[sl] @ fk[sl].T))
        num = Sm @ v[sl] + fq[sl] @ R(A)
        den[sl] = Sm.sum(1) + fq[sl] @ Z
        c[sl] = (dout[sl] * num).sum(1) / den[sl] ** 2
        g = R(dout[sl] / den[sl][:, None])
        Tp = R(np.tril((dout[sl] @ v[sl].T) / den[sl][:, None] - c[sl][:, None]))
        dfq[sl] = Tp @ fk[sl] + g @ R(A).T - c[sl][:, None] * Z[None, :]
        A += fk[sl].T @ v[sl]
        Z += fk[sl].sum(0)
    Bn, Y = np.zeros((d, d)), np.zeros(d)
    dfk, dv = np.zeros((N, d)), np.zeros((N, d))
    for n in reversed(range(nch)):            # reverse scan
        sl = slice(n * CH, min(N, (n + 1) * CH))
        Sm = R(np.tril(fq[sl] @ fk[sl].T))
        g = R(dout[sl] / den[sl][:, None])
        Tp = R(np.tril((dout[sl] @ v[sl].T) / den[sl][:, None] - c[sl][:, None]))
        dfk[sl] = Tp.T @ fq[sl] + v[sl] @ R(Bn).T - Y[None, :]
        dv[sl] = Sm.T @ g + fk[sl] @ R(Bn)
        Bn += fq[sl].T @ g
        Y += fq[sl].T @ c[sl]
    slope = lambda f: np.where(f > 1, 1.0, f)
    return dfq * slope(fq), dfk * slope(fk), dv


def _case():
    wl = gi.Workload("case", 1, 1, 281, 64, 1, "bf16", 1182)
    q, k, v = gi.make_qkv(wl)
    dout = gi.make_qkv(gi.Workload("case", 1, 1, 281, 64, 1, "bf16", 1183))[2]
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
    assert 1e-2 < worst < 4e-2    # single rows are not within 2e-2, whatever the kernel does
