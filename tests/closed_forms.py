"""Closed forms of masked attention with uniform probabilities, in O(N d^2) per head.

TEST INFRASTRUCTURE, independent of the oracle and of the HIP path: nothing here expands a mask or
forms an N x N array.  When every score is 0 (Q = 0 or K = 0), Equations 1-2 give P_ij = 1 / c_i on the
keys row i may see (c_i of them) and Algorithm 2 reduces to sums over those sets:

    lse_i = log c_i                         out_i = (1 / c_i) sum_{j in A_i} V_j
    D_i   = dO_i . out_i                    dV_j  = sum_{i sees j} dO_i / c_i
    dS_ij = (dO_i . V_j - D_i) / c_i
    dQ_i  = scale / c_i * ( (sum_{j in A_i} K_j V_j^T) dO_i  -  D_i sum_{j in A_i} K_j )
    dK_j  = scale * ( (sum_{i sees j} q_i dO_i^T / c_i) V_j  -  sum_{i sees j} D_i q_i / c_i )

For the causal-type masks of the benchmark configurations the keys a row sees form ONE contiguous
range A_i = [a_i, e_i) and the rows that see a key form one contiguous range [r_j, b_j), both with
non-decreasing end points, so every sum is a difference of prefix sums.  The ranges are written here
from the task structure (document spans, window width, prefix length), not from the four vectors.
"""
from __future__ import annotations

import numpy as np


def ranges_causal_document(n, spans):
    """Row i of document [s, e) sees keys [s, i + 1); key j is seen by rows [j, e)."""
    a = np.zeros(n, dtype=np.int64)
    b = np.zeros(n, dtype=np.int64)
    for s, e in spans:
        a[s:e] = s
        b[s:e] = e
    idx = np.arange(n, dtype=np.int64)
    return a, idx + 1, idx.copy(), b


def ranges_sliding_window(n, w):
    """Row i sees keys [max(0, i - w + 1), i + 1); key j is seen by rows [j, min(j + w, n))."""
    idx = np.arange(n, dtype=np.int64)
    return np.maximum(idx - w + 1, 0), idx + 1, idx.copy(), np.minimum(idx + w, n)


def ranges_prefix_lm(n, p):
    """Row i sees keys [0, max(i + 1, p)); key j < p is seen by every row, key j >= p by rows [j, n)."""
    idx = np.arange(n, dtype=np.int64)
    return np.zeros(n, dtype=np.int64), np.maximum(idx + 1, p), np.where(idx < p, 0, idx), np.full(n, n, dtype=np.int64)


def ranges_of(workload, b):
    """(a, e, r, bb) for batch row b of a Workload whose mask kind is one of the three above."""
    st = workload.structure[b]
    if workload.mask_kind == "causal_document":
        return ranges_causal_document(workload.N, st)
    if workload.mask_kind == "sliding_window":
        return ranges_sliding_window(workload.N, st["window"])
    if workload.mask_kind == "prefix_lm":
        return ranges_prefix_lm(workload.N, st["prefix"])
    raise ValueError(workload.mask_kind)


def prefix_rows(x):
    """[N + 1, ...] prefix sums along axis 0: result[t] = sum_{i < t} x_i."""
    out = np.zeros((x.shape[0] + 1,) + x.shape[1:], dtype=np.float64)
    np.cumsum(x, axis=0, out=out[1:])
    return out


def prefix_apply(A, B, x, U, block=192):
    """y_t = sum_{i < x_t} A_i (B_i . U_t) = (sum_{i < x_t} A_i B_i^T) U_t for t = 0..len(x)-1.

    A, B: [M, d]; U: [T, d]; x: int [T], non-decreasing, 0 <= x_t <= M.  The d x d prefix matrix is
    carried as a running sum up to `base` and the at most `block` terms between base and x_t are added
    per group of rows, so the cost is O((M + T) d^2) and no [M, d, d] array exists."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    x = np.asarray(x, dtype=np.int64)
    assert x.ndim == 1 and U.shape[0] == x.shape[0]
    assert np.all(np.diff(x) >= 0) and (x.size == 0 or (x[0] >= 0 and x[-1] <= A.shape[0]))
    d = A.shape[1]
    y = np.zeros((x.shape[0], d), dtype=np.float64)
    R = np.zeros((d, d), dtype=np.float64)       # R[p, q] = sum_{i < base} A_i[p] B_i[q]
    base, t, total = 0, 0, x.shape[0]
    while t < total:
        nb = int(x[t])
        for c0 in range(base, nb, 4096):
            c1 = min(c0 + 4096, nb)
            R += A[c0:c1].T @ B[c0:c1]
        base = nb
        # rows t..t1-1: those whose end point lies within `block` of base (at least row t itself)
        t1 = t + int(np.searchsorted(x[t:t + block], base + block, side="right"))
        span = int(x[t1 - 1]) - base
        u = U[t:t1]
        acc = u @ R.T
        if span > 0:
            g = u @ B[base:base + span].T                                       # [rows, span]
            g *= (np.arange(span)[None, :] < (x[t:t1] - base)[:, None])
            acc += g @ A[base:base + span]
        y[t:t1] = acc
        t = t1
    return y


def range_apply(A, B, lo, hi, U):
    """y_t = sum_{lo_t <= i < hi_t} A_i (B_i . U_t); empty ranges (hi <= lo) give 0."""
    hi = np.maximum(hi, lo)
    return prefix_apply(A, B, hi, U) - prefix_apply(A, B, lo, U)


def forward_uniform(v, a, e):
    """lse [N], out [N, d] for S = 0: uniform attention over keys [a_i, e_i)."""
    v = np.asarray(v, dtype=np.float64)
    c = (e - a).astype(np.float64)
    pv = prefix_rows(v)
    with np.errstate(divide="ignore", invalid="ignore"):
        out = np.where(c[:, None] > 0, (pv[e] - pv[a]) / c[:, None], 0.0)
        lse = np.log(c)
    return lse, out


def backward_uniform(q, k, v, dout, scale, a, e, r, bb, out=None):
    """dq, dk, dv [N, d] for S = 0 (the caller passes q = 0 or k = 0, which makes dk resp. dq exactly
    zero).  `out`: the forward output D is formed from (default: the exact closed form)."""
    q, k, v, dout = (np.asarray(t, dtype=np.float64) for t in (q, k, v, dout))
    c = (e - a).astype(np.float64)
    live = c > 0
    inv_c = np.where(live, 1.0 / np.where(live, c, 1.0), 0.0)
    if out is None:
        _, out = forward_uniform(v, a, e)
    big_d = (dout * out).sum(axis=1)
    # dV_j = sum_{i in [r_j, b_j)} dO_i / c_i
    pw = prefix_rows(dout * inv_c[:, None])
    hi = np.maximum(bb, r)
    dv = pw[hi] - pw[r]
    # dQ_i = scale / c_i * ( (sum_{j in A_i} K_j V_j^T) dO_i - D_i sum_{j in A_i} K_j )
    if k.any():
        pk = prefix_rows(k)
        dq = range_apply(k, v, a, e, dout) - big_d[:, None] * (pk[np.maximum(e, a)] - pk[a])
        dq *= (scale * inv_c)[:, None]
    else:
        dq = np.zeros_like(q)       # every term carries a factor K_j
    # dK_j = scale * ( (sum_{i sees j} q_i dO_i^T / c_i) V_j - sum_{i sees j} D_i q_i / c_i )
    if q.any():
        qs = q * inv_c[:, None]
        pqd = prefix_rows(qs * big_d[:, None])
        dk = scale * (range_apply(qs, dout, r, bb, v) - (pqd[hi] - pqd[r]))
    else:
        dk = np.zeros_like(k)       # every term carries a factor q_i
    return dq, dk, dv
