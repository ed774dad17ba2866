"""Plain fp64 CPU oracle for column-wise sparse masked attention (FlashMask).

TEST INFRASTRUCTURE.  This file is the slow, obviously-correct definition the
HIP kernels are compared against.  It shares no code with the GPU path and the
product never calls it.

What it computes, and where the paper defines it:

* The mask.  Each key column j carries two half-open intervals of query rows,
  [LTS_j, LTE_j) and [UTS_j, UTE_j); a query row inside either interval may
  not attend to key j (Section 4.1; the element rule of Algorithm 1, "apply
  mask" steps, with 0-based rows and columns).
* Attention.  S = scale * Q K^T, masked entries set to -inf, P = softmax over
  each row, O = P V (Equations 1 and 2).  The paper's tiled algorithm reaches
  exactly this result (Section 4.4), so the oracle is the dense definition.
  The log-sum-exp L_i = m_i + log(l_i) is the quantity Algorithm 1 returns.
* Gradients.  Algorithm 2 written densely:  dV = P^T dO,  dP = dO V^T,
  D_i = sum_c dO_ic O_ic,  dS = P o (dP - D),  dQ = scale dS K,
  dK = scale dS^T Q.
* The preprocessing tables: min and max of each of the four vectors over every
  block of B_c key columns (Section 4.2 "Preprocessing"), in the order
  LTStart^max, LTStart^min, LTEnd^max, LTEnd^min, UTStart^max, UTStart^min,
  UTEnd^max, UTEnd^min.
* The tile classes of Equation 4, applied once to the lower-triangle pair and
  once to the upper-triangle pair, exactly as the skip tests and the element
  mask tests of Algorithm 1 apply them.
* Block sparsity rho (Section 4.3) and the FLOP counts derived from it
  (Appendix "Testing Method").

Readings where the paper is silent (all listed in the design notes):
a row whose keys are all masked gives out = 0, lse = -inf and contributes no
gradient; an interval with start >= end is empty; the row range of the last
(ragged) row block ends at N, not at i*B_r; scale multiplies S before the mask.

Large N: every function that would need an N x N array works on a chunk of
query rows at a time.  Softmax is row-wise, so chunking rows changes nothing
but the memory footprint.

Parity pins (tests/test_oracle_*.py): mask expansion vs each mask family's
defining predicate by brute force; the interval example printed in Section 4.1;
textbook softmax attention for the empty mask; closed forms for Q = 0; rows of
P sum to one; gradients vs central finite differences; tables vs brute force;
tile counts and TFLOP figures printed in the paper's kernel tables for the
deterministic masks; the grouped-head gradients vs finite differences of the
summed loss.  The random document / shared-question workloads of the
paper are unpublished: for those inputs parity is pinned only by predicates,
closed forms and invariants ("parity unpinned" by printed values).
"""
from __future__ import annotations

import math

import numpy as np

NEG_INF = -np.inf

# Tile-class byte, low two bits: kind.  Bits 4 and 5: which element masks a
# partially masked tile needs (lower-triangle pair / upper-triangle pair).
UNMASKED = 0
PARTIAL = 1
FULLY = 2
NEED_LT = 1 << 4
NEED_UT = 1 << 5

ROW_CHUNK = 1024


def _vec(x):
    return np.asarray(x, dtype=np.int64).reshape(-1)


# --------------------------------------------------------------------------
# Mask expansion (Section 4.1)
# --------------------------------------------------------------------------
def expand_mask(lts, lte, uts, ute, rows=None):
    """Dense boolean mask, True = masked.  Shape [len(rows), N].

    masked[i, j] = (LTS_j <= i < LTE_j) or (UTS_j <= i < UTE_j), with i the
    0-based query row and j the 0-based key column.
    """
    lts, lte, uts, ute = _vec(lts), _vec(lte), _vec(uts), _vec(ute)
    n = lts.shape[0]
    if rows is None:
        rows = np.arange(n, dtype=np.int64)
    i = np.asarray(rows, dtype=np.int64).reshape(-1, 1)
    in_lt = (lts[None, :] <= i) & (i < lte[None, :])
    in_ut = (uts[None, :] <= i) & (i < ute[None, :])
    return in_lt | in_ut


# --------------------------------------------------------------------------
# Forward (Equations 1-2; outputs of Algorithm 1)
# --------------------------------------------------------------------------
def _softmax_rows(q_rows, k, masked, scale):
    """P, lse for a chunk of rows.  q_rows [r,d], k [N,d], masked [r,N]."""
    s = scale * (q_rows @ k.T)
    s = np.where(masked, NEG_INF, s)
    m = s.max(axis=1)
    dead = ~np.isfinite(m)            # every key of the row is masked
    m_safe = np.where(dead, 0.0, m)
    e = np.exp(s - m_safe[:, None])   # exp(-inf) = 0 exactly
    l = e.sum(axis=1)
    l_safe = np.where(dead, 1.0, l)
    p = e / l_safe[:, None]
    lse = np.where(dead, NEG_INF, m_safe + np.log(l_safe))
    return p, lse


def forward_rows(q, k, v, lts, lte, uts, ute, scale, rows):
    """out [r,d] and lse [r] for the listed query rows of one (batch, head)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    out = np.zeros((rows.shape[0], v.shape[1]), dtype=np.float64)
    lse = np.zeros(rows.shape[0], dtype=np.float64)
    for c0 in range(0, rows.shape[0], ROW_CHUNK):
        r = rows[c0:c0 + ROW_CHUNK]
        masked = expand_mask(lts, lte, uts, ute, r)
        p, l = _softmax_rows(q[r], k, masked, scale)
        out[c0:c0 + ROW_CHUNK] = p @ v
        lse[c0:c0 + ROW_CHUNK] = l
    return out, lse


def forward(q, k, v, lts, lte, uts, ute, scale):
    """out [N,d], lse [N] for one (batch, head)."""
    n = np.asarray(q).shape[0]
    return forward_rows(q, k, v, lts, lte, uts, ute, scale, np.arange(n))


def probabilities(q, k, lts, lte, uts, ute, scale):
    """Dense P [N,N] (small N only; used by invariants tests)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    p, _ = _softmax_rows(q, k, expand_mask(lts, lte, uts, ute), scale)
    return p


# --------------------------------------------------------------------------
# Backward (Algorithm 2, written densely)
# --------------------------------------------------------------------------
def backward_row_block(q, k, v, dout, lts, lte, uts, ute, scale, rows):
    """Everything Algorithm 2 derives from the listed query rows: their out,
    lse and dq, and the amounts they add to dk and dv (full [N,d] arrays)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    r = np.asarray(rows, dtype=np.int64)
    masked = expand_mask(lts, lte, uts, ute, r)
    p, lse = _softmax_rows(q[r], k, masked, scale)
    out = p @ v
    do = dout[r]
    dv_part = p.T @ do
    dp = do @ v.T
    big_d = (do * out).sum(axis=1)
    ds = p * (dp - big_d[:, None])
    dq = scale * (ds @ k)
    dk_part = scale * (ds.T @ q[r])
    return dq, dk_part, dv_part, out, lse


def backward(q, k, v, dout, lts, lte, uts, ute, scale):
    """dq, dk, dv (and out, lse) for one (batch, head); all [N,d] / [N]."""
    n, d = np.asarray(q).shape
    dv_cols = np.asarray(v).shape[1]
    dq = np.zeros((n, d)); dk = np.zeros((n, d)); dv = np.zeros((n, dv_cols))
    out = np.zeros((n, dv_cols)); lse = np.zeros(n)
    for r0 in range(0, n, ROW_CHUNK):
        r = np.arange(r0, min(r0 + ROW_CHUNK, n))
        dq[r], dk_part, dv_part, out[r], lse[r] = backward_row_block(q, k, v, dout, lts, lte, uts, ute, scale, r)
        dk += dk_part
        dv += dv_part
    return dq, dk, dv, out, lse


def backward_grouped(q, k, v, dout, lts, lte, uts, ute, scale):
    """Grouped K/V heads (the head layout of the paper's inference appendix: H query heads on
    H_kv < H key/value heads; query head h attends to K/V head h // (H // H_kv)).

    q, dout: [H, N, d]; k, v: [H_kv, N, d].  Each query head is plain attention on its K/V head;
    a K/V head's gradient is the sum of what its query heads send back (chain rule through the
    shared tensor).  Returns dq [H,N,d], dk, dv [H_kv,N,d], out [H,N,d], lse [H,N].
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    heads, kv_heads = q.shape[0], k.shape[0]
    assert heads % kv_heads == 0
    group = heads // kv_heads
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    out = np.zeros_like(dout); lse = np.zeros(q.shape[:2])
    for h in range(heads):
        dq[h], dk_h, dv_h, out[h], lse[h] = backward(q[h], k[h // group], v[h // group], dout[h], lts, lte, uts, ute, scale)
        dk[h // group] += dk_h
        dv[h // group] += dv_h
    return dq, dk, dv, out, lse


def backward_rows(q, k, v, dout, lts, lte, uts, ute, scale, rows):
    """dq for the listed query rows only (dq_i needs nothing but row i)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    dq = np.zeros((rows.shape[0], q.shape[1]))
    for c0 in range(0, rows.shape[0], ROW_CHUNK):
        r = rows[c0:c0 + ROW_CHUNK]
        masked = expand_mask(lts, lte, uts, ute, r)
        p, _ = _softmax_rows(q[r], k, masked, scale)
        do = dout[r]
        dp = do @ v.T
        big_d = (do * (p @ v)).sum(axis=1)
        ds = p * (dp - big_d[:, None])
        dq[c0:c0 + ROW_CHUNK] = scale * (ds @ k)
    return dq


def backward_cols(q, k, v, dout, lts, lte, uts, ute, scale, cols):
    """dk, dv for the listed key columns only.

    dK_j = scale * sum_i dS_ij q_i and dV_j = sum_i P_ij dO_i run over the
    query rows that may see column j; P_ij needs the whole of row i, so every
    such row is evaluated densely over all N keys and then only the listed
    columns of P and dS are kept.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    cols = np.asarray(cols, dtype=np.int64)
    lts, lte, uts, ute = _vec(lts), _vec(lte), _vec(uts), _vec(ute)
    n = q.shape[0]
    dk = np.zeros((cols.shape[0], q.shape[1]))
    dv = np.zeros((cols.shape[0], v.shape[1]))
    # rows that see at least one listed column (dense expansion of those columns)
    col_masked = expand_mask(lts[cols], lte[cols], uts[cols], ute[cols],
                             np.arange(n))            # [N, len(cols)]
    live_rows = np.nonzero(~col_masked.all(axis=1))[0]
    for c0 in range(0, live_rows.shape[0], ROW_CHUNK):
        r = live_rows[c0:c0 + ROW_CHUNK]
        masked = expand_mask(lts, lte, uts, ute, r)
        p, _ = _softmax_rows(q[r], k, masked, scale)
        do = dout[r]
        big_d = (do * (p @ v)).sum(axis=1)
        p_c = p[:, cols]
        dp_c = do @ v[cols].T
        ds_c = p_c * (dp_c - big_d[:, None])
        dv += p_c.T @ do
        dk += scale * (ds_c.T @ q[r])
    return dk, dv


# --------------------------------------------------------------------------
# Preprocessing tables (Section 4.2, "Preprocessing")
# --------------------------------------------------------------------------
TABLE_ROWS = ("LTStart_max", "LTStart_min", "LTEnd_max", "LTEnd_min",
              "UTStart_max", "UTStart_min", "UTEnd_max", "UTEnd_min")


def minmax_tables(lts, lte, uts, ute, block_c):
    """int32 [8, T_c]: max and min of each vector over each block of B_c columns.

    A ragged last block takes its min/max over the columns that exist.
    """
    vecs = [[int(x) for x in _vec(a)] for a in (lts, lte, uts, ute)]
    n = len(vecs[0])
    t_c = (n + block_c - 1) // block_c
    table = np.zeros((8, t_c), dtype=np.int32)
    for j in range(t_c):
        lo, hi = j * block_c, min((j + 1) * block_c, n)
        for a, vec in enumerate(vecs):
            block = vec[lo:hi]
            table[2 * a, j] = max(block)
            table[2 * a + 1, j] = min(block)
    return table


# --------------------------------------------------------------------------
# Tile classification (Equation 4; skip and mask tests of Algorithm 1)
# --------------------------------------------------------------------------
def classify_tiles(table, n, block_r, block_c):
    """uint8 [T_r, T_c] tile classes from the min/max table.

    For a row block covering rows [r0, r1) (r1 clipped to N) and a start/end
    pair: fully masked iff r0 >= Start^max and r1 <= End^min; partially masked
    iff r1 > Start^min and r0 < End^max.  A tile is FULLY if either pair says
    fully; else PARTIAL (with the NEED_* bits of the pairs that say partially);
    else UNMASKED.
    """
    table = np.asarray(table, dtype=np.int64)
    t_r = (n + block_r - 1) // block_r
    t_c = (n + block_c - 1) // block_c
    assert table.shape == (8, t_c)
    cls = np.zeros((t_r, t_c), dtype=np.uint8)
    for i in range(t_r):
        r0 = i * block_r
        r1 = min((i + 1) * block_r, n)
        for j in range(t_c):
            s_max, s_min, e_max, e_min = (int(x) for x in table[0:4, j])
            full_lt = r0 >= s_max and r1 <= e_min
            part_lt = r1 > s_min and r0 < e_max
            s_max, s_min, e_max, e_min = (int(x) for x in table[4:8, j])
            full_ut = r0 >= s_max and r1 <= e_min
            part_ut = r1 > s_min and r0 < e_max
            if full_lt or full_ut:
                cls[i, j] = FULLY
            elif part_lt or part_ut:
                cls[i, j] = PARTIAL | (NEED_LT if part_lt else 0) | (NEED_UT if part_ut else 0)
            else:
                cls[i, j] = UNMASKED
    return cls


def classify_tiles_fast(table, n, block_r, block_c):
    """Same table as classify_tiles, by broadcasting (for N beyond ~16K).

    tests/test_oracle_tables.py checks it equal to the loop version.
    """
    t = np.asarray(table, dtype=np.int64)
    t_r = (n + block_r - 1) // block_r
    r0 = (np.arange(t_r, dtype=np.int64) * block_r)[:, None]
    r1 = np.minimum(r0 + block_r, n)
    full_lt = (r0 >= t[0][None, :]) & (r1 <= t[3][None, :])
    part_lt = (r1 > t[1][None, :]) & (r0 < t[2][None, :])
    full_ut = (r0 >= t[4][None, :]) & (r1 <= t[7][None, :])
    part_ut = (r1 > t[5][None, :]) & (r0 < t[6][None, :])
    full = full_lt | full_ut
    part = (part_lt | part_ut) & ~full
    cls = np.where(full, FULLY, 0).astype(np.uint8)
    cls |= np.where(part, PARTIAL, 0).astype(np.uint8)
    cls |= np.where(part & part_lt, NEED_LT, 0).astype(np.uint8)
    cls |= np.where(part & part_ut, NEED_UT, 0).astype(np.uint8)
    return cls


def tile_kind(cls):
    return np.asarray(cls) & 3


def block_sparsity(cls):
    """rho = (#fully masked tiles) / (T_r * T_c)  (Section 4.3)."""
    kind = tile_kind(cls)
    return float((kind == FULLY).sum()) / float(kind.size)


# --------------------------------------------------------------------------
# Counters for the throughput metric
# --------------------------------------------------------------------------
def count_unmasked_elements(lts, lte, uts, ute):
    """Number of (i, j) pairs with masked[i, j] False, by interval arithmetic
    per column: N minus the size of the union of the two clipped intervals."""
    lts, lte, uts, ute = _vec(lts), _vec(lte), _vec(uts), _vec(ute)
    n = lts.shape[0]
    total = 0
    for j in range(n):
        a0, a1 = max(int(lts[j]), 0), min(int(lte[j]), n)
        b0, b1 = max(int(uts[j]), 0), min(int(ute[j]), n)
        la = max(a1 - a0, 0)
        lb = max(b1 - b0, 0)
        if la > 0 and lb > 0:
            overlap = max(min(a1, b1) - max(a0, b0), 0)
        else:
            overlap = 0
        total += n - (la + lb - overlap)
    return total


def allowed_keys_per_row(lts, lte, uts, ute):
    """c_i = number of keys row i may attend to, in O(N) by difference arrays."""
    lts, lte, uts, ute = _vec(lts), _vec(lte), _vec(uts), _vec(ute)
    n = lts.shape[0]
    diff = np.zeros(n + 1, dtype=np.int64)
    for j in range(n):
        a0, a1 = max(int(lts[j]), 0), min(int(lte[j]), n)
        b0, b1 = max(int(uts[j]), 0), min(int(ute[j]), n)
        ivs = []
        if a1 > a0:
            ivs.append((a0, a1))
        if b1 > b0:
            ivs.append((b0, b1))
        if len(ivs) == 2 and max(a0, b0) < min(a1, b1):      # overlapping: merge
            ivs = [(min(a0, b0), max(a1, b1))]
        for s, e in ivs:
            diff[s] += 1
            diff[e] -= 1
    masked_per_row = np.cumsum(diff[:n])
    return n - masked_per_row


def flops_tile(cls_128, batch_heads, d):
    """Paper-style FLOP count: 4*d*128*128 per non-skipped 128x128 tile for the
    forward pass, 2.5x that for the backward pass (Appendix 'Testing Method';
    the factor 2.5 is the 5-vs-2 matrix products of Algorithms 2 and 1)."""
    live = int((tile_kind(cls_128) != FULLY).sum())
    fw = 4.0 * d * 128 * 128 * live * batch_heads
    return fw, 2.5 * fw


def flops_elem(n_unmasked, batch_heads, d):
    """Strict count: 4*d FLOP per unmasked score element forward, 2.5x backward."""
    fw = 4.0 * d * float(n_unmasked) * batch_heads
    return fw, 2.5 * fw
