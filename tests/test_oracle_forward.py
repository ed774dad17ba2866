"""Pins for the oracle's forward pass (no GPU)."""
import math

import numpy as np
import pytest
import torch

import workloads
from oracle import flashmask_oracle as orc
from predicates import PREDICATES

KINDS = sorted(PREDICATES)


def rand_qkv(seed, n, d):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n, d)), rng.standard_normal((n, d)), rng.standard_normal((n, d)))


def test_empty_mask_is_textbook_softmax_attention():
    n, d = 40, 16
    q, k, v = rand_qkv(0, n, d)
    scale = 0.37
    out, lse = orc.forward(q, k, v, *workloads.full_mask(n), scale)
    # written out element by element, no shared helper
    for i in range(n):
        s = [scale * sum(q[i, c] * k[j, c] for c in range(d)) for j in range(n)]
        z = sum(math.exp(x) for x in s)
        want = [sum(math.exp(s[j]) / z * v[j, c] for j in range(n)) for c in range(d)]
        assert np.allclose(out[i], want, rtol=1e-12, atol=1e-12)
        assert abs(lse[i] - math.log(z)) < 1e-12


@pytest.mark.parametrize("kind", KINDS + ["random_intervals"])
def test_matches_library_sdpa_with_dense_mask(kind):
    """Any expanded mask: equal to a library's fp64 scaled-dot-product attention
    fed the dense boolean mask (cross-check only; rows with no key excluded)."""
    n, d = 48, 8
    for seed in range(3):
        w = workloads.small_workload(kind, n, seed=seed + 5)
        vec = w.vectors[0]
        q, k, v = rand_qkv(seed, n, d)
        scale = 1.0 / math.sqrt(d)
        out, lse = orc.forward(q, k, v, *vec, scale)
        allowed = ~orc.expand_mask(*vec)
        live = allowed.any(axis=1)
        tq, tk, tv = (torch.from_numpy(x)[None, None] for x in (q, k, v))
        am = torch.from_numpy(allowed | ~live[:, None])[None, None]   # give dead rows something
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=am, scale=scale)[0, 0].numpy()
        assert np.allclose(out[live], ref[live], rtol=1e-10, atol=1e-12)
        s = torch.from_numpy(scale * q @ k.T).masked_fill(torch.from_numpy(~allowed), -math.inf)
        ref_lse = torch.logsumexp(s, dim=1).numpy()
        assert np.allclose(lse[live], ref_lse[live], rtol=1e-12, atol=1e-12)
        # rows with every key masked: zero output, lse = -inf
        assert np.all(out[~live] == 0.0)
        assert np.all(np.isneginf(lse[~live]))


@pytest.mark.parametrize("kind", KINDS)
def test_zero_query_closed_form(kind):
    """Q = 0 => S = 0: lse_i = log(#allowed keys), out_i = mean of allowed V rows,
    with the allowed set taken from the family's predicate, not from the oracle."""
    n, d = 33, 4
    w = workloads.small_workload(kind, n, seed=11)
    st = w.structure[0]
    if isinstance(st, dict):
        st = dict(st, N=n)
    _, k, v = rand_qkv(3, n, d)
    out, lse = orc.forward(np.zeros((n, d)), k, v, *w.vectors[0], 0.5)
    for i in range(n):
        cols = [j for j in range(n) if PREDICATES[kind](i, j, st)]
        if not cols:       # a row that sees no key (a dropped query): out = 0, lse = -inf
            assert np.isneginf(lse[i]) and np.all(out[i] == 0.0)
            continue
        assert abs(lse[i] - math.log(len(cols))) < 1e-12
        assert np.allclose(out[i], v[cols].mean(axis=0), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("kind", KINDS + ["random_intervals"])
def test_softmax_rows_and_invariants(kind):
    n, d = 40, 8
    w = workloads.small_workload(kind, n, seed=21)
    vec = w.vectors[0]
    q, k, v = rand_qkv(4, n, d)
    masked = orc.expand_mask(*vec)
    p = orc.probabilities(q, k, *vec, 0.3)
    live = ~masked.all(axis=1)
    assert np.allclose(p[live].sum(axis=1), 1.0, atol=1e-12)
    assert np.all(p[masked] == 0.0)
    assert np.all(p[~live] == 0.0)
    # identical V rows => every live output row equals that row
    v0 = np.arange(d, dtype=float)
    out, _ = orc.forward(q, k, np.tile(v0, (n, 1)), *vec, 0.3)
    assert np.allclose(out[live], v0, atol=1e-12)
    assert np.all(out[~live] == 0.0)
    # adding the same vector to every key shifts each row's scores by a row constant:
    # out unchanged, lse shifted by scale * q_i . delta
    delta = np.linspace(-1, 1, d)
    out1, lse1 = orc.forward(q, k, v, *vec, 0.3)
    out2, lse2 = orc.forward(q, k + delta, v, *vec, 0.3)
    assert np.allclose(out1[live], out2[live], atol=1e-11)
    assert np.allclose(lse2[live] - lse1[live], 0.3 * (q @ delta)[live], atol=1e-11)


def test_forward_rows_equals_full_and_chunking_is_invisible():
    n, d = 70, 8
    w = workloads.small_workload("shared_question", n, seed=2)
    q, k, v = rand_qkv(9, n, d)
    out, lse = orc.forward(q, k, v, *w.vectors[0], 0.2)
    rows = np.array([0, 3, 17, 69, 41])
    o2, l2 = orc.forward_rows(q, k, v, *w.vectors[0], 0.2, rows)
    assert np.array_equal(o2, out[rows]) and np.array_equal(l2, lse[rows])
    old = orc.ROW_CHUNK
    try:
        orc.ROW_CHUNK = 7
        o3, l3 = orc.forward(q, k, v, *w.vectors[0], 0.2)
    finally:
        orc.ROW_CHUNK = old
    assert np.allclose(o3, out, atol=1e-14) and np.allclose(l3, lse, atol=1e-14)


def test_large_n_closed_form_without_dense_work():
    """N = 131072 (config 5's mask): lse = log(c_i) on sampled rows, with c_i
    from the document spans directly."""
    w = workloads.config("5")
    spans = w.structure[0]
    n, d = w.N, 4
    rng = np.random.default_rng(0)
    v = rng.standard_normal((n, d))
    rows = np.unique(np.concatenate([[0, n - 1], [s for s, _ in spans], [e - 1 for _, e in spans],
                                     rng.integers(0, n, 64)]))
    out, lse = orc.forward_rows(np.zeros((n, d)), np.zeros((n, d)), v, *w.vectors[0], 1.0, rows)
    csum = np.concatenate([np.zeros((1, d)), np.cumsum(v, axis=0)])
    for r, i in enumerate(rows):
        s = [s for s, e in spans if s <= i < e][0]
        cnt = i - s + 1
        assert abs(lse[r] - math.log(cnt)) < 1e-10
        assert np.allclose(out[r], (csum[i + 1] - csum[s]) / cnt, atol=1e-9)
