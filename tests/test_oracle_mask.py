"""Pins for the oracle's mask expansion (no GPU)."""
import os

import numpy as np
import pytest

import workloads
from oracle import flashmask_oracle as orc
from predicates import PREDICATES

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_paper_interval_example():
    """The one worked interval the paper prints (Section 4.1)."""
    line = [l for l in open(os.path.join(GOLDEN, "paper_interval_example.txt")) if not l.startswith("#")][0]
    vals = [int(x) for x in line.split()]
    lts, lte, uts, ute, n = vals[:5]
    want = set(vals[5:])
    # one column, n rows: pad the vectors so the column count equals n (expand wants square)
    L = np.full(n, n); E = np.full(n, n); U = np.zeros(n, int); V = np.zeros(n, int)
    col = 5
    L[col], E[col], U[col], V[col] = lts, lte, uts, ute
    m = orc.expand_mask(L, E, U, V)
    assert set(np.nonzero(m[:, col])[0].tolist()) == want
    assert not m[:, [c for c in range(n) if c != col]].any()


def brute_force(N, kind, st):
    pred = PREDICATES[kind]
    if isinstance(st, dict):
        st = dict(st, N=N)
    allowed = np.zeros((N, N), dtype=bool)
    for i in range(N):
        for j in range(N):
            allowed[i, j] = pred(i, j, st)
    return allowed


@pytest.mark.parametrize("kind", sorted(PREDICATES))
@pytest.mark.parametrize("N", [8, 13, 32, 64])
def test_expansion_equals_predicate(kind, N):
    for seed in range(6):
        w = workloads.small_workload(kind, N, seed=1000 * N + seed)
        lts, lte, uts, ute = w.vectors[0]
        masked = orc.expand_mask(lts, lte, uts, ute)
        allowed = brute_force(N, kind, w.structure[0])
        assert np.array_equal(~masked, allowed), (kind, N, seed, w.structure[0])


def test_config1_spans_are_the_stated_documents():
    w = workloads.config("1")
    assert w.structure[0] == [(0, 200), (200, 380), (380, 512)]
    masked = orc.expand_mask(*w.vectors[0])
    allowed = brute_force(512, "causal_document", w.structure[0])
    assert np.array_equal(~masked, allowed)


def test_empty_interval_sentinels_and_inverted_pairs():
    n = 10
    # start >= end is empty whatever the values
    L = np.array([5] * n); E = np.array([5, 4, 0, -3, 5, 5, 5, 5, 5, 5])
    U = np.array([9] * n); V = np.array([9, 3, 0, -1, 9, 9, 9, 9, 9, 9])
    assert not orc.expand_mask(L, E, U, V).any()
    # out-of-range bounds are simply clipped by the row range
    m = orc.expand_mask(np.full(n, -7), np.full(n, 3), np.full(n, 8), np.full(n, 99))
    assert np.array_equal(np.nonzero(m[:, 0])[0], [0, 1, 2, 8, 9])


def test_counters_match_dense_counts():
    for kind in sorted(PREDICATES) + ["random_intervals"]:
        for seed in range(4):
            w = workloads.small_workload(kind, 48, seed=77 + seed)
            v = w.vectors[0]
            masked = orc.expand_mask(*v)
            assert orc.count_unmasked_elements(*v) == int((~masked).sum())
            assert np.array_equal(orc.allowed_keys_per_row(*v), (~masked).sum(axis=1))


def test_large_configs_have_no_dead_rows_and_right_shapes():
    for name in workloads.CONFIG_NAMES:
        w = workloads.config(name)
        assert len(w.vectors) == w.B
        for v in w.vectors:
            assert all(a.shape == (w.N,) and a.dtype == np.int32 for a in v)
            c = orc.allowed_keys_per_row(*v)
            assert c.min() >= 1          # every token sees at least itself
