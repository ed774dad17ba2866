"""Pins for tests/closed_forms.py (no GPU): the range tables against the mask families' predicates, the
blocked prefix routine against the plain sum, and the uniform-probability closed forms against the
oracle's dense gradients with Q = 0 and with K = 0.  The last one is also a pin of the oracle: two
derivations that share no code (dense Algorithm 2 / prefix sums over the task structure) must agree."""
import numpy as np
import pytest

import closed_forms as cf
import workloads
from oracle import flashmask_oracle as orc
from predicates import PREDICATES


def _workload(kind, n, seed):
    w = workloads.small_workload(kind, n, seed=seed)
    return w, w.vectors[0], cf.ranges_of(w, 0)


@pytest.mark.parametrize("kind", ["causal_document", "sliding_window", "prefix_lm"])
@pytest.mark.parametrize("n", [2, 9, 40])
def test_ranges_are_the_predicates(kind, n):
    for seed in range(4):
        w, vec, (a, e, r, bb) = _workload(kind, n, 50 + seed)
        pred = PREDICATES[kind]
        st = w.structure[0]
        for i in range(n):
            for j in range(n):
                allowed = pred(i, j, st)
                assert allowed == (a[i] <= j < e[i]), (kind, i, j)
                assert allowed == (r[j] <= i < bb[j]), (kind, i, j)
        for x in (a, e, r, bb):
            assert np.all(np.diff(x) >= 0)


@pytest.mark.parametrize("block", [1, 3, 192])
def test_prefix_apply_is_the_plain_sum(block):
    rng = np.random.default_rng(4)
    m, t, d = 37, 29, 5
    A, B, U = rng.standard_normal((m, d)), rng.standard_normal((m, d)), rng.standard_normal((t, d))
    for x in (np.sort(rng.integers(0, m + 1, t)), np.zeros(t, dtype=np.int64), np.full(t, m),
              np.minimum(np.arange(t) + 4, m), np.repeat([0, 11, 30], [9, 10, 10])):
        got = cf.prefix_apply(A, B, x, U, block=block)
        for k in range(t):
            want = sum((A[i] * (B[i] @ U[k]) for i in range(int(x[k]))), np.zeros(d))
            assert np.allclose(got[k], want, atol=1e-11)


@pytest.mark.parametrize("kind", ["causal_document", "sliding_window", "prefix_lm"])
@pytest.mark.parametrize("which_zero", ["q", "k"])
def test_closed_forms_equal_the_dense_oracle(kind, which_zero):
    n, d, scale = 230, 6, 0.37
    for seed in (1, 2):
        w, vec, (a, e, r, bb) = _workload(kind, n, 90 + seed)
        rng = np.random.default_rng(seed)
        q, k, v, do = (rng.standard_normal((n, d)) for _ in range(4))
        if which_zero == "q":
            q = np.zeros_like(q)
        else:
            k = np.zeros_like(k)
        dq, dk, dv, out, lse = orc.backward(q, k, v, do, *vec, scale)
        lse_c, out_c = cf.forward_uniform(v, a, e)
        dq_c, dk_c, dv_c = cf.backward_uniform(q, k, v, do, scale, a, e, r, bb)
        assert np.allclose(lse, lse_c, atol=1e-12) and np.allclose(out, out_c, atol=1e-12)
        assert np.allclose(dv, dv_c, atol=1e-11)
        assert np.allclose(dq, dq_c, atol=1e-11) and np.allclose(dk, dk_c, atol=1e-11)
        if which_zero == "q":
            assert np.all(dk_c == 0.0) and np.abs(dq_c).max() > 1e-3
        else:
            assert np.all(dq_c == 0.0) and np.abs(dk_c).max() > 1e-3
