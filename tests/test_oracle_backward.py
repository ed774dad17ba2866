"""Pins for the oracle's gradients (no GPU)."""
import math

import numpy as np
import pytest
import torch

import workloads
from oracle import flashmask_oracle as orc
from predicates import PREDICATES

KINDS = sorted(PREDICATES)


def rand(seed, n, d):
    rng = np.random.default_rng(seed)
    return tuple(rng.standard_normal((n, d)) for _ in range(4))


@pytest.mark.parametrize("kind", KINDS + ["random_intervals"])
@pytest.mark.parametrize("n,d", [(7, 3), (16, 8)])
def test_gradients_match_central_finite_differences(kind, n, d):
    w = workloads.small_workload(kind, n, seed=31 + n)
    vec = w.vectors[0]
    q, k, v, do = rand(n, n, d)
    scale = 0.6
    dq, dk, dv, out, lse = orc.backward(q, k, v, do, *vec, scale)

    def loss(q_, k_, v_):
        o, _ = orc.forward(q_, k_, v_, *vec, scale)
        return float((o * do).sum())

    eps = 1e-6
    rng = np.random.default_rng(5)
    for arr, grad, which in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        idx = [(int(rng.integers(n)), int(rng.integers(d))) for _ in range(12)] + [(0, 0), (n - 1, d - 1)]
        for (r, c) in idx:
            args = [q.copy(), k.copy(), v.copy()]
            args[which][r, c] += eps
            up = loss(*args)
            args[which][r, c] -= 2 * eps
            dn = loss(*args)
            fd = (up - dn) / (2 * eps)
            assert abs(fd - grad[r, c]) < 1e-7 * max(1.0, abs(fd)), (kind, which, r, c, fd, grad[r, c])


@pytest.mark.parametrize("kind", KINDS + ["random_intervals"])
def test_gradients_match_library_autograd(kind):
    n, d = 24, 8
    w = workloads.small_workload(kind, n, seed=3)
    vec = w.vectors[0]
    q, k, v, do = rand(1, n, d)
    scale = 1 / math.sqrt(d)
    dq, dk, dv, out, lse = orc.backward(q, k, v, do, *vec, scale)
    allowed = ~orc.expand_mask(*vec)
    live = allowed.any(axis=1)
    tq, tk, tv = (torch.from_numpy(x).clone().requires_grad_(True) for x in (q, k, v))
    s = scale * tq @ tk.T
    s = s.masked_fill(torch.from_numpy(~allowed), -math.inf)
    s = torch.where(torch.from_numpy(live)[:, None], s, torch.zeros_like(s))
    p = torch.softmax(s, dim=1) * torch.from_numpy(live)[:, None]
    (p @ tv * torch.from_numpy(do)).sum().backward()
    assert np.allclose(dq, tq.grad.numpy(), atol=1e-11)
    assert np.allclose(dk, tk.grad.numpy(), atol=1e-11)
    assert np.allclose(dv, tv.grad.numpy(), atol=1e-11)


@pytest.mark.parametrize("kind", KINDS + ["random_intervals"])
def test_gradient_invariants(kind):
    n, d = 36, 8
    w = workloads.small_workload(kind, n, seed=8)
    vec = w.vectors[0]
    q, k, v, do = rand(2, n, d)
    dq, dk, dv, out, lse = orc.backward(q, k, v, do, *vec, 0.4)
    masked = orc.expand_mask(*vec)
    live = ~masked.all(axis=1)
    # sum_j dV_j = sum over live rows of dO_i  (rows of P sum to one)
    assert np.allclose(dv.sum(axis=0), do[live].sum(axis=0), atol=1e-11)
    # a key column no row may see receives no gradient at all
    unseen = masked.all(axis=0)
    assert np.all(dk[unseen] == 0.0) and np.all(dv[unseen] == 0.0)
    # a row with no visible key has zero dq
    assert np.all(dq[~live] == 0.0)
    # D = rowsum(dO o O) equals rowsum(P o dP)  (Algorithm 2, D pre-pass)
    p = orc.probabilities(q, k, *vec, 0.4)
    assert np.allclose((do * out).sum(axis=1), (p * (do @ v.T)).sum(axis=1), atol=1e-11)


def test_partial_backward_helpers_equal_full():
    n, d = 50, 8
    w = workloads.small_workload("causal_document", n, seed=4)
    vec = w.vectors[0]
    q, k, v, do = rand(6, n, d)
    dq, dk, dv, _, _ = orc.backward(q, k, v, do, *vec, 0.25)
    rows = np.array([0, 49, 13, 27])
    cols = np.array([1, 48, 20])
    assert np.allclose(orc.backward_rows(q, k, v, do, *vec, 0.25, rows), dq[rows], atol=1e-13)
    dk2, dv2 = orc.backward_cols(q, k, v, do, *vec, 0.25, cols)
    assert np.allclose(dk2, dk[cols], atol=1e-13) and np.allclose(dv2, dv[cols], atol=1e-13)


@pytest.mark.parametrize("heads,kv_heads", [(4, 2), (3, 1), (6, 3)])
def test_grouped_head_gradients_match_central_finite_differences(heads, kv_heads):
    """K/V heads shared by several query heads: dk, dv of a K/V head are the derivatives of the
    loss summed over ALL heads, which is what finite differences of that loss see."""
    n, d, scale = 12, 4, 0.7
    w = workloads.small_workload("causal_document", n, seed=41)
    vec = w.vectors[0]
    rng = np.random.default_rng(17)
    q, do = rng.standard_normal((heads, n, d)), rng.standard_normal((heads, n, d))
    k, v = rng.standard_normal((kv_heads, n, d)), rng.standard_normal((kv_heads, n, d))
    dq, dk, dv, out, lse = orc.backward_grouped(q, k, v, do, *vec, scale)
    group = heads // kv_heads

    def loss(q_, k_, v_):
        return sum(float((orc.forward(q_[h], k_[h // group], v_[h // group], *vec, scale)[0] * do[h]).sum())
                   for h in range(heads))

    eps = 1e-6
    for arr, grad, which in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        for _ in range(10):
            idx = tuple(int(rng.integers(sz)) for sz in arr.shape)
            args = [q.copy(), k.copy(), v.copy()]
            args[which][idx] += eps
            up = loss(*args)
            args[which][idx] -= 2 * eps
            dn = loss(*args)
            fd = (up - dn) / (2 * eps)
            assert abs(fd - grad[idx]) < 1e-7 * max(1.0, abs(fd)), (which, idx, fd, grad[idx])


# --- the chunked paths: every loop over chunks of query rows, run with several chunks -------------
CHUNKED_KINDS = ["document", "shared_question", "random_intervals", "causal_document", "sliding_window"]


class small_chunks:
    """Run the oracle with chunks of 7 query rows, so that N ~ 50 spans eight chunks."""

    def __enter__(self):
        self.old = orc.ROW_CHUNK
        orc.ROW_CHUNK = 7

    def __exit__(self, *exc):
        orc.ROW_CHUNK = self.old


@pytest.mark.parametrize("kind", CHUNKED_KINDS)
def test_chunked_backward_matches_central_finite_differences(kind):
    """The accumulation of dk and dv across row chunks in backward(): finite differences of the
    loss (forward also chunked) against gradients computed over eight chunks."""
    n, d, scale = 53, 5, 0.45
    w = workloads.small_workload(kind, n, seed=77)
    vec = w.vectors[0]
    q, k, v, do = rand(n + 3, n, d)
    with small_chunks():
        dq, dk, dv, out, lse = orc.backward(q, k, v, do, *vec, scale)

        def loss(q_, k_, v_):
            o, _ = orc.forward(q_, k_, v_, *vec, scale)
            return float((o * do).sum())

        eps = 1e-6
        rng = np.random.default_rng(9)
        for grad, which in ((dq, 0), (dk, 1), (dv, 2)):
            # rows of every chunk, first and last chunk included
            idx = [(int(r), int(rng.integers(d))) for r in list(range(0, n, 5)) + [n - 1]]
            for (r, c) in idx:
                args = [q.copy(), k.copy(), v.copy()]
                args[which][r, c] += eps
                up = loss(*args)
                args[which][r, c] -= 2 * eps
                dn = loss(*args)
                fd = (up - dn) / (2 * eps)
                assert abs(fd - grad[r, c]) < 1e-7 * max(1.0, abs(fd)), (kind, which, r, c, fd, grad[r, c])
    # and the chunking itself is invisible: one chunk gives the same arrays
    dq1, dk1, dv1, out1, lse1 = orc.backward(q, k, v, do, *vec, scale)
    for a, b in ((dq, dq1), (dk, dk1), (dv, dv1), (out, out1)):
        assert np.allclose(a, b, atol=1e-13)
    assert np.array_equal(np.isneginf(lse), np.isneginf(lse1))
    assert np.allclose(lse[np.isfinite(lse)], lse1[np.isfinite(lse1)], atol=1e-13)


@pytest.mark.parametrize("kind", CHUNKED_KINDS)
def test_chunked_partial_helpers_equal_full(kind):
    """backward_rows and backward_cols over several chunks (the row list, and the live rows of the
    listed columns, both span more than one chunk) against the single-chunk full backward, which the
    finite-difference tests pin."""
    n, d, scale = 50, 6, 0.3
    w = workloads.small_workload(kind, n, seed=12)
    vec = w.vectors[0]
    q, k, v, do = rand(21, n, d)
    dq, dk, dv, _, _ = orc.backward(q, k, v, do, *vec, scale)     # ROW_CHUNK = 1024: one chunk
    rng = np.random.default_rng(3)
    rows = rng.permutation(n)[:31]                                # unsorted, five chunks of seven
    cols = np.array(sorted(set(rng.integers(0, n, 9).tolist()) | {0, n - 1}))
    masked = orc.expand_mask(*vec)
    live_rows = int((~masked[:, cols].all(axis=1)).sum())
    with small_chunks():
        got_dq = orc.backward_rows(q, k, v, do, *vec, scale, rows)
        got_dk, got_dv = orc.backward_cols(q, k, v, do, *vec, scale, cols)
    if kind != "random_intervals":
        assert live_rows > 2 * 7, "the listed columns must be seen by rows of several chunks"
    assert np.allclose(got_dq, dq[rows], atol=1e-13)
    assert np.allclose(got_dk, dk[cols], atol=1e-13) and np.allclose(got_dv, dv[cols], atol=1e-13)


def test_backward_cols_live_row_filter_on_bidirectional_and_two_interval_masks():
    """The rows backward_cols skips (those that see none of the listed columns) add nothing: compare
    with the same sums taken over ALL rows, written out here, on masks with both intervals in use."""
    n, d, scale = 40, 4, 0.5
    for kind, seed in (("document", 5), ("global_sliding_window", 6), ("prefix_document", 7), ("random_intervals", 8)):
        w = workloads.small_workload(kind, n, seed=seed)
        vec = w.vectors[0]
        q, k, v, do = rand(seed, n, d)
        p = orc.probabilities(q, k, *vec, scale)
        out = p @ v
        ds = p * (do @ v.T - (do * out).sum(axis=1)[:, None])
        cols = np.array([0, 7, 19, 20, 39])
        with small_chunks():
            got_dk, got_dv = orc.backward_cols(q, k, v, do, *vec, scale, cols)
        assert np.allclose(got_dv, (p.T @ do)[cols], atol=1e-13)
        assert np.allclose(got_dk, scale * (ds.T @ q)[cols], atol=1e-13)
