"""GPU: parity at the full benchmark sizes, in the launch configuration bench.py
times, on sampled outputs the oracle computes one by one.

out / lse / dq are checked on sampled query rows (each needs only its own row of
scores); dk / dv on sampled key columns (the oracle evaluates every query row
that may see one of them).  A closed form that holds at any size covers every
head: with Q = 0, lse_i = log(#keys row i may see)."""
import math

import numpy as np
import pytest
import torch

import workloads
from gpu_util import ABS_FWD, bf16_to_np, check_bwd, check_fwd, f64, to_device
from oracle import flashmask_oracle as orc

pytestmark = pytest.mark.gpu


def sample_rows(w, vec, rng, n_random=96):
    n = w.N
    edges = set()
    for arr in vec:
        for x in np.unique(arr)[:64]:
            for dx in (-1, 0, 1):
                if 0 <= x + dx < n:
                    edges.add(int(x + dx))
    edges = sorted(edges)[:96]
    tiles = [t * 128 + o for t in rng.integers(0, n // 128, 8) for o in (0, 63, 64, 127)]
    rows = np.unique(np.concatenate([[0, n - 1], edges, tiles, rng.integers(0, n, n_random)])).astype(np.int64)
    return rows


def sample_cols(w, vec, rng, row_budget=6144):
    """Key columns whose sets of visible rows stay within a row budget."""
    n = w.N
    lts, lte, uts, ute = (np.asarray(a, dtype=np.int64) for a in vec)
    cand = np.unique(np.concatenate([[0, n - 1], rng.integers(0, n, 400),
                                     np.clip(np.unique(lts)[:40] - 1, 0, n - 1), np.clip(np.unique(lts)[:40] - 2, 0, n - 1)]))
    rng.shuffle(cand)
    chosen, live = [], np.zeros(n, dtype=bool)
    for j in cand:
        col_live = ~orc.expand_mask(lts[[j]], lte[[j]], uts[[j]], ute[[j]], np.arange(n))[:, 0]
        if (live | col_live).sum() <= row_budget:
            live |= col_live
            chosen.append(int(j))
        if len(chosen) >= 48:
            break
    return np.array(sorted(chosen), dtype=np.int64)


@pytest.mark.parametrize("name", ["2", "3", "4a", "4b", "5"])
def test_config_parity_on_sampled_outputs(name):
    import paper_2410_01359_amd as fm
    w = workloads.config(name)
    bits, dev, vecs = to_device(w)
    out, lse = fm.flashmask_fwd(dev["q"], dev["k"], dev["v"], *vecs, w.scale)
    dq, dk, dv = fm.flashmask_bwd(dev["q"], dev["k"], dev["v"], out, lse, dev["dout"], *vecs, w.scale)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    for t in (dq, dk, dv):
        assert torch.isfinite(t.float()).all()
    rng = np.random.default_rng(w.seed)
    heads = sorted({0, w.H - 1})
    for b in range(w.B):
        vec = w.vectors[b]
        rows = sample_rows(w, vec, rng)
        cols = sample_cols(w, vec, rng)
        assert len(cols) >= 8
        for h in heads:
            args = [f64(bits[n][b, h]) for n in ("q", "k", "v", "dout")]
            what = f"config {name} b={b} h={h}"
            ro, rl = orc.forward_rows(args[0], args[1], args[2], *vec, w.scale, rows)
            check_fwd(bf16_to_np(out[b, h][rows]), lse[b, h][rows].cpu().numpy(), ro, rl, what)
            rdq = orc.backward_rows(*args, *vec, w.scale, rows)
            check_bwd(bf16_to_np(dq[b, h][rows]), rdq, "dq", what)
            rdk, rdv = orc.backward_cols(*args, *vec, w.scale, cols)
            check_bwd(bf16_to_np(dk[b, h][cols]), rdk, "dk", what)
            check_bwd(bf16_to_np(dv[b, h][cols]), rdv, "dv", what)


@pytest.mark.parametrize("name", ["2", "3", "4a", "4b", "5"])
def test_config_zero_query_closed_form_every_head(name):
    """Q = 0 => every score is 0: lse_i = log(c_i) and out_i = mean of the visible
    V rows, for every row of every head, with c_i from interval arithmetic."""
    import paper_2410_01359_amd as fm
    w = workloads.config(name)
    bits, dev, vecs = to_device(w, ("q", "v"))
    q0 = torch.zeros_like(dev["q"])
    # keys irrelevant when q = 0; reuse v as k
    out, lse = fm.flashmask_fwd(q0, dev["v"], dev["v"], *vecs, w.scale)
    torch.cuda.synchronize()
    for b in range(w.B):
        c = orc.allowed_keys_per_row(*w.vectors[b]).astype(np.float64)
        want = torch.from_numpy(np.log(c)).cuda()
        err = (lse[b].double() - want[None, :]).abs().max().item()
        assert err <= ABS_FWD, f"config {name} b={b}: lse vs log(count) max-abs {err}"
    # causal-type masks of these configs: visible keys of row i form one or two prefix-sum ranges;
    # check out on sampled rows of head 0 against the oracle's row routine with q = 0
    rng = np.random.default_rng(1)
    rows = np.unique(rng.integers(0, w.N, 64))
    v0 = f64(bits["v"][0, 0])
    ro, _ = orc.forward_rows(np.zeros_like(v0), v0, v0, *w.vectors[0], w.scale, rows)
    got = bf16_to_np(out[0, 0][rows])
    assert np.abs(got - ro).max() <= ABS_FWD


OTHER_FAMILIES = ["document", "prefix_document", "global_sliding_window", "causal_blockwise", "random_eviction",
                  "qk_sparse", "random_intervals"]


@pytest.mark.parametrize("kind", OTHER_FAMILIES)
def test_other_mask_families_at_16k(kind):
    """The mask families outside the five configurations (both interval pairs active, union
    covers, mostly-partial tiles), at N = 16384, d = 128, on sampled rows and columns."""
    import paper_2410_01359_amd as fm
    w = workloads.small_workload(kind, 16384, seed=4100 + len(kind), B=1, H=2, d=128)
    bits, dev, vecs = to_device(w)
    out, lse = fm.flashmask_fwd(dev["q"], dev["k"], dev["v"], *vecs, w.scale)
    dq, dk, dv = fm.flashmask_bwd(dev["q"], dev["k"], dev["v"], out, lse, dev["dout"], *vecs, w.scale)
    torch.cuda.synchronize()
    rng = np.random.default_rng(w.seed)
    vec = w.vectors[0]
    rows = sample_rows(w, vec, rng, n_random=64)
    cols = sample_cols(w, vec, rng, row_budget=8192)
    for h in range(w.H):
        args = [f64(bits[n][0, h]) for n in ("q", "k", "v", "dout")]
        what = f"{kind} N=16384 h={h}"
        ro, rl = orc.forward_rows(args[0], args[1], args[2], *vec, w.scale, rows)
        check_fwd(bf16_to_np(out[0, h][rows]), lse[0, h][rows].cpu().numpy(), ro, rl, what)
        rdq = orc.backward_rows(*args, *vec, w.scale, rows)
        check_bwd(bf16_to_np(dq[0, h][rows]), rdq, "dq", what)
        if len(cols):
            rdk, rdv = orc.backward_cols(*args, *vec, w.scale, cols)
            check_bwd(bf16_to_np(dk[0, h][cols]), rdk, "dk", what)
            check_bwd(bf16_to_np(dv[0, h][cols]), rdv, "dv", what)
    # every head: with Q = 0, lse = log(number of visible keys), -inf where a row sees nothing
    out0, lse0 = fm.flashmask_fwd(torch.zeros_like(dev["q"]), dev["v"], dev["v"], *vecs, w.scale)
    torch.cuda.synchronize()
    c = orc.allowed_keys_per_row(*vec).astype(np.float64)
    with np.errstate(divide="ignore"):
        want = np.log(c)
    got = lse0[0].cpu().numpy().astype(np.float64)
    assert np.array_equal(np.isneginf(got), np.isneginf(want)[None, :].repeat(w.H, 0))
    fin = np.isfinite(want)
    assert np.abs(got[:, fin] - want[fin][None, :]).max() <= ABS_FWD
